// Internal declarations shared by the HIP translation units of libdsnet.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "dsnet.h"

typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even float -> bf16 through the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16_t f2bf(float f) {
    const __bf16 b = (__bf16)f;
    return __builtin_bit_cast(bf16_t, b);
}
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
// two floats -> packed bf16 pair (lo in bits 0..15)
__device__ __forceinline__ uint32_t f2bf2(float lo, float hi) {
    const f32x2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}

// ---- error reporting --------------------------------------------------------
void ds_set_error(const char* fmt, ...);
#define DS_FAIL(code, ...)            \
    do {                              \
        ds_set_error(__VA_ARGS__);    \
        return (code);                \
    } while (0)
#define DS_CHECK_LAUNCH(what)                                                  \
    do {                                                                       \
        hipError_t e__ = hipGetLastError();                                    \
        if (e__ != hipSuccess) DS_FAIL(DS_EHIP, "%s: %s", what, hipGetErrorString(e__)); \
    } while (0)

// reserves `bytes` of dynamic LDS for a kernel: once per (device, kernel), safe to call from any thread
int32_t ds_reserve_lds(const void* kernel, int bytes, const char* what);

static inline bool ds_aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }
static inline size_t ds_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- group table passed by value to kernels ---------------------------------
struct GroupTable {
    int32_t T;
    int32_t k_in[DS_MAX_GROUPS];
    int32_t k_out[DS_MAX_GROUPS];
    int32_t row[DS_MAX_GROUPS];
};

// per-group spatial slice of a stored KS x KS filter (Section 3.2, Eq. 11-13): the taps k0 + i*l, i < n, per axis
// (centred k x k block, every l-th tap), applied at dilation l with `pad` zeros per side
struct SpatialTable {
    int32_t k0[DS_MAX_GROUPS];
    int32_t n[DS_MAX_GROUPS];
    int32_t l[DS_MAX_GROUPS];
    int32_t pad[DS_MAX_GROUPS];
};

// ---- grouped GEMM / implicit-GEMM convolution -------------------------------
#define DS_GEMM_BM 128

struct GemmArgs {
    // operands
    const bf16_t* A;       // activations
    const bf16_t* Wt;      // weights [N_full][KK][w_tap_stride] (w_ld elements per output row)
    void* C;               // output
    const bf16_t* R;       // residual (nullable), addressed like C unless r_sample_stride is set
    const float* scale;    // [rows][tab_ld] nullable (=1)
    const float* shift;    // [rows][tab_ld] nullable (=0)
    // addressing: element offset of (slot, local row p, col) =
    //   index[slot] * sample_stride + (p + row0) * ld + col ;  ld <= 0 -> group's own width
    const int32_t* a_index;  // slot -> sample (nullable = identity)
    const int32_t* c_index;
    int64_t a_sample_stride, c_sample_stride, r_sample_stride;
    int32_t a_ld, c_ld, r_ld;
    int32_t c_row0;          // output/residual row shift inside a sample
    int32_t r_use_index;     // 0: residual ignores c_index (broadcast table such as a position embedding)
    // weights
    int64_t w_ld, w_tap_stride, w_seg_stride, c_seg_stride;
    int32_t n_seg, tab_ld, tab_seg_stride;
    // geometry: rows of a sample are the Ho*Wo output pixels of a KxK convolution over HxW
    int32_t H, W, Ho, Wo, K, stride, pad, rows;
    int32_t Kw, stride_w;    // filter width and horizontal stride where they differ from K / stride (0 = the same)
    // schedule
    const int32_t* offsets;  // device [T+1] slots
    const int4* mtiles;      // device [(group, first row inside group, first slot, rows of group)]
    const int32_t* n_mtiles; // device scalar
    int32_t act, out_f32;
    GroupTable gt;
};

size_t ds_mtile_capacity(int32_t B, int32_t rows, int32_t T);
// builds the m-tile list for (offsets, rows); list needs ds_mtile_capacity()*16 + 16 bytes
int32_t ds_build_mtiles(const int32_t* offsets, int32_t T, int32_t rows, void* list, hipStream_t s);
int32_t ds_launch_gemm(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s);
// 1x1 / linear layers with input slices of at most 64 channels and several 64-column passes: one workgroup per 128 rows
// and all their columns; DS_EUNSUPPORTED otherwise
int32_t ds_launch_thin(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s);
// a second 1x1 layer applied to the rows of a thin layer before they leave the workgroup (Section 3.2: the next
// bottleneck's first convolution reads exactly the rows the previous bottleneck's last convolution wrote)
struct ThinChain {
    const bf16_t* Wt;              // [N2_full][w_ld]; its input slice is the first layer's output slice
    const float *scale, *shift;    // [rows][tab_ld], row = the group's row of the first layer; nullable (1 / 0)
    bf16_t* C;                     // second output: c_index[slot] * c_sample_stride + p * c_ld + col
    int64_t w_ld, c_sample_stride;
    int32_t c_ld, tab_ld, act;     // c_ld <= 0: the group's own width
    int32_t k_out[DS_MAX_GROUPS];  // per group; <= 0: the group ends with the first layer
};
int32_t ds_launch_thin_chain(const GemmArgs& a, const ThinChain& ch, int32_t max_mtiles, int32_t max_kout, hipStream_t s);
// 3x3 stride-1 padding-1 layers on maps up to 59 pixels wide; DS_EUNSUPPORTED for any other shape
int32_t ds_launch_conv3(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s);

static inline const int4* ds_mtile_entries(const void* list) { return (const int4*)((const char*)list + 16); }
static inline const int32_t* ds_mtile_count(const void* list) { return (const int32_t*)list; }

// ---- routing agent ------------------------------------------------------------
constexpr int POOL_SPLIT_MAX = 8;   // most partial sums per (item, channel) the spatial pool leaves for its consumer
struct GateArgs {
    const void* x;            // feature maps; nullptr = route on logit_bias alone
    int32_t dtype, layout;
    int32_t B, C, HW;         // items, stored channels, pixels
    const int32_t* c_in;      // per item valid channels (nullable = C)
    const int32_t* x_index;   // item -> sample block in x (nullable = identity)
    int64_t x_sample_stride;
    int32_t x_ld;             // NHWC row stride; <= 0 -> the item's own channel count
    const float *w1, *b1, *w2, *b2;
    int32_t C_mlp, T;
    const float* logit_bias;        // [*, T] indexed by output row, nullable
    const int32_t* out_index;       // item -> output row (nullable = identity)
    const int32_t* route_override;  // indexed by output row, nullable
    float* logits;
    int32_t* route;
    float* partial;           // [B][splits][C] scratch
};
size_t ds_gate_partial_bytes(int32_t B, int32_t C);
int32_t ds_launch_gate(const GateArgs& a, hipStream_t s);
// y[b][p][c] = x[b][p][c] * scale[b][c] on the valid channels (NHWC) / y[b][c][p] (NCHW); fp32 or bf16
int32_t ds_launch_channel_scale(const void* x, void* y, const float* scale, const int32_t* c_in, int32_t dtype,
                                int32_t layout, int32_t B, int32_t C, int32_t HW, hipStream_t s);
struct BucketArgs {
    const int32_t* route;     // [B]
    const int32_t* lo;        // nullable: key = route * mul + lo
    int32_t mul, B, T;
    int32_t *perm, *inv_perm, *offsets, *slot_group;   // inv_perm, slot_group nullable
    const int32_t* inv_prev;  // with src_index: src_index[slot] = inv_prev ? inv_prev[sample] : sample
    int32_t* src_index;       // nullable
    // optional extras done by the same launch (T <= DS_MAX_GROUPS): up to two m-tile lists for the new offsets
    // (as ds_build_mtiles writes them, for list_rows[i] rows per sample) and slot_lut[slot] = lut[group of slot]
    int32_t n_lists, list_rows[2];
    void* lists[2];
    int32_t* slot_lut;        // nullable
    int32_t lut[DS_MAX_GROUPS];
};
int32_t ds_launch_bucket_ex(const BucketArgs& a, hipStream_t s);
int32_t ds_launch_bucket(const int32_t* route, int32_t B, int32_t T, int32_t* perm, int32_t* inv_perm,
                         int32_t* offsets, int32_t* slot_group, hipStream_t s);

// ---- memory-bound layers ------------------------------------------------------
// Activations are [slot][pixel or token][channel]; a slot's block starts at
// index[slot] * sample_stride and its rows have stride ld (<= 0: the slot's own width).
struct ActView {
    void* p;
    const int32_t* index;
    int64_t sample_stride;
    int32_t ld;
};

int32_t ds_launch_expand_groups(const int32_t* offsets, int32_t T, int32_t* slot_group, hipStream_t s);
int32_t ds_launch_dwconv(ActView x, ActView y, const bf16_t* w, const float* scale, const float* shift,
                         int32_t tab_ld, const int32_t* slot_group, const GroupTable& gt, int32_t B, int32_t C,
                         int32_t H, int32_t W, int32_t stride, int32_t act, hipStream_t s);
// spatially sliced filter; y is packed [Ho_t][Wo_t][ld] per slot, the resolution following the group's padding
int32_t ds_launch_dwconv_spatial(ActView x, ActView y, const bf16_t* w, int32_t KS, const float* scale, const float* shift,
                                 int32_t tab_ld, const int32_t* slot_group, const GroupTable& gt, const SpatialTable& st,
                                 int32_t B, int32_t C, int32_t H, int32_t W, int32_t stride, int32_t act, hipStream_t s);
int32_t ds_launch_layernorm(ActView x, ActView y, const float* gamma, const float* beta, float eps,
                            const int32_t* slot_group, const GroupTable& gt, int32_t B, int32_t rows,
                            int32_t row0, int32_t n_rows, hipStream_t s);
int32_t ds_launch_stem(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                       const float* shift, int32_t B, int32_t H, int32_t W, int32_t K, int32_t stride,
                       int32_t pad, int32_t Cout, hipStream_t s);
// 3x3 depthwise + batch-norm + ReLU and 1x1 pointwise + batch-norm + ReLU of an unsliced block in one kernel
// (x [B][H][W][C] -> y [B][Ho][Wo][N]); DS_EUNSUPPORTED when the shape has no fused variant
int32_t ds_launch_dwpw(const bf16_t* x, int32_t B, int32_t H, int32_t W, int32_t C, int32_t stride, const bf16_t* wd,
                       const float* sd, const float* hd, const bf16_t* wp, int32_t w_ld, int32_t N, const float* sp,
                       const float* hp, bf16_t* y, hipStream_t s);
int32_t ds_launch_stem_mfma(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                            const float* shift, int32_t B, int32_t H, int32_t W, int32_t K, int32_t stride,
                            int32_t pad, int32_t Cout, hipStream_t s);
int32_t ds_launch_maxpool(const bf16_t* x, bf16_t* y, int32_t B, int32_t H, int32_t W, int32_t C, hipStream_t s);
// fused 7x7/2 stem (64 filters) + 3x3/2 max-pool; DS_EUNSUPPORTED for other shapes
int32_t ds_launch_stem_pool(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                            const float* shift, int32_t B, int32_t H, int32_t W, int32_t K, int32_t stride,
                            int32_t pad, int32_t Cout, hipStream_t s);
// classifier: logits[out_index[slot]][o] = sum_{c < slot_c[slot]} W[o][c] * v[c] + b[o]; v = spatial mean of x
// (HW > 0; partial needs ds_gate_partial_bytes(B, C)) or row 0 of the slot (HW == 0)
int32_t ds_launch_head(ActView x, int32_t HW, const bf16_t* w, int32_t w_ld, const float* bias, int32_t n_out,
                       const int32_t* slot_c, const int32_t* out_index, float* logits, float* partial, int32_t B,
                       int32_t C, hipStream_t s);
int32_t ds_launch_patchify(const bf16_t* img, const int32_t* index, bf16_t* patches, int32_t B, int32_t H,
                           int32_t W, int32_t P, hipStream_t s);
int32_t ds_launch_cls_rows(ActView x, const bf16_t* cls, const bf16_t* pos, const int32_t* slot_group,
                           const GroupTable& gt, int32_t B, hipStream_t s);
int32_t ds_launch_conv_f32_nchw(const float* x, const float* w, const float* scale, const float* shift,
                                int32_t tab_ld, const float* residual, float* y, const int32_t* slot_group,
                                const int32_t* perm, const GroupTable& gt, int32_t B, int32_t C_I, int32_t C_O,
                                int32_t H, int32_t W, int32_t K, int32_t stride, int32_t pad, int32_t act,
                                hipStream_t s);
int32_t ds_launch_compose_index(const int32_t* inner, const int32_t* outer, int32_t* out, int32_t B, hipStream_t s);
int32_t ds_launch_lookup(const int32_t* idx, const GroupTable& gt, int32_t which, int32_t* out, int32_t B, hipStream_t s);

// ---- attention ----------------------------------------------------------------
// q, k, v, o: bf16 [slot][N][ld]; head j uses columns j*Dh..j*Dh+Dh-1; group g runs heads < k_out[g]/Dh;
// head_dim Dh: 32, 48 or 64
int32_t ds_launch_attention(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* o, int64_t sample_stride,
                            int32_t ld, int32_t o_ld, int64_t o_sample_stride, const int32_t* slot_group,
                            const GroupTable& gt, int32_t B, int32_t N, int32_t H, int32_t head_dim, hipStream_t s);

// ---- small index helpers ---------------------------------------------------------
int32_t ds_launch_set_offsets(int32_t* offsets, int32_t B, hipStream_t s);  // offsets[0..1] = {0, B}
// key[b] = hi[b] * mul + (lo ? lo[b] : 0)
int32_t ds_launch_make_key(const int32_t* hi, const int32_t* lo, int32_t mul, int32_t* key, int32_t B, hipStream_t s);

// ---- per-kernel timing with HIP events (off unless ds_profile_enable(1)) ---------
enum {
    DS_K_GEMM = 0,   // gemm_kernel on linear / 1x1 layers
    DS_K_GEMM_TAPS,  // gemm_kernel walking KxK taps (implicit-GEMM convolution)
    DS_K_ATTENTION,
    DS_K_DWCONV,
    DS_K_LAYERNORM,
    DS_K_STEM,
    DS_K_MAXPOOL,
    DS_K_HEAD,
    DS_K_GATE,
    DS_K_BUCKET,
    DS_K_MISC,
    DS_K_CONV3,      // conv3_kernel (3x3 stride-1 layers with the input patch staged once)
    DS_K_THIN,       // thin_kernel (short reductions, one workgroup per row tile; with or without a chained second layer)
    DS_K_COUNT
};
struct ProfScope {
    int rec;
    hipStream_t s;
    ProfScope(int kind, hipStream_t stream);
    ~ProfScope();
};

struct ProfPause {   // no launch made by this thread inside its scope is recorded (and no event is created)
    bool was;
    ProfPause();
    ~ProfPause();
};

// ---- small dense layer on one vector per item --------------------------------------
struct FcArgs {
    const float* v_partial;   // [items][splits][C] partial sums (scaled by v_scale), or
    const bf16_t* v_rows;     // one bf16 row per item at v_rows + item * v_row_stride
    int64_t v_row_stride;
    int32_t splits;
    float v_scale;
    const int32_t* c_item;    // valid input width per item (nullable = C)
    int32_t C;                // stored input width / stride of v_partial
    const void* w;            // [n_out][w_ld] fp32 or bf16
    int32_t w_ld;
    const float* bias;        // nullable
    int32_t n_out, relu;      // relu: 0 none, 1 ReLU, 2 one plus tanh (attention head of the gate)
    const int32_t* out_index; // item -> output row (nullable = identity)
    float* out;
    int32_t out_ld, items;
};
int32_t ds_launch_fc(const FcArgs& a, int32_t w_bf16, int32_t acc_f64, int32_t kind, hipStream_t s);
// spatial partial sums of NHWC/NCHW feature maps into a.partial [B][splits][C]; returns splits
int32_t ds_launch_pool(const GateArgs& a, int32_t kind, int32_t* splits_out, hipStream_t s);
