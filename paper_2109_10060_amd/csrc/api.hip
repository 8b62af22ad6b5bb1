// extern "C" entry points of the sliced layers: argument validation on the host,
// then launches of the grouped kernels.  Samples keep their original order in
// the caller's tensors; the kernels gather and scatter whole samples through the
// bucket permutation.
#include <stdarg.h>
#include <string.h>

#include <mutex>
#include <set>
#include <utility>

#include "common.h"

static thread_local char g_err[512] = "";

void ds_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int32_t ds_reserve_lds(const void* kernel, int bytes, const char* what) {
    static std::mutex mu;
    static std::set<std::pair<int, const void*>> done;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) DS_FAIL(DS_EHIP, "%s: no current device", what);
    std::lock_guard<std::mutex> lock(mu);
    const auto key = std::make_pair(dev, kernel);
    if (done.count(key)) return DS_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        DS_FAIL(DS_EHIP, "%s: cannot reserve %d bytes of LDS", what, bytes);
    done.insert(key);
    return DS_OK;
}

extern "C" const char* ds_last_error(void) { return g_err; }
extern "C" int32_t ds_version(void) { return 1; }

namespace {

int32_t check_groups(const char* who, const ds_groups* g, int32_t k_full, int32_t n_full, bool need8,
                     GroupTable* gt, int32_t* max_in, int32_t* max_out) {
    if (!g) DS_FAIL(DS_EINVAL, "%s: null groups", who);
    if (g->T < 1 || g->T > DS_MAX_GROUPS) DS_FAIL(DS_EINVAL, "%s: T=%d outside 1..%d", who, g->T, DS_MAX_GROUPS);
    if (!g->offsets) DS_FAIL(DS_EINVAL, "%s: null offsets", who);
    gt->T = g->T;
    int mi = 0, mo = 0;
    for (int t = 0; t < g->T; ++t) {
        const int ki = g->k_in[t], ko = g->k_out[t];
        if (ki < 0 || ko < 0 || ki > k_full || ko > n_full)
            DS_FAIL(DS_EINVAL, "%s: group %d slice (%d,%d) exceeds stored size (%d,%d)", who, t, ki, ko, k_full, n_full);
        if (need8 && ((ki % 8) || (ko % 8))) DS_FAIL(DS_EALIGN, "%s: group %d slice (%d,%d) not a multiple of 8", who, t, ki, ko);
        if (g->table_row[t] < 0) DS_FAIL(DS_EINVAL, "%s: negative table row", who);
        gt->k_in[t] = ki;
        gt->k_out[t] = ko;
        gt->row[t] = g->table_row[t];
        mi = ki > mi ? ki : mi;
        mo = ko > mo ? ko : mo;
    }
    *max_in = mi;
    *max_out = mo;
    return DS_OK;
}

void linear_geometry(GemmArgs& a, int rows) {
    a.H = 1; a.W = rows; a.Ho = 1; a.Wo = rows; a.K = 1; a.stride = 1; a.pad = 0; a.rows = rows;
}

}  // namespace

extern "C" size_t ds_gate_workspace(int32_t B, int32_t C) { return B > 0 && C > 0 ? ds_gate_partial_bytes(B, C) : 0; }
extern "C" size_t ds_slot_workspace(int32_t B) { return ds_align_up((size_t)(B > 0 ? B : 0) * 4 + 4, 256); }

extern "C" size_t ds_sliced_linear_workspace(int32_t B, int32_t rows, int32_t T) {
    if (B < 0 || rows < 0 || T < 0) return 0;
    return ds_align_up(16 + ds_mtile_capacity(B, rows, T) * 16, 256);
}

extern "C" int32_t ds_sliced_linear(const void* x, int64_t x_ld, const void* w, int64_t w_ld, int32_t N_full,
                                    int32_t K_full, const float* bias, const ds_groups* g, int32_t B, int32_t rows,
                                    int32_t act, const void* residual, int64_t r_ld, void* y, int32_t y_dtype,
                                    int64_t y_ld, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "ds_sliced_linear";
    if (B < 0 || rows < 0 || N_full < 1 || K_full < 1) DS_FAIL(DS_EINVAL, "%s: negative or zero size", who);
    GroupTable gt;
    int mi, mo;
    int32_t rc = check_groups(who, g, K_full, N_full, true, &gt, &mi, &mo);
    if (rc) return rc;
    if (y_dtype != DS_BF16 && y_dtype != DS_F32) DS_FAIL(DS_EUNSUPPORTED, "%s: y dtype", who);
    if (act < DS_ACT_NONE || act > DS_ACT_GELU) DS_FAIL(DS_EINVAL, "%s: activation", who);
    if (B == 0 || rows == 0) return DS_OK;
    if (!x || !w || !y) DS_FAIL(DS_EINVAL, "%s: null tensor", who);
    if (x_ld < mi || w_ld < mi || y_ld < mo || (residual && r_ld < mo)) DS_FAIL(DS_ESHAPE, "%s: leading stride smaller than slice", who);
    if ((x_ld % 8) || (w_ld % 8) || (y_ld % 8) || (residual && (r_ld % 8)) || !ds_aligned16(x) || !ds_aligned16(w) ||
        !ds_aligned16(y) || !ds_aligned16(residual))
        DS_FAIL(DS_EALIGN, "%s: pointers need 16-byte alignment and strides multiples of 8", who);
    if (!ws || ws_bytes < ds_sliced_linear_workspace(B, rows, g->T))
        DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes", who, ds_sliced_linear_workspace(B, rows, g->T));
    hipStream_t s = (hipStream_t)stream;
    rc = ds_build_mtiles(g->offsets, g->T, rows, ws, s);
    if (rc) return rc;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.A = (const bf16_t*)x; a.Wt = (const bf16_t*)w; a.C = y; a.R = (const bf16_t*)residual;
    a.scale = nullptr; a.shift = bias; a.tab_ld = 0; a.tab_seg_stride = 0;
    a.a_index = g->perm; a.c_index = g->perm;
    a.a_sample_stride = (int64_t)rows * x_ld; a.c_sample_stride = (int64_t)rows * y_ld;
    a.r_sample_stride = (int64_t)rows * r_ld;
    a.a_ld = (int32_t)x_ld; a.c_ld = (int32_t)y_ld; a.r_ld = (int32_t)(residual ? r_ld : y_ld);
    a.c_row0 = 0; a.r_use_index = 1;
    a.w_ld = w_ld; a.w_tap_stride = 0; a.w_seg_stride = 0; a.c_seg_stride = 0; a.n_seg = 1;
    linear_geometry(a, rows);
    a.offsets = g->offsets; a.mtiles = ds_mtile_entries(ws); a.n_mtiles = ds_mtile_count(ws);
    a.act = act; a.out_f32 = y_dtype == DS_F32;
    a.gt = gt;
    {
        // thin reductions with several column passes have a kernel of their own
        const int32_t rt = ds_launch_thin(a, (int32_t)ds_mtile_capacity(B, rows, g->T), mo, s);
        if (rt != DS_EUNSUPPORTED) return rt;
    }
    return ds_launch_gemm(a, (int32_t)ds_mtile_capacity(B, rows, g->T), mo, s);
}

extern "C" size_t ds_sliced_conv_workspace(int32_t B, int32_t Ho, int32_t Wo, int32_t T) {
    if (B < 0 || Ho < 0 || Wo < 0 || T < 0) return 0;
    return ds_align_up(16 + ds_mtile_capacity(B, Ho * Wo, T) * 16, 256) + ds_slot_workspace(B);
}

extern "C" int32_t ds_sliced_conv(const void* x, int32_t dtype, int32_t layout, int32_t B, int32_t C_I, int32_t H,
                                  int32_t W, const void* w, int32_t C_O, int32_t K, const float* scale,
                                  const float* shift, const ds_groups* g, int32_t stride, int32_t pad, int32_t act,
                                  const void* residual, void* y, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "ds_sliced_conv";
    if (B < 0 || C_I < 1 || C_O < 1 || H < 1 || W < 1 || K < 1 || stride < 1 || pad < 0)
        DS_FAIL(DS_EINVAL, "%s: bad size", who);
    const bool f32 = dtype == DS_F32 && layout == DS_NCHW;
    const bool b16 = dtype == DS_BF16 && layout == DS_NHWC;
    if (!f32 && !b16) DS_FAIL(DS_EUNSUPPORTED, "%s: only (f32, NCHW) and (bf16, NHWC)", who);
    if (act != DS_ACT_NONE && act != DS_ACT_RELU) DS_FAIL(DS_EUNSUPPORTED, "%s: activation", who);
    if (H + 2 * pad < K || W + 2 * pad < K) DS_FAIL(DS_ESHAPE, "%s: kernel larger than padded input", who);
    GroupTable gt;
    int mi, mo;
    int32_t rc = check_groups(who, g, C_I, C_O, b16, &gt, &mi, &mo);
    if (rc) return rc;
    if (B == 0) return DS_OK;
    if (!x || !w || !y) DS_FAIL(DS_EINVAL, "%s: null tensor", who);
    const int Ho = (H + 2 * pad - K) / stride + 1, Wo = (W + 2 * pad - K) / stride + 1;
    if (!ws || ws_bytes < ds_sliced_conv_workspace(B, Ho, Wo, g->T))
        DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes", who, ds_sliced_conv_workspace(B, Ho, Wo, g->T));
    hipStream_t s = (hipStream_t)stream;
    if (f32) {
        int32_t* slot_group = (int32_t*)ws;
        rc = ds_launch_expand_groups(g->offsets, g->T, slot_group, s);
        if (rc) return rc;
        return ds_launch_conv_f32_nchw((const float*)x, (const float*)w, scale, shift, C_O, (const float*)residual,
                                       (float*)y, slot_group, g->perm, gt, B, C_I, C_O, H, W, K, stride, pad, act, s);
    }
    if ((C_I % 8) || (C_O % 8) || !ds_aligned16(x) || !ds_aligned16(w) || !ds_aligned16(y) || !ds_aligned16(residual))
        DS_FAIL(DS_EALIGN, "%s: bf16 path needs 16-byte aligned pointers and channel counts multiples of 8", who);
    const int rows = Ho * Wo;
    rc = ds_build_mtiles(g->offsets, g->T, rows, ws, s);
    if (rc) return rc;
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.A = (const bf16_t*)x; a.Wt = (const bf16_t*)w; a.C = y; a.R = (const bf16_t*)residual;
    a.scale = scale; a.shift = shift; a.tab_ld = C_O; a.tab_seg_stride = 0;
    a.a_index = g->perm; a.c_index = g->perm;
    a.a_sample_stride = (int64_t)H * W * C_I; a.c_sample_stride = (int64_t)rows * C_O;
    a.r_sample_stride = a.c_sample_stride;
    a.a_ld = C_I; a.c_ld = C_O; a.r_ld = C_O; a.c_row0 = 0; a.r_use_index = 1;
    a.w_ld = (int64_t)K * K * C_I; a.w_tap_stride = C_I; a.n_seg = 1;
    a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo; a.K = K; a.stride = stride; a.pad = pad; a.rows = rows;
    a.offsets = g->offsets; a.mtiles = ds_mtile_entries(ws); a.n_mtiles = ds_mtile_count(ws);
    a.act = act; a.out_f32 = 0;
    a.gt = gt;
    {
        // thin reductions with several column passes have a kernel of their own
        const int32_t rt = ds_launch_thin(a, (int32_t)ds_mtile_capacity(B, rows, g->T), mo, s);
        if (rt != DS_EUNSUPPORTED) return rt;
    }
    return ds_launch_gemm(a, (int32_t)ds_mtile_capacity(B, rows, g->T), mo, s);
}

extern "C" int32_t ds_sliced_dwconv(const void* x, int32_t B, int32_t C, int32_t H, int32_t W, const void* w,
                                    const float* scale, const float* shift, const ds_groups* g, int32_t stride,
                                    int32_t act, void* y, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "ds_sliced_dwconv";
    if (B < 0 || C < 1 || H < 1 || W < 1 || (stride != 1 && stride != 2)) DS_FAIL(DS_EINVAL, "%s: bad size", who);
    if (act != DS_ACT_NONE && act != DS_ACT_RELU) DS_FAIL(DS_EUNSUPPORTED, "%s: activation", who);
    GroupTable gt;
    int mi, mo;
    int32_t rc = check_groups(who, g, C, C, true, &gt, &mi, &mo);
    if (rc) return rc;
    if (B == 0) return DS_OK;
    if (!x || !w || !y || !scale || !shift) DS_FAIL(DS_EINVAL, "%s: null tensor", who);
    if ((C % 8) || !ds_aligned16(x) || !ds_aligned16(w) || !ds_aligned16(y) || !ds_aligned16(scale) || !ds_aligned16(shift))
        DS_FAIL(DS_EALIGN, "%s: needs 16-byte aligned pointers and C %% 8 == 0", who);
    if (!ws || ws_bytes < ds_slot_workspace(B)) DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes", who, ds_slot_workspace(B));
    hipStream_t s = (hipStream_t)stream;
    int32_t* slot_group = (int32_t*)ws;
    rc = ds_launch_expand_groups(g->offsets, g->T, slot_group, s);
    if (rc) return rc;
    const int Ho = (H + 2 - 3) / stride + 1, Wo = (W + 2 - 3) / stride + 1;
    ActView xv = {(void*)x, g->perm, (int64_t)H * W * C, C};
    ActView yv = {y, g->perm, (int64_t)Ho * Wo * C, C};
    return ds_launch_dwconv(xv, yv, (const bf16_t*)w, scale, shift, C, slot_group, gt, B, C, H, W, stride, act, s);
}

extern "C" int32_t ds_sliced_dwconv_spatial(const void* x, int32_t B, int32_t C, int32_t H, int32_t W, const void* w,
                                            int32_t K, const float* scale, const float* shift, const ds_groups* g,
                                            const ds_spatial* sp, int32_t stride, int32_t act, void* y,
                                            int64_t y_sample_stride, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "ds_sliced_dwconv_spatial";
    if (B < 0 || C < 1 || H < 1 || W < 1 || stride < 1 || stride > 4) DS_FAIL(DS_EINVAL, "%s: bad size", who);
    if (K < 1 || K > 7 || (K % 2) == 0) DS_FAIL(DS_EUNSUPPORTED, "%s: stored filter size %d (odd, at most 7)", who, K);
    if (act != DS_ACT_NONE && act != DS_ACT_RELU) DS_FAIL(DS_EUNSUPPORTED, "%s: activation", who);
    if (!sp) DS_FAIL(DS_EINVAL, "%s: null spatial table", who);
    GroupTable gt;
    int mi, mo;
    int32_t rc = check_groups(who, g, C, C, true, &gt, &mi, &mo);
    if (rc) return rc;
    SpatialTable st;
    memset(&st, 0, sizeof(st));
    for (int t = 0; t < g->T; ++t) {
        const int k = sp->ksize[t], l = sp->dilation[t], pad = sp->pad[t];
        if (k < 1 || k > K || ((K - k) % 2)) DS_FAIL(DS_EINVAL, "%s: group %d kernel size %d is no centred block of %d", who, t, k, K);
        if (l < 1 || pad < 0 || pad > 16) DS_FAIL(DS_EINVAL, "%s: group %d dilation %d / padding %d", who, t, l, pad);
        st.k0[t] = (K - k) / 2;
        st.n[t] = (k + l - 1) / l;
        st.l[t] = l;
        st.pad[t] = pad;
        const int span = (st.n[t] - 1) * l + 1;
        const int Ho = (H + 2 * pad - span) / stride + 1, Wo = (W + 2 * pad - span) / stride + 1;
        if (H + 2 * pad < span || W + 2 * pad < span) DS_FAIL(DS_ESHAPE, "%s: group %d has no output pixel", who, t);
        if ((int64_t)Ho * Wo * C > y_sample_stride) DS_FAIL(DS_ESHAPE, "%s: group %d output exceeds y_sample_stride", who, t);
    }
    if (B == 0) return DS_OK;
    if (!x || !w || !y || !scale || !shift) DS_FAIL(DS_EINVAL, "%s: null tensor", who);
    if ((C % 8) || (y_sample_stride % 8) || !ds_aligned16(x) || !ds_aligned16(w) || !ds_aligned16(y) || !ds_aligned16(scale) ||
        !ds_aligned16(shift))
        DS_FAIL(DS_EALIGN, "%s: needs 16-byte aligned pointers, C %% 8 == 0 and y_sample_stride %% 8 == 0", who);
    if ((int64_t)H * W * C * 2 >= 0x7fffffffLL) DS_FAIL(DS_EUNSUPPORTED, "%s: a sample spans 2 GiB or more", who);
    if (!ws || ws_bytes < ds_slot_workspace(B)) DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes", who, ds_slot_workspace(B));
    hipStream_t s = (hipStream_t)stream;
    int32_t* slot_group = (int32_t*)ws;
    rc = ds_launch_expand_groups(g->offsets, g->T, slot_group, s);
    if (rc) return rc;
    ActView xv = {(void*)x, g->perm, (int64_t)H * W * C, C};
    ActView yv = {y, g->perm, y_sample_stride, C};
    return ds_launch_dwconv_spatial(xv, yv, (const bf16_t*)w, K, scale, shift, C, slot_group, gt, st, B, C, H, W, stride, act, s);
}

extern "C" int32_t ds_sliced_layernorm(const void* x, int64_t x_ld, const float* gamma, const float* beta, float eps,
                                       const ds_groups* g, int32_t B, int32_t rows, void* y, int64_t y_ld, void* ws,
                                       size_t ws_bytes, void* stream) {
    const char* who = "ds_sliced_layernorm";
    if (B < 0 || rows < 0) DS_FAIL(DS_EINVAL, "%s: negative size", who);
    GroupTable gt;
    int mi, mo;
    int32_t rc = check_groups(who, g, (int32_t)x_ld, INT32_MAX, true, &gt, &mi, &mo);
    if (rc) return rc;
    if (mi > 2048) DS_FAIL(DS_EUNSUPPORTED, "%s: width above 2048", who);
    if (B == 0 || rows == 0) return DS_OK;
    if (!x || !y || !gamma || !beta) DS_FAIL(DS_EINVAL, "%s: null tensor", who);
    if (y_ld < mi) DS_FAIL(DS_ESHAPE, "%s: y_ld smaller than slice", who);
    if ((x_ld % 8) || (y_ld % 8) || !ds_aligned16(x) || !ds_aligned16(y) || !ds_aligned16(gamma) || !ds_aligned16(beta))
        DS_FAIL(DS_EALIGN, "%s: needs 16-byte aligned pointers and strides multiples of 8", who);
    if (!ws || ws_bytes < ds_slot_workspace(B)) DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes", who, ds_slot_workspace(B));
    hipStream_t s = (hipStream_t)stream;
    int32_t* slot_group = (int32_t*)ws;
    rc = ds_launch_expand_groups(g->offsets, g->T, slot_group, s);
    if (rc) return rc;
    ActView xv = {(void*)x, g->perm, (int64_t)rows * x_ld, (int32_t)x_ld};
    ActView yv = {y, g->perm, (int64_t)rows * y_ld, (int32_t)y_ld};
    return ds_launch_layernorm(xv, yv, gamma, beta, eps, slot_group, gt, B, rows, 0, rows, s);
}

extern "C" size_t ds_sliced_mhsa_workspace(int32_t B, int32_t N, int32_t H, int32_t head_dim, int32_t T) {
    if (B < 0 || N < 0 || H < 0 || head_dim < 0 || T < 0) return 0;
    return ds_align_up(16 + ds_mtile_capacity(B, N, T) * 16, 256) + ds_slot_workspace(B) +
           4 * ds_align_up((size_t)B * N * H * head_dim * sizeof(bf16_t), 256);
}

extern "C" int32_t ds_sliced_mhsa(const void* x, int32_t B, int32_t N, int32_t D_e, const void* wqkv,
                                  const float* bqkv, const void* wproj, const float* bproj, int32_t H,
                                  int32_t head_dim, const ds_groups* g, const void* residual, void* y, void* ws,
                                  size_t ws_bytes, void* stream) {
    const char* who = "ds_sliced_mhsa";
    if (B < 0 || N < 1 || D_e < 1 || H < 1) DS_FAIL(DS_EINVAL, "%s: bad size", who);
    if (head_dim != 32 && head_dim != 48 && head_dim != 64) DS_FAIL(DS_EUNSUPPORTED, "%s: head_dim must be 32, 48 or 64", who);
    if (N > 224) DS_FAIL(DS_EUNSUPPORTED, "%s: N above 224", who);
    const int Hd = H * head_dim;
    GroupTable gt;
    int mi, mo;
    int32_t rc = check_groups(who, g, D_e, Hd, true, &gt, &mi, &mo);
    if (rc) return rc;
    for (int t = 0; t < gt.T; ++t)
        if (gt.k_out[t] % head_dim) DS_FAIL(DS_EINVAL, "%s: k_out must be heads * head_dim", who);
    if (B == 0) return DS_OK;
    if (!x || !wqkv || !wproj || !y) DS_FAIL(DS_EINVAL, "%s: null tensor", who);
    if ((D_e % 8) || !ds_aligned16(x) || !ds_aligned16(wqkv) || !ds_aligned16(wproj) || !ds_aligned16(y) || !ds_aligned16(residual))
        DS_FAIL(DS_EALIGN, "%s: needs 16-byte aligned pointers and D_e %% 8 == 0", who);
    if (!ws || ws_bytes < ds_sliced_mhsa_workspace(B, N, H, head_dim, g->T))
        DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes", who, ds_sliced_mhsa_workspace(B, N, H, head_dim, g->T));
    hipStream_t s = (hipStream_t)stream;
    char* p = (char*)ws;
    void* mlist = p;
    p += ds_align_up(16 + ds_mtile_capacity(B, N, g->T) * 16, 256);
    int32_t* slot_group = (int32_t*)p;
    p += ds_slot_workspace(B);
    const size_t bufsz = ds_align_up((size_t)B * N * Hd * sizeof(bf16_t), 256);
    bf16_t* qkv = (bf16_t*)p;          // [3][B][N][Hd], slot order
    bf16_t* obuf = (bf16_t*)(p + 3 * bufsz);
    rc = ds_build_mtiles(g->offsets, g->T, N, mlist, s);
    if (rc) return rc;
    rc = ds_launch_expand_groups(g->offsets, g->T, slot_group, s);
    if (rc) return rc;
    const int cap = (int)ds_mtile_capacity(B, N, g->T);

    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.A = (const bf16_t*)x; a.Wt = (const bf16_t*)wqkv; a.C = qkv; a.R = nullptr;
    a.scale = nullptr; a.shift = bqkv; a.tab_ld = 0; a.tab_seg_stride = Hd;
    a.a_index = g->perm; a.c_index = nullptr;
    a.a_sample_stride = (int64_t)N * D_e; a.a_ld = D_e;
    a.c_sample_stride = (int64_t)N * Hd; a.c_ld = Hd;
    a.w_ld = D_e; a.w_tap_stride = 0; a.w_seg_stride = (int64_t)Hd * D_e; a.n_seg = 3;
    a.c_seg_stride = (int64_t)(bufsz / sizeof(bf16_t));
    linear_geometry(a, N);
    a.offsets = g->offsets; a.mtiles = ds_mtile_entries(mlist); a.n_mtiles = ds_mtile_count(mlist);
    a.act = DS_ACT_NONE; a.out_f32 = 0; a.gt = gt;
    rc = ds_launch_gemm(a, cap, mo, s);
    if (rc) return rc;

    const int64_t seg = (int64_t)(bufsz / sizeof(bf16_t));
    rc = ds_launch_attention(qkv, qkv + seg, qkv + 2 * seg, obuf, (int64_t)N * Hd, Hd, Hd, (int64_t)N * Hd, slot_group,
                             gt, B, N, H, head_dim, s);
    if (rc) return rc;

    GemmArgs b;
    memset(&b, 0, sizeof(b));
    GroupTable gp = gt;
    for (int t = 0; t < gt.T; ++t) { gp.k_in[t] = gt.k_out[t]; gp.k_out[t] = gt.k_in[t]; }
    b.A = obuf; b.Wt = (const bf16_t*)wproj; b.C = y; b.R = (const bf16_t*)residual;
    b.scale = nullptr; b.shift = bproj; b.tab_ld = 0;
    b.a_index = nullptr; b.c_index = g->perm;
    b.a_sample_stride = (int64_t)N * Hd; b.a_ld = Hd;
    b.c_sample_stride = (int64_t)N * D_e; b.c_ld = D_e;
    b.r_sample_stride = (int64_t)N * D_e; b.r_ld = D_e; b.r_use_index = 1;
    b.w_ld = Hd; b.n_seg = 1;
    linear_geometry(b, N);
    b.offsets = g->offsets; b.mtiles = ds_mtile_entries(mlist); b.n_mtiles = ds_mtile_count(mlist);
    b.act = DS_ACT_NONE; b.out_f32 = 0; b.gt = gp;
    return ds_launch_gemm(b, cap, mi, s);
}

// ---- pool + classifier and max-pool as calls of their own ("Pool + FC" rows of the routing-space tables, Section 5.2) ----
extern "C" size_t ds_pool_head_workspace(int32_t B, int32_t C) {
    if (B <= 0 || C <= 0) return 0;
    return 2 * ds_slot_workspace(B) + ds_align_up(ds_gate_partial_bytes(B, C), 256);
}

extern "C" int32_t ds_pool_head(const void* x, int32_t B, int32_t HW, int32_t C, const void* w, const float* bias,
                                int32_t n_out, const ds_groups* g, float* logits, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "ds_pool_head";
    if (B < 0 || HW < 1 || C < 1 || n_out < 1) DS_FAIL(DS_EINVAL, "%s: bad size", who);
    GroupTable gt;
    int mi, mo;
    int32_t rc = check_groups(who, g, C, INT32_MAX, true, &gt, &mi, &mo);
    if (rc) return rc;
    if (B == 0) return DS_OK;
    if (!x || !w || !logits) DS_FAIL(DS_EINVAL, "%s: null tensor", who);
    if ((C % 8) || !ds_aligned16(x) || !ds_aligned16(w)) DS_FAIL(DS_EALIGN, "%s: needs 16-byte aligned pointers and C %% 8 == 0", who);
    if (!ws || ws_bytes < ds_pool_head_workspace(B, C)) DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes", who, ds_pool_head_workspace(B, C));
    hipStream_t s = (hipStream_t)stream;
    int32_t* slot_group = (int32_t*)ws;
    int32_t* slot_c = (int32_t*)((char*)ws + ds_slot_workspace(B));
    float* partial = (float*)((char*)ws + 2 * ds_slot_workspace(B));
    rc = ds_launch_expand_groups(g->offsets, g->T, slot_group, s);
    if (rc) return rc;
    rc = ds_launch_lookup(slot_group, gt, 0, slot_c, B, s);
    if (rc) return rc;
    ActView xv = {(void*)x, g->perm, (int64_t)HW * C, C};
    return ds_launch_head(xv, HW, (const bf16_t*)w, C, bias, n_out, slot_c, g->perm, logits, partial, B, C, s);
}

extern "C" int32_t ds_maxpool(const void* x, int32_t B, int32_t H, int32_t W, int32_t C, void* y, void* stream) {
    const char* who = "ds_maxpool";
    if (B < 0 || H < 1 || W < 1 || C < 1) DS_FAIL(DS_EINVAL, "%s: bad size", who);
    if (B == 0) return DS_OK;
    if (!x || !y) DS_FAIL(DS_EINVAL, "%s: null tensor", who);
    if ((C % 8) || !ds_aligned16(x) || !ds_aligned16(y)) DS_FAIL(DS_EALIGN, "%s: needs 16-byte aligned pointers and C %% 8 == 0", who);
    return ds_launch_maxpool((const bf16_t*)x, (bf16_t*)y, B, H, W, C, (hipStream_t)stream);
}
