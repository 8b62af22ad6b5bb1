// Memory-bound layers of the sliced networks: depthwise convolution (Section 3.3,
// Eq. 10 with one channel per group) with split batch-norm (Eq. 14), LayerNorm over
// the valid embedding slice, the unsliced stem convolution, max-pool, the
// pool + classifier head with sliced input width, patch extraction, and the fp32
// NCHW direct convolution used by the single-block configuration (Eq. 9).
// All bf16 kernels move 8 channels (16 bytes) per lane and keep lanes of a
// wavefront on consecutive channels of one pixel so that global accesses coalesce.
#include "common.h"

namespace {

__device__ __forceinline__ void unpack8(const uint4 q, float* v) {
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ uint4 pack8(const float* v) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = f2bf2(v[2 * i], v[2 * i + 1]);
    return make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ void loadf8(const float* p, float* v) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

__global__ void expand_groups_kernel(const int32_t* offsets, int T, int32_t* slot_group) {
    for (int t = 0; t < T; ++t) {
        const int b0 = offsets[t], b1 = offsets[t + 1];
        for (int j = b0 + threadIdx.x; j < b1; j += blockDim.x) slot_group[j] = t;
    }
}

// ---- depthwise 3x3 + scale/shift + activation ---------------------------------
// grid (ceil(Ho*Wo*C/8 / 256), B); thread = (output pixel, 8-channel chunk)
__global__ __launch_bounds__(256) void dwconv_kernel(ActView x, ActView y, const bf16_t* w, const float* scale,
                                                     const float* shift, int tab_ld, const int32_t* slot_group,
                                                     const GroupTable gt, int C, int H, int W, int Ho, int Wo,
                                                     int stride, int act) {
    const int slot = blockIdx.y;
    const int g = slot_group ? slot_group[slot] : 0;
    const int c = gt.k_in[g];
    const int chunks = c >> 3;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= Ho * Wo * chunks) return;
    const int pix = idx / chunks, ch = (idx - pix * chunks) * 8;
    const int oy = pix / Wo, ox = pix - oy * Wo;
    const int xs = x.index ? x.index[slot] : slot;
    const int ys = y.index ? y.index[slot] : slot;
    const int xld = x.ld > 0 ? x.ld : c, yld = y.ld > 0 ? y.ld : c;
    const bf16_t* xp = (const bf16_t*)x.p + (int64_t)xs * x.sample_stride + ch;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < 3; ++u) {
        const int iy = oy * stride + u - 1;
        if (iy < 0 || iy >= H) continue;
#pragma unroll
        for (int v = 0; v < 3; ++v) {
            const int ix = ox * stride + v - 1;
            if (ix < 0 || ix >= W) continue;
            float xv[8], wv[8];
            unpack8(*(const uint4*)(xp + (int64_t)(iy * W + ix) * xld), xv);
            unpack8(*(const uint4*)(w + (u * 3 + v) * C + ch), wv);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = fmaf(xv[i], wv[i], acc[i]);
        }
    }
    const int64_t ti = (int64_t)gt.row[g] * tab_ld + ch;
    float sc[8], sh[8];
    loadf8(scale + ti, sc);
    loadf8(shift + ti, sh);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        acc[i] = acc[i] * sc[i] + sh[i];
        if (act == DS_ACT_RELU) acc[i] = fmaxf(acc[i], 0.f);
    }
    *(uint4*)((bf16_t*)y.p + (int64_t)ys * y.sample_stride + (int64_t)pix * yld + ch) = pack8(acc);
}

constexpr int DW_PX_S2 = 2;   // output pixels per thread at stride 2 (4 at stride 1)

// Same layer, PX consecutive output pixels of a row per thread: the 3 x (3 + 3 STRIDE) input window
// and the 9 filter chunks are loaded once for 4 outputs, which cuts the load instructions per
// output from 18 to 6.75 (stride 1) / 9 (stride 2).
// one-dimensional grid of ceil(Ho * ceil(Wo/PX) * C/8 / 256) tiles x (B rounded up to 8) slots, slot fastest
template <int STRIDE, int PX>
__global__ __launch_bounds__(256, 3) void dwconv4_kernel(ActView x, ActView y, const bf16_t* w, const float* scale,
                                                      const float* shift, int tab_ld, const int32_t* slot_group,
                                                      const GroupTable gt, int C, int H, int W, int Ho, int Wo,
                                                      int act, int B, int slots8) {
    constexpr int NCOL = (PX - 1) * STRIDE + 3;
    // The slot is the fastest index of the launch order (padded to a multiple of 8): workgroups go to the 8 dies
    // in turn, so every tile of one sample lands on the same die and the rows that vertically neighbouring
    // tiles share are served by that die's L2 instead of being fetched from memory once per die.
    const int slot = blockIdx.x % slots8;
    if (slot >= B) return;
    const int g = slot_group ? slot_group[slot] : 0;
    const int c = gt.k_in[g];
    const int chunks = c >> 3;
    const int xgroups = (Wo + PX - 1) / PX;
    const int idx = (blockIdx.x / slots8) * 256 + threadIdx.x;
    if (idx >= Ho * xgroups * chunks) return;
    const int pg = idx / chunks, ch = (idx - pg * chunks) * 8;
    const int oy = pg / xgroups, ox0 = (pg - oy * xgroups) * PX;
    const int xs = x.index ? x.index[slot] : slot;
    const int ys = y.index ? y.index[slot] : slot;
    const int xld = x.ld > 0 ? x.ld : c, yld = y.ld > 0 ? y.ld : c;
    float acc[PX][8];
#pragma unroll
    for (int p = 0; p < PX; ++p)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[p][i] = 0.f;
    const int ix0 = ox0 * STRIDE - 1;
    // The whole 3 x NCOL window is fetched with buffer loads before any arithmetic: a tap outside
    // the image gets an out-of-range offset and comes back as zeros, so there is no branch around a
    // load and all of them are in flight together (with branches the compiler emits load, wait,
    // use per tap, and the kernel is bound by that chain of latencies).  The sample is addressed
    // through a descriptor of its own, so offsets stay small.
    constexpr uint32_t OOB = 0x80000000u;
    // (the descriptor must be uniform over the wavefront: sample base only; the channel goes into the offset)
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const bf16_t*)x.p + (int64_t)xs * x.sample_stride), 0, 0x7fffffff, 0x00020000);
    uint4 xin[3][NCOL];
#pragma unroll
    for (int u = 0; u < 3; ++u) {
        const int iy = oy * STRIDE + u - 1;
        const bool rok = iy >= 0 && iy < H;
#pragma unroll
        for (int col = 0; col < NCOL; ++col) {
            const int ix = ix0 + col;
            const uint32_t off = (rok && ix >= 0 && ix < W) ? (uint32_t)(((iy * W + ix) * xld + ch) * 2) : OOB;
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
            xin[u][col] = make_uint4(t[0], t[1], t[2], t[3]);
        }
    }
    uint4 win[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) win[t] = *(const uint4*)(w + t * C + ch);
    // the bf16 pairs stay packed: v_dot2_f32_bf16 against a weight pair with one half zeroed is the
    // multiply-add of the other half (the bf16 product is exact in fp32, so this equals an fma) and
    // saves the unpacking of every loaded pixel
#pragma unroll
    for (int u = 0; u < 3; ++u) {
        bf16x2_t wlo[3][4], whi[3][4];
#pragma unroll
        for (int v = 0; v < 3; ++v) {
            const uint32_t qq[4] = {win[u * 3 + v].x, win[u * 3 + v].y, win[u * 3 + v].z, win[u * 3 + v].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wlo[v][j] = __builtin_bit_cast(bf16x2_t, qq[j] & 0x0000ffffu);
                whi[v][j] = __builtin_bit_cast(bf16x2_t, qq[j] & 0xffff0000u);
            }
        }
#pragma unroll
        for (int col = 0; col < NCOL; ++col) {
            const uint4 q = xin[u][col];
            const bf16x2_t xq[4] = {__builtin_bit_cast(bf16x2_t, q.x), __builtin_bit_cast(bf16x2_t, q.y),
                                    __builtin_bit_cast(bf16x2_t, q.z), __builtin_bit_cast(bf16x2_t, q.w)};
#pragma unroll
            for (int p = 0; p < PX; ++p) {
                const int v = col - p * STRIDE;      // filter column this input column meets for output p
                if (v >= 0 && v < 3) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc[p][2 * j] = __builtin_amdgcn_fdot2_f32_bf16(xq[j], wlo[v][j], acc[p][2 * j], false);
                        acc[p][2 * j + 1] = __builtin_amdgcn_fdot2_f32_bf16(xq[j], whi[v][j], acc[p][2 * j + 1], false);
                    }
                }
            }
        }
    }
    const int64_t ti = (int64_t)gt.row[g] * tab_ld + ch;
    float sc[8], sh[8];
    loadf8(scale + ti, sc);
    loadf8(shift + ti, sh);
    bf16_t* yp = (bf16_t*)y.p + (int64_t)ys * y.sample_stride + ((int64_t)oy * Wo + ox0) * yld + ch;
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        if (ox0 + p >= Wo) break;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc[p][i] = acc[p][i] * sc[i] + sh[i];
            if (act == DS_ACT_RELU) acc[p][i] = fmaxf(acc[p][i], 0.f);
        }
        *(uint4*)(yp + (int64_t)p * yld) = pack8(acc[p]);
    }
}

// ---- depthwise convolution with a spatially sliced filter (Section 3.2, Eq. 11-13) --------------
// The filter is stored once as KS x KS taps ([KS][KS][C]); a route uses the centred k x k block of it
// (Eq. 11), every l-th tap of that block at dilation l (Eq. 12) and its own padding (Eq. 13), which also
// sets its output resolution.  One slot per workgroup, so the route's tap count N is uniform over the
// workgroup and picks a fully unrolled row routine: the N input pixels and N filter taps of a row are
// all requested (branch-free buffer loads, zeros outside the image) before the first multiply.
// A lane owns 8 channels of one output pixel; the output is packed [Ho_t][Wo_t][width] per slot.
constexpr int DWS_PX = 4;   // output pixels per lane on undilated routes

template <int N>
__device__ __forceinline__ void dws_rows(float (&acc)[8], const __amdgpu_buffer_rsrc_t rsrc, const bf16_t* w, int KS, int C,
                                         int k0, int l, int iy0, int ix0, int H, int W, int xld, int ch) {
    constexpr uint32_t OOB = 0x80000000u;
#pragma unroll 1
    for (int i = 0; i < N; ++i) {
        const int iy = iy0 + i * l;
        const bool rok = iy >= 0 && iy < H;
        uint4 xin[N], win[N];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const int ix = ix0 + j * l;
            const uint32_t off = (rok && ix >= 0 && ix < W) ? (uint32_t)(((iy * W + ix) * xld + ch) * 2) : OOB;
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
            xin[j] = make_uint4(t[0], t[1], t[2], t[3]);
            win[j] = *(const uint4*)(w + ((k0 + i * l) * KS + k0 + j * l) * C + ch);
        }
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const uint32_t xq[4] = {xin[j].x, xin[j].y, xin[j].z, xin[j].w};
            const uint32_t wq[4] = {win[j].x, win[j].y, win[j].z, win[j].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bf16x2_t xv = __builtin_bit_cast(bf16x2_t, xq[q]);
                acc[2 * q] = __builtin_amdgcn_fdot2_f32_bf16(xv, __builtin_bit_cast(bf16x2_t, wq[q] & 0x0000ffffu), acc[2 * q], false);
                acc[2 * q + 1] = __builtin_amdgcn_fdot2_f32_bf16(xv, __builtin_bit_cast(bf16x2_t, wq[q] & 0xffff0000u), acc[2 * q + 1], false);
            }
        }
    }
}

// Undilated routes: PX neighbouring output pixels of a row per lane, so that the (PX - 1) STRIDE + N input
// columns of a filter row are loaded once and every tap's weight pair masks are made once for all PX outputs.
template <int N, int STRIDE, int PX>
__device__ __forceinline__ void dws_rows_px(float (&acc)[PX][8], const __amdgpu_buffer_rsrc_t rsrc, const bf16_t* w, int KS,
                                            int C, int k0, int iy0, int ix0, int H, int W, int xld, int ch) {
    constexpr uint32_t OOB = 0x80000000u;
    constexpr int NCOL = (PX - 1) * STRIDE + N;
#pragma unroll 1
    for (int i = 0; i < N; ++i) {
        const int iy = iy0 + i;
        const bool rok = iy >= 0 && iy < H;
        uint4 xin[NCOL], win[N];
#pragma unroll
        for (int col = 0; col < NCOL; ++col) {
            const int ix = ix0 + col;
            const uint32_t off = (rok && ix >= 0 && ix < W) ? (uint32_t)(((iy * W + ix) * xld + ch) * 2) : OOB;
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
            xin[col] = make_uint4(t[0], t[1], t[2], t[3]);
        }
#pragma unroll
        for (int j = 0; j < N; ++j) win[j] = *(const uint4*)(w + ((k0 + i) * KS + k0 + j) * C + ch);
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const uint32_t wq[4] = {win[j].x, win[j].y, win[j].z, win[j].w};
            bf16x2_t wlo[4], whi[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                wlo[q] = __builtin_bit_cast(bf16x2_t, wq[q] & 0x0000ffffu);
                whi[q] = __builtin_bit_cast(bf16x2_t, wq[q] & 0xffff0000u);
            }
#pragma unroll
            for (int p = 0; p < PX; ++p) {
                const uint4 xv = xin[p * STRIDE + j];
                const uint32_t xq[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bf16x2_t xx = __builtin_bit_cast(bf16x2_t, xq[q]);
                    acc[p][2 * q] = __builtin_amdgcn_fdot2_f32_bf16(xx, wlo[q], acc[p][2 * q], false);
                    acc[p][2 * q + 1] = __builtin_amdgcn_fdot2_f32_bf16(xx, whi[q], acc[p][2 * q + 1], false);
                }
            }
        }
    }
}

template <int STRIDE, int PX>
__global__ __launch_bounds__(256) void dwconv_spatial_kernel(ActView x, ActView y, const bf16_t* w, int KS,
                                                             const float* scale, const float* shift, int tab_ld,
                                                             const int32_t* slot_group, const GroupTable gt,
                                                             const SpatialTable st, int C, int H, int W, int stride,
                                                             int act, int B, int slots8) {
    // slot-fastest launch order, as in dwconv4_kernel: a sample's tiles share one die's L2
    const int slot = blockIdx.x % slots8;
    if (slot >= B) return;
    const int g = slot_group ? slot_group[slot] : 0;
    const int c = gt.k_in[g];
    const int chunks = c >> 3;
    const int n = st.n[g], l = st.l[g], pad = st.pad[g], k0 = st.k0[g];
    const int span = (n - 1) * l + 1;
    const int Ho = (H + 2 * pad - span) / stride + 1, Wo = (W + 2 * pad - span) / stride + 1;
    // STRIDE == 0: any stride, one pixel per lane.  Otherwise undilated routes take PX pixels per lane.
    const bool wide = STRIDE > 0 && l == 1;                     // uniform over the workgroup
    const int px = wide ? PX : 1;
    const int xgroups = (Wo + px - 1) / px;
    const int idx = (blockIdx.x / slots8) * 256 + threadIdx.x;
    if (Ho <= 0 || Wo <= 0 || idx >= Ho * xgroups * chunks) return;
    const int pg = idx / chunks, ch = (idx - pg * chunks) * 8;
    const int oy = pg / xgroups, ox0 = (pg - oy * xgroups) * px;
    const int xs = x.index ? x.index[slot] : slot;
    const int ys = y.index ? y.index[slot] : slot;
    const int xld = x.ld > 0 ? x.ld : c, yld = y.ld > 0 ? y.ld : c;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)((const bf16_t*)x.p + (int64_t)xs * x.sample_stride), 0, 0x7fffffff, 0x00020000);
    float acc[PX][8];
#pragma unroll
    for (int p = 0; p < PX; ++p)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[p][i] = 0.f;
    const int iy0 = oy * stride - pad, ix0 = ox0 * stride - pad;
    if (wide) {
        if constexpr (STRIDE > 0) {
            switch (n) {
                case 1: dws_rows_px<1, STRIDE, PX>(acc, rsrc, w, KS, C, k0, iy0, ix0, H, W, xld, ch); break;
                case 3: dws_rows_px<3, STRIDE, PX>(acc, rsrc, w, KS, C, k0, iy0, ix0, H, W, xld, ch); break;
                case 5: dws_rows_px<5, STRIDE, PX>(acc, rsrc, w, KS, C, k0, iy0, ix0, H, W, xld, ch); break;
                default: dws_rows_px<7, STRIDE, PX>(acc, rsrc, w, KS, C, k0, iy0, ix0, H, W, xld, ch); break;
            }
        }
    } else {
        switch (n) {
            case 1: dws_rows<1>(acc[0], rsrc, w, KS, C, k0, l, iy0, ix0, H, W, xld, ch); break;
            case 2: dws_rows<2>(acc[0], rsrc, w, KS, C, k0, l, iy0, ix0, H, W, xld, ch); break;
            case 3: dws_rows<3>(acc[0], rsrc, w, KS, C, k0, l, iy0, ix0, H, W, xld, ch); break;
            case 4: dws_rows<4>(acc[0], rsrc, w, KS, C, k0, l, iy0, ix0, H, W, xld, ch); break;
            case 5: dws_rows<5>(acc[0], rsrc, w, KS, C, k0, l, iy0, ix0, H, W, xld, ch); break;
            case 6: dws_rows<6>(acc[0], rsrc, w, KS, C, k0, l, iy0, ix0, H, W, xld, ch); break;
            default: dws_rows<7>(acc[0], rsrc, w, KS, C, k0, l, iy0, ix0, H, W, xld, ch); break;
        }
    }
    const int64_t ti = (int64_t)gt.row[g] * tab_ld + ch;
    float sc[8], sh[8];
    loadf8(scale + ti, sc);
    loadf8(shift + ti, sh);
    bf16_t* yp = (bf16_t*)y.p + (int64_t)ys * y.sample_stride + ((int64_t)oy * Wo + ox0) * yld + ch;
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        if (p >= px || ox0 + p >= Wo) break;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc[p][i] = acc[p][i] * sc[i] + sh[i];
            if (act == DS_ACT_RELU) acc[p][i] = fmaxf(acc[p][i], 0.f);
        }
        *(uint4*)(yp + (int64_t)p * yld) = pack8(acc[p]);
    }
}

// ---- channel re-weighting by the attention head of the gate (Section 3.5, Eq. 23) ---------
// NHWC bf16: 8 channels per thread; channels at or beyond the sample's width are not touched
__global__ __launch_bounds__(256) void channel_scale_nhwc_bf16_kernel(const bf16_t* x, bf16_t* y, const float* scale,
                                                                      const int32_t* c_in, int C, int HW) {
    const int b = blockIdx.y;
    const int c = c_in ? c_in[b] : C;
    const int chunks = c >> 3;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= HW * chunks) return;
    const int p = idx / chunks, ch = (idx - p * chunks) * 8;
    const int64_t off = ((int64_t)b * HW + p) * C + ch;
    float v[8], f[8];
    unpack8(*(const uint4*)(x + off), v);
    loadf8(scale + (int64_t)b * C + ch, f);
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= f[i];
    *(uint4*)(y + off) = pack8(v);
}

template <typename T>
__device__ __forceinline__ float ld_as_float(const T* p);
template <>
__device__ __forceinline__ float ld_as_float<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float ld_as_float<bf16_t>(const bf16_t* p) { return bf2f(*p); }
__device__ __forceinline__ void st_from_float(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_from_float(bf16_t* p, float v) { *p = f2bf(v); }

// any other layout / type: one element per thread; grid (ceil(C*HW/256), B)
template <typename T, bool NHWC>
__global__ __launch_bounds__(256) void channel_scale_kernel(const T* x, T* y, const float* scale, const int32_t* c_in,
                                                            int C, int HW) {
    const int b = blockIdx.y;
    const int c = c_in ? c_in[b] : C;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= C * HW) return;
    const int ch = NHWC ? idx % C : idx / HW;
    if (ch >= c) return;
    const int64_t off = (int64_t)b * C * HW + idx;
    st_from_float(y + off, ld_as_float<T>(x + off) * scale[(int64_t)b * C + ch]);
}

// ---- LayerNorm over the valid slice; one wavefront per row ----------------------
__global__ __launch_bounds__(256) void layernorm_kernel(ActView x, ActView y, const float* gamma,
                                                        const float* beta, float eps, const int32_t* slot_group,
                                                        const GroupTable gt, int B, int rows, int row0, int n_rows) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (r >= B * n_rows) return;
    const int slot = r / n_rows, p = row0 + (r - slot * n_rows);
    (void)rows;
    const int g = slot_group ? slot_group[slot] : 0;
    const int d = gt.k_in[g];
    const int xs = x.index ? x.index[slot] : slot, ys = y.index ? y.index[slot] : slot;
    const int xld = x.ld > 0 ? x.ld : d, yld = y.ld > 0 ? y.ld : d;
    const bf16_t* xr = (const bf16_t*)x.p + (int64_t)xs * x.sample_stride + (int64_t)p * xld;
    bf16_t* yr = (bf16_t*)y.p + (int64_t)ys * y.sample_stride + (int64_t)p * yld;
    constexpr int MAXC = 4;  // up to 4 chunks of 8 per lane: d <= 2048
    float v[MAXC][8];
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
        const int ch = (k * 64 + lane) * 8;
        if (ch < d) {
            unpack8(*(const uint4*)(xr + ch), v[k]);
#pragma unroll
            for (int i = 0; i < 8; ++i) s += v[k][i];
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    const float mu = s / (float)d;
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
        const int ch = (k * 64 + lane) * 8;
        if (ch < d) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float t = v[k][i] - mu;
                q += t * t;
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o, 64);
    const float rstd = 1.0f / sqrtf(q / (float)d + eps);
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
        const int ch = (k * 64 + lane) * 8;
        if (ch < d) {
            float gm[8], bt[8], o8[8];
            loadf8(gamma + ch, gm);
            loadf8(beta + ch, bt);
#pragma unroll
            for (int i = 0; i < 8; ++i) o8[i] = (v[k][i] - mu) * rstd * gm[i] + bt[i];
            *(uint4*)(yr + ch) = pack8(o8);
        }
    }
}

// Narrow rows (d <= 512): 16 lanes per row, 4 rows per wavefront, so a wavefront keeps four
// independent rows of loads in flight and the reductions take 4 exchange steps instead of 6.
// gamma and beta (fp32, four times the bytes of a bf16 row between them) go through LDS once per
// workgroup instead of through the vector cache once per row.
__global__ __launch_bounds__(256) void layernorm16_kernel(ActView x, ActView y, const float* gamma,
                                                          const float* beta, float eps, const int32_t* slot_group,
                                                          const GroupTable gt, int B, int row0, int n_rows, int dmax) {
    __shared__ __attribute__((aligned(16))) float gl[512], bl[512];
    const int r = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int l16 = threadIdx.x & 15;
    const bool live = r < B * n_rows;
    const int rr = live ? r : 0;
    const int slot = rr / n_rows, p = row0 + (rr - slot * n_rows);
    const int g = slot_group ? slot_group[slot] : 0;
    const int d = gt.k_in[g];
    const int xs = x.index ? x.index[slot] : slot, ys = y.index ? y.index[slot] : slot;
    const int xld = x.ld > 0 ? x.ld : d, yld = y.ld > 0 ? y.ld : d;
    const bf16_t* xr = (const bf16_t*)x.p + (int64_t)xs * x.sample_stride + (int64_t)p * xld;
    bf16_t* yr = (bf16_t*)y.p + (int64_t)ys * y.sample_stride + (int64_t)p * yld;
    constexpr int MAXC = 4;
    // the affine parameters: one float2 of each per thread (256 threads x 2 = 512 channels), requested with the row
    const int pc = threadIdx.x * 2;
    float2 gq = make_float2(0.f, 0.f), bq = make_float2(0.f, 0.f);
    if (pc < dmax) {
        gq = *(const float2*)(gamma + pc);
        bq = *(const float2*)(beta + pc);
    }
    float v[MAXC][8];
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
        const int ch = (k * 16 + l16) * 8;
        if (live && ch < d) {
            unpack8(*(const uint4*)(xr + ch), v[k]);
#pragma unroll
            for (int i = 0; i < 8; ++i) s += v[k][i];
        }
    }
    *(float2*)(gl + pc) = gq;
    *(float2*)(bl + pc) = bq;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 16);
    const float mu = s / (float)d;
    float q = 0.f;
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
        const int ch = (k * 16 + l16) * 8;
        if (live && ch < d) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float t = v[k][i] - mu;
                q += t * t;
            }
        }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) q += __shfl_xor(q, o, 16);
    const float rstd = 1.0f / sqrtf(q / (float)d + eps);
    __syncthreads();
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
        const int ch = (k * 16 + l16) * 8;
        if (live && ch < d) {
            float o8[8];
            const float4 g0 = *(const float4*)(gl + ch), g1 = *(const float4*)(gl + ch + 4);
            const float4 b0 = *(const float4*)(bl + ch), b1 = *(const float4*)(bl + ch + 4);
            const float gm[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
            const float bt[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i) o8[i] = (v[k][i] - mu) * rstd * gm[i] + bt[i];
            *(uint4*)(yr + ch) = pack8(o8);
        }
    }
}

// ---- stem: KxK stride-s convolution of a 3-channel NCHW image -> NHWC ----------
// weights [K*K*3][Cout] bf16 staged in LDS as fp32; thread = (pixel, 8 output channels)
__global__ __launch_bounds__(256) void stem_kernel(const bf16_t* img, const int32_t* index, bf16_t* y,
                                                   const bf16_t* w, const float* scale, const float* shift, int H,
                                                   int W, int Ho, int Wo, int K, int stride, int pad, int Cout) {
    extern __shared__ float wl[];  // [K*K*3][Cout]
    const int nw = K * K * 3 * Cout;
    for (int i = threadIdx.x; i < nw; i += 256) wl[i] = bf2f(w[i]);
    __syncthreads();
    const int chunks = Cout >> 3;
    const int ppb = 256 / chunks;  // pixels per block
    const int slot = blockIdx.y;
    const int pl = threadIdx.x / chunks, ch = (threadIdx.x - pl * chunks) * 8;
    const int pix = blockIdx.x * ppb + pl;
    if (pl >= ppb || pix >= Ho * Wo) return;
    const int oy = pix / Wo, ox = pix - oy * Wo;
    const int sample = index ? index[slot] : slot;
    const bf16_t* ip = img + (int64_t)sample * 3 * H * W;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int u = 0; u < K; ++u) {
        const int iy = oy * stride + u - pad;
        if (iy < 0 || iy >= H) continue;
        for (int v = 0; v < K; ++v) {
            const int ix = ox * stride + v - pad;
            if (ix < 0 || ix >= W) continue;
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const float xv = bf2f(ip[((int64_t)c * H + iy) * W + ix]);
                const float* wp = wl + ((u * K + v) * 3 + c) * Cout + ch;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = fmaf(xv, wp[i], acc[i]);
            }
        }
    }
    float sc[8], sh[8];
    loadf8(scale + ch, sc);
    loadf8(shift + ch, sh);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = fmaxf(acc[i] * sc[i] + sh[i], 0.f);
    *(uint4*)(y + ((int64_t)slot * Ho * Wo + pix) * Cout + ch) = pack8(acc);
}

// ---- 3x3 stride-2 pad-1 max-pool, NHWC -----------------------------------------
__global__ __launch_bounds__(256) void maxpool_kernel(const bf16_t* x, bf16_t* y, int H, int W, int Ho, int Wo, int C) {
    const int chunks = C >> 3;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= Ho * Wo * chunks) return;
    const int b = blockIdx.y;
    const int pix = idx / chunks, ch = (idx - pix * chunks) * 8;
    const int oy = pix / Wo, ox = pix - oy * Wo;
    float m[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) m[i] = -INFINITY;
#pragma unroll
    for (int u = 0; u < 3; ++u) {
        const int iy = oy * 2 + u - 1;
        if (iy < 0 || iy >= H) continue;
#pragma unroll
        for (int v = 0; v < 3; ++v) {
            const int ix = ox * 2 + v - 1;
            if (ix < 0 || ix >= W) continue;
            float xv[8];
            unpack8(*(const uint4*)(x + (((int64_t)b * H + iy) * W + ix) * C + ch), xv);
#pragma unroll
            for (int i = 0; i < 8; ++i) m[i] = fmaxf(m[i], xv[i]);
        }
    }
    *(uint4*)(y + (((int64_t)b * Ho + oy) * Wo + ox) * C + ch) = pack8(m);
}

// ---- patch extraction: NCHW image -> [slot][patch][(c,u,v)] ----------------------
__global__ __launch_bounds__(256) void patchify_kernel(const bf16_t* img, const int32_t* index, bf16_t* out, int H,
                                                       int W, int P) {
    const int gw = W / P, gh = H / P;
    const int kchunks = 3 * P * P / 8;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= gh * gw * kchunks) return;
    const int slot = blockIdx.y;
    const int sample = index ? index[slot] : slot;
    const int patch = idx / kchunks, kc = (idx - patch * kchunks) * 8;
    const int gy = patch / gw, gx = patch - gy * gw;
    const int c = kc / (P * P), rem = kc - c * P * P;
    const int u = rem / P, v = rem - u * P;
    const uint4 q = *(const uint4*)(img + (((int64_t)sample * 3 + c) * H + gy * P + u) * W + gx * P + v);
    *(uint4*)(out + ((int64_t)slot * gh * gw + patch) * (3 * P * P) + kc) = q;
}

// class-token row: x[slot][0][:d] = cls[:d] + pos[0][:d]
__global__ void cls_rows_kernel(ActView x, const bf16_t* cls, const bf16_t* pos, const int32_t* slot_group,
                                const GroupTable gt) {
    const int slot = blockIdx.x;
    const int g = slot_group ? slot_group[slot] : 0;
    const int d = gt.k_in[g];
    const int xs = x.index ? x.index[slot] : slot;
    bf16_t* xr = (bf16_t*)x.p + (int64_t)xs * x.sample_stride;
    for (int i = threadIdx.x; i < d; i += blockDim.x) xr[i] = f2bf(bf2f(cls[i]) + bf2f(pos[i]));
}

// ---- fp32 NCHW direct convolution (single dynamic block, Eq. 9 + Eq. 14) ---------
// grid (ceil(Ho*Wo/256), C_O, B); thread = one output element; samples keep their order
__global__ __launch_bounds__(256) void conv_f32_kernel(const float* x, const float* w, const float* scale,
                                                       const float* shift, int tab_ld, const float* residual,
                                                       float* y, const int32_t* slot_group, const int32_t* perm,
                                                       const GroupTable gt, int C_I, int C_O, int H, int W, int Ho,
                                                       int Wo, int K, int stride, int pad, int act) {
    const int slot = blockIdx.z;
    const int g = slot_group ? slot_group[slot] : 0;
    const int o = blockIdx.y;
    if (o >= gt.k_out[g]) return;
    const int pix = blockIdx.x * 256 + threadIdx.x;
    if (pix >= Ho * Wo) return;
    const int b = perm ? perm[slot] : slot;
    const int c_in = gt.k_in[g];
    const int oy = pix / Wo, ox = pix - oy * Wo;
    const float* xb = x + (int64_t)b * C_I * H * W;
    const float* wo = w + (int64_t)o * C_I * K * K;
    float acc = 0.f;
    for (int i = 0; i < c_in; ++i) {
        for (int u = 0; u < K; ++u) {
            const int iy = oy * stride + u - pad;
            if (iy < 0 || iy >= H) continue;
            for (int v = 0; v < K; ++v) {
                const int ix = ox * stride + v - pad;
                if (ix < 0 || ix >= W) continue;
                acc = fmaf(wo[(i * K + u) * K + v], xb[((int64_t)i * H + iy) * W + ix], acc);
            }
        }
    }
    const int64_t ti = (int64_t)gt.row[g] * tab_ld + o;
    float val = acc * (scale ? scale[ti] : 1.f) + (shift ? shift[ti] : 0.f);
    const int64_t yi = (((int64_t)b * C_O + o) * Ho + oy) * Wo + ox;
    if (residual) val += residual[yi];
    if (act == DS_ACT_RELU) val = fmaxf(val, 0.f);
    y[yi] = val;
}

__global__ void compose_index_kernel(const int32_t* inner, const int32_t* outer, int32_t* out, int B) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < B) out[j] = inner[outer[j]];
}

__global__ void lookup_kernel(const int32_t* idx, const GroupTable gt, int which, int32_t* out, int B) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= B) return;
    const int g = idx[j];
    out[j] = which == 0 ? gt.k_in[g] : (which == 1 ? gt.k_out[g] : gt.row[g]);
}

__global__ void set_offsets_kernel(int32_t* offsets, int B) {
    if (threadIdx.x == 0) { offsets[0] = 0; offsets[1] = B; }
}

__global__ void make_key_kernel(const int32_t* hi, const int32_t* lo, int mul, int32_t* key, int B) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < B) key[j] = hi[j] * mul + (lo ? lo[j] : 0);
}

}  // namespace

int32_t ds_launch_set_offsets(int32_t* offsets, int32_t B, hipStream_t s) {
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(set_offsets_kernel, dim3(1), dim3(64), 0, s, offsets, B);
    DS_CHECK_LAUNCH("set offsets");
    return DS_OK;
}

int32_t ds_launch_make_key(const int32_t* hi, const int32_t* lo, int32_t mul, int32_t* key, int32_t B, hipStream_t s) {
    if (B <= 0) return DS_OK;
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(make_key_kernel, dim3((B + 255) / 256), dim3(256), 0, s, hi, lo, mul, key, B);
    DS_CHECK_LAUNCH("make key");
    return DS_OK;
}

int32_t ds_launch_expand_groups(const int32_t* offsets, int32_t T, int32_t* slot_group, hipStream_t s) {
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(expand_groups_kernel, dim3(1), dim3(256), 0, s, offsets, T, slot_group);
    DS_CHECK_LAUNCH("expand groups");
    return DS_OK;
}

int32_t ds_launch_dwconv(ActView x, ActView y, const bf16_t* w, const float* scale, const float* shift,
                         int32_t tab_ld, const int32_t* slot_group, const GroupTable& gt, int32_t B, int32_t C,
                         int32_t H, int32_t W, int32_t stride, int32_t act, hipStream_t s) {
    if (B <= 0) return DS_OK;
    const int Ho = (H + 2 - 3) / stride + 1, Wo = (W + 2 - 3) / stride + 1;
    int cmax = 0;
    for (int t = 0; t < gt.T; ++t) cmax = gt.k_in[t] > cmax ? gt.k_in[t] : cmax;
    const int px = stride == 1 ? 4 : DW_PX_S2;
    const int64_t n = (int64_t)Ho * ((Wo + px - 1) / px) * (cmax / 8);
    if (n <= 0) return DS_OK;
    const int slots8 = (B + 7) & ~7;
    const int64_t nwg = ((n + 255) / 256) * slots8;
    if (nwg > 0x7fffffffll) DS_FAIL(DS_ESHAPE, "depthwise conv: %lld workgroups exceed the launch limit", (long long)nwg);
    dim3 grid((unsigned)nwg);
    ProfScope prof(DS_K_DWCONV, s);
    if (stride == 1)
        hipLaunchKernelGGL((dwconv4_kernel<1, 4>), grid, dim3(256), 0, s, x, y, w, scale, shift, tab_ld, slot_group, gt, C, H, W,
                           Ho, Wo, act, B, slots8);
    else
        hipLaunchKernelGGL((dwconv4_kernel<2, DW_PX_S2>), grid, dim3(256), 0, s, x, y, w, scale, shift, tab_ld, slot_group, gt, C, H, W,
                           Ho, Wo, act, B, slots8);
    DS_CHECK_LAUNCH("depthwise conv");
    return DS_OK;
}

int32_t ds_launch_dwconv_spatial(ActView x, ActView y, const bf16_t* w, int32_t KS, const float* scale, const float* shift,
                                 int32_t tab_ld, const int32_t* slot_group, const GroupTable& gt, const SpatialTable& st,
                                 int32_t B, int32_t C, int32_t H, int32_t W, int32_t stride, int32_t act, hipStream_t s) {
    if (B <= 0) return DS_OK;
    int64_t nmax = 0;
    for (int t = 0; t < gt.T; ++t) {
        if (st.n[t] < 1 || st.n[t] > 7) DS_FAIL(DS_EUNSUPPORTED, "spatial depthwise conv: %d taps per axis (1..7)", st.n[t]);
        const int span = (st.n[t] - 1) * st.l[t] + 1;
        const int Ho = (H + 2 * st.pad[t] - span) / stride + 1, Wo = (W + 2 * st.pad[t] - span) / stride + 1;
        if (Ho <= 0 || Wo <= 0) continue;
        const int px = (stride <= 2 && st.l[t] == 1) ? DWS_PX : 1;   // pixels per lane, as the kernel chooses them
        const int64_t n = (int64_t)Ho * ((Wo + px - 1) / px) * (gt.k_in[t] / 8);
        nmax = n > nmax ? n : nmax;
    }
    if (nmax <= 0) return DS_OK;
    const int slots8 = (B + 7) & ~7;
    const int64_t nwg = ((nmax + 255) / 256) * slots8;
    if (nwg > 0x7fffffffll) DS_FAIL(DS_ESHAPE, "spatial depthwise conv: %lld workgroups exceed the launch limit", (long long)nwg);
    dim3 grid((unsigned)nwg);
    ProfScope prof(DS_K_DWCONV, s);
    if (stride == 1)
        hipLaunchKernelGGL((dwconv_spatial_kernel<1, DWS_PX>), grid, dim3(256), 0, s, x, y, w, KS, scale, shift, tab_ld,
                           slot_group, gt, st, C, H, W, stride, act, B, slots8);
    else if (stride == 2)
        hipLaunchKernelGGL((dwconv_spatial_kernel<2, DWS_PX>), grid, dim3(256), 0, s, x, y, w, KS, scale, shift, tab_ld,
                           slot_group, gt, st, C, H, W, stride, act, B, slots8);
    else
        hipLaunchKernelGGL((dwconv_spatial_kernel<0, 1>), grid, dim3(256), 0, s, x, y, w, KS, scale, shift, tab_ld,
                           slot_group, gt, st, C, H, W, stride, act, B, slots8);
    DS_CHECK_LAUNCH("spatial depthwise conv");
    return DS_OK;
}

int32_t ds_launch_channel_scale(const void* x, void* y, const float* scale, const int32_t* c_in, int32_t dtype,
                                int32_t layout, int32_t B, int32_t C, int32_t HW, hipStream_t s) {
    if (B <= 0 || C <= 0 || HW <= 0) return DS_OK;
    ProfScope prof(DS_K_GATE, s);
    if (layout == DS_NHWC && dtype == DS_BF16 && (C % 8) == 0) {
        dim3 grid((unsigned)(((int64_t)HW * (C / 8) + 255) / 256), (unsigned)B);
        hipLaunchKernelGGL(channel_scale_nhwc_bf16_kernel, grid, dim3(256), 0, s, (const bf16_t*)x, (bf16_t*)y, scale, c_in, C,
                           HW);
    } else {
        dim3 grid((unsigned)(((int64_t)C * HW + 255) / 256), (unsigned)B);
        if (dtype == DS_BF16 && layout == DS_NHWC)
            hipLaunchKernelGGL((channel_scale_kernel<bf16_t, true>), grid, dim3(256), 0, s, (const bf16_t*)x, (bf16_t*)y, scale, c_in, C, HW);
        else if (dtype == DS_BF16)
            hipLaunchKernelGGL((channel_scale_kernel<bf16_t, false>), grid, dim3(256), 0, s, (const bf16_t*)x, (bf16_t*)y, scale, c_in, C, HW);
        else if (layout == DS_NHWC)
            hipLaunchKernelGGL((channel_scale_kernel<float, true>), grid, dim3(256), 0, s, (const float*)x, (float*)y, scale, c_in, C, HW);
        else
            hipLaunchKernelGGL((channel_scale_kernel<float, false>), grid, dim3(256), 0, s, (const float*)x, (float*)y, scale, c_in, C, HW);
    }
    DS_CHECK_LAUNCH("channel scale");
    return DS_OK;
}

int32_t ds_launch_layernorm(ActView x, ActView y, const float* gamma, const float* beta, float eps,
                            const int32_t* slot_group, const GroupTable& gt, int32_t B, int32_t rows,
                            int32_t row0, int32_t n_rows, hipStream_t s) {
    if (B <= 0 || n_rows <= 0) return DS_OK;
    const int64_t total = (int64_t)B * n_rows;
    ProfScope prof(DS_K_LAYERNORM, s);
    int dmax = 0;
    for (int t = 0; t < gt.T; ++t) dmax = gt.k_in[t] > dmax ? gt.k_in[t] : dmax;
    if (dmax <= 512) {
        hipLaunchKernelGGL(layernorm16_kernel, dim3((unsigned)((total + 15) / 16)), dim3(256), 0, s, x, y, gamma, beta, eps,
                           slot_group, gt, B, row0, n_rows, dmax);
        DS_CHECK_LAUNCH("layernorm");
        return DS_OK;
    }
    hipLaunchKernelGGL(layernorm_kernel, dim3((unsigned)((total + 3) / 4)), dim3(256), 0, s, x, y, gamma, beta, eps,
                       slot_group, gt, B, rows, row0, n_rows);
    DS_CHECK_LAUNCH("layernorm");
    return DS_OK;
}

int32_t ds_launch_stem(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                       const float* shift, int32_t B, int32_t H, int32_t W, int32_t K, int32_t stride,
                       int32_t pad, int32_t Cout, hipStream_t s) {
    if (B <= 0) return DS_OK;
    const int32_t rc = ds_launch_stem_mfma(img, index, y, w, scale, shift, B, H, W, K, stride, pad, Cout, s);
    if (rc != DS_EUNSUPPORTED) return rc;
    const int Ho = (H + 2 * pad - K) / stride + 1, Wo = (W + 2 * pad - K) / stride + 1;
    const int chunks = Cout / 8, ppb = 256 / chunks;
    dim3 grid((unsigned)((Ho * Wo + ppb - 1) / ppb), (unsigned)B);
    const size_t shm = (size_t)K * K * 3 * Cout * sizeof(float);
    ProfScope prof(DS_K_STEM, s);
    hipLaunchKernelGGL(stem_kernel, grid, dim3(256), shm, s, img, index, y, w, scale, shift, H, W, Ho, Wo, K, stride,
                       pad, Cout);
    DS_CHECK_LAUNCH("stem conv");
    return DS_OK;
}

int32_t ds_launch_maxpool(const bf16_t* x, bf16_t* y, int32_t B, int32_t H, int32_t W, int32_t C, hipStream_t s) {
    if (B <= 0) return DS_OK;
    const int Ho = (H + 2 - 3) / 2 + 1, Wo = (W + 2 - 3) / 2 + 1;
    const int64_t n = (int64_t)Ho * Wo * (C / 8);
    dim3 grid((unsigned)((n + 255) / 256), (unsigned)B);
    ProfScope prof(DS_K_MAXPOOL, s);
    hipLaunchKernelGGL(maxpool_kernel, grid, dim3(256), 0, s, x, y, H, W, Ho, Wo, C);
    DS_CHECK_LAUNCH("maxpool");
    return DS_OK;
}

int32_t ds_launch_head(ActView x, int32_t HW, const bf16_t* w, int32_t w_ld, const float* bias, int32_t n_out,
                       const int32_t* slot_c, const int32_t* out_index, float* logits, float* partial, int32_t B,
                       int32_t C, hipStream_t s) {
    if (B <= 0) return DS_OK;
    FcArgs f = {};
    f.c_item = slot_c; f.C = C; f.w = w; f.w_ld = w_ld; f.bias = bias; f.n_out = n_out; f.relu = 0;
    f.out_index = out_index; f.out = logits; f.out_ld = n_out; f.items = B;
    if (HW > 0) {
        GateArgs g = {};
        g.x = x.p; g.dtype = DS_BF16; g.layout = DS_NHWC; g.B = B; g.C = C; g.HW = HW;
        g.c_in = slot_c; g.x_index = x.index; g.x_sample_stride = x.sample_stride; g.x_ld = x.ld;
        g.partial = partial;
        int splits = 1;
        const int32_t rc = ds_launch_pool(g, DS_K_HEAD, &splits, s);
        if (rc) return rc;
        f.v_partial = partial; f.splits = splits; f.v_scale = 1.0f / (float)HW;
    } else {
        f.v_rows = (const bf16_t*)x.p; f.v_row_stride = x.sample_stride;
    }
    return ds_launch_fc(f, 1, 0, DS_K_HEAD, s);
}

int32_t ds_launch_patchify(const bf16_t* img, const int32_t* index, bf16_t* patches, int32_t B, int32_t H,
                           int32_t W, int32_t P, hipStream_t s) {
    if (B <= 0) return DS_OK;
    const int64_t n = (int64_t)(H / P) * (W / P) * (3 * P * P / 8);
    dim3 grid((unsigned)((n + 255) / 256), (unsigned)B);
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(patchify_kernel, grid, dim3(256), 0, s, img, index, patches, H, W, P);
    DS_CHECK_LAUNCH("patchify");
    return DS_OK;
}

int32_t ds_launch_cls_rows(ActView x, const bf16_t* cls, const bf16_t* pos, const int32_t* slot_group,
                           const GroupTable& gt, int32_t B, hipStream_t s) {
    if (B <= 0) return DS_OK;
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(cls_rows_kernel, dim3((unsigned)B), dim3(128), 0, s, x, cls, pos, slot_group, gt);
    DS_CHECK_LAUNCH("class-token rows");
    return DS_OK;
}

int32_t ds_launch_conv_f32_nchw(const float* x, const float* w, const float* scale, const float* shift,
                                int32_t tab_ld, const float* residual, float* y, const int32_t* slot_group,
                                const int32_t* perm, const GroupTable& gt, int32_t B, int32_t C_I, int32_t C_O,
                                int32_t H, int32_t W, int32_t K, int32_t stride, int32_t pad, int32_t act,
                                hipStream_t s) {
    if (B <= 0) return DS_OK;
    const int Ho = (H + 2 * pad - K) / stride + 1, Wo = (W + 2 * pad - K) / stride + 1;
    int omax = 0;
    for (int t = 0; t < gt.T; ++t) omax = gt.k_out[t] > omax ? gt.k_out[t] : omax;
    if (omax <= 0) return DS_OK;
    dim3 grid((unsigned)((Ho * Wo + 255) / 256), (unsigned)omax, (unsigned)B);
    ProfScope prof(DS_K_GEMM_TAPS, s);
    hipLaunchKernelGGL(conv_f32_kernel, grid, dim3(256), 0, s, x, w, scale, shift, tab_ld, residual, y, slot_group,
                       perm, gt, C_I, C_O, H, W, Ho, Wo, K, stride, pad, act);
    DS_CHECK_LAUNCH("fp32 conv");
    return DS_OK;
}

int32_t ds_launch_compose_index(const int32_t* inner, const int32_t* outer, int32_t* out, int32_t B, hipStream_t s) {
    if (B <= 0) return DS_OK;
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(compose_index_kernel, dim3((B + 255) / 256), dim3(256), 0, s, inner, outer, out, B);
    DS_CHECK_LAUNCH("compose index");
    return DS_OK;
}

int32_t ds_launch_lookup(const int32_t* idx, const GroupTable& gt, int32_t which, int32_t* out, int32_t B, hipStream_t s) {
    if (B <= 0) return DS_OK;
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(lookup_kernel, dim3((B + 255) / 256), dim3(256), 0, s, idx, gt, which, out, B);
    DS_CHECK_LAUNCH("lookup");
    return DS_OK;
}
