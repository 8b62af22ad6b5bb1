// Stem convolution on the matrix cores: KxK stride-2 convolution of a 3-channel NCHW
// bf16 image (never sliced; it feeds the first gate) with folded batch-norm and ReLU,
// written channels-last.
//
// A workgroup keeps the repacked filter bank in LDS and walks output tiles of 8x16
// pixels.  For each tile the input patch (3 x (2*8+K-2) x 40 pixels) is staged in LDS;
// the reduction index is ordered (channel, filter row, filter column) with the filter
// columns padded to 8 (7x7) or 4 (3x3) slots, so that the 8 reduction values a lane
// feeds to v_mfma_f32_32x32x16_bf16 are 8 (or 2x4) consecutive input pixels of one
// patch row: four 4-byte LDS reads, no gather.  Slot 0 of every padded group has a
// zero weight, which keeps those reads 4-byte aligned for stride 2.
#include "common.h"

namespace {

template <int KS, int PAD, int VP, int NTILES>
__global__ __launch_bounds__(256) void stem_mfma_kernel(const bf16_t* __restrict__ img, const int32_t* index,
                                                        bf16_t* __restrict__ y, const bf16_t* __restrict__ w,
                                                        const float* scale, const float* shift, int H, int W, int Ho,
                                                        int Wo, int tiles_x, int tiles_y, int total_tiles, int cout) {
    // cout <= COUT filters are stored ([taps][cout]) and written (cout channels per pixel); the matrix
    // columns beyond them carry zero weights and are dropped
    constexpr int COUT = NTILES * 32, PAIRS = 3 * KS, KP = ((PAIRS * VP + 15) / 16) * 16, KSTEPS = KP / 16;
    constexpr int W_LD = KP + 8, TH = 8, TW = 16, PR = 2 * TH + KS - 2, PC = 40, CBASE = 4 - PAD - 1;
    __shared__ __attribute__((aligned(16))) bf16_t Wl[COUT * W_LD];
    __shared__ __attribute__((aligned(16))) bf16_t patch[3 * PR * PC];
    const int tid = threadIdx.x;
    // filter bank: Wl[n][(c*KS + u)*VP + e] = w[u][e-1][c][n] for 1 <= e <= KS, else 0
    for (int i = tid; i < COUT * KP; i += 256) {
        const int n = i / KP, k = i - n * KP;
        const int pair = k / VP, e = k - pair * VP;
        const int c = pair / KS, u = pair - c * KS, v = e - 1;
        bf16_t val = 0;
        if (pair < PAIRS && v >= 0 && v < KS && n < cout) val = w[((u * KS + v) * 3 + c) * cout + n];
        Wl[n * W_LD + k] = val;
    }
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int py = wave * 2 + (l32 >> 4), px = l32 & 15;
    float sc[NTILES], sh[NTILES];
#pragma unroll
    for (int t = 0; t < NTILES; ++t) {
        sc[t] = t * 32 + l32 < cout ? scale[t * 32 + l32] : 0.f;
        sh[t] = t * 32 + l32 < cout ? shift[t * 32 + l32] : 0.f;
    }
    for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        const int slot = tile / (tiles_x * tiles_y);
        const int t2 = tile - slot * tiles_x * tiles_y;
        const int ty = t2 / tiles_x, tx = t2 - ty * tiles_x;
        const int oy0 = ty * TH, ox0 = tx * TW;
        const int sample = index ? index[slot] : slot;
        __syncthreads();  // filter bank ready / previous patch no longer read
        for (int c = tid; c < 3 * PR * (PC / 4); c += 256) {
            const int row = c / (PC / 4), ch = c - row * (PC / 4);
            const int cc = row / PR, r = row - cc * PR;
            const int iy = oy0 * 2 - PAD + r, col0 = ox0 * 2 - 4 + ch * 4;
            uint2 v = make_uint2(0, 0);
            if (iy >= 0 && iy < H && col0 >= 0 && col0 + 3 < W)
                v = *(const uint2*)(img + (((int64_t)sample * 3 + cc) * H + iy) * W + col0);
            *(uint2*)(patch + row * PC + ch * 4) = v;
        }
        __syncthreads();
        f32x16_t acc[NTILES];
#pragma unroll
        for (int t = 0; t < NTILES; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int kbase = ks * 16 + lhi * 8;
            union { uint32_t u[4]; bf16x8_t v; } af;
#pragma unroll
            for (int h = 0; h < 8 / VP; ++h) {
                const int pair = kbase / VP + h;
                const int c = pair / KS, u = pair - c * KS;
                const bf16_t* p = patch + (c * PR + 2 * py + u) * PC + 2 * px + CBASE;
#pragma unroll
                for (int q = 0; q < VP / 2; ++q)
                    af.u[h * (VP / 2) + q] = pair < PAIRS ? *(const uint32_t*)(p + 2 * q) : 0u;
            }
#pragma unroll
            for (int t = 0; t < NTILES; ++t) {
                const bf16x8_t bfr = *(const bf16x8_t*)(Wl + (t * 32 + l32) * W_LD + kbase);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bfr, acc[t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int i = 8 * (e >> 2) + 4 * lhi + (e & 3);
            const int oy = oy0 + wave * 2 + (i >> 4), ox = ox0 + (i & 15);
            if (oy < Ho && ox < Wo) {
                bf16_t* op = y + (((int64_t)slot * Ho + oy) * Wo + ox) * cout + l32;
#pragma unroll
                for (int t = 0; t < NTILES; ++t)
                    if (t * 32 + l32 < cout) op[t * 32] = f2bf(fmaxf(acc[t][e] * sc[t] + sh[t], 0.f));
            }
        }
    }
}

// 7x7 stride-2 stem fused with the 3x3 stride-2 padding-1 max-pool that follows it (the ResNet
// layout): the 112x112 map is never written.  A workgroup of 5 wavefronts computes the 9 x 17
// convolution pixels (153 of its 160 matrix rows) under a 4 x 8 tile of pooled pixels, applies
// batch-norm and ReLU, rounds to bf16 (the value the unfused path would have stored) into LDS,
// and pools from there with 16-byte stores.  Convolution pixels outside the map are stored as 0:
// after the ReLU every value is >= 0 and every pooling window holds at least its centre pixel,
// so 0 acts as the pool's padding.
template <int NTILES>
__global__ __launch_bounds__(320) void stem_pool_kernel(const bf16_t* __restrict__ img, const int32_t* index,
                                                        bf16_t* __restrict__ y, const bf16_t* __restrict__ w,
                                                        const float* scale, const float* shift, int H, int W, int Ho,
                                                        int Wo, int Hp, int Wp, int tiles_x, int tiles_y,
                                                        int total_tiles) {
    constexpr int KS = 7, PAD = 3, VP = 8, NTH = 320;
    constexpr int COUT = NTILES * 32, PAIRS = 3 * KS, KP = ((PAIRS * VP + 15) / 16) * 16, KSTEPS = KP / 16;
    constexpr int W_LD = KP + 8, CH = 9, CW = 17, NPIX = CH * CW, PR = 2 * CH + KS - 2, PC = 44, CBASE = 2;
    constexpr int C_LD = COUT + 8;                     // conv tile row stride in LDS (bf16)
    __shared__ __attribute__((aligned(16))) bf16_t Wl[COUT * W_LD];
    __shared__ __attribute__((aligned(16))) bf16_t patch[3 * PR * PC];
    __shared__ __attribute__((aligned(16))) bf16_t ctile[NPIX * C_LD];
    const int tid = threadIdx.x;
    for (int i = tid; i < COUT * KP; i += NTH) {
        const int n = i / KP, k = i - n * KP;
        const int pair = k / VP, e = k - pair * VP;
        const int c = pair / KS, u = pair - c * KS, v = e - 1;
        bf16_t val = 0;
        if (pair < PAIRS && v >= 0 && v < KS) val = w[((u * KS + v) * 3 + c) * COUT + n];
        Wl[n * W_LD + k] = val;
    }
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int pi = wave * 32 + l32;                    // this lane's convolution pixel as the A-operand row
    const int pcy = pi < NPIX ? pi / CW : 0, pcx = pi < NPIX ? pi - (pi / CW) * CW : 0;
    float sc[NTILES], sh[NTILES];
#pragma unroll
    for (int t = 0; t < NTILES; ++t) {
        sc[t] = scale[t * 32 + l32];
        sh[t] = shift[t * 32 + l32];
    }
    // patch offset of this lane's 8 reduction values at every k-step (-1: padding beyond the last pair)
    int koff[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
        const int pair = (ks * 16 + lhi * 8) / VP;
        const int c = pair / KS, u = pair - c * KS;
        koff[ks] = pair < PAIRS ? (c * PR + 2 * pcy + u) * PC + 2 * pcx + CBASE : -1;
    }
    for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
        const int slot = tile / (tiles_x * tiles_y);
        const int t2 = tile - slot * tiles_x * tiles_y;
        const int ty = t2 / tiles_x, tx = t2 - ty * tiles_x;
        const int p0 = ty * 4, q0 = tx * 8;            // pooled tile origin
        const int oy0 = 2 * p0 - 1, ox0 = 2 * q0 - 1;  // first convolution pixel
        const int sample = index ? index[slot] : slot;
        __syncthreads();  // filter bank ready / previous patch and conv tile no longer read
        // input rows 2 oy0 - 3 .., columns 2 ox0 - 6 .. (a multiple of 4, so the 8-byte loads are aligned)
        for (int c = tid; c < 3 * PR * (PC / 4); c += NTH) {
            const int row = c / (PC / 4), ch = c - row * (PC / 4);
            const int cc = row / PR, r = row - cc * PR;
            const int iy = oy0 * 2 - PAD + r, col0 = ox0 * 2 - 6 + ch * 4;
            uint2 v = make_uint2(0, 0);
            if (iy >= 0 && iy < H && col0 >= 0 && col0 + 3 < W)
                v = *(const uint2*)(img + (((int64_t)sample * 3 + cc) * H + iy) * W + col0);
            *(uint2*)(patch + row * PC + ch * 4) = v;
        }
        __syncthreads();
        f32x16_t acc[NTILES];
#pragma unroll
        for (int t = 0; t < NTILES; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            const int kbase = ks * 16 + lhi * 8;
            union { uint32_t u[4]; bf16x8_t v; } af;
            const bf16_t* p = patch + (koff[ks] < 0 ? 0 : koff[ks]);
#pragma unroll
            for (int q = 0; q < VP / 2; ++q) af.u[q] = koff[ks] >= 0 ? *(const uint32_t*)(p + 2 * q) : 0u;
#pragma unroll
            for (int t = 0; t < NTILES; ++t) {
                const bf16x8_t bfr = *(const bf16x8_t*)(Wl + (t * 32 + l32) * W_LD + kbase);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af.v, bfr, acc[t], 0, 0, 0);
            }
        }
        // batch-norm, ReLU, bf16 rounding; the accumulator holds pixel i of the wavefront, channel l32 (+32 t)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int i = wave * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
            if (i < NPIX) {
                const int cy = i / CW, cx = i - cy * CW;
                const int oy = oy0 + cy, ox = ox0 + cx;
                const bool in = oy >= 0 && oy < Ho && ox >= 0 && ox < Wo;
#pragma unroll
                for (int t = 0; t < NTILES; ++t)
                    ctile[i * C_LD + t * 32 + l32] = in ? f2bf(fmaxf(acc[t][e] * sc[t] + sh[t], 0.f)) : (bf16_t)0;
            }
        }
        __syncthreads();
        // pooled pixel (pr, pc) of the tile, 8 channels per thread
        constexpr int CHUNKS = COUT / 8;
        for (int it = tid; it < 32 * CHUNKS; it += NTH) {
            const int ch = (it % CHUNKS) * 8, pp = it / CHUNKS;
            const int pr = pp >> 3, pc = pp & 7;
            if (p0 + pr >= Hp || q0 + pc >= Wp) continue;
            float m[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) m[k] = 0.f;
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int v = 0; v < 3; ++v) {
                    const uint4 q = *(const uint4*)(ctile + ((2 * pr + u) * CW + 2 * pc + v) * C_LD + ch);
                    const uint32_t qq[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        m[2 * k] = fmaxf(m[2 * k], __uint_as_float(qq[k] << 16));
                        m[2 * k + 1] = fmaxf(m[2 * k + 1], __uint_as_float(qq[k] & 0xffff0000u));
                    }
                }
            uint4 o;
            o.x = f2bf2(m[0], m[1]);
            o.y = f2bf2(m[2], m[3]);
            o.z = f2bf2(m[4], m[5]);
            o.w = f2bf2(m[6], m[7]);
            *(uint4*)(y + (((int64_t)slot * Hp + p0 + pr) * Wp + q0 + pc) * COUT + ch) = o;
        }
    }
}

template <int KS, int PAD, int VP, int NTILES>
int32_t launch_stem(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                    const float* shift, int B, int H, int W, int Ho, int Wo, int cout, hipStream_t s) {
    const int tiles_x = (Wo + 15) / 16, tiles_y = (Ho + 7) / 8;
    const long long total = (long long)B * tiles_x * tiles_y;
    const int grid = (int)(total < 256 * 5 ? total : 256 * 5);
    ProfScope prof(DS_K_STEM, s);
    hipLaunchKernelGGL((stem_mfma_kernel<KS, PAD, VP, NTILES>), dim3(grid), dim3(256), 0, s, img, index, y, w, scale, shift,
                       H, W, Ho, Wo, tiles_x, tiles_y, (int)total, cout);
    DS_CHECK_LAUNCH("stem conv (mfma)");
    return DS_OK;
}

}  // namespace

// 7x7 stride-2 padding-3 stem (64 filters) + 3x3 stride-2 padding-1 max-pool in one kernel;
// y is the pooled map [B][Hp][Wp][64].  DS_EUNSUPPORTED for any other shape.
int32_t ds_launch_stem_pool(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                            const float* shift, int32_t B, int32_t H, int32_t W, int32_t K, int32_t stride,
                            int32_t pad, int32_t Cout, hipStream_t s) {
    if (K != 7 || stride != 2 || pad != 3 || Cout != 64 || (W % 4) != 0) return DS_EUNSUPPORTED;
    const int Ho = (H + 6 - 7) / 2 + 1, Wo = (W + 6 - 7) / 2 + 1;
    const int Hp = (Ho + 2 - 3) / 2 + 1, Wp = (Wo + 2 - 3) / 2 + 1;
    const int tiles_x = (Wp + 7) / 8, tiles_y = (Hp + 3) / 4;
    const long long total = (long long)B * tiles_x * tiles_y;
    if (total <= 0) return DS_OK;
    const int grid = (int)(total < 256 * 3 ? total : 256 * 3);
    ProfScope prof(DS_K_STEM, s);
    hipLaunchKernelGGL((stem_pool_kernel<2>), dim3(grid), dim3(320), 0, s, img, index, y, w, scale, shift, H, W, Ho, Wo, Hp,
                       Wp, tiles_x, tiles_y, (int)total);
    DS_CHECK_LAUNCH("stem conv + max-pool");
    return DS_OK;
}

// returns DS_EUNSUPPORTED when the shape has no matrix-core variant (the caller then uses the direct kernel)
int32_t ds_launch_stem_mfma(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                            const float* shift, int32_t B, int32_t H, int32_t W, int32_t K, int32_t stride,
                            int32_t pad, int32_t Cout, hipStream_t s) {
    if (stride != 2 || (W % 4) != 0) return DS_EUNSUPPORTED;
    const int Ho = (H + 2 * pad - K) / 2 + 1, Wo = (W + 2 * pad - K) / 2 + 1;
    if (Cout < 1 || Cout > 64) return DS_EUNSUPPORTED;
    if (K == 7 && pad == 3 && Cout > 32) return launch_stem<7, 3, 8, 2>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, Cout, s);
    if (K == 7 && pad == 3) return launch_stem<7, 3, 8, 1>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, Cout, s);
    if (K == 3 && pad == 1 && Cout > 32) return launch_stem<3, 1, 4, 2>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, Cout, s);
    if (K == 3 && pad == 1) return launch_stem<3, 1, 4, 1>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, Cout, s);
    return DS_EUNSUPPORTED;
}
