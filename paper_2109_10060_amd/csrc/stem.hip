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
                                                        int Wo, int tiles_x, int tiles_y, int total_tiles) {
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
        if (pair < PAIRS && v >= 0 && v < KS) val = w[((u * KS + v) * 3 + c) * COUT + n];
        Wl[n * W_LD + k] = val;
    }
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int py = wave * 2 + (l32 >> 4), px = l32 & 15;
    float sc[NTILES], sh[NTILES];
#pragma unroll
    for (int t = 0; t < NTILES; ++t) {
        sc[t] = scale[t * 32 + l32];
        sh[t] = shift[t * 32 + l32];
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
                bf16_t* op = y + (((int64_t)slot * Ho + oy) * Wo + ox) * COUT + l32;
#pragma unroll
                for (int t = 0; t < NTILES; ++t) op[t * 32] = f2bf(fmaxf(acc[t][e] * sc[t] + sh[t], 0.f));
            }
        }
    }
}

template <int KS, int PAD, int VP, int NTILES>
int32_t launch_stem(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                    const float* shift, int B, int H, int W, int Ho, int Wo, hipStream_t s) {
    const int tiles_x = (Wo + 15) / 16, tiles_y = (Ho + 7) / 8;
    const long long total = (long long)B * tiles_x * tiles_y;
    const int grid = (int)(total < 256 * 5 ? total : 256 * 5);
    ProfScope prof(DS_K_STEM, s);
    hipLaunchKernelGGL((stem_mfma_kernel<KS, PAD, VP, NTILES>), dim3(grid), dim3(256), 0, s, img, index, y, w, scale, shift,
                       H, W, Ho, Wo, tiles_x, tiles_y, (int)total);
    DS_CHECK_LAUNCH("stem conv (mfma)");
    return DS_OK;
}

}  // namespace

// returns DS_EUNSUPPORTED when the shape has no matrix-core variant (the caller then uses the direct kernel)
int32_t ds_launch_stem_mfma(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                            const float* shift, int32_t B, int32_t H, int32_t W, int32_t K, int32_t stride,
                            int32_t pad, int32_t Cout, hipStream_t s) {
    if (stride != 2 || (W % 4) != 0) return DS_EUNSUPPORTED;
    const int Ho = (H + 2 * pad - K) / 2 + 1, Wo = (W + 2 * pad - K) / 2 + 1;
    if (K == 7 && pad == 3 && Cout == 64) return launch_stem<7, 3, 8, 2>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, s);
    if (K == 7 && pad == 3 && Cout == 32) return launch_stem<7, 3, 8, 1>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, s);
    if (K == 3 && pad == 1 && Cout == 32) return launch_stem<3, 1, 4, 1>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, s);
    if (K == 3 && pad == 1 && Cout == 64) return launch_stem<3, 1, 4, 2>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, s);
    return DS_EUNSUPPORTED;
}
