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

typedef short i16x2_t __attribute__((ext_vector_type(2)));

// Input patch of one tile: 3 x PR rows of PC pixels, fetched as 8-byte pieces.  Which piece a thread
// owns does not depend on the tile, so the decomposition is done once; per tile the pieces are requested
// with branch-free buffer loads (a piece outside the image gets an out-of-range offset and reads as
// zeros) and are held in registers while the previous tile is still being worked on.
template <int PR, int PC, int NTH, int XOFF>
struct PatchLoader {
    static constexpr int NCH = 3 * PR * (PC / 4), NL = (NCH + NTH - 1) / NTH;
    static constexpr uint32_t OOB = 0x80000000u;
    int r[NL], x[NL], plane[NL], lds[NL];
    uint2 v[NL];
    __device__ void init(int tid, int H, int W) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int c = tid + i * NTH;
            const int row = c / (PC / 4), ch = c - row * (PC / 4);
            const int cc = row / PR;
            r[i] = row - cc * PR;
            x[i] = ch * 4 - XOFF;
            plane[i] = cc * H * W;
            lds[i] = c < NCH ? row * PC + ch * 4 : -1;
        }
    }
    // iy0, ix0: image row / column of patch row 0 / the patch's column XOFF
    __device__ void issue(const bf16_t* img, int sample, int iy0, int ix0, int H, int W) {
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(img + (int64_t)sample * 3 * H * W), 0, 0x7fffffff, 0x00020000);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int iy = iy0 + r[i], col0 = ix0 + x[i];
            const bool ok = lds[i] >= 0 && iy >= 0 && iy < H && col0 >= 0 && col0 + 3 < W;
            const uint32_t off = ok ? (uint32_t)((plane[i] + iy * W + col0) * 2) : OOB;
            const auto t = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)off, 0, 0);
            v[i] = make_uint2(t[0], t[1]);
        }
    }
    __device__ void store(bf16_t* patch) const {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            if (lds[i] >= 0) *(uint2*)(patch + lds[i]) = v[i];
    }
};

// Tile order.  Workgroups are dealt to the 8 dies in turn (blockIdx.x % 8), each die with an L2 of its own, and the
// input patches of neighbouring tiles overlap (the filter's halo, and 64-byte lines shared across a tile edge): with
// tiles walked in plain order every die fetches those lines from memory for itself, about four times the image in
// all.  With by_die (grid and batch multiples of 8) walk index v stands for tile (v / 8) % tiles_per_image of sample
// v % 8 + 8 * (v / 8 / tiles_per_image), so every tile of one sample is worked on by the same die.
__device__ __forceinline__ int tile_of(int v, int tiles_per_image, bool by_die) {
    if (!by_die) return v;
    const int vq = v >> 3, s8 = vq / tiles_per_image;
    return ((v & 7) + 8 * s8) * tiles_per_image + (vq - s8 * tiles_per_image);
}

template <int KS, int PAD, int VP, int NTILES>
__global__ __launch_bounds__(256) void stem_mfma_kernel(const bf16_t* __restrict__ img, const int32_t* index,
                                                        bf16_t* __restrict__ y, const bf16_t* __restrict__ w,
                                                        const float* scale, const float* shift, int H, int W, int Ho,
                                                        int Wo, int tiles_x, int tiles_y, int total_tiles, int cout, int by_die) {
    // cout <= COUT filters are stored ([taps][cout]) and written (cout channels per pixel); the matrix
    // columns beyond them carry zero weights and are dropped
    constexpr int COUT = NTILES * 32, PAIRS = 3 * KS, KP = ((PAIRS * VP + 15) / 16) * 16, KSTEPS = KP / 16;
    constexpr int W_LD = KP + 8, TH = 8, TW = 16, PR = 2 * TH + KS - 2, PC = 40, CBASE = 4 - PAD - 1;
    __shared__ __attribute__((aligned(16))) bf16_t Wl[COUT * W_LD];
    __shared__ __attribute__((aligned(16))) bf16_t patch[3 * PR * PC];
    // output tile, one row of S_LD channels per pixel: a lane finishes runs of four channels of its own pixel (8-byte
    // writes), then the tile leaves as 16-byte pieces, 16 consecutive pixels of a map row making one contiguous run
    constexpr int S_LD = COUT + 8;
    __shared__ __attribute__((aligned(16))) bf16_t stile[TH * TW * S_LD];
    __shared__ __attribute__((aligned(16))) float scl[COUT], shl[COUT];
    const int tid = threadIdx.x;
    if (tid < COUT) {
        scl[tid] = tid < cout ? scale[tid] : 0.f;
        shl[tid] = tid < cout ? shift[tid] : 0.f;
    }
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
    const int chunks = cout >> 3;                       // 16-byte pieces per output pixel
    PatchLoader<PR, PC, 256, 4> pl;
    pl.init(tid, H, W);
    auto fetch = [&](int tile) {
        const int slot = tile / (tiles_x * tiles_y);
        const int t2 = tile - slot * tiles_x * tiles_y;
        const int ty = t2 / tiles_x, tx = t2 - ty * tiles_x;
        const int sample = __builtin_amdgcn_readfirstlane(index ? index[slot] : slot);
        pl.issue(img, sample, ty * TH * 2 - PAD, tx * TW * 2, H, W);
    };
    for (int v = blockIdx.x; v < total_tiles; v += gridDim.x) {
        const int tile = tile_of(v, tiles_x * tiles_y, by_die);
        const int slot = tile / (tiles_x * tiles_y);
        const int t2 = tile - slot * tiles_x * tiles_y;
        const int ty = t2 / tiles_x, tx = t2 - ty * tiles_x;
        const int oy0 = ty * TH, ox0 = tx * TW;
        fetch(tile);      // all pieces in flight together
        __syncthreads();  // filter bank ready / previous patch no longer read
        pl.store(patch);
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
                // filters as the row operand: the accumulator holds this lane's pixel (column l32) and channels
                // 32 t + 8 g + 4 lhi + 0..3 in elements 4 g .. 4 g + 3
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af.v, acc[t], 0, 0, 0);
            }
        }
        // batch-norm, ReLU, bf16 rounding into the tile
#pragma unroll
        for (int t = 0; t < NTILES; ++t)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ch = t * 32 + g * 8 + lhi * 4;
                const float4 s4 = *(const float4*)(scl + ch), h4 = *(const float4*)(shl + ch);
                uint2 o;
                o.x = f2bf2(fmaxf(acc[t][4 * g] * s4.x + h4.x, 0.f), fmaxf(acc[t][4 * g + 1] * s4.y + h4.y, 0.f));
                o.y = f2bf2(fmaxf(acc[t][4 * g + 2] * s4.z + h4.z, 0.f), fmaxf(acc[t][4 * g + 3] * s4.w + h4.w, 0.f));
                *(uint2*)(stile + (wave * 32 + l32) * S_LD + ch) = o;
            }
        __syncthreads();
        for (int c = tid; c < TH * TW * chunks; c += 256) {
            const int pix = c / chunks, ch = (c - pix * chunks) * 8;
            const int oy = oy0 + (pix >> 4), ox = ox0 + (pix & 15);
            if (oy < Ho && ox < Wo)
                *(uint4*)(y + (((int64_t)slot * Ho + oy) * Wo + ox) * cout + ch) = *(const uint4*)(stile + pix * S_LD + ch);
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
                                                        int total_tiles, int by_die) {
    constexpr int KS = 7, PAD = 3, VP = 8, NTH = 320;
    constexpr int COUT = NTILES * 32, PAIRS = 3 * KS, KP = ((PAIRS * VP + 15) / 16) * 16, KSTEPS = KP / 16;
    constexpr int W_LD = KP + 8, CH = 9, CW = 17, NPIX = CH * CW, PR = 2 * CH + KS - 2, PC = 48, CBASE = 2;
    constexpr int C_LD = COUT + 8;                     // conv tile row stride in LDS (bf16)
    __shared__ __attribute__((aligned(16))) bf16_t Wl[COUT * W_LD];
    __shared__ __attribute__((aligned(16))) bf16_t patch[3 * PR * PC];
    __shared__ __attribute__((aligned(16))) bf16_t ctile[NPIX * C_LD];
    __shared__ __attribute__((aligned(16))) float scl[COUT], shl[COUT];
    const int tid = threadIdx.x;
    if (tid < COUT) {
        scl[tid] = scale[tid];
        shl[tid] = shift[tid];
    }
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
    // patch offset of this lane's 8 reduction values at every k-step (-1: padding beyond the last pair)
    int koff[KSTEPS];
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
        const int pair = (ks * 16 + lhi * 8) / VP;
        const int c = pair / KS, u = pair - c * KS;
        koff[ks] = pair < PAIRS ? (c * PR + 2 * pcy + u) * PC + 2 * pcx + CBASE : -1;
    }
    // input rows 2 oy0 - 3 .., columns 2 ox0 - 6 .. (a multiple of 4, so the 8-byte loads are aligned)
    PatchLoader<PR, PC, NTH, 6> pl;
    pl.init(tid, H, W);
    auto fetch = [&](int tile) {
        const int slot = tile / (tiles_x * tiles_y);
        const int t2 = tile - slot * tiles_x * tiles_y;
        const int ty = t2 / tiles_x, tx = t2 - ty * tiles_x;
        const int sample = __builtin_amdgcn_readfirstlane(index ? index[slot] : slot);
        pl.issue(img, sample, (8 * ty - 1) * 2 - PAD, (16 * tx - 1) * 2, H, W);
    };
    if ((int)blockIdx.x < total_tiles) fetch(tile_of(blockIdx.x, tiles_x * tiles_y, by_die));
    for (int v = blockIdx.x; v < total_tiles; v += gridDim.x) {
        const int tile = tile_of(v, tiles_x * tiles_y, by_die);
        const int slot = tile / (tiles_x * tiles_y);
        const int t2 = tile - slot * tiles_x * tiles_y;
        const int ty = t2 / tiles_x, tx = t2 - ty * tiles_x;
        const int p0 = ty * 4, q0 = tx * 8;            // pooled tile origin
        const int oy0 = 2 * p0 - 1, ox0 = 2 * q0 - 1;  // first convolution pixel
        __syncthreads();  // filter bank ready / previous patch and conv tile no longer read
        pl.store(patch);
        __syncthreads();
        if (v + (int)gridDim.x < total_tiles) fetch(tile_of(v + gridDim.x, tiles_x * tiles_y, by_die));   // in flight during this tile's arithmetic
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
                // filters as the row operand: the accumulator then holds this lane's own pixel (column l32)
                // and channels 32 t + 8 g + 4 lhi + 0..3 in elements 4 g .. 4 g + 3, i.e. runs of four
                // consecutive channels that go to LDS as one 8-byte write
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af.v, acc[t], 0, 0, 0);
            }
        }
        // batch-norm, ReLU, bf16 rounding
        if (pi < NPIX) {
            const int oy = oy0 + pcy, ox = ox0 + pcx;
            const bool in = oy >= 0 && oy < Ho && ox >= 0 && ox < Wo;
#pragma unroll
            for (int t = 0; t < NTILES; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int ch = t * 32 + g * 8 + lhi * 4;
                    const float4 s4 = *(const float4*)(scl + ch), h4 = *(const float4*)(shl + ch);
                    uint2 o;
                    o.x = f2bf2(fmaxf(acc[t][4 * g] * s4.x + h4.x, 0.f), fmaxf(acc[t][4 * g + 1] * s4.y + h4.y, 0.f));
                    o.y = f2bf2(fmaxf(acc[t][4 * g + 2] * s4.z + h4.z, 0.f), fmaxf(acc[t][4 * g + 3] * s4.w + h4.w, 0.f));
                    *(uint2*)(ctile + pi * C_LD + ch) = in ? o : make_uint2(0u, 0u);
                }
        }
        __syncthreads();
        // pooled pixel (pr, pc) of the tile, 8 channels per thread
        constexpr int CHUNKS = COUT / 8;
        for (int it = tid; it < 32 * CHUNKS; it += NTH) {
            const int ch = (it % CHUNKS) * 8, pp = it / CHUNKS;
            const int pr = pp >> 3, pc = pp & 7;
            if (p0 + pr >= Hp || q0 + pc >= Wp) continue;
            // every value is >= 0 after the ReLU, and non-negative bf16 values order like their bit patterns:
            // the maximum is a packed signed 16-bit integer maximum (a -0 loses to everything), no unpacking
            i16x2_t m[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) m[k] = i16x2_t{0, 0};
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int v = 0; v < 3; ++v) {
                    const uint4 q = *(const uint4*)(ctile + ((2 * pr + u) * CW + 2 * pc + v) * C_LD + ch);
                    const uint32_t qq[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                    for (int k = 0; k < 4; ++k) m[k] = __builtin_elementwise_max(m[k], __builtin_bit_cast(i16x2_t, qq[k]));
                }
            uint4 o;
            o.x = __builtin_bit_cast(uint32_t, m[0]);
            o.y = __builtin_bit_cast(uint32_t, m[1]);
            o.z = __builtin_bit_cast(uint32_t, m[2]);
            o.w = __builtin_bit_cast(uint32_t, m[3]);
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
    const int by_die = (B % 8) == 0 && (grid % 8) == 0;
    ProfScope prof(DS_K_STEM, s);
    hipLaunchKernelGGL((stem_mfma_kernel<KS, PAD, VP, NTILES>), dim3(grid), dim3(256), 0, s, img, index, y, w, scale, shift,
                       H, W, Ho, Wo, tiles_x, tiles_y, (int)total, cout, by_die);
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
    const int by_die = (B % 8) == 0 && (grid % 8) == 0;
    ProfScope prof(DS_K_STEM, s);
    hipLaunchKernelGGL((stem_pool_kernel<2>), dim3(grid), dim3(320), 0, s, img, index, y, w, scale, shift, H, W, Ho, Wo, Hp,
                       Wp, tiles_x, tiles_y, (int)total, by_die);
    DS_CHECK_LAUNCH("stem conv + max-pool");
    return DS_OK;
}

// returns DS_EUNSUPPORTED when the shape has no matrix-core variant (the caller then uses the direct kernel)
int32_t ds_launch_stem_mfma(const bf16_t* img, const int32_t* index, bf16_t* y, const bf16_t* w, const float* scale,
                            const float* shift, int32_t B, int32_t H, int32_t W, int32_t K, int32_t stride,
                            int32_t pad, int32_t Cout, hipStream_t s) {
    if (stride != 2 || (W % 4) != 0) return DS_EUNSUPPORTED;
    const int Ho = (H + 2 * pad - K) / 2 + 1, Wo = (W + 2 * pad - K) / 2 + 1;
    if (Cout < 8 || Cout > 64 || (Cout % 8) != 0) return DS_EUNSUPPORTED;  // the tile leaves in 8-channel pieces
    if (K == 7 && pad == 3 && Cout > 32) return launch_stem<7, 3, 8, 2>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, Cout, s);
    if (K == 7 && pad == 3) return launch_stem<7, 3, 8, 1>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, Cout, s);
    if (K == 3 && pad == 1 && Cout > 32) return launch_stem<3, 1, 4, 2>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, Cout, s);
    if (K == 3 && pad == 1) return launch_stem<3, 1, 4, 1>(img, index, y, w, scale, shift, B, H, W, Ho, Wo, Cout, s);
    return DS_EUNSUPPORTED;
}
