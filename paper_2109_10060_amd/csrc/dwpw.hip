// Depthwise-separable block in one kernel: 3x3 depthwise convolution + batch-norm + ReLU feeding the 1x1 pointwise
// convolution + batch-norm + ReLU (Section 3.2, Eq. 9 and Eq. 10 at full width: the blocks in front of the gate are
// not sliced, so there is one group and no route table).  The depthwise output of a tile of 128 consecutive output
// pixels never leaves the compute unit: it is written to LDS as the pixel operand of the pointwise GEMM, which saves
// one write and one read of the widest maps of the network.
//
// Workgroup = 128 consecutive output pixels of one sample (row-major), 4 wavefronts.
//   phase 1  each lane computes runs of PX output pixels x 8 channels exactly as the stand-alone depthwise kernel does
//            (whole input window requested up front with branch-free buffer loads, v_dot2 on channel pairs against
//            masked weight pairs), applies the depthwise batch-norm and ReLU, rounds to bf16 -- the value the unfused
//            path would have stored -- and writes it into the operand tile A[C/32][128][32] (XOR-swizzled 64-byte rows);
//   phase 2  for every 64 output channels: the pointwise weights of all C input channels go through LDS once, each
//            wavefront multiplies its 32 pixels (v_mfma_f32_32x32x16_bf16, the weights as the row operand so that a lane
//            ends with runs of four channels of its own pixel), batch-norm, ReLU, bf16, an LDS tile, 16-byte stores.
#include "common.h"

namespace {

constexpr int S_LD = 64 + 8;                   // staging tile row (bf16)
constexpr uint32_t OOB = 0x80000000u;

__device__ __forceinline__ int swz(int r) { return ((r >> 1) ^ (r >> 2)) & 3; }

__device__ __forceinline__ uint4 pack8r(const float* v) {
    uint4 q;
    q.x = f2bf2(v[0], v[1]); q.y = f2bf2(v[2], v[3]); q.z = f2bf2(v[4], v[5]); q.w = f2bf2(v[6], v[7]);
    return q;
}

struct DwPwArgs {
    const bf16_t* x;        // [B][H][W][C]
    bf16_t* y;              // [B][Ho][Wo][N]
    const bf16_t* wd;       // [9][C]
    const float *sd, *hd;   // [C]
    const bf16_t* wp;       // [N][w_ld]
    const float *sp, *hp;   // [N]
    int B, H, W, C, Ho, Wo, N, w_ld, tiles_per_image, by_die;
};

// all tiles of one sample on one die (workgroups are dealt to the 8 dies in turn): neighbouring tiles share input rows
__device__ __forceinline__ int tile_of(int v, int tiles_per_image, bool by_die) {
    if (!by_die) return v;
    const int vq = v >> 3, s8 = vq / tiles_per_image;
    return ((v & 7) + 8 * s8) * tiles_per_image + (vq - s8 * tiles_per_image);
}

// RT: 32-pixel row tiles per wavefront; the workgroup's tile is TPX = 128 RT consecutive output pixels.
// KCH: 32-channel chunks of the reduction (the last may be partly zeros)
template <int STRIDE, int PX, int RT, int KCH>
__global__ __launch_bounds__(256, 3) void dwpw_kernel(const DwPwArgs a) {
    constexpr int NCOL = (PX - 1) * STRIDE + 3, TPX = 128 * RT;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int C = a.C, N = a.N, Wo = a.Wo, H = a.H, W = a.W;
    constexpr int kch = KCH;
    char* As = smem;                                       // [kch][128][32] bf16
    char* Bs = smem + kch * TPX * 64;                      // [kch][64][32] bf16, later the staging tile [128][S_LD]
    const int tid = threadIdx.x;
    const int tile = tile_of(blockIdx.x, a.tiles_per_image, a.by_die);
    const int slot = tile / a.tiles_per_image;
    const int p0 = (tile - slot * a.tiles_per_image) * TPX;
    const int HoWo = a.Ho * Wo;

    // pointwise weights of the first 64 filters and their batch-norm constants: requested now, parked in registers
    // during phase 1, so that the tile's only exposed memory round trip is the one of its input window
    const int wchunks = C >> 3;                            // 16-byte pieces of real channels per weight row
    constexpr int wslots = KCH * 4;                        // pieces per row of the LDS tile (those past wchunks are zeros)
    constexpr int wpieces = 64 * wslots;                   // per 64-filter tile: 256 KCH, KCH per lane
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.wp, 0, 0x7fffffff, 0x00020000);
    uint4 wreg0 = make_uint4(0, 0, 0, 0), wreg1 = wreg0, wreg2 = wreg0, wreg3 = wreg0;
    float creg;
    // piece e of the 64-filter tile at n0: filter n0 + e / wslots, channels 8 (e % wslots) ..; zeros past N or C
#define DWPW_WLOAD(e_, n0_)                                                                            \
    ([&] {                                                                                             \
        const int nl = (e_) / wslots, c8 = (e_) - nl * wslots;                                         \
        const bool ok = (e_) < wpieces && (n0_) + nl < N && c8 < wchunks;                              \
        const auto t = __builtin_amdgcn_raw_buffer_load_b128(                                          \
            rsrc_w, (int)(ok ? (uint32_t)((((n0_) + nl) * a.w_ld + c8 * 8) * 2) : OOB), 0, 0);         \
        return make_uint4(t[0], t[1], t[2], t[3]);                                                     \
    }())
#define DWPW_FETCH(n0_)                                                                                \
    do {                                                                                               \
        wreg0 = DWPW_WLOAD(tid, n0_);                                                                  \
        if constexpr (KCH > 1) wreg1 = DWPW_WLOAD(tid + 256, n0_);                                     \
        if constexpr (KCH > 2) { wreg2 = DWPW_WLOAD(tid + 512, n0_); wreg3 = DWPW_WLOAD(tid + 768, n0_); } \
        creg = 0.f;                                                                                    \
        if (tid < 128 && (n0_) + (tid & 63) < N) creg = (tid < 64 ? a.sp : a.hp)[(n0_) + (tid & 63)];  \
    } while (0)
    DWPW_FETCH(0);

    // ---- phase 1: depthwise rows of this tile into the operand tile ------------------------------------------
    {
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(a.x + (int64_t)slot * H * W * C), 0, 0x7fffffff, 0x00020000);
        const int chunks = C >> 3;
        const int items = (TPX / PX) * chunks;
        // the last 32-channel chunk of a width that is no multiple of 32: its missing channels multiply as zeros
        for (int e = tid; e < TPX * (kch * 4 - chunks); e += 256) {
            const int row = e / (kch * 4 - chunks), c8 = chunks + (e - row * (kch * 4 - chunks));
            *(uint4*)(As + ((c8 >> 2) * TPX + row) * 64 + (((c8 & 3) ^ swz(row)) * 16)) = make_uint4(0, 0, 0, 0);
        }
        for (int e = tid; e < items; e += 256) {
            const int gl = e / chunks, c8 = e - gl * chunks, ch = c8 * 8;
            const int pl = gl * PX, p = p0 + pl;
            char* arow = As + ((c8 >> 2) * TPX + pl) * 64;
            if (p >= HoWo) {                               // rows past the sample: zeros (never stored, but multiplied)
#pragma unroll
                for (int q = 0; q < PX; ++q) *(uint4*)(arow + q * 64 + (((c8 & 3) ^ swz(pl + q)) * 16)) = make_uint4(0, 0, 0, 0);
                continue;
            }
            const int oy = p / Wo, ox0 = p - oy * Wo;
            const int ix0 = ox0 * STRIDE - 1;
            uint4 xin[3][NCOL];
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int iy = oy * STRIDE + u - 1;
                const bool rok = iy >= 0 && iy < H;
#pragma unroll
                for (int col = 0; col < NCOL; ++col) {
                    const int ix = ix0 + col;
                    const uint32_t off = (rok && ix >= 0 && ix < W) ? (uint32_t)(((iy * W + ix) * C + ch) * 2) : OOB;
                    const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
                    xin[u][col] = make_uint4(t[0], t[1], t[2], t[3]);
                }
            }
            uint4 win[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) win[t] = *(const uint4*)(a.wd + t * C + ch);
            float acc[PX][8];
#pragma unroll
            for (int q = 0; q < PX; ++q)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[q][i] = 0.f;
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
                    const uint4 q4 = xin[u][col];
                    const bf16x2_t xq[4] = {__builtin_bit_cast(bf16x2_t, q4.x), __builtin_bit_cast(bf16x2_t, q4.y),
                                            __builtin_bit_cast(bf16x2_t, q4.z), __builtin_bit_cast(bf16x2_t, q4.w)};
#pragma unroll
                    for (int q = 0; q < PX; ++q) {
                        const int v = col - q * STRIDE;
                        if (v >= 0 && v < 3) {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                acc[q][2 * j] = __builtin_amdgcn_fdot2_f32_bf16(xq[j], wlo[v][j], acc[q][2 * j], false);
                                acc[q][2 * j + 1] = __builtin_amdgcn_fdot2_f32_bf16(xq[j], whi[v][j], acc[q][2 * j + 1], false);
                            }
                        }
                    }
                }
            }
            float sc[8], sh[8];
            {
                const float4 s0 = *(const float4*)(a.sd + ch), s1 = *(const float4*)(a.sd + ch + 4);
                const float4 h0 = *(const float4*)(a.hd + ch), h1 = *(const float4*)(a.hd + ch + 4);
                sc[0] = s0.x; sc[1] = s0.y; sc[2] = s0.z; sc[3] = s0.w; sc[4] = s1.x; sc[5] = s1.y; sc[6] = s1.z; sc[7] = s1.w;
                sh[0] = h0.x; sh[1] = h0.y; sh[2] = h0.z; sh[3] = h0.w; sh[4] = h1.x; sh[5] = h1.y; sh[6] = h1.z; sh[7] = h1.w;
            }
#pragma unroll
            for (int q = 0; q < PX; ++q) {
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[q][i] = fmaxf(acc[q][i] * sc[i] + sh[i], 0.f);
                *(uint4*)(arow + q * 64 + (((c8 & 3) ^ swz(pl + q)) * 16)) = pack8r(acc[q]);
            }
        }
    }

    // ---- phase 2: pointwise GEMM, 64 output channels at a time ---------------------------------------------------
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int prow = wave * 32 * RT + l32;                 // this lane's pixel row in its wavefront's first row tile
    float* cst = (float*)(Bs + (kch * 64 * 64 > TPX * S_LD * 2 ? kch * 64 * 64 : TPX * S_LD * 2));   // [64] scale, [64] shift
    for (int n0 = 0; n0 < N; n0 += 64) {
        __syncthreads();                                   // operand tile complete / staging tile of the last pass read
        {
            const uint4 wr[4] = {wreg0, wreg1, wreg2, wreg3};
#pragma unroll
            for (int i = 0; i < KCH; ++i) {
                const int e = tid + 256 * i;
                {
                    const int nl = e / wslots, c8 = e - nl * wslots;
                    *(uint4*)(Bs + ((c8 >> 2) * 64 + nl) * 64 + (((c8 & 3) ^ swz(nl)) * 16)) = wr[i];
                }
            }
        }
        if (tid < 128) cst[tid] = creg;
        __syncthreads();
        if (n0 + 64 < N) DWPW_FETCH(n0 + 64);              // the next pass's weights travel during this pass
        f32x16_t acc[RT][2];
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[r][t][e] = 0.f;
        for (int kc = 0; kc < kch; ++kc) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int c = kk * 2 + lhi;
                bf16x8_t wf[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int nr = t * 32 + l32;
                    wf[t] = *(const bf16x8_t*)(Bs + (kc * 64 + nr) * 64 + ((c ^ swz(nr)) * 16));
                }
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    const int pr = prow + r * 32;
                    const bf16x8_t pf = *(const bf16x8_t*)(As + (kc * TPX + pr) * 64 + ((c ^ swz(pr)) * 16));
                    // filters as the row operand: the accumulator holds pixel pr and channels 32 t + 8 g + 4 lhi + 0..3
#pragma unroll
                    for (int t = 0; t < 2; ++t) acc[r][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[t], pf, acc[r][t], 0, 0, 0);
                }
            }
        }
        __syncthreads();                                   // weight tile read by every wavefront: reuse it for staging
        bf16_t* stile = (bf16_t*)Bs;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int chn = t * 32 + g * 8 + lhi * 4;
                const float4 s4 = *(const float4*)(cst + chn), h4 = *(const float4*)(cst + 64 + chn);
#pragma unroll
                for (int r = 0; r < RT; ++r) {
                    uint2 o;
                    o.x = f2bf2(fmaxf(acc[r][t][4 * g] * s4.x + h4.x, 0.f), fmaxf(acc[r][t][4 * g + 1] * s4.y + h4.y, 0.f));
                    o.y = f2bf2(fmaxf(acc[r][t][4 * g + 2] * s4.z + h4.z, 0.f), fmaxf(acc[r][t][4 * g + 3] * s4.w + h4.w, 0.f));
                    *(uint2*)(stile + (prow + r * 32) * S_LD + chn) = o;
                }
            }
        __syncthreads();
        bf16_t* yp = a.y + ((int64_t)slot * HoWo + p0) * N + n0;
        for (int c = tid; c < TPX * 8; c += 256) {
            const int pix = c >> 3, ch = (c & 7) * 8;
            if (p0 + pix < HoWo && n0 + ch < N) *(uint4*)(yp + (int64_t)pix * N + ch) = *(const uint4*)(stile + pix * S_LD + ch);
        }
    }
}

}  // namespace

// x [B][H][W][C] -> y [B][Ho][Wo][N], 3x3 depthwise (padding 1, stride 1 or 2) + folded batch-norm + ReLU, then 1x1
// pointwise + folded batch-norm + ReLU.  DS_EUNSUPPORTED for shapes the kernel is not written for (the caller then
// runs the two layers one after the other).
int32_t ds_launch_dwpw(const bf16_t* x, int32_t B, int32_t H, int32_t W, int32_t C, int32_t stride, const bf16_t* wd,
                       const float* sd, const float* hd, const bf16_t* wp, int32_t w_ld, int32_t N, const float* sp,
                       const float* hp, bf16_t* y, hipStream_t s) {
    if (B <= 0) return DS_OK;
    const int Ho = (H + 2 - 3) / stride + 1, Wo = (W + 2 - 3) / stride + 1;
    const int px = stride == 1 ? 4 : 2;
    if ((stride != 1 && stride != 2) || (C % 8) || C < 8 || C > 128 || (N % 8) || N < 8 || N > 128 || (w_ld % 8) || (Wo % px) || Ho < 1 ||
        (int64_t)H * W * C * 2 >= 0x7fffffffll)
        return DS_EUNSUPPORTED;
    DwPwArgs a;
    a.x = x; a.y = y; a.wd = wd; a.sd = sd; a.hd = hd; a.wp = wp; a.sp = sp; a.hp = hp;
    a.B = B; a.H = H; a.W = W; a.C = C; a.Ho = Ho; a.Wo = Wo; a.N = N; a.w_ld = w_ld;
    // 32 channels: 256-pixel tiles, so that every lane has a run of 4 pixels x 8 channels to compute
    const int rt = (stride == 1 && C <= 32) ? 2 : 1, tpx = 128 * rt;
    a.tiles_per_image = (Ho * Wo + tpx - 1) / tpx;
    const int64_t grid = (int64_t)B * a.tiles_per_image;
    if (grid > 0x7fffffffll) return DS_EUNSUPPORTED;
    a.by_die = (B % 8) == 0;
    const int kch = C <= 32 ? 1 : (C <= 64 ? 2 : 4);
    const int b_bytes = kch * 64 * 64, st_bytes = tpx * S_LD * 2;
    const int smem = kch * tpx * 64 + (b_bytes > st_bytes ? b_bytes : st_bytes) + 2 * 64 * 4;
    ProfScope prof(DS_K_DWCONV, s);
    const dim3 g((unsigned)grid), b(256);
#define DWPW_LAUNCH(S_, P_, R_)                                                                         \
    do {                                                                                               \
        if (kch == 1) hipLaunchKernelGGL((dwpw_kernel<S_, P_, R_, 1>), g, b, smem, s, a);              \
        else if (kch == 2) hipLaunchKernelGGL((dwpw_kernel<S_, P_, R_, 2>), g, b, smem, s, a);         \
        else hipLaunchKernelGGL((dwpw_kernel<S_, P_, R_, 4>), g, b, smem, s, a);                       \
    } while (0)
    if (stride == 1 && rt == 2) {
        hipLaunchKernelGGL((dwpw_kernel<1, 4, 2, 1>), g, b, smem, s, a);
    } else if (stride == 1) {
        DWPW_LAUNCH(1, 4, 1);
    } else {
        DWPW_LAUNCH(2, 2, 1);
    }
#undef DWPW_LAUNCH
    DS_CHECK_LAUNCH("depthwise + pointwise");
    return DS_OK;
}
