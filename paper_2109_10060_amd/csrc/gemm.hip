// Grouped prefix-slice GEMM / implicit-GEMM convolution on the gfx950 matrix cores.
//
// One launch serves every route group of a layer.  Group g owns a contiguous
// range of bucket slots and multiplies its rows by the leading block
// W[:k_out[g], :k_in[g]] of the stored weight, read in place through the
// full-size leading stride (weight slicing, Section 3.2 Eq. 8; convolution
// filters, Section 3.3 Eq. 9).  A row of a sample is one token (linear layers)
// or one output pixel of a KxK convolution over an NHWC image; in the second
// case the K*K taps are walked inside the reduction loop and the A operand is
// gathered from the shifted input pixels (zero outside the image).
//
// Tiling: 128 x BN output tile per 256-thread workgroup (BN = 64, 128 or 256,
// chosen from the widest slice of the layer), 4 wavefronts, each holding a grid
// of v_mfma_f32_32x32x16_bf16 accumulators.  Operands go through LDS in 32-deep
// slabs (row stride padded to 40 elements: conflict-free 16-byte reads), double
// buffered, with the next slab's global loads in flight during the matrix
// instructions and one barrier per slab.  The epilogue (split batch-norm scale and
// shift or bias, residual, ReLU/GELU, bf16 rounding) re-reads the accumulators
// through LDS so that every lane stores 4 consecutive channels of one row.
//
// Work items are (m-tile, n-tile) pairs with the n-tile fastest; the linear block
// index is dealt round-robin to the 8 XCDs by the hardware, so each XCD is given
// a contiguous run of work items and the blocks that share an activation tile hit
// the same L2.
#include <stdlib.h>

#include "common.h"

namespace {

constexpr int BM = DS_GEMM_BM, BK = 32, LDS_LD = BK + 8, NT = 256;

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

template <int WROWS, int WCOLS, int WMT, int WNT>
struct Tile {
    static constexpr int BN = WCOLS * WNT * 32;
    static constexpr int COLS = WNT * 32;                      // columns staged per wavefront
    static constexpr int SROWS = COLS > 64 ? 16 : 32;          // rows staged per pass
    static constexpr int ST_LD = COLS + 4;
    static constexpr int LOOP_BYTES = 2 * (BM + BN) * LDS_LD * 2;
    static constexpr int STAGE_BYTES = 4 * SROWS * ST_LD * 4;
    static constexpr int MAIN_BYTES = LOOP_BYTES > STAGE_BYTES ? LOOP_BYTES : STAGE_BYTES;
    static constexpr int TABLE_BYTES = BM * (8 + 8 + 8 + 8);
    static constexpr int SMEM = MAIN_BYTES + TABLE_BYTES;
    static_assert(WROWS * WCOLS == 4 && WROWS * WMT * 32 == BM, "4 wavefronts cover a 128-row tile");
};

template <int WROWS, int WCOLS, int WMT, int WNT>
__global__ __launch_bounds__(NT) void gemm_kernel(const GemmArgs a, const int ny, const int max_mtiles) {
    using TL = Tile<WROWS, WCOLS, WMT, WNT>;
    constexpr int BN = TL::BN;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t* As = (bf16_t*)smem;                       // [2][BM][LDS_LD]
    bf16_t* Bs = As + 2 * BM * LDS_LD;                // [2][BN][LDS_LD]
    long long* rowA = (long long*)(smem + TL::MAIN_BYTES);
    long long* rowC = rowA + BM;
    long long* rowR = rowC + BM;
    int2* rowYX = (int2*)(rowR + BM);

    // ---- work item ------------------------------------------------------------------
    // m-tiles are dealt to the 8 XCDs round-robin; on one XCD consecutive blocks walk the n-tiles
    // of one m-tile, so the activation tile they share stays in that XCD's L2
    const int j = (int)(blockIdx.x >> 3);
    const int jm = j / ny, y = j - jm * ny;
    const int mt = jm * 8 + (int)(blockIdx.x & 7);
    if (mt >= max_mtiles) return;
    const int4 me = a.mtiles[mt];            // in-bounds even beyond the live count; checked next
    if (mt >= *a.n_mtiles) return;
    const int g = me.x, grow0 = me.y, slot0 = me.z, rows_g = me.w;
    const int k_in = a.gt.k_in[g], k_out = a.gt.k_out[g];
    if (k_in <= 0 || k_out <= 0) return;
    const int ntiles = (k_out + BN - 1) / BN;
    const int seg = y / ntiles;
    if (seg >= a.n_seg) return;
    const int n0 = (y - seg * ntiles) * BN;

    const int tid = threadIdx.x;
    const int a_ld = a.a_ld > 0 ? a.a_ld : k_in;
    const int c_ld = a.c_ld > 0 ? a.c_ld : k_out;
    const int r_ld = a.r_ld > 0 ? a.r_ld : k_out;

    // ---- per-row table: where each of the 128 rows lives --------------------------------
    if (tid < BM) {
        const int m = grow0 + tid;
        long long ra = -1, rc = -1, rr = 0;
        int2 yx = make_int2(0, 0);
        if (m < rows_g) {
            const int sl = m / a.rows;
            const int p = m - sl * a.rows;
            const int slot = slot0 + sl;
            const int sa = a.a_index ? a.a_index[slot] : slot;
            const int cs = a.c_index ? a.c_index[slot] : slot;
            const int oy = p / a.Wo, ox = p - oy * a.Wo;
            ra = (long long)sa * a.a_sample_stride;
            yx = make_int2(oy * a.stride - a.pad, ox * a.stride - a.pad);
            const long long pc = p + a.c_row0;
            rc = (long long)cs * a.c_sample_stride + pc * c_ld + (long long)seg * a.c_seg_stride;
            rr = (long long)(a.r_use_index ? cs : 0) * a.r_sample_stride + pc * r_ld;
        }
        rowA[tid] = ra;
        rowC[tid] = rc;
        rowR[tid] = rr;
        rowYX[tid] = yx;
    }
    __syncthreads();

    // ---- load assignment: A 2 chunks, B BN/64 chunks of 8 elements per thread ---------
    constexpr int NB = BN / 64;
    const int kc8 = (tid & 3) * 8;
    const int lrow = tid >> 2;
    long long abase[2];
    int2 ayx[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        abase[i] = rowA[lrow + 64 * i];
        ayx[i] = rowYX[lrow + 64 * i];
    }
    long long wrow[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int n = n0 + lrow + 64 * i;
        wrow[i] = n < k_out ? (long long)seg * a.w_seg_stride + (long long)n * a.w_ld : -1;
    }

    uint4 ra[2], rb[NB];
    auto load_global = [&](int tap, int kc) {
        const int u = tap / a.K, v = tap - u * a.K;
        const bool kok = (kc + kc8) < k_in;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int iy = ayx[i].x + u, ix = ayx[i].y + v;
            const bool ok = abase[i] >= 0 && kok && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
            ra[i] = make_uint4(0, 0, 0, 0);
            if (ok) ra[i] = *(const uint4*)(a.A + abase[i] + (long long)(iy * a.W + ix) * a_ld + kc + kc8);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            rb[i] = make_uint4(0, 0, 0, 0);
            if (wrow[i] >= 0 && kok) rb[i] = *(const uint4*)(a.Wt + wrow[i] + (long long)tap * a.w_tap_stride + kc + kc8);
        }
    };
    auto store_lds = [&](int buf) {
        bf16_t* as = As + buf * BM * LDS_LD;
        bf16_t* bs = Bs + buf * BN * LDS_LD;
#pragma unroll
        for (int i = 0; i < 2; ++i) *(uint4*)(as + (lrow + 64 * i) * LDS_LD + kc8) = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *(uint4*)(bs + (lrow + 64 * i) * LDS_LD + kc8) = rb[i];
    };

    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WCOLS, wn = wave - wm * WCOLS;
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16_t acc[WMT][WNT];
#pragma unroll
    for (int i = 0; i < WMT; ++i)
#pragma unroll
        for (int j = 0; j < WNT; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // epilogue constants, loaded early so their latency hides behind the main loop
    constexpr int COLS = TL::COLS, SROWS = TL::SROWS, ST_LD = TL::ST_LD;
    constexpr int CG = COLS / 4, RPP = 64 / CG, PASSES = 32 / SROWS, VPP = 16 / PASSES;
    const int cg = lane % CG, rr0 = lane / CG;
    const int ncol = n0 + wn * COLS + cg * 4;
    const bool nok = ncol < k_out;
    float sc[4] = {1.f, 1.f, 1.f, 1.f}, sh[4] = {0.f, 0.f, 0.f, 0.f};
    if (nok) {
        const long long ti = (long long)a.gt.row[g] * a.tab_ld + (long long)seg * a.tab_seg_stride + ncol;
        if (a.scale) {
            const float4 t = *(const float4*)(a.scale + ti);
            sc[0] = t.x; sc[1] = t.y; sc[2] = t.z; sc[3] = t.w;
        }
        if (a.shift) {
            const float4 t = *(const float4*)(a.shift + ti);
            sh[0] = t.x; sh[1] = t.y; sh[2] = t.z; sh[3] = t.w;
        }
    }
    const int kchunks = (k_in + BK - 1) / BK;
    const int nk = a.K * a.K * kchunks;
    int tap = 0, kc = 0;
    load_global(0, 0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        kc += BK;
        if (kc >= k_in) { kc = 0; ++tap; }
        const bool more = kt + 1 < nk;
        if (more) load_global(tap, kc);
        const bf16_t* as = As + buf * BM * LDS_LD + (wm * WMT * 32 + l32) * LDS_LD + lhi * 8;
        const bf16_t* bs = Bs + buf * BN * LDS_LD + (wn * WNT * 32 + l32) * LDS_LD + lhi * 8;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8_t af[WMT], bfr[WNT];
#pragma unroll
            for (int t = 0; t < WMT; ++t) af[t] = *(const bf16x8_t*)(as + t * 32 * LDS_LD + kk * 16);
#pragma unroll
            for (int t = 0; t < WNT; ++t) bfr[t] = *(const bf16x8_t*)(bs + t * 32 * LDS_LD + kk * 16);
#pragma unroll
            for (int i = 0; i < WMT; ++i)
#pragma unroll
                for (int j = 0; j < WNT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (more) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue through LDS: each lane finishes 4 consecutive channels of one row -----
    float* st = (float*)smem + wave * SROWS * ST_LD;
#pragma unroll
    for (int tm = 0; tm < WMT; ++tm) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
#pragma unroll
            for (int tn = 0; tn < WNT; ++tn)
#pragma unroll
                for (int vv = 0; vv < VPP; ++vv) {
                    const int v = ps * VPP + vv;
                    const int lr = 8 * ((v >> 2) - ps * (4 / PASSES)) + 4 * lhi + (v & 3);
                    st[lr * ST_LD + tn * 32 + l32] = acc[tm][tn][v];
                }
            __syncthreads();
            if (nok) {
#pragma unroll
                for (int rr = rr0; rr < SROWS; rr += RPP) {
                    const int r = wm * WMT * 32 + tm * 32 + ps * SROWS + rr;
                    const long long coff = rowC[r];
                    if (coff < 0) continue;
                    const float4 t = *(const float4*)(st + rr * ST_LD + cg * 4);
                    float val[4] = {t.x * sc[0] + sh[0], t.y * sc[1] + sh[1], t.z * sc[2] + sh[2], t.w * sc[3] + sh[3]};
                    if (a.R) {
                        const uint2 q = *(const uint2*)(a.R + rowR[r] + ncol);
                        val[0] += __uint_as_float(q.x << 16);
                        val[1] += __uint_as_float(q.x & 0xffff0000u);
                        val[2] += __uint_as_float(q.y << 16);
                        val[3] += __uint_as_float(q.y & 0xffff0000u);
                    }
                    if (a.act == DS_ACT_RELU) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) val[j] = fmaxf(val[j], 0.f);
                    } else if (a.act == DS_ACT_GELU) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) val[j] = gelu_erf(val[j]);
                    }
                    if (a.out_f32) {
                        *(float4*)((float*)a.C + coff + ncol) = make_float4(val[0], val[1], val[2], val[3]);
                    } else {
                        uint2 q;
                        q.x = (uint32_t)f2bf(val[0]) | ((uint32_t)f2bf(val[1]) << 16);
                        q.y = (uint32_t)f2bf(val[2]) | ((uint32_t)f2bf(val[3]) << 16);
                        *(uint2*)((bf16_t*)a.C + coff + ncol) = q;
                    }
                }
            }
            __syncthreads();
        }
    }
}

__global__ void build_mtiles_kernel(const int32_t* offsets, int T, int rows, int32_t* count, int4* entries) {
    __shared__ int pre[DS_MAX_GROUPS + 1];
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int g = 0; g < T; ++g) {
            pre[g] = acc;
            const int rg = (offsets[g + 1] - offsets[g]) * rows;
            acc += (rg + BM - 1) / BM;
        }
        pre[T] = acc;
        *count = acc;
    }
    __syncthreads();
    for (int g = 0; g < T; ++g) {
        const int n = pre[g + 1] - pre[g];
        const int slot0 = offsets[g], rg = (offsets[g + 1] - slot0) * rows;
        for (int i = threadIdx.x; i < n; i += blockDim.x) entries[pre[g] + i] = make_int4(g, i * BM, slot0, rg);
    }
}

template <int WROWS, int WCOLS, int WMT, int WNT>
int32_t launch(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    using TL = Tile<WROWS, WCOLS, WMT, WNT>;
    static bool configured = false;
    auto kern = gemm_kernel<WROWS, WCOLS, WMT, WNT>;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, TL::SMEM) != hipSuccess)
            DS_FAIL(DS_EHIP, "sliced gemm: cannot reserve %d bytes of LDS", TL::SMEM);
        configured = true;
    }
    const int ny = a.n_seg * ((max_kout + TL::BN - 1) / TL::BN);
    const unsigned grid = (unsigned)(((max_mtiles + 7) / 8) * ny * 8);
    ProfScope prof(a.K > 1 ? DS_K_GEMM_TAPS : DS_K_GEMM, s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), TL::SMEM, s, a, ny, max_mtiles);
    DS_CHECK_LAUNCH("sliced gemm");
    return DS_OK;
}

}  // namespace

size_t ds_mtile_capacity(int32_t B, int32_t rows, int32_t T) {
    return (size_t)(((int64_t)B * rows + BM - 1) / BM + T);
}

int32_t ds_build_mtiles(const int32_t* offsets, int32_t T, int32_t rows, void* list, hipStream_t s) {
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(build_mtiles_kernel, dim3(1), dim3(256), 0, s, offsets, T, rows, (int32_t*)list,
                       (int4*)((char*)list + 16));
    DS_CHECK_LAUNCH("build_mtiles");
    return DS_OK;
}

int32_t ds_launch_gemm(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    if (max_mtiles <= 0 || max_kout <= 0) return DS_OK;
    static const int forced = [] {
        const char* e = getenv("DSNET_GEMM_TILE");   // tuning knob: force the n-tile width (64, 128, 256)
        return e ? atoi(e) : 0;
    }();
    const int bn = forced ? forced : (max_kout <= 64 ? 64 : (max_kout <= 128 ? 128 : 256));
    if (bn == 64) return launch<4, 1, 1, 2>(a, max_mtiles, max_kout, s);
    if (bn == 128) return launch<2, 2, 2, 2>(a, max_mtiles, max_kout, s);
    return launch<2, 2, 2, 4>(a, max_mtiles, max_kout, s);
}
