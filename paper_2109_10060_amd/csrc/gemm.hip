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
// Tiling: 128 x 64 output tile per 256-thread workgroup, 4 wavefronts, each holding a 32 x 64 grid of
// v_mfma_f32_32x32x16_bf16 accumulators (the dispatcher uses this shape for every layer: with ragged route
// groups and slices as narrow as 64 channels the wider 128 x 128 / 128 x 256 instantiations lose more to
// quantisation and residency than their lower operand traffic gains).  Operands go through one LDS tile in
// 32-deep slabs, 64-deep ones for reductions of 256 steps and more, or 128-deep ones where a launch is about one
// generation of workgroups and a filter tap has 512 channels or more (the last ResNet stage: half as many dependent
// load -> LDS -> barrier rounds per workgroup; 64-, 128- or 256-byte rows, 16-byte chunks XOR-swizzled by row so
// stores and reads are bank-conflict free); the next slab's global loads are issued into
// registers before the current slab's matrix instructions and stored to LDS after them, and 5-6 resident
// workgroups per compute unit hide each other's round trips.  The epilogue (split batch-norm scale and
// shift or bias, residual, ReLU/GELU, bf16 rounding) re-reads the accumulators through LDS so that every lane
// stores 4 consecutive channels of one row.
//
// Work items are (m-tile, n-tile) pairs with the n-tile fastest; the linear block
// index is dealt round-robin to the 8 XCDs by the hardware, so each XCD is given
// a contiguous run of work items and the blocks that share an activation tile hit
// the same L2.
#include "common.h"

namespace {

constexpr int BM = DS_GEMM_BM, NT = 256;

// 16-byte chunk c of LDS row r is stored at chunk position c ^ swz(r): rows are BK * 2 bytes with no
// padding; the row-major stores and the operand reads (32 consecutive rows, one chunk column) are
// bank-conflict free for 8- and 16-lane access groups alike
template <int BK>
__device__ __forceinline__ int swz(int r) {
    return BK == 128 ? (r & 15) : BK == 64 ? ((r ^ (r >> 3)) & 7) : (((r >> 1) ^ (r >> 2)) & 3);
}

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

template <int WROWS, int WCOLS, int WMT, int WNT, int BK>
struct Tile {
    static constexpr int BN = WCOLS * WNT * 32, LDS_LD = BK;
    static constexpr int COLS = WNT * 32;                      // columns staged per wavefront
    static constexpr int SROWS = 16;                           // rows staged per pass
    static constexpr int ST_LD = COLS + 4;
    static constexpr int LOOP_BYTES = (BM + BN) * LDS_LD * 2;
    static constexpr int STAGE_BYTES = 4 * SROWS * ST_LD * 4;
    static constexpr int MAIN_BYTES = LOOP_BYTES > STAGE_BYTES ? LOOP_BYTES : STAGE_BYTES;
    static constexpr int TABLE_BYTES = BM * (4 + 8 + 8 + 8) + 2 * BN * 4;   // row tables + scale / shift of the tile's columns
    static constexpr int SMEM = MAIN_BYTES + TABLE_BYTES;
    static_assert(WROWS * WCOLS == 4 && WROWS * WMT * 32 == BM, "4 wavefronts cover a 128-row tile");
};

template <int WROWS, int WCOLS, int WMT, int WNT, int BK, bool CONV, bool HASR>
__global__ __launch_bounds__(NT, BK == 128 ? 3 : (WMT * WNT == 2 && !CONV) ? (BK == 32 ? (HASR ? 5 : 6) : 5) : 1) void gemm_kernel(const GemmArgs a, const int ny, const int max_mtiles) {
    using TL = Tile<WROWS, WCOLS, WMT, WNT, BK>;
    constexpr int BN = TL::BN, LDS_LD = BK, CPR = BK / 8, RPT = NT / CPR;   // chunks per row, rows per pass
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t* As = (bf16_t*)smem;                       // [BM][BK]
    bf16_t* Bs = As + BM * LDS_LD;                    // [BN][BK]
    long long* rowC = (long long*)(smem + TL::MAIN_BYTES);
    long long* rowR = rowC + BM;
    int2* rowYX = (int2*)(rowR + BM);
    uint32_t* rowA = (uint32_t*)(rowYX + BM);
    float* scl = (float*)(rowA + BM);                 // [BN] scale, then [BN] shift of this tile's output columns
    // operands are fetched with buffer loads: 32-bit byte offsets against a uniform base, and an
    // offset beyond the descriptor's range returns zeros, which supplies every tail (rows beyond
    // the group, channels beyond the slice, taps outside the image) without branches
    constexpr uint32_t OOB = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.Wt, 0, 0x7fffffff, 0x00020000);

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
        long long rc = -1, rr = 0;
        uint32_t ra = OOB;
        int2 yx = make_int2(0, 0);
        if (m < rows_g) {
            const int sl = m / a.rows;
            const int p = m - sl * a.rows;
            const int slot = slot0 + sl;
            const int sa = a.a_index ? a.a_index[slot] : slot;
            const int cs = a.c_index ? a.c_index[slot] : slot;
            const int oy = p / a.Wo, ox = p - oy * a.Wo;
            // byte offset of the sample (convolution) or of the row itself (linear layers)
            ra = (uint32_t)(((long long)sa * a.a_sample_stride + (CONV ? 0 : (long long)p * a_ld)) * 2);
            yx = make_int2(oy * a.stride - a.pad, ox * (a.stride_w > 0 ? a.stride_w : a.stride) - a.pad);
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

    // ---- load assignment: a thread owns chunk (tid % CPR) of rows (tid / CPR) + RPT i ----
    constexpr int NA = BM / RPT, NB = BN / RPT;
    const int lchunk = tid % CPR;
    const int kc8 = lchunk * 8;
    const int lrow = tid / CPR;
    uint32_t aoff[NA], apix[NA], woff[NB];
    int2 ayx[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        aoff[i] = rowA[lrow + RPT * i];
        ayx[i] = rowYX[lrow + RPT * i];
        apix[i] = aoff[i] == OOB ? OOB : aoff[i] + kc8 * 2;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int n = n0 + lrow + RPT * i;
        woff[i] = n < k_out ? (uint32_t)(((long long)seg * a.w_seg_stride + (long long)n * a.w_ld + kc8) * 2) : OOB;
    }
    // per filter tap: byte offset of the input pixel each owned row reads (OOB outside the image)
    auto set_tap = [&](int tap) {
        if constexpr (CONV) {
            const int kw = a.Kw > 0 ? a.Kw : a.K;
            const int u = tap / kw, v = tap - u * kw;
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                const int iy = ayx[i].x + u, ix = ayx[i].y + v;
                const bool ok = aoff[i] != OOB && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
                apix[i] = ok ? aoff[i] + (uint32_t)(((iy * a.W + ix) * a_ld + kc8) * 2) : OOB;
            }
        }
    };

    uint4 ra[NA], rb[NB];
    auto load_global = [&](int tap, int kc) {
        const bool kok = (kc + kc8) < k_in;
        const int soff_a = kc * 2;
        const int soff_w = (int)((tap * a.w_tap_stride + kc) * 2);
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, (int)(kok ? apix[i] : OOB), soff_a, 0);
            ra[i] = make_uint4(t[0], t[1], t[2], t[3]);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, (int)(kok ? woff[i] : OOB), soff_w, 0);
            rb[i] = make_uint4(t[0], t[1], t[2], t[3]);
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int r = lrow + RPT * i;
            *(uint4*)(As + r * LDS_LD + ((lchunk ^ swz<BK>(r)) * 8)) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int r = lrow + RPT * i;
            *(uint4*)(Bs + r * LDS_LD + ((lchunk ^ swz<BK>(r)) * 8)) = rb[i];
        }
    };

    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave / WCOLS, wn = wave - wm * WCOLS;
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16_t acc[WMT][WNT];
#pragma unroll
    for (int i = 0; i < WMT; ++i)
#pragma unroll
        for (int jj = 0; jj < WNT; ++jj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jj][v] = 0.f;

    // operand rows of this lane: row (32 t + l32) of the wave's A / B block; with 128-byte rows the
    // swizzle key of row + 32 t is the key of the row ^ (4 t & 7), with 64-byte rows it does not change
    const bf16_t* as = As + (wm * WMT * 32 + l32) * LDS_LD;
    const bf16_t* bs = Bs + (wn * WNT * 32 + l32) * LDS_LD;
    const int fa = swz<BK>(wm * WMT * 32 + l32), fb = swz<BK>(wn * WNT * 32 + l32);
    constexpr int TK = BK == 64 ? 4 : 0;   // 256-byte rows: the key is the row's low four bits, the same 32 rows on

    const int kchunks = (k_in + BK - 1) / BK;
    const int nk = a.K * (a.Kw > 0 ? a.Kw : a.K) * kchunks;
    int tap = 0, kc = 0;
    set_tap(0);
    load_global(0, 0);

    // The first operand slab is requested before anything else: loads return in order, so whatever is issued
    // ahead of it would have to arrive before the slab can go to LDS.
    // epilogue constants, loaded now so their latency hides behind the main loop
    constexpr int COLS = TL::COLS, SROWS = TL::SROWS, ST_LD = TL::ST_LD;
    constexpr int CG = COLS / 4, RPP = 64 / CG, PASSES = 32 / SROWS, VPP = 16 / PASSES;
    const int cg = lane % CG, rr0 = lane / CG;
    const int ncol = n0 + wn * COLS + cg * 4;
    const bool nok = ncol < k_out;
    // scale and shift of the tile's columns wait in LDS, not in registers, until the epilogue (registers set the residency)
    if (tid < BN) {
        const int n = n0 + tid;
        float vs = 1.f, vh = 0.f;
        if (n < k_out) {
            const long long ti = (long long)a.gt.row[g] * a.tab_ld + (long long)seg * a.tab_seg_stride + n;
            if (a.scale) vs = a.scale[ti];
            if (a.shift) vh = a.shift[ti];
        }
        scl[tid] = vs;
        scl[BN + tid] = vh;
    }

    // the residual rows this lane will add are fetched ahead of the main loop, so that their latency hides behind it
    // instead of sitting between the last matrix instruction and the stores -- except with the 64-deep slabs, where
    // their 16 registers would cost a resident workgroup: there they are requested right after the loop
    constexpr bool RES_EARLY = BK == 32;
    uint2 rres[HASR ? WMT * PASSES * (SROWS / RPP) : 1];
    auto fetch_residual = [&]() {
#pragma unroll
        for (int tm = 0; tm < WMT; ++tm)
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps)
#pragma unroll
                for (int q = 0; q < SROWS / RPP; ++q) {
                    const int r = wm * WMT * 32 + tm * 32 + ps * SROWS + rr0 + q * RPP;
                    uint2 t = make_uint2(0, 0);
                    if (nok && rowC[r] >= 0) t = *(const uint2*)(a.R + rowR[r] + ncol);
                    rres[(tm * PASSES + ps) * (SROWS / RPP) + q] = t;
                }
    };
    if constexpr (HASR && RES_EARLY) fetch_residual();

    store_lds();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        kc += BK;
        if (kc >= k_in) {
            kc = 0;
            ++tap;
            if (kt + 1 < nk) set_tap(tap);
        }
        const bool more = kt + 1 < nk;
        if (more) load_global(tap, kc);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8_t af[WMT], bfr[WNT];
            const int c = kk * 2 + lhi;
#pragma unroll
            for (int t = 0; t < WMT; ++t) af[t] = *(const bf16x8_t*)(as + t * 32 * LDS_LD + ((c ^ fa ^ ((TK * t) & 7)) * 8));
#pragma unroll
            for (int t = 0; t < WNT; ++t) bfr[t] = *(const bf16x8_t*)(bs + t * 32 * LDS_LD + ((c ^ fb ^ ((TK * t) & 7)) * 8));
#pragma unroll
            for (int i = 0; i < WMT; ++i)
#pragma unroll
                for (int jj = 0; jj < WNT; ++jj)
                    acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[jj], acc[i][jj], 0, 0, 0);
        }
        __syncthreads();
        if (more) {
            store_lds();
            __syncthreads();
        }
    }

    if constexpr (HASR && !RES_EARLY) fetch_residual();

    // ---- epilogue through LDS: each lane finishes 4 consecutive channels of one row -----
    // The staging rows belong to one wavefront (written and read back by its own lanes, and the main loop's last
    // barrier has already retired every read of the operand tiles they alias), and a wavefront's LDS accesses
    // complete in order, so the passes only need the compiler kept from moving LDS accesses across them.
    auto wave_sync = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
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
            wave_sync();
            if (nok) {
#pragma unroll
                for (int rr = rr0; rr < SROWS; rr += RPP) {
                    const int r = wm * WMT * 32 + tm * 32 + ps * SROWS + rr;
                    const long long coff = rowC[r];
                    if (coff < 0) continue;
                    const float4 t = *(const float4*)(st + rr * ST_LD + cg * 4);
                    const float4 s4 = *(const float4*)(scl + wn * COLS + cg * 4), h4 = *(const float4*)(scl + BN + wn * COLS + cg * 4);
                    float val[4] = {t.x * s4.x + h4.x, t.y * s4.y + h4.y, t.z * s4.z + h4.z, t.w * s4.w + h4.w};
                    if constexpr (HASR) {
                        const uint2 q = rres[(tm * PASSES + ps) * (SROWS / RPP) + (rr - rr0) / RPP];
                        val[0] += __uint_as_float(q.x << 16);
                        val[1] += __uint_as_float(q.x & 0xffff0000u);
                        val[2] += __uint_as_float(q.y << 16);
                        val[3] += __uint_as_float(q.y & 0xffff0000u);
                    }
                    if (a.act == DS_ACT_RELU) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) val[e] = fmaxf(val[e], 0.f);
                    } else if (a.act == DS_ACT_GELU) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) val[e] = gelu_erf(val[e]);
                    }
                    if (a.out_f32) {
                        *(float4*)((float*)a.C + coff + ncol) = make_float4(val[0], val[1], val[2], val[3]);
                    } else {
                        uint2 q;
                        q.x = f2bf2(val[0], val[1]);
                        q.y = f2bf2(val[2], val[3]);
                        *(uint2*)((bf16_t*)a.C + coff + ncol) = q;
                    }
                }
            }
            wave_sync();
        }
    }
}

// The list walks the groups from the last to the first: route tables are ordered from the narrowest
// to the widest slice, so the longest work items are dispatched first and the short ones fill the
// tail of the launch.
__global__ void build_mtiles_kernel(const int32_t* offsets, int T, int rows, int32_t* count, int4* entries) {
    __shared__ int pre[DS_MAX_GROUPS + 1];
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int q = 0; q < T; ++q) {
            const int g = T - 1 - q;
            pre[q] = acc;
            const int rg = (offsets[g + 1] - offsets[g]) * rows;
            acc += (rg + BM - 1) / BM;
        }
        pre[T] = acc;
        *count = acc;
    }
    __syncthreads();
    for (int q = 0; q < T; ++q) {
        const int g = T - 1 - q;
        const int n = pre[q + 1] - pre[q];
        const int slot0 = offsets[g], rg = (offsets[g + 1] - slot0) * rows;
        for (int i = threadIdx.x; i < n; i += blockDim.x) entries[pre[q] + i] = make_int4(g, i * BM, slot0, rg);
    }
}

template <int WROWS, int WCOLS, int WMT, int WNT, int BK, bool CONV, bool HASR>
int32_t launch(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    using TL = Tile<WROWS, WCOLS, WMT, WNT, BK>;
    auto kern = gemm_kernel<WROWS, WCOLS, WMT, WNT, BK, CONV, HASR>;
    {
        const int32_t rc = ds_reserve_lds((const void*)kern, TL::SMEM, "sliced gemm");
        if (rc) return rc;
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
    // ragged route slices favour the narrow 128x64 tile at high occupancy in every layer of the batch-256 networks.
    // Its slabs are 32 deep for short reductions and 64 deep from 256 reduction steps on: half the barriers and
    // twice the bytes in flight per workgroup outweigh the lower residency there (measured per layer: ViT MLP
    // down-projection 62 -> 52 us, ResNet stage-4 strided 3x3 83 -> 66 us; 128-step layers 44 -> 48 us the other way)
    // (a slab never crosses a filter tap: with fewer than 64 channels per tap the deep slab would be mostly padding --
    // the 8x8 patch embedding over 24 channels ran 144 -> 226 us with it)
    int kmax = 0;
    for (int t = 0; t < a.gt.T; ++t) kmax = a.gt.k_in[t] > kmax ? a.gt.k_in[t] : kmax;
    const long long taps = (long long)a.K * (a.Kw > 0 ? a.Kw : a.K);
    // (exactly 256 steps: the 64-deep slabs pay only where a residual is streamed as well -- without one the 32-deep
    // kernel keeps six workgroups per compute unit: DS-MBNet's 256-channel pointwise layers -1.1 % per step, DS-ResNet -0.4 %)
    const bool deep = kmax >= 64 && (kmax * taps >= 320 || (kmax * taps >= 256 && a.R != nullptr));
    // 32-bit byte offsets inside the kernel: activations and weights must each span less than 2 GiB
    const long long slots = (long long)max_mtiles * BM / (a.rows > 0 ? a.rows : 1) + 1;
    if (slots * a.a_sample_stride * 2 >= 0x7fffffffLL)
        DS_FAIL(DS_EUNSUPPORTED, "sliced gemm: activation tensor spans 2 GiB or more");
    if (((long long)a.n_seg * a.w_seg_stride + (long long)max_kout * a.w_ld + taps * a.w_tap_stride + kmax) * 2 >= 0x7fffffffLL)
        DS_FAIL(DS_EUNSUPPORTED, "sliced gemm: weight tensor spans 2 GiB or more");
    const bool conv = a.K > 1 || a.stride > 1 || a.pad > 0;
    if (conv) {
        const int32_t rc = ds_launch_conv3(a, max_mtiles, max_kout, s);
        if (rc != DS_EUNSUPPORTED) return rc;
    }
#define DS_GEMM_DISPATCH(...)                                                                          \
    (conv ? (a.R ? launch<__VA_ARGS__, true, true>(a, max_mtiles, max_kout, s)                         \
                 : launch<__VA_ARGS__, true, false>(a, max_mtiles, max_kout, s))                       \
          : (a.R ? launch<__VA_ARGS__, false, true>(a, max_mtiles, max_kout, s)                        \
                 : launch<__VA_ARGS__, false, false>(a, max_mtiles, max_kout, s)))
    if (!deep) return DS_GEMM_DISPATCH(4, 1, 1, 2, 32);   // 64-wide tile, 32-deep slabs
    // launches of about one generation with long reductions: 128-deep slabs halve the number of dependent rounds
    const long long wgs = (long long)max_mtiles * a.n_seg * ((max_kout + 63) / 64);
    if (kmax >= 512 && wgs <= 256 * 6) return DS_GEMM_DISPATCH(4, 1, 1, 2, 128);
    return DS_GEMM_DISPATCH(4, 1, 1, 2, 64);
#undef DS_GEMM_DISPATCH
}
