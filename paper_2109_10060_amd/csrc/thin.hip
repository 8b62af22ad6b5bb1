// Grouped prefix-slice linear / 1x1 layer with a short reduction (slices of at most 64, with a residual 128, input channels): Section 3.2,
// Eq. 8 / Eq. 9 with split batch-norm (Eq. 14), optional residual and ReLU -- the third convolution of the first-stage
// bottlenecks (64 r -> 256 r channels on 56x56 maps) and that stage's projection shortcut.
//
// With so short a reduction these layers are streams: per output element one residual read, one write and a handful
// of multiply-adds.  gemm_kernel runs them as one workgroup per (128 rows, 64 columns) whose lifetime is its fixed
// head (tile record, row table, first operand slab) and its epilogue.  Here a workgroup owns 128 rows and ALL their
// output columns: the activation rows are staged in LDS once, and per 64 columns the weights, the batch-norm constants
// and the residual tile are requested one pass ahead (registers), so a pass waits for nothing it has not asked for a
// whole pass earlier.  The residual tile is parked in LDS, each lane adds its own 8-byte runs in place, and the tile
// leaves as 16-byte pieces.  Same m-tile list, row addressing and results as gemm_kernel.
#include "common.h"
#include <cstring>

namespace {

constexpr int BM = DS_GEMM_BM, NT = 256, T_LD = 64 + 8;
constexpr uint32_t OOB = 0x80000000u;
constexpr int TILE_BYTES = BM * T_LD * 2;
constexpr int smem_bytes(int kch) { return kch * BM * 64 + kch * 64 * 64 + TILE_BYTES + BM * (8 + 8 + 4) + 2 * 64 * 4; }
// chained variant (2 chunks): plus the second layer's 64 x 64 slab; the pass constants take the place of the activation
// row table, which is spent by then (42 allocation units of 1280 bytes: three workgroups per compute unit still fit)
constexpr int W2_BYTES = 64 * 64 * 2;
constexpr int smem_bytes_chain() { return smem_bytes(2) + W2_BYTES - 2 * 64 * 4; }

__device__ __forceinline__ int swz(int r) { return ((r >> 1) ^ (r >> 2)) & 3; }

// KCH: 32-channel chunks of the widest input slice (2: up to 64 channels, 4: up to 128)
// CHAIN: the rows' results feed a second 1x1 layer of at most 64 output channels before they leave the workgroup
// (the next bottleneck's first convolution): each pass's 64 result columns are one reduction slab of that layer, whose
// accumulators stay in registers over the passes, so the wide map is written once and not read back.
// N2B: 32-column blocks of the second layer's output (2: up to 64 channels, 4: up to 128).  With 128-channel input slices
// (KCH = 4) the second layer's slab takes the place of the first layer's weights once the pass's own matrix
// instructions are done (one more barrier per pass), so that two workgroups per compute unit still fit.
template <bool HASR, int KCH, bool CHAIN, int N2B = 2>
__global__ __launch_bounds__(NT, CHAIN ? (KCH == 4 ? 2 : 3) : 1) void thin_kernel(const GemmArgs a, const int max_mtiles, const ThinChain ch) {
    constexpr int A_BYTES = KCH * BM * 64, B_BYTES = KCH * 64 * 64, CP = KCH * 4;   // CP 16-byte pieces per operand row
    constexpr int NAP = BM * CP / NT, NWP = 64 * CP / NT;                            // pieces per lane: activations, weights
    constexpr bool W2_ALIAS = CHAIN && KCH == 4;
    constexpr int N2R = 32 * N2B;                      // rows (output channels) of the second layer's slab
    static_assert(!W2_ALIAS || 2 * N2R * 64 <= B_BYTES, "the second layer's slab fits the first layer's weight tile");
    static_assert(W2_ALIAS || N2B == 2, "the separate slab holds 64 output channels");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* As = smem;                                   // [KCH][128][32] bf16
    char* Bs = smem + A_BYTES;                         // [KCH][64][32] bf16
    char* W2s = W2_ALIAS ? Bs : smem + A_BYTES + B_BYTES;   // CHAIN only: [2][N2R][32] bf16, the second layer's slab of the pass
    constexpr int T_OFF = A_BYTES + B_BYTES + (CHAIN && !W2_ALIAS ? W2_BYTES : 0);
    bf16_t* tile = (bf16_t*)(smem + T_OFF);            // [128][T_LD]: residual in, result out
    long long* rowC = (long long*)(smem + T_OFF + TILE_BYTES);
    long long* rowR = rowC + BM;                       // CHAIN: rows of the second output (the residual is addressed like C)
    uint32_t* rowA = (uint32_t*)(rowR + BM);
    float* cst = (float*)(CHAIN ? rowA : rowA + BM);   // [64] scale, [64] shift of the pass (CHAIN: over the spent rowA)
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.Wt, 0, 0x7fffffff, 0x00020000);

    const int mt = blockIdx.x;
    if (mt >= max_mtiles) return;
    const int4 me = a.mtiles[mt];                      // in-bounds even beyond the live count; checked next
    if (mt >= *a.n_mtiles) return;
    const int g = me.x, grow0 = me.y, slot0 = me.z, rows_g = me.w;
    const int k_in = a.gt.k_in[g], k_out = a.gt.k_out[g];
    if (k_in <= 0 || k_out <= 0) return;
    const int tid = threadIdx.x;
    const int a_ld = a.a_ld > 0 ? a.a_ld : k_in;
    const int c_ld = a.c_ld > 0 ? a.c_ld : k_out;
    const int r_ld = a.r_ld > 0 ? a.r_ld : k_out;
    const int k_out2 = CHAIN ? ch.k_out[g] : 0;        // <= 0: this group ends with the first layer
    const int c2_ld = ch.c_ld > 0 ? ch.c_ld : k_out2;

    if (tid < BM) {
        const int m = grow0 + tid;
        long long rc = -1, rr = 0;
        uint32_t ra = OOB;
        if (m < rows_g) {
            const int sl = m / a.rows;
            const int p = m - sl * a.rows;
            const int slot = slot0 + sl;
            const int sa = a.a_index ? a.a_index[slot] : slot;
            const int cs = a.c_index ? a.c_index[slot] : slot;
            ra = (uint32_t)(((long long)sa * a.a_sample_stride + (long long)p * a_ld) * 2);
            const long long pc = p + a.c_row0;
            rc = (long long)cs * a.c_sample_stride + pc * c_ld;
            rr = CHAIN ? (long long)cs * ch.c_sample_stride + (long long)p * c2_ld
                       : (long long)(a.r_use_index ? cs : 0) * a.r_sample_stride + pc * r_ld;
        }
        rowA[tid] = ra;
        rowC[tid] = rc;
        rowR[tid] = rr;
    }
    __syncthreads();

    // ---- what travels one pass ahead: weights (NWP pieces), constants (1 value), residual (4 pieces) per lane ----
    const int prow8 = tid >> 3, pc8 = (tid & 7) * 8;   // tile piece e = tid + 256 i: row (e >> 3), columns 8 (e & 7) ..
    const int orow = tid / CP, oc8 = tid % CP;         // operand piece e = tid + 256 i: row (e / CP), channels 8 (e % CP) ..
    const long long trow = (long long)a.gt.row[g] * a.tab_ld;
    uint4 wreg[NWP], rreg[4];
    float creg;
    auto fetch_pass = [&](int n0) {
#pragma unroll
        for (int i = 0; i < NWP; ++i) {
            const int nl = orow + (NT / CP) * i;
            const bool ok = n0 + nl < k_out && oc8 * 8 < k_in;
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(
                rsrc_w, (int)(ok ? (uint32_t)(((long long)(n0 + nl) * a.w_ld + oc8 * 8) * 2) : OOB), 0, 0);
            wreg[i] = make_uint4(t[0], t[1], t[2], t[3]);
        }
        {
            const int col = n0 + (tid & 63), which = tid >> 6;          // 0: scale, 1: shift (lanes 128.. idle)
            const float* tab = which == 0 ? a.scale : a.shift;
            creg = which == 0 ? 1.f : 0.f;
            if (which < 2 && tab && col < k_out) creg = tab[trow + col];
        }
        if constexpr (HASR) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = prow8 + 32 * i;
                uint4 t = make_uint4(0, 0, 0, 0);
                if (rowC[row] >= 0 && n0 + pc8 < k_out) t = *(const uint4*)(a.R + (CHAIN ? rowC[row] : rowR[row]) + n0 + pc8);
                rreg[i] = t;
            }
        }
    };

    // ---- the activation rows, once -------------------------------------------------------------------------
    {
        uint4 areg[NAP];
#pragma unroll
        for (int i = 0; i < NAP; ++i) {
            const int row = orow + (NT / CP) * i;
            const uint32_t ra = rowA[row];
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, (int)((ra != OOB && oc8 * 8 < k_in) ? ra + oc8 * 16 : OOB), 0, 0);
            areg[i] = make_uint4(t[0], t[1], t[2], t[3]);
        }
        fetch_pass(0);
#pragma unroll
        for (int i = 0; i < NAP; ++i) {
            const int row = orow + (NT / CP) * i;
            *(uint4*)(As + ((oc8 >> 2) * BM + row) * 64 + (((oc8 & 3) ^ swz(row)) * 16)) = areg[i];
        }
    }

    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int prow = wave * 32 + l32;
    const int kch = (k_in + 31) >> 5;                  // chunks of this group's reduction, at most KCH
    // second layer: its weights for the 64 channels of a pass, 2 pieces per lane (row tid / 8 + 32 i, channels 8 (tid % 8) ..)
    const __amdgpu_buffer_rsrc_t rsrc_w2 = __builtin_amdgcn_make_buffer_rsrc((void*)(CHAIN ? ch.Wt : a.Wt), 0, 0x7fffffff, 0x00020000);
    uint4 w2reg[N2B];
    f32x16_t acc2[N2B];
    auto fetch_w2 = [&](int n0) {
#pragma unroll
        for (int i = 0; i < N2B; ++i) {
            const int nl = (tid >> 3) + 32 * i, c0 = n0 + (tid & 7) * 8;
            const bool ok = nl < k_out2 && c0 < k_out;
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w2, (int)(ok ? (uint32_t)(((long long)nl * ch.w_ld + c0) * 2) : OOB), 0, 0);
            w2reg[i] = make_uint4(t[0], t[1], t[2], t[3]);
        }
    };
    auto store_w2 = [&]() {
#pragma unroll
        for (int i = 0; i < N2B; ++i) {
            const int nl = (tid >> 3) + 32 * i, pc = tid & 7;
            *(uint4*)(W2s + ((pc >> 2) * N2R + nl) * 64 + (((pc & 3) ^ swz(nl)) * 16)) = w2reg[i];
        }
    };
    if constexpr (CHAIN) {
        if (k_out2 > 0) fetch_w2(0);
#pragma unroll
        for (int t = 0; t < N2B; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc2[t][e] = 0.f;
    }
    for (int n0 = 0; n0 < k_out; n0 += 64) {
        __syncthreads();                               // activation rows staged / last pass's tile copied out
#pragma unroll
        for (int i = 0; i < NWP; ++i) {
            const int nl = orow + (NT / CP) * i;
            *(uint4*)(Bs + ((oc8 >> 2) * 64 + nl) * 64 + (((oc8 & 3) ^ swz(nl)) * 16)) = wreg[i];
        }
        if (tid < 128) cst[tid] = creg;
        if constexpr (CHAIN && !W2_ALIAS) {
            if (k_out2 > 0) store_w2();
        }
        if constexpr (HASR) {
#pragma unroll
            for (int i = 0; i < 4; ++i) *(uint4*)(tile + (prow8 + 32 * i) * T_LD + pc8) = rreg[i];
        }
        __syncthreads();
        if (n0 + 64 < k_out) {                         // in flight during this pass
            fetch_pass(n0 + 64);
            if constexpr (CHAIN && !W2_ALIAS) {
                if (k_out2 > 0) fetch_w2(n0 + 64);
            }
        }
        f32x16_t acc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
        for (int kc = 0; kc < kch; ++kc) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int c = kk * 2 + lhi;
                const bf16x8_t pf = *(const bf16x8_t*)(As + (kc * BM + prow) * 64 + ((c ^ swz(prow)) * 16));
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int nr = t * 32 + l32;
                    const bf16x8_t wf = *(const bf16x8_t*)(Bs + (kc * 64 + nr) * 64 + ((c ^ swz(nr)) * 16));
                    // weights as the row operand: the accumulator holds row prow and columns 32 t + 8 q + 4 lhi + 0..3
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, pf, acc[t], 0, 0, 0);
                }
            }
        }
        // epilogue in place: this lane's 8-byte runs of the residual tile become its results
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = t * 32 + q * 8 + lhi * 4;
                const float4 s4 = *(const float4*)(cst + col), h4 = *(const float4*)(cst + 64 + col);
                float v[4] = {acc[t][4 * q] * s4.x + h4.x, acc[t][4 * q + 1] * s4.y + h4.y, acc[t][4 * q + 2] * s4.z + h4.z,
                              acc[t][4 * q + 3] * s4.w + h4.w};
                uint2* tp = (uint2*)(tile + prow * T_LD + col);
                if constexpr (HASR) {
                    const uint2 r2 = *tp;
                    v[0] += __uint_as_float(r2.x << 16);
                    v[1] += __uint_as_float(r2.x & 0xffff0000u);
                    v[2] += __uint_as_float(r2.y << 16);
                    v[3] += __uint_as_float(r2.y & 0xffff0000u);
                }
                if (a.act == DS_ACT_RELU) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
                }
                uint2 o;
                o.x = f2bf2(v[0], v[1]);
                o.y = f2bf2(v[2], v[3]);
                *tp = o;
            }
        __syncthreads();
        if constexpr (W2_ALIAS) {
            // every wavefront is done with the first layer's weights of this pass: the second layer's slab takes their
            // place, and the slab of the next pass is requested (a whole pass ahead of its use)
            if (k_out2 > 0) {                          // uniform over the workgroup
                store_w2();
                if (n0 + 64 < k_out) fetch_w2(n0 + 64);
                __syncthreads();
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = prow8 + 32 * i;
            const long long rc = rowC[row];
            if (rc >= 0 && n0 + pc8 < k_out) *(uint4*)((bf16_t*)a.C + rc + n0 + pc8) = *(const uint4*)(tile + row * T_LD + pc8);
        }
        if constexpr (CHAIN) {
            if (k_out2 > 0) {
                // the pass's 64 result columns (bf16, as stored) are one reduction slab of the second layer
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const bf16x8_t pf = *(const bf16x8_t*)(tile + prow * T_LD + kk * 16 + lhi * 8);
                    const int c = (kk & 1) * 2 + lhi;
#pragma unroll
                    for (int t = 0; t < N2B; ++t) {
                        const int nr = t * 32 + l32;
                        const bf16x8_t wf = *(const bf16x8_t*)(W2s + ((kk >> 1) * N2R + nr) * 64 + ((c ^ swz(nr)) * 16));
                        acc2[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, pf, acc2[t], 0, 0, 0);
                    }
                }
            }
        }
    }
    if constexpr (CHAIN) {
        if (k_out2 <= 0) return;
        const long long trow2 = (long long)a.gt.row[g] * ch.tab_ld;
        // the second layer's results leave through the same tile, 64 columns at a time
#pragma unroll
        for (int hb = 0; hb < N2B / 2; ++hb) {
            if (hb * 64 >= k_out2) break;              // uniform over the workgroup
            __syncthreads();                           // the last pass's tile (or the previous 64 columns) has been read
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int col = t * 32 + q * 8 + lhi * 4, gcol = hb * 64 + col;
                    float4 s4 = make_float4(1.f, 1.f, 1.f, 1.f), h4 = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (gcol < k_out2) {
                        if (ch.scale) s4 = *(const float4*)(ch.scale + trow2 + gcol);
                        if (ch.shift) h4 = *(const float4*)(ch.shift + trow2 + gcol);
                    }
                    const f32x16_t& av = acc2[2 * hb + t];
                    float v[4] = {av[4 * q] * s4.x + h4.x, av[4 * q + 1] * s4.y + h4.y, av[4 * q + 2] * s4.z + h4.z,
                                  av[4 * q + 3] * s4.w + h4.w};
                    if (ch.act == DS_ACT_RELU) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
                    }
                    uint2 o;
                    o.x = f2bf2(v[0], v[1]);
                    o.y = f2bf2(v[2], v[3]);
                    *(uint2*)(tile + prow * T_LD + col) = o;
                }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = prow8 + 32 * i;
                if (rowC[row] >= 0 && hb * 64 + pc8 < k_out2)
                    *(uint4*)(ch.C + rowR[row] + hb * 64 + pc8) = *(const uint4*)(tile + row * T_LD + pc8);
            }
        }
    }
}

}  // namespace

namespace {

int32_t thin_supported(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, int* kmax_out) {
    if (a.K > 1 || a.stride > 1 || a.pad > 0 || a.n_seg != 1 || a.out_f32 || (a.act != DS_ACT_NONE && a.act != DS_ACT_RELU))
        return DS_EUNSUPPORTED;
    int kmax = 0;
    for (int t = 0; t < a.gt.T; ++t) {
        kmax = a.gt.k_in[t] > kmax ? a.gt.k_in[t] : kmax;
        if ((a.gt.k_in[t] % 8) || (a.gt.k_out[t] % 8)) return DS_EUNSUPPORTED;
    }
    // measured: up to 64 input channels always wins (-27..-33 % per layer), 65..128 only where a residual is streamed too
    // (2 workgroups per compute unit there); one pass per workgroup gains nothing over the general kernel
    if (kmax > 128 || (kmax > 64 && !a.R) || max_kout < 128) return DS_EUNSUPPORTED;
    const long long slots = (long long)max_mtiles * BM / (a.rows > 0 ? a.rows : 1) + 1;
    if (slots * a.a_sample_stride * 2 >= 0x7fffffffLL) return DS_EUNSUPPORTED;
    if (((long long)max_kout * a.w_ld + kmax) * 2 >= 0x7fffffffLL) return DS_EUNSUPPORTED;   // 32-bit weight offsets
    *kmax_out = kmax;
    return DS_OK;
}

int32_t thin_configure() {
    const int32_t rc[6] = {ds_reserve_lds((const void*)thin_kernel<true, 4, true, 4>, smem_bytes(4), "thin layer"),
                           ds_reserve_lds((const void*)thin_kernel<true, 2, false>, smem_bytes(2), "thin layer"),
                           ds_reserve_lds((const void*)thin_kernel<false, 2, false>, smem_bytes(2), "thin layer"),
                           ds_reserve_lds((const void*)thin_kernel<true, 4, false>, smem_bytes(4), "thin layer"),
                           ds_reserve_lds((const void*)thin_kernel<false, 4, false>, smem_bytes(4), "thin layer"),
                           ds_reserve_lds((const void*)thin_kernel<true, 2, true>, smem_bytes_chain(), "thin layer")};
    for (int i = 0; i < 6; ++i)
        if (rc[i]) return rc[i];
    return DS_OK;
}

}  // namespace

// 1x1 / linear layers whose widest input slice is at most 64 channels, bf16 output, no activation or ReLU, one
// segment; DS_EUNSUPPORTED otherwise (the caller then uses the general kernel)
int32_t ds_launch_thin(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    if (max_mtiles <= 0 || max_kout <= 0) return DS_OK;
    int kmax = 0;
    if (thin_supported(a, max_mtiles, max_kout, &kmax) != DS_OK) return DS_EUNSUPPORTED;
    const int32_t rc = thin_configure();
    if (rc != DS_OK) return rc;
    ProfScope prof(DS_K_THIN, s);
    const dim3 grid((unsigned)max_mtiles), block(NT);
    ThinChain none;
    memset(&none, 0, sizeof(none));
    if (kmax <= 64) {
        if (a.R) hipLaunchKernelGGL((thin_kernel<true, 2, false>), grid, block, smem_bytes(2), s, a, max_mtiles, none);
        else hipLaunchKernelGGL((thin_kernel<false, 2, false>), grid, block, smem_bytes(2), s, a, max_mtiles, none);
    } else {
        if (a.R) hipLaunchKernelGGL((thin_kernel<true, 4, false>), grid, block, smem_bytes(4), s, a, max_mtiles, none);
        else hipLaunchKernelGGL((thin_kernel<false, 4, false>), grid, block, smem_bytes(4), s, a, max_mtiles, none);
    }
    DS_CHECK_LAUNCH("thin layer");
    return DS_OK;
}

// The same layer (input slices up to 128 channels, residual addressed like the output) followed, inside the workgroup, by
// a second 1x1 layer over the result rows with at most 128 output channels per group (64 / 64: three workgroups per
// compute unit; beyond: two); DS_EUNSUPPORTED otherwise (the caller then launches the two layers one after the other)
int32_t ds_launch_thin_chain(const GemmArgs& a, const ThinChain& ch, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    if (max_mtiles <= 0 || max_kout <= 0) return DS_EUNSUPPORTED;
    int kmax = 0;
    if (thin_supported(a, max_mtiles, max_kout, &kmax) != DS_OK) return DS_EUNSUPPORTED;
    if (!a.R || !a.r_use_index || a.r_sample_stride != a.c_sample_stride || a.r_ld != a.c_ld) return DS_EUNSUPPORTED;
    if (!ch.Wt || !ch.C || (ch.act != DS_ACT_NONE && ch.act != DS_ACT_RELU) || (ch.tab_ld % 4)) return DS_EUNSUPPORTED;
    // 16-byte pieces of the second output and of its weights, float4 reads of its batch-norm constants
    if ((ch.c_sample_stride % 8) || (ch.c_ld > 0 && ch.c_ld % 8) || (ch.w_ld % 8) ||
        (((uintptr_t)ch.scale | (uintptr_t)ch.shift | (uintptr_t)ch.C | (uintptr_t)ch.Wt) & 15))
        return DS_EUNSUPPORTED;
    int k2max = 0;
    for (int t = 0; t < a.gt.T; ++t) {
        if (ch.k_out[t] > 128 || (ch.k_out[t] > 0 && ch.k_out[t] % 8)) return DS_EUNSUPPORTED;
        k2max = ch.k_out[t] > k2max ? ch.k_out[t] : k2max;
    }
    if (((long long)k2max * ch.w_ld + max_kout) * 2 >= 0x7fffffffLL) return DS_EUNSUPPORTED;   // 32-bit weight offsets
    const int32_t rc = thin_configure();
    if (rc != DS_OK) return rc;
    ProfScope prof(DS_K_THIN, s);
    if (kmax <= 64 && k2max <= 64)
        hipLaunchKernelGGL((thin_kernel<true, 2, true>), dim3((unsigned)max_mtiles), dim3(NT), smem_bytes_chain(), s, a, max_mtiles, ch);
    else
        hipLaunchKernelGGL((thin_kernel<true, 4, true, 4>), dim3((unsigned)max_mtiles), dim3(NT), smem_bytes(4), s, a, max_mtiles, ch);
    DS_CHECK_LAUNCH("chained thin layers");
    return DS_OK;
}
