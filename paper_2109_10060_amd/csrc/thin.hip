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

namespace {

constexpr int BM = DS_GEMM_BM, NT = 256, T_LD = 64 + 8;
constexpr uint32_t OOB = 0x80000000u;
constexpr int TILE_BYTES = BM * T_LD * 2;
constexpr int smem_bytes(int kch) { return kch * BM * 64 + kch * 64 * 64 + TILE_BYTES + BM * (8 + 8 + 4) + 2 * 64 * 4; }

__device__ __forceinline__ int swz(int r) { return ((r >> 1) ^ (r >> 2)) & 3; }

// KCH: 32-channel chunks of the widest input slice (2: up to 64 channels, 4: up to 128)
template <bool HASR, int KCH>
__global__ __launch_bounds__(NT) void thin_kernel(const GemmArgs a, const int max_mtiles) {
    constexpr int A_BYTES = KCH * BM * 64, B_BYTES = KCH * 64 * 64, CP = KCH * 4;   // CP 16-byte pieces per operand row
    constexpr int NAP = BM * CP / NT, NWP = 64 * CP / NT;                            // pieces per lane: activations, weights
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* As = smem;                                   // [KCH][128][32] bf16
    char* Bs = smem + A_BYTES;                         // [KCH][64][32] bf16
    bf16_t* tile = (bf16_t*)(smem + A_BYTES + B_BYTES);   // [128][T_LD]: residual in, result out
    long long* rowC = (long long*)(smem + A_BYTES + B_BYTES + TILE_BYTES);
    long long* rowR = rowC + BM;
    uint32_t* rowA = (uint32_t*)(rowR + BM);
    float* cst = (float*)(rowA + BM);                  // [64] scale, [64] shift of the pass
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
            rr = (long long)(a.r_use_index ? cs : 0) * a.r_sample_stride + pc * r_ld;
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
                if (rowC[row] >= 0 && n0 + pc8 < k_out) t = *(const uint4*)(a.R + rowR[row] + n0 + pc8);
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
    for (int n0 = 0; n0 < k_out; n0 += 64) {
        __syncthreads();                               // activation rows staged / last pass's tile copied out
#pragma unroll
        for (int i = 0; i < NWP; ++i) {
            const int nl = orow + (NT / CP) * i;
            *(uint4*)(Bs + ((oc8 >> 2) * 64 + nl) * 64 + (((oc8 & 3) ^ swz(nl)) * 16)) = wreg[i];
        }
        if (tid < 128) cst[tid] = creg;
        if constexpr (HASR) {
#pragma unroll
            for (int i = 0; i < 4; ++i) *(uint4*)(tile + (prow8 + 32 * i) * T_LD + pc8) = rreg[i];
        }
        __syncthreads();
        if (n0 + 64 < k_out) fetch_pass(n0 + 64);      // in flight during this pass
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
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = prow8 + 32 * i;
            const long long rc = rowC[row];
            if (rc >= 0 && n0 + pc8 < k_out) *(uint4*)((bf16_t*)a.C + rc + n0 + pc8) = *(const uint4*)(tile + row * T_LD + pc8);
        }
    }
}

}  // namespace

// 1x1 / linear layers whose widest input slice is at most 64 channels, bf16 output, no activation or ReLU, one
// segment; DS_EUNSUPPORTED otherwise (the caller then uses the general kernel)
int32_t ds_launch_thin(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    if (max_mtiles <= 0 || max_kout <= 0) return DS_OK;
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
    static bool configured = false;
    if (!configured) {
        if (hipFuncSetAttribute((const void*)thin_kernel<true, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes(2)) != hipSuccess ||
            hipFuncSetAttribute((const void*)thin_kernel<false, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes(2)) != hipSuccess ||
            hipFuncSetAttribute((const void*)thin_kernel<true, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes(4)) != hipSuccess ||
            hipFuncSetAttribute((const void*)thin_kernel<false, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes(4)) != hipSuccess)
            DS_FAIL(DS_EHIP, "thin layer: cannot reserve %d bytes of LDS", smem_bytes(4));
        configured = true;
    }
    ProfScope prof(DS_K_GEMM, s);
    const dim3 grid((unsigned)max_mtiles), block(NT);
    if (kmax <= 64) {
        if (a.R) hipLaunchKernelGGL((thin_kernel<true, 2>), grid, block, smem_bytes(2), s, a, max_mtiles);
        else hipLaunchKernelGGL((thin_kernel<false, 2>), grid, block, smem_bytes(2), s, a, max_mtiles);
    } else {
        if (a.R) hipLaunchKernelGGL((thin_kernel<true, 4>), grid, block, smem_bytes(4), s, a, max_mtiles);
        else hipLaunchKernelGGL((thin_kernel<false, 4>), grid, block, smem_bytes(4), s, a, max_mtiles);
    }
    DS_CHECK_LAUNCH("thin layer");
    return DS_OK;
}
