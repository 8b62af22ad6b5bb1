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
// Tiling: 128x128 output tile per 256-thread workgroup, 4 wavefronts in a 2x2
// arrangement, each holding 2x2 accumulators of v_mfma_f32_32x32x16_bf16.
// Operands are staged through LDS in 128x32 slabs (row stride padded to 40
// elements), with the next slab's global loads issued before the current slab's
// matrix instructions.
#include "common.h"

namespace {

constexpr int BM = DS_GEMM_BM, BN = 128, BK = 32, LDS_LD = BK + 8, NT = 256;

struct RowInfo {
    int64_t base;   // element offset of the sample
    int iy0, ix0;   // top-left input pixel of the receptive field
    bool valid;
};

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

__global__ __launch_bounds__(NT) void gemm_kernel(const GemmArgs a) {
    __shared__ __attribute__((aligned(16))) bf16_t As[BM * LDS_LD];
    __shared__ __attribute__((aligned(16))) bf16_t Bs[BN * LDS_LD];

    const int mt = blockIdx.x;
    if (mt >= *a.n_mtiles) return;
    const int2 me = a.mtiles[mt];
    const int g = me.x, grow0 = me.y;
    const int k_in = a.gt.k_in[g], k_out = a.gt.k_out[g];
    if (k_in <= 0 || k_out <= 0) return;
    const int ntiles = (k_out + BN - 1) / BN;
    const int seg = blockIdx.y / ntiles;
    if (seg >= a.n_seg) return;
    const int n0 = (blockIdx.y - seg * ntiles) * BN;
    const int slot0 = a.offsets[g];
    const int rows_g = (a.offsets[g + 1] - slot0) * a.rows;

    const int tid = threadIdx.x;
    const int a_ld = a.a_ld > 0 ? a.a_ld : k_in;

    // ---- per-thread load assignment: 2 A chunks + 2 B chunks of 8 elements --
    RowInfo ri[2];
    int64_t wrow[2];
    bool wvalid[2];
    const int kc8 = (tid & 3) * 8;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = (tid >> 2) + i * 64;
        const int m = grow0 + r;
        ri[i].valid = m < rows_g;
        const int mm = ri[i].valid ? m : 0;
        const int slot = slot0 + mm / a.rows;
        const int p = mm % a.rows;
        const int sample = a.a_index ? a.a_index[slot] : slot;
        ri[i].base = (int64_t)sample * a.a_sample_stride;
        ri[i].iy0 = (p / a.Wo) * a.stride - a.pad;
        ri[i].ix0 = (p % a.Wo) * a.stride - a.pad;
        const int n = n0 + r;
        wvalid[i] = n < k_out;
        wrow[i] = (int64_t)seg * a.w_seg_stride + (int64_t)(wvalid[i] ? n : 0) * a.w_ld;
    }

    const int kchunks = (k_in + BK - 1) / BK;
    const int nk = a.K * a.K * kchunks;

    uint4 ra[2], rb[2];
    auto load_global = [&](int tap, int kc) {
        const int u = tap / a.K, v = tap - u * a.K;
        const bool kok = (kc + kc8) < k_in;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int iy = ri[i].iy0 + u, ix = ri[i].ix0 + v;
            const bool ok = ri[i].valid && kok && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
            ra[i] = make_uint4(0, 0, 0, 0);
            if (ok) ra[i] = *(const uint4*)(a.A + ri[i].base + (int64_t)(iy * a.W + ix) * a_ld + kc + kc8);
            rb[i] = make_uint4(0, 0, 0, 0);
            if (wvalid[i] && kok) rb[i] = *(const uint4*)(a.Wt + wrow[i] + (int64_t)tap * a.w_tap_stride + kc + kc8);
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int r = (tid >> 2) + i * 64;
            *(uint4*)(As + r * LDS_LD + kc8) = ra[i];
            *(uint4*)(Bs + r * LDS_LD + kc8) = rb[i];
        }
    };

    const int wave = tid >> 6, lane = tid & 63;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    int tap = 0, kc = 0;
    load_global(tap, kc);
    store_lds();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        int ntap = tap, nkc = kc + BK;
        if (nkc >= k_in) { nkc = 0; ntap = tap + 1; }
        if (kt + 1 < nk) load_global(ntap, nkc);
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8_t af[2], bfg[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                af[t] = *(const bf16x8_t*)(As + (wm * 64 + t * 32 + l32) * LDS_LD + kk * 16 + lhi * 8);
                bfg[t] = *(const bf16x8_t*)(Bs + (wn * 64 + t * 32 + l32) * LDS_LD + kk * 16 + lhi * 8);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfg[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
        if (kt + 1 < nk) {
            store_lds();
            __syncthreads();
        }
        tap = ntap;
        kc = nkc;
    }

    // ---- epilogue: scale/shift (+bias), residual, activation, store ---------
    const int trow = a.gt.row[g];
    const int c_ld = a.c_ld > 0 ? a.c_ld : k_out;
    const int r_ld = a.r_ld > 0 ? a.r_ld : k_out;
    float sc[2], sh[2];
    int ncol[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + j * 32 + l32;
        ncol[j] = n;
        const int64_t ti = (int64_t)trow * a.tab_ld + (int64_t)seg * a.tab_seg_stride + (n < k_out ? n : 0);
        sc[j] = a.scale ? a.scale[ti] : 1.f;
        sh[j] = a.shift ? a.shift[ti] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v >> 2) + 4 * lhi + (v & 3);
            const int m = grow0 + wm * 64 + i * 32 + row;
            if (m >= rows_g) continue;
            const int slot = slot0 + m / a.rows;
            const int p = m % a.rows + a.c_row0;
            const int cs = a.c_index ? a.c_index[slot] : slot;
            const int64_t crow = (int64_t)cs * a.c_sample_stride + (int64_t)p * c_ld + (int64_t)seg * a.c_seg_stride;
            const int64_t rrow = (int64_t)(a.r_use_index ? cs : 0) * a.r_sample_stride + (int64_t)p * r_ld;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = ncol[j];
                if (n >= k_out) continue;
                float val = acc[i][j][v] * sc[j] + sh[j];
                if (a.R) val += bf2f(a.R[rrow + n]);
                if (a.act == DS_ACT_RELU) val = fmaxf(val, 0.f);
                else if (a.act == DS_ACT_GELU) val = gelu_erf(val);
                if (a.out_f32) ((float*)a.C)[crow + n] = val;
                else ((bf16_t*)a.C)[crow + n] = f2bf(val);
            }
        }
    }
}

__global__ void build_mtiles_kernel(const int32_t* offsets, int T, int rows, int32_t* count, int2* entries) {
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
        for (int i = threadIdx.x; i < n; i += blockDim.x) entries[pre[g] + i] = make_int2(g, i * BM);
    }
}

}  // namespace

size_t ds_mtile_capacity(int32_t B, int32_t rows, int32_t T) {
    return (size_t)(((int64_t)B * rows + BM - 1) / BM + T);
}

int32_t ds_build_mtiles(const int32_t* offsets, int32_t T, int32_t rows, void* list, hipStream_t s) {
    ProfScope prof(DS_K_MISC, s);
    hipLaunchKernelGGL(build_mtiles_kernel, dim3(1), dim3(256), 0, s, offsets, T, rows, (int32_t*)list,
                       (int2*)((char*)list + 16));
    DS_CHECK_LAUNCH("build_mtiles");
    return DS_OK;
}

int32_t ds_launch_gemm(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    if (max_mtiles <= 0 || max_kout <= 0) return DS_OK;
    dim3 grid((unsigned)max_mtiles, (unsigned)(a.n_seg * ((max_kout + BN - 1) / BN)));
    ProfScope prof(a.K > 1 ? DS_K_GEMM_TAPS : DS_K_GEMM, s);
    hipLaunchKernelGGL(gemm_kernel, grid, dim3(NT), 0, s, a);
    DS_CHECK_LAUNCH("sliced gemm");
    return DS_OK;
}
