// Grouped prefix-slice 3x3 convolution (stride 1, padding 1) as an implicit GEMM whose input patch
// is staged once per channel chunk (filter slicing, Section 3.3 Eq. 9; split batch-norm, Eq. 14).
//
// gemm_kernel walks the 9 taps as 9 separate reduction slabs and fetches the 128 shifted input
// pixels of each tap from L2 again.  Here a workgroup (same 128-pixel x 64-filter tile, same
// epilogue) loads, for every 32-channel chunk, the contiguous run of input pixels that its 128
// output pixels touch -- pixel indices m - (W+1) .. m + 127 + (W+1) in the group's row-major pixel
// order, 128 + 2 (W+1) rows -- once into LDS, and every tap reads its operand rows from that patch
// at a fixed row offset ((u-1) W + (v-1)); lanes whose tap falls outside the image (or the group)
// read a row of zeros instead.  A tap that is inside the image never leaves the sample, so the
// linear pixel order needs no per-sample bookkeeping.  The weights of one filter row (3 taps) are
// staged per phase: 12 matrix instructions per wavefront between barriers instead of 4, and the
// activation traffic from L2 drops from 9 x 128 rows per chunk to 128 + 2 (W+1).
#include "common.h"

namespace {

constexpr int BM = DS_GEMM_BM, BN = 64, NT = 256;
constexpr int RMAX = 248;                      // patch rows: 128 + 2 (W + 1), so W <= 59
constexpr int ZROW = RMAX;                     // one more row, all zeros
constexpr int TPP = 3;                         // taps staged per phase: 3 (one filter row) or 9 (the whole filter)
constexpr int PPC = 9 / TPP;                   // phases per channel chunk
constexpr int A_BYTES = (RMAX + 1) * 64, B_BYTES = TPP * BN * 64;
constexpr int SROWS = 16, ST_LD = BN + 4, STAGE_BYTES = 4 * SROWS * ST_LD * 4;
constexpr int MAIN_BYTES = A_BYTES + B_BYTES > STAGE_BYTES ? A_BYTES + B_BYTES : STAGE_BYTES;
constexpr int TABLE_BYTES = BM * 16;
constexpr int SMEM = MAIN_BYTES + TABLE_BYTES;
constexpr int NR = (RMAX * 4 + NT - 1) / NT;   // 16-byte patch loads per thread and chunk

// chunk c of a 64-byte LDS row r is stored at position c ^ sw(r): any run of consecutive rows read
// with one chunk column spreads over the banks, whatever row the run starts at, for access groups of
// 8 lanes (128 bytes) and of 16 lanes (256 bytes) alike -- a key of (r >> 1) & 3 serves only the former
// and cost 40 % of the LDS cycles in conflicts
__device__ __forceinline__ int sw(int r) { return ((r >> 1) ^ (r >> 2)) & 3; }
__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

template <bool HASR>
__global__ __launch_bounds__(NT) void conv3_kernel(const GemmArgs a, const int ny, const int max_mtiles) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* As = smem;                                   // [RMAX + 1][32] bf16
    char* Bs = smem + A_BYTES;                         // [TPP][BN][32] bf16
    long long* rowC = (long long*)(smem + MAIN_BYTES);
    long long* rowR = rowC + BM;
    constexpr uint32_t OOB = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, 0x7fffffff, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_w = __builtin_amdgcn_make_buffer_rsrc((void*)a.Wt, 0, 0x7fffffff, 0x00020000);

    const int j = (int)(blockIdx.x >> 3);
    const int jm = j / ny, y = j - jm * ny;
    const int mt = jm * 8 + (int)(blockIdx.x & 7);
    if (mt >= max_mtiles) return;
    const int4 me = a.mtiles[mt];
    if (mt >= *a.n_mtiles) return;
    const int g = me.x, grow0 = me.y, slot0 = me.z, rows_g = me.w;
    const int k_in = a.gt.k_in[g], k_out = a.gt.k_out[g];
    if (k_in <= 0 || k_out <= 0) return;
    const int n0 = y * BN;
    if (n0 >= k_out) return;

    const int tid = threadIdx.x;
    const int a_ld = a.a_ld > 0 ? a.a_ld : k_in;
    const int c_ld = a.c_ld > 0 ? a.c_ld : k_out;
    const int r_ld = a.r_ld > 0 ? a.r_ld : k_out;
    const int W = a.W, H = a.H, rows = a.rows;
    const int halo = W + 1, R = BM + 2 * halo;

    if (tid < 4) *(uint4*)(As + ZROW * 64 + tid * 16) = make_uint4(0, 0, 0, 0);

    // ---- patch loader: item e = tid + 256 i is chunk (e & 3) of patch row (e >> 2) --------------
    const int lchunk = tid & 3;
    uint32_t poff[NR];
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        const int jr = (tid + NT * i) >> 2;
        const int L = grow0 - halo + jr;              // pixel index in the group's row-major order
        uint32_t o = OOB;
        if (jr < R && L >= 0 && L < rows_g) {
            const int sl = L / rows;
            const int p = L - sl * rows;
            const int slot = slot0 + sl;
            const int sa = a.a_index ? a.a_index[slot] : slot;
            o = (uint32_t)(((long long)sa * a.a_sample_stride + (long long)p * a_ld + lchunk * 8) * 2);
        }
        poff[i] = o;
    }
    // ---- weight loader: chunk (tid & 3) of filter row n0 + (tid >> 2), one load per tap ---------
    const int wn_row = tid >> 2;
    const uint32_t woff = (n0 + wn_row) < k_out ? (uint32_t)(((long long)(n0 + wn_row) * a.w_ld + lchunk * 8) * 2) : OOB;

    uint4 ra[NR], rb[TPP];
    auto load_phase = [&](int c, int u) {
        const int kc = c * 32;
        const bool kok = kc + lchunk * 8 < k_in;
        if (u == 0) {
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_a, (int)(kok ? poff[i] : OOB), kc * 2, 0);
                ra[i] = make_uint4(t[0], t[1], t[2], t[3]);
            }
        }
#pragma unroll
        for (int v = 0; v < TPP; ++v) {
            const int soff = (int)(((u * TPP + v) * a.w_tap_stride + kc) * 2);
            const auto t = __builtin_amdgcn_raw_buffer_load_b128(rsrc_w, (int)(kok ? woff : OOB), soff, 0);
            rb[v] = make_uint4(t[0], t[1], t[2], t[3]);
        }
    };
    auto store_phase = [&](int u) {
        if (u == 0) {
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                const int jr = (tid + NT * i) >> 2;
                if (jr < R) *(uint4*)(As + jr * 64 + ((lchunk ^ sw(jr)) * 16)) = ra[i];
            }
        }
#pragma unroll
        for (int v = 0; v < TPP; ++v) *(uint4*)(Bs + (v * BN + wn_row) * 64 + ((lchunk ^ sw(wn_row)) * 16)) = rb[v];
    };

    // the first patch and filter-row loads are requested as soon as their addresses are known: everything below (output
    // row table, tap mask, epilogue constants) is worked out while they travel
    load_phase(0, 0);

    if (tid < BM) {
        const int m = grow0 + tid;
        long long rc = -1, rr = 0;
        if (m < rows_g) {
            const int sl = m / rows;
            const int p = m - sl * rows;
            const int slot = slot0 + sl;
            const int cs = a.c_index ? a.c_index[slot] : slot;
            rc = (long long)cs * a.c_sample_stride + (long long)(p + a.c_row0) * c_ld;
            rr = (long long)(a.r_use_index ? cs : 0) * a.r_sample_stride + (long long)(p + a.c_row0) * r_ld;
        }
        rowC[tid] = rc;
        rowR[tid] = rr;
    }
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    // ---- this lane's output pixel: which taps are inside the image ---------------------------
    const int trow = wave * 32 + l32;
    int tapmask = 0;
    {
        const int m = grow0 + trow;
        if (m < rows_g) {
            const int p = m % rows;
            const int oy = p / W, ox = p - oy * W;
#pragma unroll
            for (int u = 0; u < 3; ++u)
#pragma unroll
                for (int v = 0; v < 3; ++v) {
                    const int iy = oy + u - 1, ix = ox + v - 1;
                    if (iy >= 0 && iy < H && ix >= 0 && ix < W) tapmask |= 1 << (u * 3 + v);
                }
        }
    }

    f32x16_t acc[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;

    // epilogue constants and residual rows, fetched early so that their latency hides behind the loop
    constexpr int COLS = BN, CG = COLS / 4, RPP = 64 / CG, PASSES = 32 / SROWS, VPP = 16 / PASSES;
    const int cg = lane % CG, rr0 = lane / CG;
    const int ncol = n0 + cg * 4;
    const bool nok = ncol < k_out;
    float sc[4] = {1.f, 1.f, 1.f, 1.f}, sh[4] = {0.f, 0.f, 0.f, 0.f};
    if (nok) {
        const long long ti = (long long)a.gt.row[g] * a.tab_ld + ncol;
        if (a.scale) {
            const float4 t = *(const float4*)(a.scale + ti);
            sc[0] = t.x; sc[1] = t.y; sc[2] = t.z; sc[3] = t.w;
        }
        if (a.shift) {
            const float4 t = *(const float4*)(a.shift + ti);
            sh[0] = t.x; sh[1] = t.y; sh[2] = t.z; sh[3] = t.w;
        }
    }
    __syncthreads();                                   // row table visible
    uint2 rres[HASR ? PASSES * (SROWS / RPP) : 1];
    if constexpr (HASR) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps)
#pragma unroll
            for (int q = 0; q < SROWS / RPP; ++q) {
                const int r = wave * 32 + ps * SROWS + rr0 + q * RPP;
                uint2 t = make_uint2(0, 0);
                if (nok && rowC[r] >= 0) t = *(const uint2*)(a.R + rowR[r] + ncol);
                rres[ps * (SROWS / RPP) + q] = t;
            }
    }

    const int nph = ((k_in + 31) / 32) * PPC;
    store_phase(0);
    __syncthreads();
    int c = 0, u = 0;
    for (int ph = 0; ph < nph; ++ph) {
        int cn = c, un = u + 1;
        if (un == PPC) {
            un = 0;
            ++cn;
        }
        const bool more = ph + 1 < nph;
        if (more) load_phase(cn, un);
#pragma unroll
        for (int v = 0; v < TPP; ++v) {
            const int tap = u * TPP + v;
            const int tu = tap / 3, tv = tap - tu * 3;
            const int arow = ((tapmask >> tap) & 1) ? trow + halo + (tu - 1) * W + (tv - 1) : ZROW;
            const char* ap = As + arow * 64;
            const int fa = sw(arow);
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const int ch = kk * 2 + lhi;
                const bf16x8_t af = *(const bf16x8_t*)(ap + ((ch ^ fa) * 16));
                bf16x8_t bfr[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int nr = t * 32 + l32;
                    bfr[t] = *(const bf16x8_t*)(Bs + (v * BN + nr) * 64 + ((ch ^ sw(nr)) * 16));
                }
#pragma unroll
                for (int t = 0; t < 2; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfr[t], acc[t], 0, 0, 0);
            }
        }
        __syncthreads();
        if (more) {
            store_phase(un);
            __syncthreads();
        }
        c = cn;
        u = un;
    }

    // ---- epilogue through LDS: each lane finishes 4 consecutive channels of one row -----------
    // staging rows are private to a wavefront and the loop's last barrier has retired every read of the tiles they
    // alias: between the passes only the compiler has to be kept from moving LDS accesses
    auto wave_sync = [] {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    float* st = (float*)smem + wave * SROWS * ST_LD;
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int vv = 0; vv < VPP; ++vv) {
                const int v = ps * VPP + vv;
                const int lr = 8 * ((v >> 2) - ps * (4 / PASSES)) + 4 * lhi + (v & 3);
                st[lr * ST_LD + tn * 32 + l32] = acc[tn][v];
            }
        wave_sync();
        if (nok) {
#pragma unroll
            for (int rr = rr0; rr < SROWS; rr += RPP) {
                const int r = wave * 32 + ps * SROWS + rr;
                const long long coff = rowC[r];
                if (coff < 0) continue;
                const float4 t = *(const float4*)(st + rr * ST_LD + cg * 4);
                float val[4] = {t.x * sc[0] + sh[0], t.y * sc[1] + sh[1], t.z * sc[2] + sh[2], t.w * sc[3] + sh[3]};
                if constexpr (HASR) {
                    const uint2 q = rres[ps * (SROWS / RPP) + (rr - rr0) / RPP];
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

template <bool HASR>
int32_t launch(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    auto kern = conv3_kernel<HASR>;
    {
        const int32_t rc = ds_reserve_lds((const void*)kern, SMEM, "sliced 3x3 conv");
        if (rc) return rc;
    }
    const int ny = (max_kout + BN - 1) / BN;
    const unsigned grid = (unsigned)(((max_mtiles + 7) / 8) * ny * 8);
    ProfScope prof(DS_K_CONV3, s);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NT), SMEM, s, a, ny, max_mtiles);
    DS_CHECK_LAUNCH("sliced 3x3 conv");
    return DS_OK;
}

}  // namespace

// 3x3, stride 1, padding 1, one segment, maps up to 59 pixels wide; DS_EUNSUPPORTED otherwise
int32_t ds_launch_conv3(const GemmArgs& a, int32_t max_mtiles, int32_t max_kout, hipStream_t s) {
    if (a.K != 3 || a.stride != 1 || a.pad != 1 || a.n_seg != 1 || a.Ho != a.H || a.Wo != a.W || a.rows != a.H * a.W ||
        BM + 2 * (a.W + 1) > RMAX)
        return DS_EUNSUPPORTED;
    if (((long long)max_kout * a.w_ld + 9 * a.w_tap_stride) * 2 >= 0x7fffffffLL) return DS_EUNSUPPORTED;   // 32-bit weight offsets
    return a.R ? launch<true>(a, max_mtiles, max_kout, s) : launch<false>(a, max_mtiles, max_kout, s);
}
