// Head-sliced self-attention (Section 3.4, Eq. 17): one workgroup per (slot, head),
// heads at or beyond the slot's head count exit at once.  Head dimension 32, 48 or 64
// (DS-ViT++ stores 8 heads of 48: its Q-K-V widths 192..384 in steps of 48 go with 4..8 heads),
// sequence length up to 224 (7 key tiles of 32).
//
// K and V^T of the head live in LDS.  One wavefront per 32-query tile (up to 7 per workgroup):
//   S^T[key][q] = K . Q^T   (v_mfma_f32_32x32x16_bf16; A = K rows from LDS, B = Q rows from global)
// so that one lane owns a fixed query column and half of its keys: the row
// maximum and sum of the softmax are in-lane reductions plus one exchange with
// lane^32.  The probabilities are rounded to bf16 in registers and fed straight back as the B
// operand of  O^T = V^T . P^T  (normalised by the row sum afterwards, in fp32); the key order an accumulator
// holds (runs of 4 keys) is reproduced on the V^T side with two 8-byte LDS reads,
// so no shuffle or LDS round trip of P is needed.
#include <type_traits>

#include "common.h"

namespace {

constexpr int NKT = 7, KEYS = NKT * 32, V_LD = KEYS + 8;

// DH: head dimension, a multiple of 16.  The output tiles are 32 channels tall, so V^T is padded with
// zero rows to DT * 32 channels and the channels past DH are computed and dropped.
template <int DH>
__global__ __launch_bounds__(448) __attribute__((amdgpu_waves_per_eu(4, 4))) void attention_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                        const bf16_t* __restrict__ v, bf16_t* __restrict__ o,
                                                        int64_t sample_stride, int ld, int o_ld,
                                                        int64_t o_sample_stride, const int32_t* slot_group,
                                                        const GroupTable gt, int N, float scale) {
    constexpr int K_LD = DH + 8, KK = DH / 16, DT = (DH + 31) / 32, CPR = DH / 8;
    static_assert(DH % 16 == 0 && DH <= 64, "head dimension");
    __shared__ __attribute__((aligned(16))) bf16_t Ks[KEYS * K_LD];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[DT * 32 * V_LD];
    const int slot = blockIdx.x, head = blockIdx.y;
    const int g = slot_group ? slot_group[slot] : 0;
    if (head * DH >= gt.k_out[g]) return;
    const int tid = threadIdx.x;
    const int64_t base = (int64_t)slot * sample_stride + head * DH;

    // this lane's query row, fetched first so that its latency overlaps the staging of K and V
    const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int qrow = wave * 32 + l32;
    bf16x8_t qf[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        uint4 t = make_uint4(0, 0, 0, 0);
        if (qrow < N) t = *(const uint4*)(q + base + (int64_t)qrow * ld + kk * 16 + lhi * 8);
        qf[kk] = *(bf16x8_t*)&t;
    }

    const int nthreads = blockDim.x;          // one wavefront per 32-query tile
    if constexpr (DH % 32 != 0)
        for (int c = tid; c < (DT * 32 - DH) * V_LD / 2; c += nthreads) ((uint32_t*)(Vt + DH * V_LD))[c] = 0u;
    for (int c = tid; c < KEYS * CPR; c += nthreads) {
        const int row = c / CPR, ch = (c - row * CPR) * 8;
        uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
        if (row < N) {
            kv = *(const uint4*)(k + base + (int64_t)row * ld + ch);
            vv = *(const uint4*)(v + base + (int64_t)row * ld + ch);
        }
        *(uint4*)(Ks + row * K_LD + ch) = kv;
        const uint32_t w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            Vt[(ch + 2 * i) * V_LD + row] = (bf16_t)(w[i] & 0xffffu);
            Vt[(ch + 2 * i + 1) * V_LD + row] = (bf16_t)(w[i] >> 16);
        }
    }
    __syncthreads();

    {
        // The keys are taken in two parts (tiles 0..3, then 4..6) with a running maximum and sum, so that only four
        // score tiles are alive at a time: 128 registers instead of 160, which lets two workgroups share a compute
        // unit and one of them stage its K and V while the other multiplies.  p = 2^((s - max) * scale * log2(e)),
        // masked keys get -inf; the scale is positive, so the maximum is taken on the raw scores.  The part's
        // probabilities are rounded to bf16 (relative to the running maximum), multiplied into O^T, and when the
        // maximum rises the earlier sum and O^T are scaled by 2^((old - new) * scale * log2(e)).
        const float c2 = scale * 1.44269504088896340736f;
        float m = -INFINITY, sum = 0.f;
        f32x16_t oacc[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;
        int krow = l32;                           // first key row of this lane; re-derived after each part (below)
        auto part = [&](auto lo_c, auto hi_c) {
            constexpr int LO = decltype(lo_c)::value, HI = decltype(hi_c)::value, NP = HI - LO;
            f32x16_t sacc[NP];
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int kt = LO + i;
#pragma unroll
                for (int e = 0; e < 16; ++e) sacc[i][e] = 0.f;
#pragma unroll
                for (int kk = 0; kk < KK; ++kk) {
                    const bf16x8_t kf = *(const bf16x8_t*)(Ks + (kt * 32 + krow) * K_LD + kk * 16 + lhi * 8);
                    sacc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[i], 0, 0, 0);
                }
            }
            __builtin_amdgcn_sched_barrier(0);   // keep the phases apart: interleaving them costs the registers this split saves
            float mp = -INFINITY;
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int kt = LO + i;
                if (kt * 32 + 32 > N) {           // only the tiles that reach past the sequence need the mask
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int key = kt * 32 + 8 * (e >> 2) + 4 * lhi + (e & 3);
                        if (key >= N) sacc[i][e] = -INFINITY;
                    }
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) mp = fmaxf(mp, sacc[i][e]);
            }
            mp = fmaxf(mp, __shfl_xor(mp, 32, 64));
            if (LO > 0) {
                // a part with every key masked (N <= 128) leaves the maximum where it was and adds zeros
                const float mn = fmaxf(m, mp);
                const float alpha = __builtin_amdgcn_exp2f((m - mn) * c2);
                sum *= alpha;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int e = 0; e < 16; ++e) oacc[dt][e] *= alpha;
                m = mn;
            } else {
                m = mp;                           // key 0 is never masked: finite
            }
            const float mc = m * c2;
            __builtin_amdgcn_sched_barrier(0);
            uint32_t pf[NP][8];
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                float pr[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    pr[e] = __builtin_amdgcn_exp2f(fmaf(sacc[i][e], c2, -mc));   // argument <= 0; results below 2^-126 flush to 0
                    sum += pr[e];
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[i][e] = f2bf2(pr[2 * e], pr[2 * e + 1]);
                asm volatile("" : "+v"(sum));        // the additions stay here: deferred, they keep all 16 values alive
                __builtin_amdgcn_sched_barrier(0);   // tile by tile: 16 scores become 8 packed registers before the next tile starts
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int kt = LO + i;
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    union { uint32_t u[4]; bf16x8_t v; } pv;
#pragma unroll
                    for (int e = 0; e < 4; ++e) pv.u[e] = pf[i][4 * half + e];
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        const bf16_t* vp = Vt + (dt * 32 + l32) * V_LD + kt * 32 + 16 * half + 4 * lhi;
                        union { uint2 h[2]; bf16x8_t v; } vf;
                        vf.h[0] = *(const uint2*)vp;
                        vf.h[1] = *(const uint2*)(vp + 8);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pv.v, oacc[dt], 0, 0, 0);
                    }
                }
            }
        };
        part(std::integral_constant<int, 0>{}, std::integral_constant<int, 4>{});
        // the second part's score tiles must not be started while the first part's probabilities are alive: tie the
        // address of its K reads to the end of the first part's O^T accumulation
        asm volatile("" : "+v"(krow) : "v"(oacc[0][0]), "v"(oacc[DT - 1][15]));
        part(std::integral_constant<int, 4>{}, std::integral_constant<int, NKT>{});
        sum += __shfl_xor(sum, 32, 64);
        const float inv = 1.0f / sum;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[dt][e] *= inv;
        // oacc[dt][e] = O[q = l32][d = dt*32 + 8*(e>>2) + 4*lhi + (e&3)]: 4 consecutive channels per store
        if (qrow < N) {
            bf16_t* op = o + (int64_t)slot * o_sample_stride + (int64_t)qrow * o_ld + head * DH + 4 * lhi;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    if (dt * 32 + 8 * g4 >= DH) continue;   // padding channels of the last tile
                    uint2 w;
                    w.x = f2bf2(oacc[dt][4 * g4], oacc[dt][4 * g4 + 1]);
                    w.y = f2bf2(oacc[dt][4 * g4 + 2], oacc[dt][4 * g4 + 3]);
                    *(uint2*)(op + dt * 32 + 8 * g4) = w;
                }
        }
    }
}

}  // namespace

int32_t ds_launch_attention(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* o, int64_t sample_stride,
                            int32_t ld, int32_t o_ld, int64_t o_sample_stride, const int32_t* slot_group,
                            const GroupTable& gt, int32_t B, int32_t N, int32_t H, int32_t head_dim, hipStream_t s) {
    if (B <= 0 || H <= 0) return DS_OK;
    if (N < 1 || N > KEYS) DS_FAIL(DS_EUNSUPPORTED, "attention: sequence length %d outside 1..%d", N, KEYS);
    if (head_dim != 32 && head_dim != 48 && head_dim != 64)
        DS_FAIL(DS_EUNSUPPORTED, "attention: head dimension %d (32, 48 or 64)", head_dim);
    ProfScope prof(DS_K_ATTENTION, s);
    const dim3 grid((unsigned)B, (unsigned)H), block(64 * ((N + 31) / 32));
    const float scale = 1.0f / sqrtf((float)head_dim);
#define DS_ATT(D)                                                                                                  \
    hipLaunchKernelGGL(attention_kernel<D>, grid, block, 0, s, q, k, v, o, sample_stride, ld, o_ld, o_sample_stride, \
                       slot_group, gt, N, scale)
    if (head_dim == 64) DS_ATT(64);
    else if (head_dim == 48) DS_ATT(48);
    else DS_ATT(32);
#undef DS_ATT
    DS_CHECK_LAUNCH("attention");
    return DS_OK;
}
