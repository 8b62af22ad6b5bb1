// Small dense layers applied to one vector per item: the gate's first MLP layer (Section 3.5,
// Eq. 22, input-sliced to the item's valid channels) and the classifier behind the global
// average pool.  A workgroup computes a 64-output x 16-item tile so that every weight row is
// read once per 16 items instead of once per item.
#include "common.h"

namespace {

template <typename WT>
__device__ __forceinline__ float wload(const WT* p);
template <>
__device__ __forceinline__ float wload<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float wload<bf16_t>(const bf16_t* p) { return bf2f(*p); }

constexpr int TO = 64, TI = 16, TC = 64;

template <typename WT, typename ACC>
__global__ __launch_bounds__(256) void fc_tile_kernel(const FcArgs a) {
    __shared__ float Wl[TO][TC + 1];
    __shared__ float Vl[TI][TC];
    __shared__ int cs[TI];
    const int tid = threadIdx.x;
    const int o0 = blockIdx.x * TO, i0 = blockIdx.y * TI;
    if (tid < TI) {
        const int item = i0 + tid;
        int c = 0;
        if (item < a.items) c = a.c_item ? a.c_item[item] : a.C;
        cs[tid] = c;
    }
    __syncthreads();
    int cmax = 0;
#pragma unroll
    for (int i = 0; i < TI; ++i) cmax = max(cmax, cs[i]);
    const int ol = tid & 63, ig = tid >> 6;      // a wavefront shares its 4 items: LDS broadcast reads
    ACC acc[4] = {0, 0, 0, 0};
    const WT* w = (const WT*)a.w;
    for (int c0 = 0; c0 < cmax; c0 += TC) {
        for (int e = tid; e < TO * TC; e += 256) {
            const int r = e / TC, cc = e - r * TC;
            const int o = o0 + r, c = c0 + cc;
            Wl[r][cc] = (o < a.n_out && c < cmax) ? wload<WT>(w + (int64_t)o * a.w_ld + c) : 0.f;
        }
        for (int e = tid; e < TI * TC; e += 256) {
            const int r = e / TC, cc = e - r * TC;
            const int item = i0 + r, c = c0 + cc;
            float v = 0.f;
            if (c < cs[r]) {
                if (a.v_rows) {
                    v = bf2f(a.v_rows[(int64_t)item * a.v_row_stride + c]);
                } else {
                    double s = 0.0;
                    for (int sp = 0; sp < a.splits; ++sp) s += (double)a.v_partial[((int64_t)item * a.splits + sp) * a.C + c];
                    v = (float)(s * (double)a.v_scale);
                }
            }
            Vl[r][cc] = v;
        }
        __syncthreads();
#pragma unroll 8
        for (int cc = 0; cc < TC; ++cc) {
            const ACC wv = (ACC)Wl[ol][cc];
#pragma unroll
            for (int s = 0; s < 4; ++s) acc[s] += wv * (ACC)Vl[ig * 4 + s][cc];
        }
        __syncthreads();
    }
    const int o = o0 + ol;
    if (o < a.n_out) {
        const ACC b = a.bias ? (ACC)a.bias[o] : (ACC)0;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int item = i0 + ig * 4 + s;
            if (item >= a.items) continue;
            ACC v = acc[s] + b;
            if (a.relu == 1 && v < (ACC)0) v = (ACC)0;
            else if (a.relu == 2) v = (ACC)1 + (ACC)tanh((double)v);   // delta(s) = 1 + tanh(s), Eq. 23
            const int row = a.out_index ? a.out_index[item] : item;
            a.out[(int64_t)row * a.out_ld + o] = (float)v;
        }
    }
}

// Vector variant: 16-byte global loads, the next PF 64-channel chunks travelling in registers while
// the current one is consumed from LDS, and the LDS tiles held in the accumulation type, so that the
// inner loop has no conversions (a float -> double conversion per operand read made the double-
// accumulating gate layer conversion-bound).  TO outputs x 16 items per workgroup: 64 outputs for
// wide layers, 16 when the launch would otherwise have too few workgroups to cover the chip.
// Needs C and w_ld to be multiples of 8.
constexpr int PF = 4;

template <typename WT, typename ACC, int TOV, bool MULTI>
__global__ __launch_bounds__(256) void fc_tile_vec_kernel(const FcArgs a) {
    constexpr int IPT = TI * TOV / 256;                 // items per thread
    static_assert(IPT >= 1 && TI * TOV % 256 == 0, "tile shape");
    __shared__ ACC Wl[TOV][TC + 1];
    __shared__ ACC Vl[TI][TC];
    __shared__ int cs[TI];
    const int tid = threadIdx.x;
    const int o0 = blockIdx.x * TOV, i0 = blockIdx.y * TI;
    if (tid < TI) {
        const int item = i0 + tid;
        int c = 0;
        if (item < a.items) c = a.c_item ? a.c_item[item] : a.C;
        cs[tid] = c;
    }
    __syncthreads();
    int cmax = 0;
#pragma unroll
    for (int i = 0; i < TI; ++i) cmax = max(cmax, cs[i]);
    const int ol = tid % TOV, ig = tid / TOV;
    constexpr bool WB = sizeof(WT) == 2;
    constexpr int EPL = WB ? 8 : 4;                     // weight elements per 16-byte load
    constexpr int WCH = TOV * TC / EPL;                 // 16-byte weight loads per chunk
    constexpr int NW = (WCH + 255) / 256;
    const int vr = tid >> 4, vc4 = (tid & 15) * 4;      // V: row, first of 4 channels
    const int vitem = i0 + vr, vcs = cs[vr];
    uint4 wregs[PF][NW];
    float vregs[PF][4];
    const WT* w = (const WT*)a.w;
    auto prefetch = [&](uint4 (&wreg)[NW], float (&vreg)[4], int c0) {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int e = tid + 256 * i;
            const int r = e / (TC / EPL), cc = (e % (TC / EPL)) * EPL;
            const int o = o0 + r, c = c0 + cc;
            wreg[i] = make_uint4(0, 0, 0, 0);
            if (e < WCH && o < a.n_out && c < cmax) wreg[i] = *(const uint4*)(w + (int64_t)o * a.w_ld + c);
        }
        const int c = c0 + vc4;
#pragma unroll
        for (int j = 0; j < 4; ++j) vreg[j] = 0.f;
        if (c < vcs) {
            if (a.v_rows) {
                const uint2 q = *(const uint2*)(a.v_rows + (int64_t)vitem * a.v_row_stride + c);
                vreg[0] = __uint_as_float(q.x << 16); vreg[1] = __uint_as_float(q.x & 0xffff0000u);
                vreg[2] = __uint_as_float(q.y << 16); vreg[3] = __uint_as_float(q.y & 0xffff0000u);
            } else {
                // every partial sum is requested before the first is added: a loop of load-then-add is a
                // chain of memory round trips (the slots past a.splits re-read the last one and are dropped)
                double sd[4] = {0, 0, 0, 0};
                if (!MULTI) {   // a.splits == 1
                    for (int sp = 0; sp < a.splits; ++sp) {
                        const float4 t = *(const float4*)(a.v_partial + ((int64_t)vitem * a.splits + sp) * a.C + c);
                        sd[0] += t.x; sd[1] += t.y; sd[2] += t.z; sd[3] += t.w;
                    }
                } else {
                    float4 t[POOL_SPLIT_MAX];
#pragma unroll
                    for (int sp = 0; sp < POOL_SPLIT_MAX; ++sp) {
                        const int q = sp < a.splits ? sp : a.splits - 1;
                        t[sp] = *(const float4*)(a.v_partial + ((int64_t)vitem * a.splits + q) * a.C + c);
                    }
#pragma unroll
                    for (int sp = 0; sp < POOL_SPLIT_MAX; ++sp)
                        if (sp < a.splits) {
                            sd[0] += t[sp].x; sd[1] += t[sp].y; sd[2] += t[sp].z; sd[3] += t[sp].w;
                        }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) vreg[j] = (float)(sd[j] * (double)a.v_scale);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (c + j >= vcs) vreg[j] = 0.f;
        }
    };
    auto store = [&](const uint4 (&wreg)[NW], const float (&vreg)[4]) {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int e = tid + 256 * i;
            if (e >= WCH) continue;
            const int r = e / (TC / EPL), cc = (e % (TC / EPL)) * EPL;
            const uint32_t q[4] = {wreg[i].x, wreg[i].y, wreg[i].z, wreg[i].w};
            if constexpr (WB) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    Wl[r][cc + 2 * j] = (ACC)__uint_as_float(q[j] << 16);
                    Wl[r][cc + 2 * j + 1] = (ACC)__uint_as_float(q[j] & 0xffff0000u);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) Wl[r][cc + j] = (ACC)__uint_as_float(q[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) Vl[vr][vc4 + j] = (ACC)vreg[j];
    };
    ACC acc[IPT];
#pragma unroll
    for (int s = 0; s < IPT; ++s) acc[s] = 0;
#pragma unroll
    for (int st = 0; st < PF; ++st)
        if (st * TC < cmax) prefetch(wregs[st], vregs[st], st * TC);
    for (int cb = 0; cb < cmax; cb += PF * TC) {
#pragma unroll
        for (int st = 0; st < PF; ++st) {
            const int c0 = cb + st * TC;
            if (c0 < cmax) {                       // uniform over the workgroup
                store(wregs[st], vregs[st]);
                __syncthreads();
                if (c0 + PF * TC < cmax) prefetch(wregs[st], vregs[st], c0 + PF * TC);
#pragma unroll 8
                for (int cc = 0; cc < TC; ++cc) {
                    const ACC wv = Wl[ol][cc];
#pragma unroll
                    for (int s = 0; s < IPT; ++s) acc[s] += wv * Vl[ig * IPT + s][cc];
                }
                __syncthreads();
            }
        }
    }
    const int o = o0 + ol;
    if (o < a.n_out) {
        const ACC b = a.bias ? (ACC)a.bias[o] : (ACC)0;
#pragma unroll
        for (int s = 0; s < IPT; ++s) {
            const int item = i0 + ig * IPT + s;
            if (item >= a.items) continue;
            ACC v = acc[s] + b;
            if (a.relu == 1 && v < (ACC)0) v = (ACC)0;
            else if (a.relu == 2) v = (ACC)1 + (ACC)tanh((double)v);   // delta(s) = 1 + tanh(s), Eq. 23
            const int row = a.out_index ? a.out_index[item] : item;
            a.out[(int64_t)row * a.out_ld + o] = (float)v;
        }
    }
}

// Matrix-core variant for the classifier (bf16 weights, fp32 pooled vector or bf16 rows, fp32 accumulation, no
// activation, one partial sum per channel): v_mfma_f32_32x32x2_f32 on a tile of 32 items x 32 outputs.  The
// wavefronts of a workgroup take interleaved 16-channel steps of the reduction and their tiles are added in
// wavefront order, so the result does not depend on timing.  Within a step the lower half of the lanes feeds channels
// k .. k+7 and the upper half k+8 .. k+15 (one matrix instruction per channel pair), so a lane loads 8 consecutive
// channels of its item and of its output's weight row.  Channels at or beyond the item's width enter as zeros.
constexpr int FC_NW = 8;   // wavefronts per workgroup of the classifier kernel
__global__ __launch_bounds__(64 * FC_NW) void fc_mfma_kernel(const FcArgs a) {
    __shared__ float red[FC_NW - 1][32][33];
    __shared__ int cs[32];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lhi = lane >> 5;
    const int o0 = blockIdx.x * 32, i0 = blockIdx.y * 32;
    if (tid < 32) {
        const int item = i0 + tid;
        cs[tid] = item < a.items ? (a.c_item ? a.c_item[item] : a.C) : 0;
    }
    __syncthreads();
    int cmax = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) cmax = max(cmax, cs[i]);
    const int item = i0 + l32, c = cs[l32];
    const int o = o0 + l32;
    const bool ook = o < a.n_out;
    const bf16_t* wrow = (const bf16_t*)a.w + (int64_t)(ook ? o : 0) * a.w_ld;
    const int nsteps = (cmax + 15) / 16;
    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    auto fetch = [&](int step, float (&av)[8], uint4& bw) {
        const int k = step * 16 + 8 * lhi;
#pragma unroll
        for (int q = 0; q < 8; ++q) av[q] = 0.f;
        bw = make_uint4(0, 0, 0, 0);
        if (k < cmax) {                       // cmax <= C, C % 8 == 0: the 8 channels are inside the row
            if (ook) bw = *(const uint4*)(wrow + k);
            if (k < c) {
                if (a.v_rows) {
                    const uint4 t = *(const uint4*)(a.v_rows + (int64_t)item * a.v_row_stride + k);
                    const uint32_t w4[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        av[2 * q] = __uint_as_float(w4[q] << 16);
                        av[2 * q + 1] = __uint_as_float(w4[q] & 0xffff0000u);
                    }
                } else {
                    const float4 t0 = *(const float4*)(a.v_partial + (int64_t)item * a.C + k);
                    const float4 t1 = *(const float4*)(a.v_partial + (int64_t)item * a.C + k + 4);
                    av[0] = t0.x * a.v_scale; av[1] = t0.y * a.v_scale; av[2] = t0.z * a.v_scale; av[3] = t0.w * a.v_scale;
                    av[4] = t1.x * a.v_scale; av[5] = t1.y * a.v_scale; av[6] = t1.z * a.v_scale; av[7] = t1.w * a.v_scale;
                }
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (k + q >= c) av[q] = 0.f;
            }
        }
    };
    // FPF steps of this wavefront in flight: a step's matrix instructions take ~500 cycles, a load a few thousand
    constexpr int FPF = 4;
    float av[FPF][8];
    uint4 bw[FPF];
#pragma unroll
    for (int st = 0; st < FPF; ++st)
        if (wave + FC_NW * st < nsteps) fetch(wave + FC_NW * st, av[st], bw[st]);
    for (int base = wave; base < nsteps; base += FC_NW * FPF) {
#pragma unroll
        for (int st = 0; st < FPF; ++st) {
            const int step = base + FC_NW * st;
            if (step < nsteps) {                 // uniform over the wavefront
                const uint32_t w4[4] = {bw[st].x, bw[st].y, bw[st].z, bw[st].w};
                float cv[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) cv[q] = av[st][q];
                if (step + FC_NW * FPF < nsteps) fetch(step + FC_NW * FPF, av[st], bw[st]);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(cv[2 * q], __uint_as_float(w4[q] << 16), acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(cv[2 * q + 1], __uint_as_float(w4[q] & 0xffff0000u), acc, 0, 0, 0);
                }
            }
        }
    }
    // acc[e] = out[item i0 + 8 (e >> 2) + 4 lhi + (e & 3)][output o0 + l32], this wavefront's share of the channels
    if (wave > 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) red[wave - 1][8 * (e >> 2) + 4 * lhi + (e & 3)][l32] = acc[e];
    }
    __syncthreads();
    if (wave == 0 && ook) {
        const float b = a.bias ? a.bias[o] : 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int r = 8 * (e >> 2) + 4 * lhi + (e & 3);
            const int it = i0 + r;
            if (it >= a.items) continue;
            float v = acc[e];
#pragma unroll
            for (int w = 0; w < FC_NW - 1; ++w) v += red[w][r][l32];
            v += b;
            const int row = a.out_index ? a.out_index[it] : it;
            a.out[(int64_t)row * a.out_ld + o] = v;
        }
    }
}

// Matrix-core variant for the hidden layer of the gate (fp32 weights, fp64 accumulation over the pool's partial
// sums): v_mfma_f64_16x16x4_f64 on a tile of 16 items x 16 outputs per workgroup, the reduction dealt to the four
// wavefronts in interleaved 16-channel steps and their tiles added in wavefront order.  Lane (i, kq) of a wavefront
// feeds item i / output i and the channels k + 4 kq .. k + 4 kq + 3 of a step, one matrix instruction per channel.
typedef double f64x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void fc_mfma64_kernel(const FcArgs a) {
    __shared__ double red[3][16][17];
    __shared__ int cs[16];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, kq = lane >> 4;
    const int o0 = blockIdx.x * 16, i0 = blockIdx.y * 16;
    if (tid < 16) {
        const int item = i0 + tid;
        cs[tid] = item < a.items ? (a.c_item ? a.c_item[item] : a.C) : 0;
    }
    __syncthreads();
    int cmax = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) cmax = max(cmax, cs[i]);
    const int item = i0 + l16, c = cs[l16];
    const int o = o0 + l16;
    const bool ook = o < a.n_out;
    const float* wrow = (const float*)a.w + (int64_t)(ook ? o : 0) * a.w_ld;
    const int nsteps = (cmax + 15) / 16;
    f64x4_t acc = {0.0, 0.0, 0.0, 0.0};
    auto fetch = [&](int step, double (&av)[4], float4& bw) {
        const int k = step * 16 + 4 * kq;
#pragma unroll
        for (int q = 0; q < 4; ++q) av[q] = 0.0;
        bw = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k < cmax) {                       // cmax <= C, C % 4 == 0: the 4 channels are inside the row
            if (ook) bw = *(const float4*)(wrow + k);
            if (k < c) {
                float4 t[POOL_SPLIT_MAX];
#pragma unroll
                for (int sp = 0; sp < POOL_SPLIT_MAX; ++sp) {
                    const int q = sp < a.splits ? sp : a.splits - 1;
                    t[sp] = *(const float4*)(a.v_partial + ((int64_t)item * a.splits + q) * a.C + k);
                }
#pragma unroll
                for (int sp = 0; sp < POOL_SPLIT_MAX; ++sp)
                    if (sp < a.splits) {
                        av[0] += t[sp].x; av[1] += t[sp].y; av[2] += t[sp].z; av[3] += t[sp].w;
                    }
#pragma unroll
                for (int q = 0; q < 4; ++q) av[q] = k + q < c ? (double)(float)(av[q] * (double)a.v_scale) : 0.0;
            }
        }
    };
    constexpr int FPF = 4;
    double av[FPF][4];
    float4 bw[FPF];
#pragma unroll
    for (int st = 0; st < FPF; ++st)
        if (wave + 4 * st < nsteps) fetch(wave + 4 * st, av[st], bw[st]);
    for (int base = wave; base < nsteps; base += 4 * FPF) {
#pragma unroll
        for (int st = 0; st < FPF; ++st) {
            const int step = base + 4 * st;
            if (step < nsteps) {                 // uniform over the wavefront
                const double cv[4] = {av[st][0], av[st][1], av[st][2], av[st][3]};
                const double cw[4] = {(double)bw[st].x, (double)bw[st].y, (double)bw[st].z, (double)bw[st].w};
                if (step + 4 * FPF < nsteps) fetch(step + 4 * FPF, av[st], bw[st]);
#pragma unroll
                for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(cv[q], cw[q], acc, 0, 0, 0);
            }
        }
    }
    // acc[e] = out[item i0 + 4 e + kq][output o0 + l16] (the fp64 tile interleaves its rows over the lane quarters),
    // this wavefront's share of the channels
    if (wave > 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave - 1][4 * e + kq][l16] = acc[e];
    }
    __syncthreads();
    if (wave == 0 && ook) {
        const double b = a.bias ? (double)a.bias[o] : 0.0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int r = 4 * e + kq;
            const int it = i0 + r;
            if (it >= a.items) continue;
            double v = ((acc[e] + red[0][r][l16]) + red[1][r][l16]) + red[2][r][l16] + b;
            if (a.relu == 1 && v < 0.0) v = 0.0;
            else if (a.relu == 2) v = 1.0 + tanh(v);
            const int row = a.out_index ? a.out_index[it] : it;
            a.out[(int64_t)row * a.out_ld + o] = (float)v;
        }
    }
}

}  // namespace

int32_t ds_launch_fc(const FcArgs& a, int32_t w_bf16, int32_t acc_f64, int32_t kind, hipStream_t s) {
    if (a.items <= 0 || a.n_out <= 0) return DS_OK;
    if (!a.v_rows && (a.splits < 1 || a.splits > POOL_SPLIT_MAX))
        DS_FAIL(DS_EINVAL, "fc: %d partial sums per channel (1..%d)", a.splits, POOL_SPLIT_MAX);
    const unsigned gy = (unsigned)((a.items + TI - 1) / TI);
    ProfScope prof(kind, s);
    const bool vec = (a.C % 8) == 0 && (a.w_ld % 8) == 0 && (a.v_rows == nullptr || (a.v_row_stride % 4) == 0);
    if (vec && w_bf16 && !acc_f64 && a.relu == 0 && (a.v_rows ? (a.v_row_stride % 8) == 0 : a.splits == 1) &&
        a.items >= 32) {
        const dim3 grid((unsigned)((a.n_out + 31) / 32), (unsigned)((a.items + 31) / 32));
        hipLaunchKernelGGL(fc_mfma_kernel, grid, dim3(64 * FC_NW), 0, s, a);
        DS_CHECK_LAUNCH("fc (matrix cores)");
        return DS_OK;
    }
    if (vec && !w_bf16 && acc_f64 && !a.v_rows && a.items >= 16) {
        const dim3 grid((unsigned)((a.n_out + 15) / 16), (unsigned)((a.items + 15) / 16));
        hipLaunchKernelGGL(fc_mfma64_kernel, grid, dim3(256), 0, s, a);
        DS_CHECK_LAUNCH("fc (fp64 matrix cores)");
        return DS_OK;
    }
    if (vec) {
        // narrow output tiles when 64-wide ones would leave most compute units without a workgroup
        const bool narrow = (long long)((a.n_out + 63) / 64) * gy < 256;
        const bool multi = !a.v_rows && a.splits > 1;   // several partial sums per channel to combine
        const dim3 grid((unsigned)((a.n_out + (narrow ? 15 : 63)) / (narrow ? 16 : 64)), gy);
#define DS_FC_LAUNCH(WT, ACC)                                                                               \
    do {                                                                                                    \
        if (narrow && multi) hipLaunchKernelGGL((fc_tile_vec_kernel<WT, ACC, 16, true>), grid, dim3(256), 0, s, a);   \
        else if (narrow) hipLaunchKernelGGL((fc_tile_vec_kernel<WT, ACC, 16, false>), grid, dim3(256), 0, s, a);      \
        else if (multi) hipLaunchKernelGGL((fc_tile_vec_kernel<WT, ACC, 64, true>), grid, dim3(256), 0, s, a);        \
        else hipLaunchKernelGGL((fc_tile_vec_kernel<WT, ACC, 64, false>), grid, dim3(256), 0, s, a);                  \
    } while (0)
        if (w_bf16) DS_FC_LAUNCH(bf16_t, float);
        else if (acc_f64) DS_FC_LAUNCH(float, double);
        else DS_FC_LAUNCH(float, float);
#undef DS_FC_LAUNCH
    } else {
        const dim3 grid((unsigned)((a.n_out + TO - 1) / TO), gy);
        if (w_bf16) hipLaunchKernelGGL((fc_tile_kernel<bf16_t, float>), grid, dim3(256), 0, s, a);
        else if (acc_f64) hipLaunchKernelGGL((fc_tile_kernel<float, double>), grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL((fc_tile_kernel<float, float>), grid, dim3(256), 0, s, a);
    }
    DS_CHECK_LAUNCH("fc tile");
    return DS_OK;
}
