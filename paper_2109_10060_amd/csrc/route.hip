// Routing agent and batch bucketing.
//
// Gate (Section 3.5): the encoder averages each valid channel over H*W (Eq. 21);
// the routing head is a two-layer MLP whose first layer is input-sliced to the
// valid channels, followed at inference by an argmax over the route scores
// (Eq. 22).  Bucketing turns the per-sample route ids into a stable bucket-major
// permutation so that every route group is a contiguous range of slots.
#include "common.h"

namespace {


// ---- encoder: partial spatial sums -------------------------------------------
// NHWC: grid (items, splits); block 256 = 32 channel chunks of 8 x 8 row lanes.
template <typename T>
__device__ __forceinline__ void load8(const T* p, float* v);
template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t* p, float* v) {
    const uint4 q = *(const uint4*)p;
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
template <>
__device__ __forceinline__ void load8<float>(const float* p, float* v) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// NHWC: grid (items, splits), block 256.  The block is shaped to the channel count: CL = 2^lcl lanes
// (8 channels each) across the channels, 256 / CL rows of the map in flight per step, so narrow maps
// (24 or 64 channels) keep every lane loading.
template <typename T>
__global__ __launch_bounds__(256) void pool_nhwc_kernel(const GateArgs a, int splits, int lcl) {
    __shared__ float red[256 * 16];   // (256 >> lcl) rows of (8 << lcl) + 8 floats
    const int item = blockIdx.x, sp = blockIdx.y;
    const int c = a.c_in ? a.c_in[item] : a.C;
    const int sample = a.x_index ? a.x_index[item] : item;
    const int ld = a.x_ld > 0 ? a.x_ld : c;
    const T* x = (const T*)a.x + (int64_t)sample * a.x_sample_stride;
    const int CL = 1 << lcl, R = 256 >> lcl, red_ld = CL * 8 + 8;
    const int lane_c = threadIdx.x & (CL - 1), lane_r = threadIdx.x >> lcl;
    const int per = (a.HW + splits - 1) / splits;
    const int r0 = sp * per, r1 = min(a.HW, r0 + per);
    for (int c0 = 0; c0 < c; c0 += CL * 8) {
        const int ch = c0 + lane_c * 8;
        float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (ch < c) {
            // four rows in flight per lane: the loads are independent, only the adds chain
            int r = r0 + lane_r;
            for (; r + 3 * R < r1; r += 4 * R) {
                float v[4][8];
#pragma unroll
                for (int k = 0; k < 4; ++k) load8<T>(x + (int64_t)(r + R * k) * ld + ch, v[k]);
#pragma unroll
                for (int k = 0; k < 4; ++k)
#pragma unroll
                    for (int i = 0; i < 8; ++i) s[i] += v[k][i];
            }
            for (; r < r1; r += R) {
                float v[8];
                load8<T>(x + (int64_t)r * ld + ch, v);
#pragma unroll
                for (int i = 0; i < 8; ++i) s[i] += v[i];
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) red[lane_r * red_ld + lane_c * 8 + i] = s[i];
        __syncthreads();
        const int cc = c0 + threadIdx.x;
        if (threadIdx.x < CL * 8 && cc < c) {
            float t = 0.f;
            for (int r = 0; r < R; ++r) t += red[r * red_ld + threadIdx.x];
            a.partial[((int64_t)item * splits + sp) * a.C + cc] = t;
        }
        __syncthreads();
    }
}

// NCHW: one wavefront per (item, channel); grid (items, ceil(C/4)), block 256; splits == 1.
template <typename T>
__global__ __launch_bounds__(256) void pool_nchw_kernel(const GateArgs a) {
    const int item = blockIdx.x;
    const int ch = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int c = a.c_in ? a.c_in[item] : a.C;
    if (ch >= c) return;
    const int sample = a.x_index ? a.x_index[item] : item;
    const T* x = (const T*)a.x + (int64_t)sample * a.x_sample_stride + (int64_t)ch * a.HW;
    float s = 0.f;
    for (int i = lane; i < a.HW; i += 64) {
        if constexpr (sizeof(T) == 2) s += bf2f(x[i]);
        else s += x[i];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) a.partial[(int64_t)item * a.C + ch] = s;
}

// ---- routing head, output layer + argmax: one wavefront per item ---------------------------
// hidden [items][C_mlp] comes from the tiled first layer (fp64 accumulation, ReLU applied).
// The wavefront is split into groups of G = 64 >> lg lanes, one group per output, so that all T
// outputs (up to 64 per pass) are computed side by side: a group strides over the hidden units and
// adds its partial sums with a butterfly.  The argmax (NaN never wins, ties go to the lowest index)
// is a butterfly over (value, index) pairs.
__global__ __launch_bounds__(64) void gate_out_kernel(const GateArgs a, const float* hidden, int lg) {
    const int item = blockIdx.x;
    const int out = a.out_index ? a.out_index[item] : item;
    const int lane = threadIdx.x;
    const bool have_x = a.x != nullptr;
    const int G = 64 >> lg, per_pass = 1 << lg;
    const int sub = lane & (G - 1), tl = lane >> (6 - lg);
    float best = 0.f;
    int arg = 0;
    bool have = false;
    for (int t0 = 0; t0 < a.T; t0 += per_pass) {
        const int t = t0 + tl;
        double s = 0.0;
        if (have_x) {
            if (t < a.T) {
                const float* wr = a.w2 + (int64_t)t * a.C_mlp;
                const float* h = hidden + (int64_t)item * a.C_mlp;
                for (int j = sub; j < a.C_mlp; j += G) s += (double)wr[j] * (double)h[j];
            }
            for (int o = G >> 1; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
            if (t < a.T && a.b2) s += (double)a.b2[t];
        }
        if (t < a.T && sub == 0) {
            if (a.logit_bias) s += (double)a.logit_bias[(int64_t)out * a.T + t];
            const float v = (float)s;
            a.logits[(int64_t)out * a.T + t] = v;
            if (v == v && (!have || v > best)) { best = v; arg = t; have = true; }   // t ascends within a lane
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ob = __shfl_xor(best, o, 64);
        const int oa = __shfl_xor(arg, o, 64);
        const bool oh = __shfl_xor((int)have, o, 64) != 0;
        if (oh && (!have || ob > best || (ob == best && oa < arg))) { best = ob; arg = oa; have = true; }
    }
    if (lane == 0) a.route[out] = a.route_override ? a.route_override[out] : arg;
}

// ---- bucketing ----------------------------------------------------------------
// One workgroup.  key[b] = route[b] * mul + (lo ? lo[b] : 0).  Histogram and exclusive scan give the
// group offsets; then, 1024 samples at a time, every thread ranks its own sample among the earlier
// samples of the chunk with the same key (stable), so the scatter is parallel over samples.
__global__ __launch_bounds__(1024) void bucket_kernel(const BucketArgs a) {
    __shared__ int base[1024 + 1];
    __shared__ int chunk[1024];
    const int tid = threadIdx.x;
    const int B = a.B, T = a.T;
    auto key_of = [&](int b) {
        const int k = a.route[b] * a.mul + (a.lo ? a.lo[b] : 0);
        return (k >= 0 && k < T) ? k : -1;
    };
    for (int t = tid; t <= T; t += 1024) base[t] = 0;
    __syncthreads();
    for (int b = tid; b < B; b += 1024) {
        const int k = key_of(b);
        if (k >= 0) atomicAdd(&base[k], 1);
    }
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        for (int t = 0; t < T; ++t) {
            const int h = base[t];
            base[t] = acc;
            acc += h;
        }
        base[T] = acc;
    }
    __syncthreads();
    for (int t = tid; t <= T; t += 1024) a.offsets[t] = base[t];
    if (a.n_lists > 0) {
        // m-tile lists of the grouped GEMM for these offsets: groups from the last to the first (widest slices
        // first), DS_GEMM_BM rows per tile; entry = (group, first row inside the group, first slot, rows of the group)
        __shared__ int pre[2][DS_MAX_GROUPS + 1];
        if (tid < a.n_lists) {
            int acc = 0;
            for (int q = 0; q < T; ++q) {
                const int g = T - 1 - q;
                pre[tid][q] = acc;
                acc += ((base[g + 1] - base[g]) * a.list_rows[tid] + DS_GEMM_BM - 1) / DS_GEMM_BM;
            }
            pre[tid][T] = acc;
            *(int32_t*)a.lists[tid] = acc;
        }
        __syncthreads();
        for (int li = 0; li < a.n_lists; ++li) {
            int4* entries = (int4*)((char*)a.lists[li] + 16);
            for (int q = 0; q < T; ++q) {
                const int g = T - 1 - q;
                const int n = pre[li][q + 1] - pre[li][q];
                const int slot0 = base[g], rg = (base[g + 1] - slot0) * a.list_rows[li];
                for (int i = tid; i < n; i += 1024) entries[pre[li][q] + i] = make_int4(g, i * DS_GEMM_BM, slot0, rg);
            }
        }
    }
    for (int b0 = 0; b0 < B; b0 += 1024) {
        __syncthreads();
        const int b = b0 + tid;
        const int k = b < B ? key_of(b) : -1;
        chunk[tid] = k;
        __syncthreads();
        if (k >= 0) {
            int rank = 0;
            for (int i = 0; i < tid; ++i) rank += chunk[i] == k;
            const int pos = base[k] + rank;
            a.perm[pos] = b;
            if (a.inv_perm) a.inv_perm[b] = pos;
            if (a.slot_group) a.slot_group[pos] = k;
            if (a.src_index) a.src_index[pos] = a.inv_prev ? a.inv_prev[b] : b;
            if (a.slot_lut) a.slot_lut[pos] = a.lut[k];
        }
        __syncthreads();
        if (k >= 0) atomicAdd(&base[k], 1);
    }
}

__global__ void bn_fold_kernel(const float* gamma, const float* beta, const float* mean, const float* var,
                               float eps, int T, int C, float* scale, float* shift) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T * C) return;
    const int c = i % C;
    const float s = gamma[c] / sqrtf(var[i] + eps);
    scale[i] = s;
    shift[i] = beta[c] - mean[i] * s;
}

// ---- Re-SBN re-calibration (the paragraph above Eq. 14): streaming per-route channel statistics -------
// Pass 1, grid (slots, splits): sum and sum of squares of every valid channel over the slot's share of the
// pixels, in fp64, lanes laid out as in pool_nhwc_kernel.  Deterministic: fixed row order per lane, fixed
// order in the LDS reduction.
__global__ __launch_bounds__(256) void bn_partial_kernel(const bf16_t* x, const int32_t* index, int64_t sample_stride,
                                                         int ld, const int32_t* slot_group, const GroupTable gt, int HW,
                                                         int C, int splits, int lcl, double* psum, double* psq) {
    __shared__ double red[256 * 9];
    const int slot = blockIdx.x, sp = blockIdx.y;
    const int c = gt.k_in[slot_group[slot]];
    const int sample = index ? index[slot] : slot;
    const bf16_t* xp = x + (int64_t)sample * sample_stride;
    const int CL = 1 << lcl, R = 256 >> lcl, red_ld = CL * 8 + 1;
    const int lane_c = threadIdx.x & (CL - 1), lane_r = threadIdx.x >> lcl;
    const int per = (HW + splits - 1) / splits;
    const int r0 = sp * per, r1 = min(HW, r0 + per);
    for (int c0 = 0; c0 < c; c0 += CL * 8) {
        const int ch = c0 + lane_c * 8;
        double s[8] = {0, 0, 0, 0, 0, 0, 0, 0}, q[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (ch < c) {
            // four rows in flight per lane; their sums are taken in fp32 (a bf16 square is exact there, the
            // additions round at 2^-24) and go into the fp64 totals once per four rows
            int r = r0 + lane_r;
            for (; r + 3 * R < r1; r += 4 * R) {
                float v[4][8];
#pragma unroll
                for (int k = 0; k < 4; ++k) load8<bf16_t>(xp + (int64_t)(r + R * k) * ld + ch, v[k]);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float s4 = (v[0][i] + v[1][i]) + (v[2][i] + v[3][i]);
                    const float q4 = fmaf(v[0][i], v[0][i], v[1][i] * v[1][i]) + fmaf(v[2][i], v[2][i], v[3][i] * v[3][i]);
                    s[i] += (double)s4;
                    q[i] += (double)q4;
                }
            }
            for (; r < r1; r += R) {
                float v[8];
                load8<bf16_t>(xp + (int64_t)r * ld + ch, v);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    s[i] += (double)v[i];
                    q[i] += (double)(v[i] * v[i]);
                }
            }
        }
        const int cc = c0 + threadIdx.x;
        const int64_t o = ((int64_t)slot * splits + sp) * C + cc;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
            for (int i = 0; i < 8; ++i) red[lane_r * red_ld + lane_c * 8 + i] = pass ? q[i] : s[i];
            __syncthreads();
            if (threadIdx.x < CL * 8 && cc < c) {
                double t = 0.0;
                for (int r = 0; r < R; ++r) t += red[r * red_ld + threadIdx.x];
                (pass ? psq : psum)[o] = t;
            }
            __syncthreads();
        }
    }
}

// Pass 2, grid (T, ceil(C / 16)), block 256 = 16 channels x 16 slot lanes: a slot lane adds the partial sums of
// every 16th slot of the route (in slot, then split order), the 16 lane totals are added in lane order, and the
// result goes onto the running totals.  Fixed order throughout, so the totals are reproducible.
__global__ __launch_bounds__(256) void bn_combine_kernel(const int32_t* offsets, const GroupTable gt, int HW, int C,
                                                         int splits, const double* psum, const double* psq,
                                                         double* sum, double* sumsq, long long* count) {
    __shared__ double rs[16][17], rq[16][17];
    const int t = blockIdx.x, cl = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const int c = blockIdx.y * 16 + cl;
    const int j0 = offsets[t], j1 = offsets[t + 1];
    if (blockIdx.y == 0 && threadIdx.x == 0) count[t] += (long long)(j1 - j0) * HW;
    double s = 0.0, q = 0.0;
    if (c < gt.k_in[t])
        for (int j = j0 + sl; j < j1; j += 16)
            for (int sp = 0; sp < splits; ++sp) {
                const int64_t o = ((int64_t)j * splits + sp) * C + c;
                s += psum[o];
                q += psq[o];
            }
    rs[sl][cl] = s;
    rq[sl][cl] = q;
    __syncthreads();
    if (sl == 0 && c < gt.k_in[t]) {
        double ts = 0.0, tq = 0.0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            ts += rs[k][cl];
            tq += rq[k][cl];
        }
        sum[(int64_t)t * C + c] += ts;
        sumsq[(int64_t)t * C + c] += tq;
    }
}

// mean = S / N, variance = Q / N - mean^2 (biased); a route without samples keeps mean 0, variance 1
__global__ void bn_finish_kernel(const double* sum, const double* sumsq, const long long* count, const GroupTable gt,
                                 int T, int C, float* mean, float* var) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T * C) return;
    const long long n = count[i / C];
    if (n <= 0 || i % C >= gt.k_in[i / C]) { mean[i] = 0.f; var[i] = 1.f; return; }
    const double m = sum[i] / (double)n;
    const double v = sumsq[i] / (double)n - m * m;
    mean[i] = (float)m;
    var[i] = (float)(v > 0.0 ? v : 0.0);
}

}  // namespace

size_t ds_gate_partial_bytes(int32_t B, int32_t C) { return (size_t)B * C * (POOL_SPLIT_MAX + 1) * sizeof(float); }

int32_t ds_launch_pool(const GateArgs& a, int32_t kind, int32_t* splits_out, hipStream_t s) {
    int splits = 1;
    ProfScope prof(kind, s);
    if (a.layout == DS_NHWC) {
        splits = a.HW >= 2048 ? 8 : (a.HW >= 512 ? 4 : (a.HW >= 128 ? 2 : 1));
        dim3 grid(a.B, splits);
        int lcl = 0;
        while ((8 << lcl) < a.C && lcl < 5) ++lcl;   // lanes across the channels: 2^lcl * 8 >= C, at most 32
        if (a.dtype == DS_BF16) hipLaunchKernelGGL(pool_nhwc_kernel<bf16_t>, grid, dim3(256), 0, s, a, splits, lcl);
        else hipLaunchKernelGGL(pool_nhwc_kernel<float>, grid, dim3(256), 0, s, a, splits, lcl);
    } else {
        dim3 grid(a.B, (a.C + 3) / 4);
        if (a.dtype == DS_BF16) hipLaunchKernelGGL(pool_nchw_kernel<bf16_t>, grid, dim3(256), 0, s, a);
        else hipLaunchKernelGGL(pool_nchw_kernel<float>, grid, dim3(256), 0, s, a);
    }
    DS_CHECK_LAUNCH("spatial pool");
    *splits_out = splits;
    return DS_OK;
}

int32_t ds_launch_gate(const GateArgs& a, hipStream_t s) {
    if (a.B <= 0) return DS_OK;
    float* hidden = nullptr;
    if (a.x) {
        int splits = 1;
        int32_t rc = ds_launch_pool(a, DS_K_GATE, &splits, s);
        if (rc) return rc;
        hidden = a.partial + (size_t)a.B * a.C * POOL_SPLIT_MAX;   // [B][C_mlp], C_mlp <= C
        FcArgs f = {};
        f.v_partial = a.partial; f.splits = splits; f.v_scale = 1.0f / (float)a.HW;
        f.c_item = a.c_in; f.C = a.C;
        f.w = a.w1; f.w_ld = a.C; f.bias = a.b1; f.n_out = a.C_mlp; f.relu = 1;
        f.out = hidden; f.out_ld = a.C_mlp; f.items = a.B;
        rc = ds_launch_fc(f, 0, 1, DS_K_GATE, s);
        if (rc) return rc;
    }
    ProfScope prof(DS_K_GATE, s);
    int lg = 0;
    while ((1 << lg) < a.T && lg < 6) ++lg;   // 2^lg outputs side by side, 64 >> lg lanes each
    hipLaunchKernelGGL(gate_out_kernel, dim3(a.B), dim3(64), 0, s, a, hidden, lg);
    DS_CHECK_LAUNCH("gate head");
    return DS_OK;
}

int32_t ds_launch_bucket_ex(const BucketArgs& a, hipStream_t s) {
    if ((a.n_lists > 0 || a.slot_lut) && a.T > DS_MAX_GROUPS) DS_FAIL(DS_EINVAL, "route bucket: fused lists need T <= %d", DS_MAX_GROUPS);
    if (a.n_lists < 0 || a.n_lists > 2) DS_FAIL(DS_EINVAL, "route bucket: at most two m-tile lists");
    ProfScope prof(DS_K_BUCKET, s);
    hipLaunchKernelGGL(bucket_kernel, dim3(1), dim3(1024), 0, s, a);
    DS_CHECK_LAUNCH("route bucket");
    return DS_OK;
}

int32_t ds_launch_bucket(const int32_t* route, int32_t B, int32_t T, int32_t* perm, int32_t* inv_perm,
                         int32_t* offsets, int32_t* slot_group, hipStream_t s) {
    BucketArgs a = {};
    a.route = route; a.mul = 1; a.B = B; a.T = T;
    a.perm = perm; a.inv_perm = inv_perm; a.offsets = offsets; a.slot_group = slot_group;
    return ds_launch_bucket_ex(a, s);
}

extern "C" int32_t ds_bn_fold(const float* gamma, const float* beta, const float* mean, const float* var,
                              float eps, int32_t T, int32_t C, float* scale, float* shift, void* stream) {
    if (T < 0 || C < 0) DS_FAIL(DS_EINVAL, "ds_bn_fold: negative size");
    if (T == 0 || C == 0) return DS_OK;
    if (!gamma || !beta || !mean || !var || !scale || !shift) DS_FAIL(DS_EINVAL, "ds_bn_fold: null pointer");
    const int n = T * C;
    hipLaunchKernelGGL(bn_fold_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, gamma, beta, mean,
                       var, eps, T, C, scale, shift);
    DS_CHECK_LAUNCH("bn fold");
    return DS_OK;
}

namespace {
int bn_stats_splits(int HW) { return HW >= 2048 ? 8 : (HW >= 512 ? 4 : (HW >= 128 ? 2 : 1)); }
}  // namespace

extern "C" size_t ds_bn_stats_workspace(int32_t B, int32_t HW, int32_t C) {
    if (B <= 0 || HW <= 0 || C <= 0) return 0;
    return ds_align_up((size_t)B * 4 + 4, 256) + 2 * ds_align_up((size_t)B * bn_stats_splits(HW) * C * sizeof(double), 256);
}

extern "C" int32_t ds_bn_stats_accumulate(const void* x, int32_t B, int32_t HW, int32_t C, const ds_groups* g, double* sum,
                                          double* sumsq, int64_t* count, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "ds_bn_stats_accumulate";
    if (B < 0 || HW < 1 || C < 1) DS_FAIL(DS_EINVAL, "%s: bad size", who);
    if (!g || g->T < 1 || g->T > DS_MAX_GROUPS || !g->offsets) DS_FAIL(DS_EINVAL, "%s: bad groups", who);
    GroupTable gt = {};
    gt.T = g->T;
    for (int t = 0; t < g->T; ++t) {
        if (g->k_in[t] < 0 || g->k_in[t] > C || (g->k_in[t] % 8)) DS_FAIL(DS_EINVAL, "%s: group %d width %d (multiple of 8, at most %d)", who, t, g->k_in[t], C);
        gt.k_in[t] = gt.k_out[t] = g->k_in[t];
    }
    if (B == 0) return DS_OK;
    if (!x || !sum || !sumsq || !count) DS_FAIL(DS_EINVAL, "%s: null pointer", who);
    if ((C % 8) || !ds_aligned16(x)) DS_FAIL(DS_EALIGN, "%s: needs C %% 8 == 0 and a 16-byte aligned x", who);
    if (!ws || ws_bytes < ds_bn_stats_workspace(B, HW, C)) DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes", who, ds_bn_stats_workspace(B, HW, C));
    hipStream_t s = (hipStream_t)stream;
    const int splits = bn_stats_splits(HW);
    int32_t* slot_group = (int32_t*)ws;
    double* psum = (double*)((char*)ws + ds_align_up((size_t)B * 4 + 4, 256));
    double* psq = (double*)((char*)psum + ds_align_up((size_t)B * splits * C * sizeof(double), 256));
    int32_t rc = ds_launch_expand_groups(g->offsets, g->T, slot_group, s);
    if (rc) return rc;
    int lcl = 0;
    while ((8 << lcl) < C && lcl < 5) ++lcl;
    hipLaunchKernelGGL(bn_partial_kernel, dim3(B, splits), dim3(256), 0, s, (const bf16_t*)x, g->perm, (int64_t)HW * C, C,
                       slot_group, gt, HW, C, splits, lcl, psum, psq);
    DS_CHECK_LAUNCH("bn partial statistics");
    hipLaunchKernelGGL(bn_combine_kernel, dim3(g->T, (C + 15) / 16), dim3(256), 0, s, g->offsets, gt, HW, C, splits, psum, psq,
                       sum, sumsq, (long long*)count);
    DS_CHECK_LAUNCH("bn combine statistics");
    return DS_OK;
}

extern "C" int32_t ds_bn_stats_finish(const double* sum, const double* sumsq, const int64_t* count, int32_t T, int32_t C,
                                      const int32_t* width, float* mean, float* var, void* stream) {
    if (T < 0 || C < 0 || T > DS_MAX_GROUPS) DS_FAIL(DS_EINVAL, "ds_bn_stats_finish: T outside 0..%d or C < 0", DS_MAX_GROUPS);
    if (T == 0 || C == 0) return DS_OK;
    if (!sum || !sumsq || !count || !mean || !var) DS_FAIL(DS_EINVAL, "ds_bn_stats_finish: null pointer");
    GroupTable gt = {};
    gt.T = T;
    for (int t = 0; t < T; ++t) {
        gt.k_in[t] = width ? width[t] : C;
        if (gt.k_in[t] < 0 || gt.k_in[t] > C) DS_FAIL(DS_EINVAL, "ds_bn_stats_finish: width[%d] = %d outside 0..%d", t, gt.k_in[t], C);
    }
    const int n = T * C;
    hipLaunchKernelGGL(bn_finish_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, sum, sumsq,
                       (const long long*)count, gt, T, C, mean, var);
    DS_CHECK_LAUNCH("bn finish statistics");
    return DS_OK;
}

extern "C" int32_t ds_gate(const void* x, int32_t x_dtype, int32_t x_layout, int32_t B, int32_t C, int32_t HW,
                           const int32_t* c_in, const float* w1, const float* b1, int32_t C_mlp, const float* w2,
                           const float* b2, int32_t T, const float* logit_bias, float* logits_out,
                           int32_t* route_out, void* ws, size_t ws_bytes, void* stream) {
    if (B < 0 || T < 1) DS_FAIL(DS_EINVAL, "ds_gate: B < 0 or T < 1");
    if (B == 0) return DS_OK;
    if (!logits_out || !route_out) DS_FAIL(DS_EINVAL, "ds_gate: null output");
    GateArgs a = {};
    if (x) {
        if (C < 1 || HW < 1 || C_mlp < 1) DS_FAIL(DS_EINVAL, "ds_gate: bad C/HW/C_mlp");
        if (!w1 || !w2) DS_FAIL(DS_EINVAL, "ds_gate: null weights");
        if (x_dtype != DS_F32 && x_dtype != DS_BF16) DS_FAIL(DS_EUNSUPPORTED, "ds_gate: dtype");
        if (x_layout != DS_NCHW && x_layout != DS_NHWC) DS_FAIL(DS_EUNSUPPORTED, "ds_gate: layout");
        if (x_layout == DS_NHWC && ((C % 8) != 0 || !ds_aligned16(x))) DS_FAIL(DS_EALIGN, "ds_gate: NHWC needs C %% 8 == 0 and a 16-byte aligned x");
        if (C_mlp > C) DS_FAIL(DS_EUNSUPPORTED, "ds_gate: hidden width above the channel count");
        if (!ws || ws_bytes < ds_gate_partial_bytes(B, C)) DS_FAIL(DS_EWORKSPACE, "ds_gate: workspace needs %zu bytes", ds_gate_partial_bytes(B, C));
    } else if (!logit_bias) {
        DS_FAIL(DS_EINVAL, "ds_gate: neither x nor logit_bias given");
    } else {
        C = 0; C_mlp = 0;
    }
    a.x = x; a.dtype = x_dtype; a.layout = x_layout; a.B = B; a.C = C; a.HW = HW;
    a.c_in = c_in; a.x_index = nullptr; a.x_sample_stride = (int64_t)C * HW; a.x_ld = C;
    a.w1 = w1; a.b1 = b1; a.w2 = w2; a.b2 = b2; a.C_mlp = C_mlp; a.T = T;
    a.logit_bias = logit_bias; a.out_index = nullptr; a.route_override = nullptr;
    a.logits = logits_out; a.route = route_out; a.partial = (float*)ws;
    return ds_launch_gate(a, (hipStream_t)stream);
}

// workspace: encoder partial sums + hidden vectors (as ds_gate) followed by the channel factors [B][C]
extern "C" size_t ds_gate_double_workspace(int32_t B, int32_t C) {
    if (B <= 0 || C <= 0) return 0;
    return ds_align_up(ds_gate_partial_bytes(B, C), 256) + (size_t)B * C * sizeof(float);
}

extern "C" int32_t ds_gate_double(const void* x, int32_t x_dtype, int32_t x_layout, int32_t B, int32_t C, int32_t HW,
                                  const int32_t* c_in, const float* w1, const float* b1, int32_t C_mlp,
                                  const float* w2, const float* b2, int32_t T, const float* logit_bias,
                                  const float* w3, const float* b3, float* logits_out, int32_t* route_out, void* y,
                                  void* ws, size_t ws_bytes, void* stream) {
    if (B < 0) DS_FAIL(DS_EINVAL, "ds_gate_double: B < 0");
    if (B == 0) return DS_OK;
    if (!x || !y || !w1 || !w3) DS_FAIL(DS_EINVAL, "ds_gate_double: null pointer");
    if (C < 1 || HW < 1 || C_mlp < 1 || C_mlp > C) DS_FAIL(DS_EINVAL, "ds_gate_double: bad C/HW/C_mlp");
    if (x_dtype != DS_F32 && x_dtype != DS_BF16) DS_FAIL(DS_EUNSUPPORTED, "ds_gate_double: dtype");
    if (x_layout != DS_NCHW && x_layout != DS_NHWC) DS_FAIL(DS_EUNSUPPORTED, "ds_gate_double: layout");
    if (x_layout == DS_NHWC && ((C % 8) != 0 || !ds_aligned16(x) || !ds_aligned16(y)))
        DS_FAIL(DS_EALIGN, "ds_gate_double: NHWC needs C %% 8 == 0 and 16-byte aligned x, y");
    const bool routing = w2 != nullptr;
    if (routing && (T < 1 || !logits_out || !route_out)) DS_FAIL(DS_EINVAL, "ds_gate_double: routing head needs T >= 1 and outputs");
    if (!ws || ws_bytes < ds_gate_double_workspace(B, C))
        DS_FAIL(DS_EWORKSPACE, "ds_gate_double: workspace needs %zu bytes", ds_gate_double_workspace(B, C));
    hipStream_t s = (hipStream_t)stream;
    GateArgs a = {};
    a.x = x; a.dtype = x_dtype; a.layout = x_layout; a.B = B; a.C = C; a.HW = HW;
    a.c_in = c_in; a.x_sample_stride = (int64_t)C * HW; a.x_ld = C;
    a.w1 = w1; a.b1 = b1; a.w2 = w2; a.b2 = b2; a.C_mlp = C_mlp; a.T = T;
    a.logit_bias = logit_bias; a.logits = logits_out; a.route = route_out; a.partial = (float*)ws;
    // encoder and hidden vector once, shared by both heads
    int splits = 1;
    int32_t rc = ds_launch_pool(a, DS_K_GATE, &splits, s);
    if (rc) return rc;
    float* hidden = a.partial + (size_t)B * C * POOL_SPLIT_MAX;
    FcArgs f = {};
    f.v_partial = a.partial; f.splits = splits; f.v_scale = 1.0f / (float)HW;
    f.c_item = c_in; f.C = C; f.w = w1; f.w_ld = C; f.bias = b1; f.n_out = C_mlp; f.relu = 1;
    f.out = hidden; f.out_ld = C_mlp; f.items = B;
    rc = ds_launch_fc(f, 0, 1, DS_K_GATE, s);
    if (rc) return rc;
    if (routing) {
        ProfScope prof(DS_K_GATE, s);
        int lg = 0;
        while ((1 << lg) < T && lg < 6) ++lg;
        hipLaunchKernelGGL(gate_out_kernel, dim3(B), dim3(64), 0, s, a, (const float*)hidden, lg);
        DS_CHECK_LAUNCH("gate head");
    }
    // attention head: factor[b][c] = 1 + tanh(W3[c, :] . hidden[b] + b3[c]); rows beyond the
    // sample's width are computed too and never used
    float* factor = (float*)((char*)ws + ds_align_up(ds_gate_partial_bytes(B, C), 256));
    FcArgs h = {};
    h.v_partial = hidden; h.splits = 1; h.v_scale = 1.0f; h.c_item = nullptr; h.C = C_mlp;
    h.w = w3; h.w_ld = C_mlp; h.bias = b3; h.n_out = C; h.relu = 2;
    h.out = factor; h.out_ld = C; h.items = B;
    rc = ds_launch_fc(h, 0, 1, DS_K_GATE, s);
    if (rc) return rc;
    return ds_launch_channel_scale(x, y, factor, c_in, x_dtype, x_layout, B, C, HW, s);
}

extern "C" int32_t ds_route_bucket(const int32_t* route, int32_t B, int32_t T, int32_t* perm, int32_t* inv_perm,
                                   int32_t* offsets, void* stream) {
    if (B < 0 || T < 1 || T > 1024) DS_FAIL(DS_EINVAL, "ds_route_bucket: need B >= 0 and 1 <= T <= 1024");
    if (!offsets) DS_FAIL(DS_EINVAL, "ds_route_bucket: null offsets");
    if (B > 0 && (!route || !perm || !inv_perm)) DS_FAIL(DS_EINVAL, "ds_route_bucket: null pointer");
    return ds_launch_bucket(route, B, T, perm, inv_perm, offsets, nullptr, (hipStream_t)stream);
}
