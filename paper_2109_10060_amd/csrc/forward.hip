// Whole-network forward passes of the three dynamic nets (Section 5.2):
// DS-MBNet (one gate after the 5th depthwise-separable block), DS-ResNet (a gate in
// the first block of each of the four stages, projection shortcut sliced with it)
// and DS-ViT (one route per image chosen before the patch embedding).
//
// Host code only enqueues kernels.  Route decisions never leave the device: the
// gate writes route ids, the bucket kernel turns them into slot order, group
// offsets and per-slot group ids, and every later launch is sized for the worst
// case and reads those tables.
//
// Activation layout after a gate: slot-major.  Slot j (bucket order) owns a block
// of fixed size rows * C_stored elements; inside it the rows are packed with the
// slot's own width as leading stride, so a bucket's rows are dense and only valid
// bytes are touched.  The first sliced layer gathers whole samples through the
// permutation; the classifier scatters logits back to the original order.
#include <string.h>
#include <mutex>

#include "common.h"

namespace {

struct Bump {
    char* base;
    size_t off;
    template <typename T>
    T* take(size_t n) {
        off = ds_align_up(off, 256);
        T* p = base ? (T*)(base + off) : nullptr;
        off += n * sizeof(T);
        return p;
    }
};

GroupTable table1(int k_in, int k_out) {
    GroupTable g;
    memset(&g, 0, sizeof(g));
    g.T = 1;
    g.k_in[0] = k_in;
    g.k_out[0] = k_out;
    g.row[0] = 0;
    return g;
}

int max_out(const GroupTable& g) {
    int m = 0;
    for (int t = 0; t < g.T; ++t) m = g.k_out[t] > m ? g.k_out[t] : m;
    return m;
}

struct MList {  // m-tile list of one (bucketing, rows-per-sample) pair
    void* list;
    int cap;
    int rows;
};

#define RC(x)                  \
    do {                       \
        int32_t rc__ = (x);    \
        if (rc__) return rc__; \
    } while (0)

// ---- intermediate activations for inspection (ds_forward_taps) ---------------------------------
// A tap copies one block's output from the slot-major packed layout to [sample][row][C_full] in the original sample
// order; only the valid slice of each sample is written.
struct Taps {
    int n;
    const int32_t* ids;      // host: block indices in execution order
    void* const* out;        // host array of device buffers
};

__global__ void unpack_slots_kernel(const bf16_t* x, int64_t x_sstride, int x_ld, const int32_t* perm, const int32_t* slot_group,
                                    const GroupTable gt, int rows, int c_full, bf16_t* out) {
    const int slot = blockIdx.y;
    const int w = gt.k_out[slot_group ? slot_group[slot] : 0];
    if (w <= 0) return;
    const int ld = x_ld > 0 ? x_ld : w, w8 = w >> 3;
    const int64_t n = (int64_t)rows * w8;
    const bf16_t* src = x + (int64_t)slot * x_sstride;
    bf16_t* dst = out + (int64_t)(perm ? perm[slot] : slot) * rows * c_full;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / w8;
        const int c = (int)(i - r * w8) * 8;
        *(uint4*)(dst + r * c_full + c) = *(const uint4*)(src + r * ld + c);
    }
}

// copies block `id`'s output when it is among the requested taps
int32_t tap_block(const Taps* taps, int id, const bf16_t* x, int64_t x_sstride, int x_ld, const int32_t* perm,
                  const int32_t* slot_group, const GroupTable& gt, int B, int rows, int c_full, hipStream_t s) {
    if (!taps) return DS_OK;
    for (int i = 0; i < taps->n; ++i) {
        if (taps->ids[i] != id) continue;
        ProfScope prof(DS_K_MISC, s);
        hipLaunchKernelGGL(unpack_slots_kernel, dim3(8, B), dim3(256), 0, s, x, x_sstride, x_ld, perm, slot_group, gt, rows,
                           c_full, (bf16_t*)taps->out[i]);
        DS_CHECK_LAUNCH("tap copy");
    }
    return DS_OK;
}

// pointwise / KxK convolution through the grouped GEMM
int32_t conv_gemm(const bf16_t* A, const int32_t* a_index, int64_t a_sstride, int a_ld, const bf16_t* Wt, int C_I_full,
                  int K, int stride, int pad, int H, int W, const float* scale, const float* shift, int tab_ld,
                  const bf16_t* R, bf16_t* C, int64_t c_sstride, int c_ld, const int32_t* offsets, const MList& ml,
                  const GroupTable& gt, int act, hipStream_t s, const ThinChain* chain = nullptr, bool* chained = nullptr) {
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    const int Ho = (H + 2 * pad - K) / stride + 1, Wo = (W + 2 * pad - K) / stride + 1;
    a.A = A; a.Wt = Wt; a.C = C; a.R = R;
    a.scale = scale; a.shift = shift; a.tab_ld = tab_ld;
    a.a_index = a_index; a.c_index = nullptr;
    a.a_sample_stride = a_sstride; a.c_sample_stride = c_sstride; a.r_sample_stride = c_sstride;
    a.a_ld = a_ld; a.c_ld = c_ld; a.r_ld = c_ld; a.r_use_index = 1;
    a.w_ld = (int64_t)K * K * C_I_full; a.w_tap_stride = C_I_full; a.n_seg = 1;
    a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo; a.K = K; a.stride = stride; a.pad = pad; a.rows = Ho * Wo;
    a.offsets = offsets; a.mtiles = ds_mtile_entries(ml.list); a.n_mtiles = ds_mtile_count(ml.list);
    a.act = act; a.out_f32 = 0; a.gt = gt;
    if (chain) {
        // the layer that reads exactly these output rows rides along where the shapes allow
        const int32_t rc = ds_launch_thin_chain(a, *chain, ml.cap, max_out(gt), s);
        *chained = rc == DS_OK;
        if (rc != DS_EUNSUPPORTED) return rc;
    }
    {
        // short reductions with several column passes stream best with one workgroup per row tile
        const int32_t rc = ds_launch_thin(a, ml.cap, max_out(gt), s);
        if (rc != DS_EUNSUPPORTED) return rc;
    }
    return ds_launch_gemm(a, ml.cap, max_out(gt), s);
}

// =====================================================================================
// DS-MBNet
//  ints:   image, stem_out, n_blocks, gate_after, gate_hidden, T, num_classes,
//          n_blocks x (C_in, C_out, stride), cin[T][n_blocks], cout[T][n_blocks]
//          [, kfull[n_blocks], ksize[T][n_blocks]]   (DS-MBNet++: stored depthwise filter size, route's kernel size)
//  params: stem.w [27][stem_out] bf16, stem.scale, stem.shift,
//          per block: dw.w [k][k][C_in] bf16 (k = 3, or kfull of the block), dw.scale, dw.shift [Tb][C_in], pw.w [C_out][C_in] bf16,
//                     pw.scale, pw.shift [Tb][C_out]   (Tb = 1 before the gate, T after),
//          gate.w1, gate.b1, gate.w2, gate.b2, fc.w [classes][C_last] bf16, fc.b
// =====================================================================================
struct MbDesc {
    int image, stem_out, nb, gate_after, gate_hidden, T, classes;
    const int32_t *blk, *cin, *cout;
    const int32_t *kfull, *ksize;   // null unless the depthwise filters are spatially sliced
};

bool parse_mb(const ds_net* net, MbDesc* d) {
    if (net->n_ints < 7) return false;
    const int32_t* v = net->ints;
    d->image = v[0]; d->stem_out = v[1]; d->nb = v[2]; d->gate_after = v[3]; d->gate_hidden = v[4]; d->T = v[5];
    d->classes = v[6];
    if (d->nb < 1 || d->nb > 64 || d->T < 1 || d->T > DS_MAX_GROUPS) return false;
    const int plain = 7 + 3 * d->nb + 2 * d->T * d->nb;
    if (net->n_ints != plain && net->n_ints != plain + d->nb + d->T * d->nb) return false;
    if (net->n_params != 3 + 6 * d->nb + 6) return false;
    d->blk = v + 7;
    d->cin = d->blk + 3 * d->nb;
    d->cout = d->cin + d->T * d->nb;
    d->kfull = d->ksize = nullptr;
    if (net->n_ints != plain) {
        d->kfull = d->cout + d->T * d->nb;
        d->ksize = d->kfull + d->nb;
    }
    if (d->image < 1 || d->stem_out < 1 || d->gate_hidden < 1 || d->classes < 1) return false;
    for (int i = 0; i < d->nb; ++i) {
        const int st = d->blk[3 * i + 2];
        if (d->blk[3 * i] < 1 || d->blk[3 * i + 1] < 1 || (st != 1 && st != 2)) return false;
    }
    for (int i = 0; i < 2 * d->T * d->nb; ++i)
        if (d->cin[i] < 1) return false;                     // cin and cout are adjacent: every valid width is positive
    return d->gate_after >= 1 && d->gate_after < d->nb;
}

struct MbPlan {
    bf16_t *bufA, *bufB;
    float *gate_logits, *gate_partial;
    float* head_partial;
    int32_t *off1, *offs, *perm, *inv, *slot_group, *route, *slot_c;
    void* lists[2 * 64 + 2];      // one tile list per (resolution, before / after the gate): at most one per block and phase
    int n_lists;
};

void plan_mb(const MbDesc& d, int B, Bump& bp, MbPlan* p) {
    const int r1 = (d.image + 2 - 3) / 2 + 1;
    size_t maxel = (size_t)r1 * r1 * d.stem_out;
    int r = r1;
    for (int i = 0; i < d.nb; ++i) {
        const int ci = d.blk[3 * i], co = d.blk[3 * i + 1], st = d.blk[3 * i + 2];
        r = (r + 2 - 3) / st + 1;
        maxel = maxel > (size_t)r * r * ci ? maxel : (size_t)r * r * ci;
        maxel = maxel > (size_t)r * r * co ? maxel : (size_t)r * r * co;
    }
    p->bufA = bp.take<bf16_t>(maxel * B);
    p->bufB = bp.take<bf16_t>(maxel * B);
    const int cg = d.blk[3 * (d.gate_after - 1) + 1];
    p->gate_logits = bp.take<float>((size_t)B * d.T);
    p->gate_partial = bp.take<float>(ds_gate_partial_bytes(B, cg) / sizeof(float));
    p->off1 = bp.take<int32_t>(2);
    p->offs = bp.take<int32_t>(d.T + 1);
    p->perm = bp.take<int32_t>(B);
    p->inv = bp.take<int32_t>(B);
    p->slot_group = bp.take<int32_t>(B);
    p->route = bp.take<int32_t>(B);
    p->slot_c = bp.take<int32_t>(B);
    p->head_partial = bp.take<float>(ds_gate_partial_bytes(B, d.blk[3 * (d.nb - 1) + 1]) / sizeof(float));
    // one m-tile list per distinct (bucketing, resolution)
    p->n_lists = 0;
    r = r1;
    int last_rows = -1, last_phase = -1;
    for (int i = 0; i < d.nb; ++i) {
        r = (r + 2 - 3) / d.blk[3 * i + 2] + 1;
        const int phase = i >= d.gate_after;
        if (r * r != last_rows || phase != last_phase) {
            p->lists[p->n_lists++] = bp.take<char>(16 + ds_mtile_capacity(B, r * r, phase ? d.T : 1) * 16);
            last_rows = r * r;
            last_phase = phase;
        }
    }
}

int32_t forward_mb(const ds_net* net, const MbDesc& d, const bf16_t* images, int B, const int32_t* route_override,
                   const float* logit_bias, float* logits, int32_t* routes_out, const MbPlan& p, hipStream_t s,
                   const Taps* taps) {
    const void* const* P = net->params;
    int r = (d.image + 2 - 3) / 2 + 1;
    RC(ds_launch_set_offsets(p.off1, B, s));
    RC(ds_launch_stem(images, nullptr, p.bufA, (const bf16_t*)P[0], (const float*)P[1], (const float*)P[2], B, d.image,
                      d.image, 3, 2, 1, d.stem_out, s));
    bf16_t *cur = p.bufA, *oth = p.bufB;
    int li = -1, last_rows = -1, last_phase = -1, fused_lists = 0;
    MList ml = {nullptr, 0, 0};
    for (int i = 0; i < d.nb; ++i) {
        const int ci = d.blk[3 * i], co = d.blk[3 * i + 1], st = d.blk[3 * i + 2];
        const void* const* Q = P + 3 + 6 * i;
        const int phase = i >= d.gate_after;
        const int rin = r;
        r = (r + 2 - 3) / st + 1;
        if (i == d.gate_after) {
            GateArgs g;
            memset(&g, 0, sizeof(g));
            const void* const* G = P + 3 + 6 * d.nb;
            g.x = cur; g.dtype = DS_BF16; g.layout = DS_NHWC; g.B = B; g.C = ci; g.HW = rin * rin;
            g.x_sample_stride = (int64_t)rin * rin * ci; g.x_ld = ci;
            g.w1 = (const float*)G[0]; g.b1 = (const float*)G[1]; g.w2 = (const float*)G[2]; g.b2 = (const float*)G[3];
            g.C_mlp = d.gate_hidden; g.T = d.T; g.logit_bias = logit_bias; g.route_override = route_override;
            g.logits = p.gate_logits; g.route = routes_out ? routes_out : p.route; g.partial = p.gate_partial;
            RC(ds_launch_gate(g, s));
            // one launch: bucket order, the tile lists of the (up to two) resolutions the sliced blocks run at, and
            // the classifier's input width per slot
            BucketArgs ba = {};
            ba.route = g.route; ba.mul = 1; ba.B = B; ba.T = d.T;
            ba.perm = p.perm; ba.inv_perm = p.inv; ba.offsets = p.offs; ba.slot_group = p.slot_group;
            int rr = rin, lrows = -1;
            for (int k = i; k < d.nb && ba.n_lists < 2; ++k) {
                rr = (rr + 2 - 3) / d.blk[3 * k + 2] + 1;
                if (rr * rr != lrows) {
                    lrows = rr * rr;
                    ba.list_rows[ba.n_lists] = lrows;
                    ba.lists[ba.n_lists] = p.lists[li + 1 + ba.n_lists];
                    ++ba.n_lists;
                }
            }
            fused_lists = ba.n_lists;
            ba.slot_lut = p.slot_c;
            for (int t = 0; t < d.T; ++t) ba.lut[t] = d.cout[t * d.nb + d.nb - 1];
            RC(ds_launch_bucket_ex(ba, s));
        }
        GroupTable gdw, gpw;
        memset(&gdw, 0, sizeof(gdw));
        if (!phase) {
            gdw = table1(ci, ci);
            gpw = table1(ci, co);
        } else {
            gdw.T = d.T;
            for (int t = 0; t < d.T; ++t) {
                gdw.k_in[t] = gdw.k_out[t] = d.cin[t * d.nb + i];
                gdw.row[t] = t;
            }
            gpw = gdw;
            for (int t = 0; t < d.T; ++t) gpw.k_out[t] = d.cout[t * d.nb + i];
        }
        if (!phase && !d.kfull) {
            // an unsliced block: depthwise and pointwise in one kernel where the shape allows, the depthwise map stays in LDS
            const int32_t rc = ds_launch_dwpw(cur, B, rin, rin, ci, st, (const bf16_t*)Q[0], (const float*)Q[1],
                                              (const float*)Q[2], (const bf16_t*)Q[3], ci, co, (const float*)Q[4],
                                              (const float*)Q[5], oth, s);
            if (rc == DS_OK) {
                bf16_t* t = cur; cur = oth; oth = t;
                RC(tap_block(taps, i, cur, (int64_t)r * r * co, co, nullptr, nullptr, gpw, B, r * r, co, s));
                continue;
            }
            if (rc != DS_EUNSUPPORTED) return rc;
        }
        const int32_t* offsets = phase ? p.offs : p.off1;
        if (r * r != last_rows || phase != last_phase) {
            ++li;
            ml.list = p.lists[li];
            ml.cap = (int)ds_mtile_capacity(B, r * r, phase ? d.T : 1);
            ml.rows = r * r;
            if (phase && fused_lists > 0) --fused_lists;      // built together with the bucket order
            else RC(ds_build_mtiles(offsets, phase ? d.T : 1, r * r, ml.list, s));
            last_rows = r * r;
            last_phase = phase;
        }
        // depthwise: the first sliced block reads the fixed-width, original-order feature map through perm
        const bool first = (i == d.gate_after);
        ActView xv = {cur, first ? p.perm : nullptr, (int64_t)rin * rin * ci, (!phase || first) ? ci : 0};
        ActView yv = {oth, nullptr, (int64_t)r * r * ci, phase ? 0 : ci};
        if (d.kfull) {
            // the route's centred block of the stored filter at the padding that keeps the resolution
            SpatialTable sp;
            memset(&sp, 0, sizeof(sp));
            for (int t = 0; t < (phase ? d.T : 1); ++t) {
                const int k = d.ksize[t * d.nb + i];
                sp.k0[t] = (d.kfull[i] - k) / 2; sp.n[t] = k; sp.l[t] = 1; sp.pad[t] = (k - 1) / 2;
            }
            RC(ds_launch_dwconv_spatial(xv, yv, (const bf16_t*)Q[0], d.kfull[i], (const float*)Q[1], (const float*)Q[2],
                                        ci, phase ? p.slot_group : nullptr, gdw, sp, B, ci, rin, rin, st, DS_ACT_RELU, s));
        } else {
            RC(ds_launch_dwconv(xv, yv, (const bf16_t*)Q[0], (const float*)Q[1], (const float*)Q[2], ci,
                                phase ? p.slot_group : nullptr, gdw, B, ci, rin, rin, st, DS_ACT_RELU, s));
        }
        // pointwise
        RC(conv_gemm(oth, nullptr, (int64_t)r * r * ci, phase ? 0 : ci, (const bf16_t*)Q[3], ci, 1, 1, 0, r, r,
                     (const float*)Q[4], (const float*)Q[5], co, nullptr, cur, (int64_t)r * r * co, phase ? 0 : co,
                     offsets, ml, gpw, DS_ACT_RELU, s));
        RC(tap_block(taps, i, cur, (int64_t)r * r * co, phase ? 0 : co, phase ? p.perm : nullptr,
                     phase ? p.slot_group : nullptr, gpw, B, r * r, co, s));
    }
    const void* const* F = P + 3 + 6 * d.nb + 4;
    const int cl = d.blk[3 * (d.nb - 1) + 1];
    ActView xv = {cur, nullptr, (int64_t)r * r * cl, 0};   // slot_c holds the last block's width per slot
    return ds_launch_head(xv, r * r, (const bf16_t*)F[0], cl, (const float*)F[1], d.classes, p.slot_c, p.perm, logits,
                          p.head_partial, B, cl, s);
}

// =====================================================================================
// DS-ResNet
//  ints:   image, stem_out, T, num_classes, widths[4], blocks[4], gate_hidden[4], mid[4][T], out[4][T] [, nblk[4][T] [, flags]]
//  params: stem.w [147][stem_out] bf16, stem.scale, stem.shift,
//          per stage: gate.w1, gate.b1, gate.w2, gate.b2, then per block:
//             c1.w [w][C_in] bf16, c1.scale, c1.shift [T][w], c2.w [w][3][3][w] bf16, c2.scale, c2.shift,
//             c3.w [4w][w] bf16, c3.scale, c3.shift [T][4w], and for the first block
//             proj.w [4w][C_in] bf16, proj.scale, proj.shift,
//          fc.w [classes][4*w_last] bf16, fc.b
// =====================================================================================
struct RnDesc {
    int image, stem_out, T, classes;
    const int32_t *widths, *blocks, *hidden, *mid, *out;
    const int32_t* nblk;     // [4][T] blocks of a stage that a route runs, or null: every stored block
    int single_gate;         // 1: the first stage's gate decides for all four stages (DS-ResNet++)
};

// route groups of a stage: (this stage's route, previous stage's route) pairs, or the route alone when one gate
// decides for every stage
inline int rn_groups(const RnDesc& d) { return d.single_gate ? d.T : d.T * d.T; }

bool parse_rn(const ds_net* net, RnDesc* d) {
    if (net->n_ints < 4) return false;
    const int32_t* v = net->ints;
    d->image = v[0]; d->stem_out = v[1]; d->T = v[2]; d->classes = v[3];
    if (d->T < 1 || d->T > DS_MAX_GROUPS) return false;
    const int base = 4 + 12 + 8 * d->T, deep = base + 4 * d->T;
    if (net->n_ints != base && net->n_ints != deep && net->n_ints != deep + 1) return false;
    d->widths = v + 4; d->blocks = v + 8; d->hidden = v + 12; d->mid = v + 16; d->out = d->mid + 4 * d->T;
    d->nblk = net->n_ints >= deep ? d->out + 4 * d->T : nullptr;
    d->single_gate = net->n_ints == deep + 1 ? (v[deep] & 1) : 0;
    if (rn_groups(*d) > DS_MAX_GROUPS) return false;
    if (d->image < 1 || d->stem_out < 1 || d->classes < 1) return false;
    for (int st = 0; st < 4; ++st)
        if (d->widths[st] < 1 || d->blocks[st] < 1 || d->blocks[st] > 64 || d->hidden[st] < 1) return false;
    for (int i = 0; i < 8 * d->T; ++i)
        if (d->mid[i] < 1) return false;                     // mid and out are adjacent: every valid width is positive
    if (d->nblk)
        for (int st = 0; st < 4; ++st)
            for (int q = 0; q < d->T; ++q)
                if (d->nblk[st * d->T + q] < 1 || d->nblk[st * d->T + q] > d->blocks[st]) return false;
    int np = 3 + 2;
    for (int s = 0; s < 4; ++s) np += 4 + 9 * d->blocks[s] + 3;
    return net->n_params == np;
}

struct RnPlan {
    bf16_t* buf[5];
    float *gate_logits, *gate_partial;
    int32_t *off1, *offs[4], *perm[4], *inv[4], *slot_group[4], *route[4], *key, *src_index, *slot_c;
    void* lists[8];
};

void plan_rn(const RnDesc& d, int B, Bump& bp, RnPlan* p) {
    const int r1 = (d.image + 6 - 7) / 2 + 1, r2 = (r1 + 2 - 3) / 2 + 1;
    size_t maxel = (size_t)r1 * r1 * d.stem_out;
    int r = r2;
    for (int s = 0; s < 4; ++s) {
        const size_t in_res = (size_t)r * r;
        if (s > 0) r = (r + 2 - 3) / 2 + 1;
        const size_t e1 = in_res * d.widths[s], e2 = (size_t)r * r * 4 * d.widths[s];
        maxel = maxel > e1 ? maxel : e1;
        maxel = maxel > e2 ? maxel : e2;
    }
    for (int i = 0; i < 5; ++i) p->buf[i] = bp.take<bf16_t>(maxel * B);
    int cmax = d.stem_out;
    for (int s = 0; s < 4; ++s) cmax = cmax > 4 * d.widths[s] ? cmax : 4 * d.widths[s];
    p->gate_logits = bp.take<float>((size_t)B * d.T);
    p->gate_partial = bp.take<float>(ds_gate_partial_bytes(B, cmax) / sizeof(float));
    p->off1 = bp.take<int32_t>(2);
    for (int s = 0; s < 4; ++s) {
        p->offs[s] = bp.take<int32_t>(rn_groups(d) + 1);
        p->perm[s] = bp.take<int32_t>(B);
        p->inv[s] = bp.take<int32_t>(B);
        p->slot_group[s] = bp.take<int32_t>(B);
        p->route[s] = bp.take<int32_t>(B);
    }
    p->key = bp.take<int32_t>(B);
    p->src_index = bp.take<int32_t>(B);
    p->slot_c = bp.take<int32_t>(B);
    r = r2;
    for (int s = 0; s < 4; ++s) {
        p->lists[2 * s] = bp.take<char>(16 + ds_mtile_capacity(B, r * r, rn_groups(d)) * 16);  // input resolution
        if (s > 0) r = (r + 2 - 3) / 2 + 1;
        p->lists[2 * s + 1] = bp.take<char>(16 + ds_mtile_capacity(B, r * r, rn_groups(d)) * 16);  // output resolution
    }
}

// Bs: batch stride of the caller's gate-major arrays (route_override, logit_bias, routes_out); B when the whole batch
// is run as one part
int32_t forward_rn(const ds_net* net, const RnDesc& d, const bf16_t* images, int B, int Bs, const int32_t* route_override,
                   const float* logit_bias, float* logits, int32_t* routes_out, const RnPlan& p, hipStream_t s,
                   const Taps* taps) {
    const void* const* P = net->params;
    const int T = d.T, G = rn_groups(d);
    const bool pairs = !d.single_gate;      // group id = q * T + q_prev, or q alone (then q_prev = q)
    const int r1 = (d.image + 6 - 7) / 2 + 1;
    int r = (r1 + 2 - 3) / 2 + 1;
    // stem and max-pool in one kernel where the shape allows, else one after the other
    int32_t fused = ds_launch_stem_pool(images, nullptr, p.buf[1], (const bf16_t*)P[0], (const float*)P[1],
                                        (const float*)P[2], B, d.image, d.image, 7, 2, 3, d.stem_out, s);
    if (fused == DS_EUNSUPPORTED) {
        RC(ds_launch_stem(images, nullptr, p.buf[0], (const bf16_t*)P[0], (const float*)P[1], (const float*)P[2], B,
                          d.image, d.image, 7, 2, 3, d.stem_out, s));
        RC(ds_launch_maxpool(p.buf[0], p.buf[1], B, r1, r1, d.stem_out, s));
    } else {
        RC(fused);
    }
    bf16_t* X = p.buf[1];          // stage input, slot order of the previous stage
    int xi = 1;                    // index of X in buf[]
    int c_prev_full = d.stem_out;
    const void* const* Q = P + 3;
    int block_id = 0;              // blocks counted over all stages, in execution order
    for (int st = 0; st < 4; ++st) {
        const int w = d.widths[st], nb = d.blocks[st];
        const int rin = r;
        const int stride = st > 0 ? 2 : 1;
        const int rout = (rin + 2 - 3) / stride + 1;
        int32_t* route = routes_out ? routes_out + (size_t)st * Bs : p.route[st];
        // ---- gate on the stage input (previous slot order), routes land in original sample order
        GateArgs g;
        memset(&g, 0, sizeof(g));
        g.x = X; g.dtype = DS_BF16; g.layout = DS_NHWC; g.B = B; g.C = c_prev_full; g.HW = rin * rin;
        g.c_in = st > 0 ? p.slot_c : nullptr;
        g.x_sample_stride = (int64_t)rin * rin * c_prev_full; g.x_ld = 0;
        g.w1 = (const float*)Q[0]; g.b1 = (const float*)Q[1]; g.w2 = (const float*)Q[2]; g.b2 = (const float*)Q[3];
        g.C_mlp = d.hidden[st]; g.T = T;
        g.logit_bias = logit_bias ? logit_bias + (size_t)st * Bs * T : nullptr;
        g.out_index = st > 0 ? p.perm[st - 1] : nullptr;
        g.route_override = route_override ? route_override + (size_t)st * Bs : nullptr;
        g.logits = p.gate_logits; g.route = route; g.partial = p.gate_partial;
        if (d.single_gate && st > 0) {
            // the first stage's decision stands: no pooling, no MLP, the route is copied
            g.x = nullptr; g.logit_bias = nullptr; g.out_index = nullptr;
            g.route_override = routes_out ? routes_out : p.route[0];
        }
        RC(ds_launch_gate(g, s));
        Q += 4;
        // ---- bucket by (this stage's route, previous stage's route)
        const int32_t* route_prev = st > 0 ? (routes_out ? routes_out + (size_t)(st - 1) * Bs : p.route[st - 1]) : nullptr;
        BucketArgs ba = {};
        ba.route = route; ba.lo = pairs ? route_prev : nullptr; ba.mul = pairs ? T : 1; ba.B = B; ba.T = G;
        ba.perm = p.perm[st]; ba.inv_perm = p.inv[st]; ba.offsets = p.offs[st]; ba.slot_group = p.slot_group[st];
        ba.inv_prev = st > 0 ? p.inv[st - 1] : nullptr;
        ba.src_index = p.src_index;          // slot of this stage -> slot of the previous stage's layout
        // the same launch builds the tile lists at both resolutions and the per-slot output width of the stage
        MList ml_in = {p.lists[2 * st], (int)ds_mtile_capacity(B, rin * rin, G), rin * rin};
        MList ml_out = {p.lists[2 * st + 1], (int)ds_mtile_capacity(B, rout * rout, G), rout * rout};
        ba.n_lists = 2;
        ba.list_rows[0] = rin * rin; ba.lists[0] = ml_in.list;
        ba.list_rows[1] = rout * rout; ba.lists[1] = ml_out.list;
        ba.slot_lut = p.slot_c;
        for (int id = 0; id < G; ++id) ba.lut[id] = d.out[st * T + (pairs ? id / T : id)];
        RC(ds_launch_bucket_ex(ba, s));
        const int32_t* src = p.src_index;
        // ---- group tables: group id = q * T + q_prev
        GroupTable g1f, gpj, g1, g2, g3;
        memset(&g1f, 0, sizeof(g1f));
        g1f.T = G;
        for (int id = 0; id < G; ++id) {
            const int q = pairs ? id / T : id, qp = pairs ? id % T : id;
            g1f.k_in[id] = st > 0 ? d.out[(st - 1) * T + qp] : d.stem_out;
            g1f.k_out[id] = d.mid[st * T + q];
            g1f.row[id] = q;
        }
        gpj = g1f; g1 = g1f; g2 = g1f; g3 = g1f;
        for (int id = 0; id < G; ++id) {
            const int q = pairs ? id / T : id;
            gpj.k_out[id] = d.out[st * T + q];
            g1.k_in[id] = d.out[st * T + q];
            g2.k_in[id] = g2.k_out[id] = d.mid[st * T + q];
            g3.k_in[id] = d.mid[st * T + q];
            g3.k_out[id] = d.out[st * T + q];
        }
        // buffers other than X: Y1, Y2, Pj, Z
        bf16_t* free4[4];
        for (int i = 0, k = 0; i < 5; ++i)
            if (i != xi) free4[k++] = p.buf[i];
        bf16_t *Y1 = free4[0], *Y2 = free4[1], *Pj = free4[2], *Z = free4[3];
        const int64_t x_ss = (int64_t)rin * rin * c_prev_full;
        bool y1_ready = false;         // the previous block's last launch has already run this block's first convolution
        for (int b = 0; b < nb; ++b, ++block_id) {
            const bool first = b == 0;
            const int bs = first ? stride : 1;
            const int rb = first ? rin : rout;  // resolution of the block input
            const void* const* L = Q;
            Q += first ? 12 : 9;
            if (d.nblk && !first) {
                // dynamic depth: a route that has run its blocks gets empty slices from here on, so the
                // kernels leave its slots of Z as they are (the block is an identity through its residual)
                bool any = false;
                for (int id = 0; id < G; ++id) {
                    if (d.nblk[st * T + (pairs ? id / T : id)] > b) { any = true; continue; }
                    g1.k_in[id] = g1.k_out[id] = g2.k_in[id] = g2.k_out[id] = g3.k_in[id] = g3.k_out[id] = 0;
                }
                if (!any) continue;
            }
            const bf16_t* in = first ? X : Z;
            const int32_t* in_idx = first ? src : nullptr;
            const int64_t in_ss = first ? x_ss : (int64_t)rout * rout * 4 * w;
            const int in_full = first ? c_prev_full : 4 * w;
            const bf16_t* shortcut;
            if (first) {
                RC(conv_gemm(in, in_idx, in_ss, 0, (const bf16_t*)L[9], in_full, 1, bs, 0, rb, rb, (const float*)L[10],
                             (const float*)L[11], 4 * w, nullptr, Pj, (int64_t)rout * rout * 4 * w, 0, p.offs[st], ml_out,
                             gpj, DS_ACT_NONE, s));
                shortcut = Pj;
            } else {
                shortcut = Z;
            }
            if (!y1_ready)
                RC(conv_gemm(in, in_idx, in_ss, 0, (const bf16_t*)L[0], in_full, 1, 1, 0, rb, rb, (const float*)L[1],
                             (const float*)L[2], w, nullptr, Y1, (int64_t)rb * rb * w, 0, p.offs[st], first ? ml_in : ml_out,
                             first ? g1f : g1, DS_ACT_RELU, s));
            y1_ready = false;
            RC(conv_gemm(Y1, nullptr, (int64_t)rb * rb * w, 0, (const bf16_t*)L[3], w, 3, bs, 1, rb, rb, (const float*)L[4],
                         (const float*)L[5], w, nullptr, Y2, (int64_t)rout * rout * w, 0, p.offs[st], ml_out, g2,
                         DS_ACT_RELU, s));
            // the next block's first convolution reads the rows this block's last one writes: where the slices are
            // narrow enough the two run as one launch and Y1 is ready when the next block starts
            ThinChain ch;
            memset(&ch, 0, sizeof(ch));
            bool next_any = false;
            if (b + 1 < nb) {
                const void* const* Ln = Q;
                ch.Wt = (const bf16_t*)Ln[0]; ch.scale = (const float*)Ln[1]; ch.shift = (const float*)Ln[2];
                ch.C = Y1; ch.w_ld = 4 * w; ch.c_sample_stride = (int64_t)rout * rout * w; ch.c_ld = 0; ch.tab_ld = w;
                ch.act = DS_ACT_RELU;
                for (int id = 0; id < G; ++id) {
                    const bool on = g1.k_out[id] > 0 && (!d.nblk || d.nblk[st * T + (pairs ? id / T : id)] > b + 1);
                    ch.k_out[id] = on ? g1.k_out[id] : 0;
                    next_any = next_any || on;
                }
            }
            // c3 adds the shortcut; later blocks update Z in place (each element is read and written by one thread)
            RC(conv_gemm(Y2, nullptr, (int64_t)rout * rout * w, 0, (const bf16_t*)L[6], w, 1, 1, 0, rout, rout,
                         (const float*)L[7], (const float*)L[8], 4 * w, shortcut, Z, (int64_t)rout * rout * 4 * w, 0,
                         p.offs[st], ml_out, g3, DS_ACT_RELU, s, next_any ? &ch : nullptr, &y1_ready));
            RC(tap_block(taps, block_id, Z, (int64_t)rout * rout * 4 * w, 0, p.perm[st], p.slot_group[st], gpj, B, rout * rout,
                         4 * w, s));
        }
        X = Z;
        for (int i = 0; i < 5; ++i)
            if (p.buf[i] == Z) xi = i;
        c_prev_full = 4 * w;
        r = rout;
    }
    ActView xv = {X, nullptr, (int64_t)r * r * c_prev_full, 0};   // slot_c holds the stage-4 output widths
    return ds_launch_head(xv, r * r, (const bf16_t*)Q[0], c_prev_full, (const float*)Q[1], d.classes, p.slot_c, p.perm[3],
                          logits, p.gate_partial, B, c_prev_full, s);
}

// =====================================================================================
// DS-ViT
//  ints:   image, patch, embed, heads, head_dim, mlp, depth, tokens, T, num_classes, routes[T][3] = (d_e, h, hidden)
//  params: embed.w [D][3*P*P] bf16, embed.b, cls [D] bf16, pos [tokens][D] bf16,
//          per layer: ln1.g, ln1.b, wqkv [3][H*Dh][D] bf16, bqkv [3][H*Dh], wproj [D][H*Dh] bf16, bproj,
//                     ln2.g, ln2.b, fc1.w [mlp][D] bf16, fc1.b, fc2.w [D][mlp] bf16, fc2.b,
//          ln.g, ln.b, head.w [classes][D] bf16, head.b
// =====================================================================================
//
// DS-ViT++ with the convolutional stem (DS_ARCH_VIT_STEM): 7x7 stride-2 convolution and two depthwise-separable
// blocks at stem_dim channels, the gate on that map, and the patch embedding as a patch x patch stride-patch
// convolution over it.
//  ints:   image, patch, embed, heads, head_dim, mlp, depth, tokens, T, num_classes, rs, stem_dim, gate_hidden,
//          routes[T][rs]
//  params: stem.c0.w [7*7*3][stem_dim] bf16, scale, shift, 2 x (dw.w [3][3][C] bf16, dw.scale, dw.shift,
//          pw.w [C][C] bf16, pw.scale, pw.shift), gate.w1, gate.b1, gate.w2, gate.b2,
//          embed.w [D][patch][patch][C] bf16, then as above from embed.b on
struct VitDesc {
    int image, patch, D, H, dh, M, depth, N, T, classes;
    int rs;                  // entries per route: 3 (d_e, heads, hidden) or 4 (+ number of blocks the route runs)
    int stem_dim, gate_hidden, pbase;   // stem width (0: none), gate MLP width, index of embed.w in params
    const int32_t* routes;
};
constexpr int VIT_STEM_PARAMS = 3 + 12 + 4;

bool parse_vit(const ds_net* net, VitDesc* d) {
    if (net->n_ints < 10) return false;
    const int32_t* v = net->ints;
    d->image = v[0]; d->patch = v[1]; d->D = v[2]; d->H = v[3]; d->dh = v[4]; d->M = v[5]; d->depth = v[6];
    d->N = v[7]; d->T = v[8]; d->classes = v[9];
    if (d->T < 1 || d->T > DS_MAX_GROUPS) return false;
    d->stem_dim = d->gate_hidden = d->pbase = 0;
    if (net->arch == DS_ARCH_VIT_STEM) {
        if (net->n_ints < 13) return false;
        d->rs = v[10]; d->stem_dim = v[11]; d->gate_hidden = v[12];
        if ((d->rs != 3 && d->rs != 4) || net->n_ints != 13 + d->rs * d->T) return false;
        if (d->stem_dim < 8 || d->gate_hidden < 1) return false;
        d->routes = v + 13;
        d->pbase = VIT_STEM_PARAMS;
    } else {
        if (net->n_ints == 10 + 3 * d->T) d->rs = 3;
        else if (net->n_ints == 10 + 4 * d->T) d->rs = 4;
        else return false;
        d->routes = v + 10;
    }
    return net->n_params == d->pbase + 4 + 12 * d->depth + 4;
}

struct VitPlan {
    bf16_t *patches, *x, *a, *qkv, *o, *h;
    bf16_t *sa, *sb;          // the stem's two feature maps
    size_t qkv_seg;
    float *gate_logits, *gate_partial;
    int32_t *off1, *offs, *perm, *inv, *slot_group, *route, *slot_c;
    void *list_p, *list_t, *list_s;
};

inline int vit_stem_res(const VitDesc& d) { return (d.image + 6 - 7) / 2 + 1; }

void plan_vit(const VitDesc& d, int B, Bump& bp, VitPlan* p) {
    const int np = d.N - 1, kp = 3 * d.patch * d.patch, Hd = d.H * d.dh;
    p->patches = p->sa = p->sb = nullptr;
    p->gate_partial = nullptr; p->off1 = nullptr; p->list_s = nullptr;
    if (d.stem_dim) {
        const int r = vit_stem_res(d);
        p->sa = bp.take<bf16_t>((size_t)B * r * r * d.stem_dim);
        p->sb = bp.take<bf16_t>((size_t)B * r * r * d.stem_dim);
        p->gate_partial = bp.take<float>(ds_gate_partial_bytes(B, d.stem_dim) / sizeof(float));
        p->off1 = bp.take<int32_t>(2);
        p->list_s = bp.take<char>(16 + ds_mtile_capacity(B, r * r, 1) * 16);
    } else {
        p->patches = bp.take<bf16_t>((size_t)B * np * kp);
    }
    p->x = bp.take<bf16_t>((size_t)B * d.N * d.D);
    p->a = bp.take<bf16_t>((size_t)B * d.N * d.D);
    p->qkv_seg = ds_align_up((size_t)B * d.N * Hd, 128);
    p->qkv = bp.take<bf16_t>(3 * p->qkv_seg);
    p->o = bp.take<bf16_t>((size_t)B * d.N * Hd);
    p->h = bp.take<bf16_t>((size_t)B * d.N * d.M);
    p->gate_logits = bp.take<float>((size_t)B * d.T);
    p->offs = bp.take<int32_t>(d.T + 1);
    p->perm = bp.take<int32_t>(B);
    p->inv = bp.take<int32_t>(B);
    p->slot_group = bp.take<int32_t>(B);
    p->route = bp.take<int32_t>(B);
    p->slot_c = bp.take<int32_t>(B);
    p->list_p = bp.take<char>(16 + ds_mtile_capacity(B, np, d.T) * 16);
    p->list_t = bp.take<char>(16 + ds_mtile_capacity(B, d.N, d.T) * 16);
}

int32_t linear_gemm(const bf16_t* A, int64_t a_ss, int a_ld, const bf16_t* Wt, int64_t w_ld, const float* bias,
                    const bf16_t* R, int64_t r_ss, int r_ld, int r_use_index, bf16_t* C, int64_t c_ss, int c_ld,
                    int c_row0, int rows, int n_seg, int64_t w_seg, int64_t c_seg, int tab_seg, const int32_t* offsets,
                    const MList& ml, const GroupTable& gt, int act, hipStream_t s) {
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.A = A; a.Wt = Wt; a.C = C; a.R = R;
    a.scale = nullptr; a.shift = bias; a.tab_ld = 0; a.tab_seg_stride = tab_seg;
    a.a_sample_stride = a_ss; a.c_sample_stride = c_ss; a.r_sample_stride = r_ss;
    a.a_ld = a_ld; a.c_ld = c_ld; a.r_ld = r_ld; a.c_row0 = c_row0; a.r_use_index = r_use_index;
    a.w_ld = w_ld; a.w_seg_stride = w_seg; a.c_seg_stride = c_seg; a.n_seg = n_seg;
    a.H = 1; a.W = rows; a.Ho = 1; a.Wo = rows; a.K = 1; a.stride = 1; a.pad = 0; a.rows = rows;
    a.offsets = offsets; a.mtiles = ds_mtile_entries(ml.list); a.n_mtiles = ds_mtile_count(ml.list);
    a.act = act; a.out_f32 = 0; a.gt = gt;
    return ds_launch_gemm(a, ml.cap, max_out(gt), s);
}

int32_t forward_vit(const ds_net* net, const VitDesc& d, const bf16_t* images, int B, const int32_t* route_override,
                    const float* logit_bias, float* logits, int32_t* routes_out, const VitPlan& p, hipStream_t s,
                    const Taps* taps) {
    const void* const* P = net->params + d.pbase;
    const int np = d.N - 1, Hd = d.H * d.dh, T = d.T;
    const int kp = d.stem_dim ? d.stem_dim : 3 * d.patch * d.patch;   // reduction length of one embedding tap
    if (!d.stem_dim && !logit_bias && !route_override)
        DS_FAIL(DS_EINVAL, "ds_forward(vit): routes need logit_bias or route_override");
    int32_t* route = routes_out ? routes_out : p.route;
    GateArgs g;
    memset(&g, 0, sizeof(g));
    g.B = B; g.T = T; g.logit_bias = logit_bias; g.route_override = route_override;
    g.logits = p.gate_logits; g.route = route;
    const int sr = vit_stem_res(d);
    if (d.stem_dim) {
        // stem: every sample at full width, original order; the gate pools its last feature map
        const void* const* S = net->params;
        const int C = d.stem_dim;
        const int64_t map = (int64_t)sr * sr * C;
        RC(ds_launch_set_offsets(p.off1, B, s));
        RC(ds_launch_stem(images, nullptr, p.sa, (const bf16_t*)S[0], (const float*)S[1], (const float*)S[2], B, d.image,
                          d.image, 7, 2, 3, C, s));
        MList ml_s = {p.list_s, (int)ds_mtile_capacity(B, sr * sr, 1), sr * sr};
        RC(ds_build_mtiles(p.off1, 1, sr * sr, ml_s.list, s));
        const GroupTable g1c = table1(C, C);
        for (int i = 0; i < 2; ++i) {
            const void* const* Q = S + 3 + 6 * i;
            // the block as one kernel where the shape allows (the depthwise map stays in LDS); it cannot run in place,
            // so two fused blocks in a row go sa -> sb -> sa and the map ends where the layers below expect it
            int32_t fused = DS_EUNSUPPORTED;
            if (i == 0) {
                fused = ds_launch_dwpw(p.sa, B, sr, sr, C, 1, (const bf16_t*)Q[0], (const float*)Q[1], (const float*)Q[2],
                                       (const bf16_t*)Q[3], C, C, (const float*)Q[4], (const float*)Q[5], p.sb, s);
                if (fused == DS_OK) {
                    const void* const* Q1 = S + 3 + 6;
                    RC(ds_launch_dwpw(p.sb, B, sr, sr, C, 1, (const bf16_t*)Q1[0], (const float*)Q1[1], (const float*)Q1[2],
                                      (const bf16_t*)Q1[3], C, C, (const float*)Q1[4], (const float*)Q1[5], p.sa, s));
                    break;
                }
                if (fused != DS_EUNSUPPORTED) return fused;
            }
            ActView xv = {p.sa, nullptr, map, C}, yv = {p.sb, nullptr, map, C};
            RC(ds_launch_dwconv(xv, yv, (const bf16_t*)Q[0], (const float*)Q[1], (const float*)Q[2], C, nullptr, g1c, B, C,
                                sr, sr, 1, DS_ACT_RELU, s));
            RC(conv_gemm(p.sb, nullptr, map, C, (const bf16_t*)Q[3], C, 1, 1, 0, sr, sr, (const float*)Q[4],
                         (const float*)Q[5], C, nullptr, p.sa, map, C, p.off1, ml_s, g1c, DS_ACT_RELU, s));
        }
        const void* const* G = S + 15;
        g.x = p.sa; g.dtype = DS_BF16; g.layout = DS_NHWC; g.C = C; g.HW = sr * sr;
        g.x_sample_stride = map; g.x_ld = C;
        g.w1 = (const float*)G[0]; g.b1 = (const float*)G[1]; g.w2 = (const float*)G[2]; g.b2 = (const float*)G[3];
        g.C_mlp = d.gate_hidden; g.partial = p.gate_partial;
    }
    RC(ds_launch_gate(g, s));
    // one launch: bucket order, the tile lists for the patch rows and the token rows, the embedding width per slot
    MList ml_p = {p.list_p, (int)ds_mtile_capacity(B, np, T), np};
    MList ml_t = {p.list_t, (int)ds_mtile_capacity(B, d.N, T), d.N};
    BucketArgs ba = {};
    ba.route = route; ba.mul = 1; ba.B = B; ba.T = T;
    ba.perm = p.perm; ba.inv_perm = p.inv; ba.offsets = p.offs; ba.slot_group = p.slot_group;
    ba.n_lists = 2;
    ba.list_rows[0] = np; ba.lists[0] = ml_p.list;
    ba.list_rows[1] = d.N; ba.lists[1] = ml_t.list;
    ba.slot_lut = p.slot_c;
    for (int t = 0; t < T; ++t) ba.lut[t] = d.routes[d.rs * t];
    RC(ds_launch_bucket_ex(ba, s));
    GroupTable ge, gq, gp, g1, g2;
    memset(&ge, 0, sizeof(ge));
    ge.T = T;
    for (int t = 0; t < T; ++t) ge.row[t] = 0;
    gq = ge; gp = ge; g1 = ge; g2 = ge;
    for (int t = 0; t < T; ++t) {
        const int de = d.routes[d.rs * t], h = d.routes[d.rs * t + 1], hid = d.routes[d.rs * t + 2];
        ge.k_in[t] = kp; ge.k_out[t] = de;
        gq.k_in[t] = de; gq.k_out[t] = h * d.dh;
        gp.k_in[t] = h * d.dh; gp.k_out[t] = de;
        g1.k_in[t] = de; g1.k_out[t] = hid;
        g2.k_in[t] = hid; g2.k_out[t] = de;
    }
    const int64_t x_ss = (int64_t)d.N * d.D;
    if (d.stem_dim) {
        // tokens 1..N-1: the stem's last convolution (kernel = stride = patch) over each sample's map, read through
        // the bucket permutation, + bias + position embedding (broadcast over samples)
        GemmArgs a;
        memset(&a, 0, sizeof(a));
        const int C = d.stem_dim, gw = sr / d.patch;
        a.A = p.sa; a.Wt = (const bf16_t*)P[0]; a.C = p.x; a.R = (const bf16_t*)P[3];
        a.scale = nullptr; a.shift = (const float*)P[1]; a.tab_ld = 0;
        a.a_index = p.perm; a.c_index = nullptr;
        a.a_sample_stride = (int64_t)sr * sr * C; a.c_sample_stride = x_ss; a.r_sample_stride = 0;
        // A patch row is patch x C contiguous values and so is the matching row of a filter: the map is read as
        // [sr][sr / patch] pixels of patch * C channels under a patch x 1 filter (vertical stride patch, horizontal 1),
        // which makes the reduction patch taps of patch * C channels instead of patch^2 taps of C (24) channels
        a.a_ld = d.patch * C; a.c_ld = 0; a.r_ld = d.D; a.c_row0 = 1; a.r_use_index = 0;
        a.w_ld = (int64_t)d.patch * d.patch * C; a.w_tap_stride = d.patch * C; a.n_seg = 1;
        a.H = sr; a.W = gw; a.Ho = gw; a.Wo = gw; a.K = d.patch; a.Kw = 1; a.stride = d.patch; a.stride_w = 1; a.pad = 0;
        a.rows = np;
        a.offsets = p.offs; a.mtiles = ds_mtile_entries(ml_p.list); a.n_mtiles = ds_mtile_count(ml_p.list);
        a.act = DS_ACT_NONE; a.out_f32 = 0; a.gt = ge;
        for (int t = 0; t < T; ++t) a.gt.k_in[t] = d.patch * C;
        RC(ds_launch_gemm(a, ml_p.cap, max_out(ge), s));
    } else {
        RC(ds_launch_patchify(images, p.perm, p.patches, B, d.image, d.image, d.patch, s));
        // tokens 1..N-1: patch embedding + bias + position embedding (broadcast over samples)
        RC(linear_gemm(p.patches, (int64_t)np * kp, kp, (const bf16_t*)P[0], kp, (const float*)P[1], (const bf16_t*)P[3], 0,
                       d.D, 0, p.x, x_ss, 0, 1, np, 1, 0, 0, 0, p.offs, ml_p, ge, DS_ACT_NONE, s));
    }
    ActView xv = {p.x, nullptr, x_ss, 0}, av = {p.a, nullptr, x_ss, 0};
    RC(ds_launch_cls_rows(xv, (const bf16_t*)P[2], (const bf16_t*)P[3], p.slot_group, gq, B, s));
    const float eps = 1e-6f;
    const GroupTable fq = gq;      // every route, for the final LayerNorm and the classifier
    for (int l = 0; l < d.depth; ++l) {
        const void* const* L = P + 4 + 12 * l;
        // dynamic depth: a route that runs fewer than l + 1 blocks gets empty slices from here on, so
        // no kernel touches its rows and the residual stream carries them through unchanged
        if (d.rs == 4) {
            bool any = false;
            for (int t = 0; t < T; ++t) {
                if (d.routes[4 * t + 3] <= l) {
                    gq.k_in[t] = gq.k_out[t] = gp.k_in[t] = gp.k_out[t] = 0;
                    g1.k_in[t] = g1.k_out[t] = g2.k_in[t] = g2.k_out[t] = 0;
                } else {
                    any = true;
                }
            }
            if (!any) break;
        }
        RC(ds_launch_layernorm(xv, av, (const float*)L[0], (const float*)L[1], eps, p.slot_group, gq, B, d.N, 0, d.N, s));
        RC(linear_gemm(p.a, x_ss, 0, (const bf16_t*)L[2], d.D, (const float*)L[3], nullptr, 0, 0, 0, p.qkv,
                       (int64_t)d.N * Hd, Hd, 0, d.N, 3, (int64_t)Hd * d.D, (int64_t)p.qkv_seg, Hd, p.offs, ml_t, gq,
                       DS_ACT_NONE, s));
        RC(ds_launch_attention(p.qkv, p.qkv + p.qkv_seg, p.qkv + 2 * p.qkv_seg, p.o, (int64_t)d.N * Hd, Hd, Hd,
                               (int64_t)d.N * Hd, p.slot_group, gq, B, d.N, d.H, d.dh, s));
        RC(linear_gemm(p.o, (int64_t)d.N * Hd, Hd, (const bf16_t*)L[4], Hd, (const float*)L[5], p.x, x_ss, 0, 1, p.x, x_ss,
                       0, 0, d.N, 1, 0, 0, 0, p.offs, ml_t, gp, DS_ACT_NONE, s));
        RC(ds_launch_layernorm(xv, av, (const float*)L[6], (const float*)L[7], eps, p.slot_group, gq, B, d.N, 0, d.N, s));
        RC(linear_gemm(p.a, x_ss, 0, (const bf16_t*)L[8], d.D, (const float*)L[9], nullptr, 0, 0, 0, p.h,
                       (int64_t)d.N * d.M, 0, 0, d.N, 1, 0, 0, 0, p.offs, ml_t, g1, DS_ACT_GELU, s));
        RC(linear_gemm(p.h, (int64_t)d.N * d.M, 0, (const bf16_t*)L[10], d.M, (const float*)L[11], p.x, x_ss, 0, 1, p.x,
                       x_ss, 0, 0, d.N, 1, 0, 0, 0, p.offs, ml_t, g2, DS_ACT_NONE, s));
        RC(tap_block(taps, l, p.x, x_ss, 0, p.perm, p.slot_group, g2, B, d.N, d.D, s));
    }
    const void* const* F = P + 4 + 12 * d.depth;
    RC(ds_launch_layernorm(xv, av, (const float*)F[0], (const float*)F[1], eps, p.slot_group, fq, B, d.N, 0, 1, s));
    return ds_launch_head(av, 0, (const bf16_t*)F[2], d.D, (const float*)F[3], d.classes, p.slot_c, p.perm, logits, nullptr,
                          B, d.D, s);
}

}  // namespace

extern "C" size_t ds_forward_workspace(const ds_net* net, int32_t B) {
    if (!net || !net->ints || B <= 0) return 0;
    Bump bp = {nullptr, 0};
    if (net->arch == DS_ARCH_MBNET) {
        MbDesc d;
        MbPlan p;
        if (!parse_mb(net, &d)) return 0;
        plan_mb(d, B, bp, &p);
    } else if (net->arch == DS_ARCH_RESNET) {
        RnDesc d;
        RnPlan p;
        if (!parse_rn(net, &d)) return 0;
        plan_rn(d, B, bp, &p);
    } else if (net->arch == DS_ARCH_VIT || net->arch == DS_ARCH_VIT_STEM) {
        VitDesc d;
        VitPlan p;
        if (!parse_vit(net, &d)) return 0;
        plan_vit(d, B, bp, &p);
    } else {
        return 0;
    }
    return ds_align_up(bp.off, 256);
}

namespace {

// argument and description checks shared by the entry points; on success *image_elems is the size of one image
int32_t check_forward(const char* who, const ds_net* net, const void* images, int32_t B, const float* logits) {
    if (!net || !net->ints || !net->params) DS_FAIL(DS_EINVAL, "%s: null net", who);
    if (B < 0) DS_FAIL(DS_EINVAL, "%s: B < 0", who);
    if (B == 0) return DS_OK;
    if (!images || !logits) DS_FAIL(DS_EINVAL, "%s: null images or logits", who);
    if (!ds_aligned16(images)) DS_FAIL(DS_EALIGN, "%s: images need 16-byte alignment", who);
    for (int i = 0; i < net->n_params; ++i)
        if (!net->params[i] || !ds_aligned16(net->params[i])) DS_FAIL(DS_EINVAL, "%s: parameter %d null or misaligned", who, i);
    if (ds_forward_workspace(net, B) == 0) DS_FAIL(DS_ESHAPE, "%s: network description inconsistent with arch %d", who, net->arch);
    if (net->arch == DS_ARCH_MBNET) {
        MbDesc d;
        parse_mb(net, &d);
        if (d.stem_out % 8) DS_FAIL(DS_EALIGN, "%s: channel counts must be multiples of 8", who);
        for (int i = 0; i < d.nb * (3 + 2 * d.T); ++i)
            if ((i >= 3 * d.nb || i % 3 != 2) && (d.blk[i] % 8)) DS_FAIL(DS_EALIGN, "%s: channel counts must be multiples of 8", who);
        if (d.kfull)
            for (int i = 0; i < d.nb; ++i) {
                const int kf = d.kfull[i];
                if (kf < 1 || kf > 7 || !(kf & 1)) DS_FAIL(DS_EUNSUPPORTED, "%s: stored depthwise filter size %d (odd, at most 7)", who, kf);
                for (int t = 0; t < d.T; ++t) {
                    const int k = d.ksize[t * d.nb + i];
                    if (k < 1 || k > kf || !(k & 1)) DS_FAIL(DS_EINVAL, "%s: kernel size %d is no centred block of %d", who, k, kf);
                }
            }
        return DS_OK;
    }
    if (net->arch == DS_ARCH_RESNET) {
        RnDesc d;
        parse_rn(net, &d);
        if (d.stem_out % 8) DS_FAIL(DS_EALIGN, "%s: channel counts must be multiples of 8", who);
        for (int i = 0; i < 8 * d.T; ++i)
            if (d.mid[i] % 8) DS_FAIL(DS_EALIGN, "%s: channel counts must be multiples of 8", who);
        return DS_OK;
    }
    VitDesc d;
    parse_vit(net, &d);
    const bool dh_ok = d.dh == 32 || d.dh == 48 || d.dh == 64;
    if (d.stem_dim) {
        const int sr = vit_stem_res(d);
        if (!dh_ok || d.N > 224 || d.patch < 1 || (sr % d.patch) || d.N != (sr / d.patch) * (sr / d.patch) + 1)
            DS_FAIL(DS_EUNSUPPORTED, "%s: vit needs head_dim 32, 48 or 64, tokens <= 224, patch dividing the stem's map", who);
        if ((d.stem_dim % 8) || d.stem_dim > 64)
            DS_FAIL(DS_EALIGN, "%s: stem width must be a multiple of 8, at most 64", who);
    } else if (!dh_ok || d.N > 224 || (d.image % d.patch) || d.N != (d.image / d.patch) * (d.image / d.patch) + 1 ||
               (d.patch % 8)) {
        DS_FAIL(DS_EUNSUPPORTED, "%s: vit needs head_dim 32, 48 or 64, tokens <= 224, patch %% 8 == 0", who);
    }
    for (int t = 0; t < d.T; ++t) {
        const int32_t* r = d.routes + d.rs * t;
        if (r[1] < 1 || r[1] > d.H) DS_FAIL(DS_EINVAL, "%s: head count outside 1..%d", who, d.H);
        if ((r[0] % 8) || (r[2] % 8) || r[0] < 8 || r[2] < 8 || r[0] > d.D || r[2] > d.M)
            DS_FAIL(DS_EALIGN, "%s: route widths must be multiples of 8 within the stored widths", who);
        if (d.rs == 4 && (r[3] < 0 || r[3] > d.depth)) DS_FAIL(DS_EINVAL, "%s: route depth outside 0..%d", who, d.depth);
    }
    return DS_OK;
}

// Samples b0 .. b0 + Bp - 1 of a batch of Bs (a checked description): the caller's arrays are addressed at the
// part's offset, the gate-major ones with the whole batch as their stride; ws holds ds_forward_workspace(net, Bp).
int32_t run_part(const ds_net* net, const bf16_t* images, int b0, int Bp, int Bs, const int32_t* route_override,
                 const float* logit_bias, float* logits, int32_t* routes_out, void* ws, hipStream_t s,
                 const Taps* taps = nullptr) {
    Bump bp = {(char*)ws, 0};
    if (net->arch == DS_ARCH_MBNET) {
        MbDesc d;
        MbPlan p;
        parse_mb(net, &d);
        plan_mb(d, Bp, bp, &p);
        return forward_mb(net, d, images + (size_t)b0 * 3 * d.image * d.image, Bp, route_override ? route_override + b0 : nullptr,
                          logit_bias ? logit_bias + (size_t)b0 * d.T : nullptr, logits + (size_t)b0 * d.classes,
                          routes_out ? routes_out + b0 : nullptr, p, s, taps);
    }
    if (net->arch == DS_ARCH_RESNET) {
        RnDesc d;
        RnPlan p;
        parse_rn(net, &d);
        plan_rn(d, Bp, bp, &p);
        return forward_rn(net, d, images + (size_t)b0 * 3 * d.image * d.image, Bp, Bs, route_override ? route_override + b0 : nullptr,
                          logit_bias ? logit_bias + (size_t)b0 * d.T : nullptr, logits + (size_t)b0 * d.classes,
                          routes_out ? routes_out + b0 : nullptr, p, s, taps);
    }
    VitDesc d;
    VitPlan p;
    parse_vit(net, &d);
    plan_vit(d, Bp, bp, &p);
    return forward_vit(net, d, images + (size_t)b0 * 3 * d.image * d.image, Bp, route_override ? route_override + b0 : nullptr,
                       logit_bias ? logit_bias + (size_t)b0 * d.T : nullptr, logits + (size_t)b0 * d.classes,
                       routes_out ? routes_out + b0 : nullptr, p, s, taps);
}

// side streams and fork / join events of ds_forward_parts, made on first use, one set per device, kept until the
// process ends (default priority, no device memory).  A device's set is shared by every call on that device, so
// the caller of part_streams holds the set's mutex while it enqueues: calls from several host threads then
// fork and join one after the other instead of recording over each other's events.
constexpr int MAX_PARTS = 4, MAX_DEVICES = 16;
struct PartStreams {
    std::mutex mu;
    bool ready = false;
    hipStream_t side[MAX_PARTS - 1];
    hipEvent_t fork, join[MAX_PARTS - 1];
};
PartStreams g_part_streams[MAX_DEVICES];

// call with ps.mu of the current device's set held by the returned lock
int32_t part_streams(PartStreams** out, std::unique_lock<std::mutex>* lock) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) DS_FAIL(DS_EHIP, "ds_forward_parts: no current device");
    PartStreams& ps = g_part_streams[dev];
    *lock = std::unique_lock<std::mutex>(ps.mu);
    if (!ps.ready) {
        if (hipEventCreateWithFlags(&ps.fork, hipEventDisableTiming) != hipSuccess) DS_FAIL(DS_EHIP, "ds_forward_parts: event creation failed");
        for (int i = 0; i < MAX_PARTS - 1; ++i)
            if (hipStreamCreateWithFlags(&ps.side[i], hipStreamNonBlocking) != hipSuccess ||
                hipEventCreateWithFlags(&ps.join[i], hipEventDisableTiming) != hipSuccess)
                DS_FAIL(DS_EHIP, "ds_forward_parts: stream creation failed");
        ps.ready = true;
    }
    *out = &ps;
    return DS_OK;
}

int part_size(int B, int parts) {          // samples per part: equal shares rounded up to a multiple of 8
    return (((B + parts - 1) / parts) + 7) & ~7;
}

}  // namespace

extern "C" int32_t ds_forward(const ds_net* net, const void* images, int32_t B, const int32_t* route_override,
                              const float* logit_bias, float* logits, int32_t* routes_out, void* ws, size_t ws_bytes,
                              void* stream) {
    const char* who = "ds_forward";
    const int32_t rc = check_forward(who, net, images, B, logits);
    if (rc || B == 0) return rc;
    const size_t need = ds_forward_workspace(net, B);
    if (!ws || ws_bytes < need || (((uintptr_t)ws) & 255u)) DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    return run_part(net, (const bf16_t*)images, 0, B, B, route_override, logit_bias, logits, routes_out, ws, (hipStream_t)stream);
}

extern "C" int32_t ds_forward_taps(const ds_net* net, const void* images, int32_t B, const int32_t* route_override,
                                   const float* logit_bias, float* logits, int32_t* routes_out, int32_t n_taps,
                                   const int32_t* tap_blocks, void* const* tap_out, void* ws, size_t ws_bytes, void* stream) {
    const char* who = "ds_forward_taps";
    if (n_taps < 0 || n_taps > 64 || (n_taps > 0 && (!tap_blocks || !tap_out))) DS_FAIL(DS_EINVAL, "%s: bad tap list", who);
    for (int i = 0; i < n_taps; ++i)
        if (tap_blocks[i] < 0 || !tap_out[i] || !ds_aligned16(tap_out[i])) DS_FAIL(DS_EINVAL, "%s: tap %d: negative block or bad buffer", who, i);
    const int32_t rc = check_forward(who, net, images, B, logits);
    if (rc || B == 0) return rc;
    const size_t need = ds_forward_workspace(net, B);
    if (!ws || ws_bytes < need || (((uintptr_t)ws) & 255u)) DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    const Taps taps = {n_taps, tap_blocks, tap_out};
    return run_part(net, (const bf16_t*)images, 0, B, B, route_override, logit_bias, logits, routes_out, ws, (hipStream_t)stream,
                    n_taps ? &taps : nullptr);
}

extern "C" size_t ds_forward_parts_workspace(const ds_net* net, int32_t B, int32_t parts) {
    if (B <= 0 || parts < 1 || parts > MAX_PARTS) return 0;
    const int h = part_size(B, parts);
    const size_t one = ds_forward_workspace(net, h < B ? h : B);
    return one * (size_t)((B + h - 1) / h);
}

extern "C" int32_t ds_forward_parts(const ds_net* net, const void* images, int32_t B, const int32_t* route_override,
                                    const float* logit_bias, float* logits, int32_t* routes_out, void* ws, size_t ws_bytes,
                                    int32_t parts, void* stream) {
    const char* who = "ds_forward_parts";
    if (parts < 1 || parts > MAX_PARTS) DS_FAIL(DS_EINVAL, "%s: parts outside 1..%d", who, MAX_PARTS);
    const int32_t rc = check_forward(who, net, images, B, logits);
    if (rc || B == 0) return rc;
    const int h = part_size(B, parts), n = (B + h - 1) / h;
    const size_t one = ds_forward_workspace(net, h < B ? h : B), need = one * (size_t)n;
    if (!ws || ws_bytes < need || (((uintptr_t)ws) & 255u)) DS_FAIL(DS_EWORKSPACE, "%s: workspace needs %zu bytes, 256-byte aligned", who, need);
    hipStream_t s = (hipStream_t)stream;
    if (n == 1) return run_part(net, (const bf16_t*)images, 0, B, B, route_override, logit_bias, logits, routes_out, ws, s);
    PartStreams* ps = nullptr;
    std::unique_lock<std::mutex> enqueue_lock;
    RC(part_streams(&ps, &enqueue_lock));
    // the side streams start after everything already queued on the caller's stream and the caller's stream continues
    // after them: to the caller the call is one piece of work on its stream
    if (hipEventRecord(ps->fork, s) != hipSuccess) DS_FAIL(DS_EHIP, "%s: event record failed", who);
    int32_t first_err = DS_OK;
    for (int i = 0; i < n; ++i) {
        hipStream_t si = i == 0 ? s : ps->side[i - 1];
        if (i > 0 && hipStreamWaitEvent(si, ps->fork, 0) != hipSuccess) DS_FAIL(DS_EHIP, "%s: stream wait failed", who);
        const int b0 = i * h, Bp = b0 + h <= B ? h : B - b0;
        const int32_t r = run_part(net, (const bf16_t*)images, b0, Bp, B, route_override, logit_bias, logits, routes_out,
                                   (char*)ws + one * (size_t)i, si);
        if (r && !first_err) first_err = r;
        if (i > 0) {
            // joined even after an error, so that no side stream is left running behind the caller's back
            if (hipEventRecord(ps->join[i - 1], si) != hipSuccess || hipStreamWaitEvent(s, ps->join[i - 1], 0) != hipSuccess)
                DS_FAIL(DS_EHIP, "%s: join failed", who);
        }
    }
    return first_err;
}
