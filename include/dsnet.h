/*
 * dsnet.h - C ABI of the gate-routed, weight-sliced inference path of DS-Net++
 * (arXiv 2109.10060) for AMD gfx950.
 *
 * The method (Section 3): a routing agent picks one route per input (Section 3.1,
 * Eq. 1; Section 3.5, Eq. 21-22) and every layer of the supernet then computes
 * with the leading contiguous block W[:k_out, :k_in] of its statically stored
 * weight (Section 3.2, Eq. 8), across filters (Eq. 9), depthwise channels
 * (Eq. 10), embedding width, heads and MLP width (Eq. 15-19).  A batch with
 * mixed routes is executed by bucketing samples by route (ds_route_bucket) and
 * running dense kernels per bucket; results equal per-sample execution.
 *
 * Conventions for every call
 *  - Pointers named "device" point to GPU memory owned by the caller; the library
 *    never allocates or frees memory and never writes weights.  Scratch comes
 *    from the caller's workspace `ws` (device, 256-byte aligned) of `ws_bytes`.
 *  - Weights are passed at FULL stored size with their full leading strides;
 *    slices are read in place.  Output elements beyond a sample's valid slice
 *    are not written.
 *  - `stream` is a hipStream_t (NULL = default stream).  Calls enqueue work and
 *    return; nothing synchronises and no route decision is read back to the host.
 *  - Return value: DS_OK or a negative code.  Arguments are validated on the
 *    host before any launch, so a failing call has no device side effects.
 *    ds_last_error() gives a thread-local message.  B == 0 is a valid no-op.
 *  - bf16 tensors need 16-byte aligned base pointers and slice sizes, leading
 *    strides and channel counts that are multiples of 8 (DS_EALIGN otherwise).
 */
#ifndef DSNET_H
#define DSNET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DS_OK            0
#define DS_EINVAL       (-1)  /* null pointer, negative size, slice larger than stored size */
#define DS_ESHAPE       (-2)  /* inconsistent shapes */
#define DS_EALIGN       (-3)  /* pointer / stride / slice not aligned for the bf16 path */
#define DS_EUNSUPPORTED (-4)  /* dtype / layout combination not implemented */
#define DS_EWORKSPACE   (-5)  /* workspace too small or missing */
#define DS_EHIP         (-6)  /* HIP launch error */

#define DS_F32  0
#define DS_BF16 1

#define DS_NCHW 0   /* [B, C, H, W]; weights [C_O, C_I, K, K]                       */
#define DS_NHWC 1   /* [B, H, W, C]; weights [C_O, K, K, C_I]; depthwise [K, K, C]  */

#define DS_ACT_NONE 0
#define DS_ACT_RELU 1
#define DS_ACT_GELU 2   /* exact erf form */

#define DS_MAX_GROUPS 64

/* Route groups of one layer.  Group t covers bucket slots offsets[t]..offsets[t+1]
 * (as written by ds_route_bucket); slot j holds sample perm[j] (NULL = identity).
 * k_in/k_out are the valid input/output widths of the group (the paper's routing
 * spaces are explicit integer lists, so no ratios cross the ABI); table_row picks
 * the row of per-route tables (split batch-norm statistics, Eq. 14).  Host struct. */
typedef struct ds_groups {
    int32_t T;
    const int32_t* offsets;             /* device [T+1] */
    const int32_t* perm;                /* device [B] or NULL */
    int32_t k_in[DS_MAX_GROUPS];
    int32_t k_out[DS_MAX_GROUPS];
    int32_t table_row[DS_MAX_GROUPS];
} ds_groups;

const char* ds_last_error(void);
int32_t ds_version(void);

/* Fold split batch-norm (Eq. 14) into per-route scale/shift tables:
 * scale[t,c] = gamma[c] / sqrt(var[t,c] + eps), shift[t,c] = beta[c] - mean[t,c] * scale[t,c].
 * All device fp32; mean/var/scale/shift are [T, C]. */
int32_t ds_bn_fold(const float* gamma, const float* beta, const float* mean, const float* var,
                   float eps, int32_t T, int32_t C, float* scale, float* shift, void* stream);

/* Re-calibration of the split batch-norm statistics (Section 3.3, the paragraph above Eq. 14:
 * mu_t and sigma_t of every route are re-estimated over a calibration set after training).
 * ds_bn_stats_accumulate streams one batch of pre-normalisation features: for each group t it
 * adds, per valid channel c < k_in[t], the sum and the sum of squares over all pixels of the
 * group's samples to sum[t, c] / sumsq[t, c] and the number of those pixels to count[t].
 * x: device bf16 [B, HW, C] (channels-last, original sample order; group t's samples hold
 * k_in[t] valid channels at channel stride C); sum, sumsq: device fp64 [T, C]; count: device
 * int64 [T]; the caller zeroes all three before the first batch and keeps them across calls.
 * The arithmetic is fp64 in a fixed order (no atomics), so a calibration pass is reproducible.
 * ds_bn_stats_finish turns the totals into mean[t, c] = S / N and the biased variance
 * var[t, c] = Q / N - mean^2 (device fp32 [T, C], ready for ds_bn_fold); width: host int32 [T],
 * the valid channels of each route (NULL = C); a route without samples and the channels at or
 * beyond a route's width get mean 0, variance 1.  T <= DS_MAX_GROUPS. */
size_t ds_bn_stats_workspace(int32_t B, int32_t HW, int32_t C);
int32_t ds_bn_stats_accumulate(const void* x, int32_t B, int32_t HW, int32_t C, const ds_groups* g,
                               double* sum, double* sumsq, int64_t* count, void* ws, size_t ws_bytes,
                               void* stream);
int32_t ds_bn_stats_finish(const double* sum, const double* sumsq, const int64_t* count, int32_t T,
                           int32_t C, const int32_t* width, float* mean, float* var, void* stream);

/* Routing agent (Section 3.5).  Encoder: mean over H*W of each valid channel
 * (Eq. 21).  Head: logits = W2 . relu(W1[:, :c_in[b]] . pooled + b1) + b2
 * (+ logit_bias[b]); route = argmax (Eq. 22 at inference; ties -> lowest index, NaN
 * never selected).  x: device [B,C,HW] (DS_NCHW) or [B,HW,C] (DS_NHWC), fp32 or
 * bf16; x == NULL skips encoder and MLP and routes on logit_bias alone.  c_in:
 * device [B] or NULL (= C).  w1 [C_mlp, C], w2 [T, C_mlp], biases nullable,
 * logit_bias [B,T] nullable: device fp32.  Outputs: logits_out [B,T] fp32,
 * route_out [B] int32 (device).  ws: at least ds_gate_workspace(B, C) bytes
 * (partial sums of the encoder); not needed when x == NULL. */
size_t ds_gate_workspace(int32_t B, int32_t C);
int32_t ds_gate(const void* x, int32_t x_dtype, int32_t x_layout, int32_t B, int32_t C, int32_t HW,
                const int32_t* c_in, const float* w1, const float* b1, int32_t C_mlp,
                const float* w2, const float* b2, int32_t T, const float* logit_bias,
                float* logits_out, int32_t* route_out, void* ws, size_t ws_bytes, void* stream);

/* Double-headed gate (Section 3.5, Eq. 23): the encoder and the hidden vector
 * h = relu(W1[:, :c_in[b]] . pooled + b1) are computed once and feed both heads.
 * Routing head (skipped when w2 == NULL): as ds_gate, logits_out [B,T], route_out [B].
 * Attention head: factor[b,c] = 1 + tanh(W3[c, :] . h + b3[c]) for c < c_in[b], and
 * y[b] = x[b] * factor[b] broadcast over the pixels; y has the type and layout of x
 * (y == x re-weights in place); elements of channels >= c_in[b] are not written.
 * w3 [C, C_mlp], b3 [C] nullable: device fp32, output-sliced to the sample's width.
 * Factors and hidden vectors are accumulated in fp64 and kept in fp32; a bf16 y is
 * rounded once (nearest even) from the fp32 product.  ws: at least
 * ds_gate_double_workspace(B, C) bytes. */
size_t ds_gate_double_workspace(int32_t B, int32_t C);
int32_t ds_gate_double(const void* x, int32_t x_dtype, int32_t x_layout, int32_t B, int32_t C, int32_t HW,
                       const int32_t* c_in, const float* w1, const float* b1, int32_t C_mlp,
                       const float* w2, const float* b2, int32_t T, const float* logit_bias,
                       const float* w3, const float* b3, float* logits_out, int32_t* route_out, void* y,
                       void* ws, size_t ws_bytes, void* stream);

/* Bucket a batch by route: offsets[t] = #samples with route < t (offsets[T] counts
 * the samples with a valid id, so offsets[T] != B flags an id outside [0,T));
 * perm lists samples bucket by bucket, ascending inside a bucket (stable);
 * inv_perm[perm[j]] = j.  All device int32.  1 <= T <= 1024. */
int32_t ds_route_bucket(const int32_t* route, int32_t B, int32_t T, int32_t* perm,
                        int32_t* inv_perm, int32_t* offsets, void* stream);

/* Sliced linear layer (Eq. 8): for every sample b of group t and each of its
 * `rows` rows, y[b, r, :k_out] = act(x[b, r, :k_in] . W[:k_out, :k_in]^T + bias[:k_out])
 * with the residual, when given, added before the activation:
 * act(x W^T + bias + residual).  x: device bf16 [B, rows, x_ld]; W: device bf16
 * [N_full, w_ld]; bias: device fp32 [N_full] or NULL; residual: device bf16
 * [B, rows, r_ld] or NULL; y: device [B, rows, y_ld], bf16 or fp32.  Samples stay
 * in their original order in x and y. */
size_t ds_sliced_linear_workspace(int32_t B, int32_t rows, int32_t T);
int32_t ds_sliced_linear(const void* x, int64_t x_ld, const void* w, int64_t w_ld, int32_t N_full,
                         int32_t K_full, const float* bias, const ds_groups* g, int32_t B,
                         int32_t rows, int32_t act, const void* residual, int64_t r_ld, void* y,
                         int32_t y_dtype, int64_t y_ld, void* ws, size_t ws_bytes, void* stream);

/* ds_sliced_linear for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments, results and errors, without the
 * workspace.  The row-tile list the kernels read is kept in a device array built into the library
 * (DS_NOALLOC_MAX_TILES records of 16 bytes, 512 KiB + 256 bytes per GPU the library has run on, held
 * until the process ends); the call allocates and frees nothing and switches the ds_profile_* recording
 * off for its duration.  (B * rows + 127) / 128 + T must not exceed DS_NOALLOC_MAX_TILES
 * (DS_EWORKSPACE otherwise, before any launch).  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams or threads) race and must be ordered by the caller. */
#define DS_NOALLOC_MAX_TILES 32768
int32_t ds_sliced_linear_noalloc(const void* x, int64_t x_ld, const void* w, int64_t w_ld, int32_t N_full,
                                 int32_t K_full, const float* bias, const ds_groups* g, int32_t B,
                                 int32_t rows, int32_t act, const void* residual, int64_t r_ld, void* y,
                                 int32_t y_dtype, int64_t y_ld, void* stream);

/* Sliced dense convolution with split batch-norm (Eq. 9 and Eq. 14):
 * y[b, :c_out] = act(scale[row, :c_out] * (W[:c_out, :c_in] * x[b, :c_in]) + shift[row, :c_out]
 *                    + residual[b, :c_out]),  row = table_row[t].
 * Supported: (DS_F32, DS_NCHW) direct kernel; (DS_BF16, DS_NHWC) matrix-core
 * implicit GEMM.  x: [B, C_I, H, W] / [B, H, W, C_I]; y: [B, C_O, Ho, Wo] /
 * [B, Ho, Wo, C_O] at full channel stride; scale/shift: device fp32 [n_rows, C_O]
 * (scale NULL = 1); residual: like y, or NULL. */
size_t ds_sliced_conv_workspace(int32_t B, int32_t Ho, int32_t Wo, int32_t T);
int32_t ds_sliced_conv(const void* x, int32_t dtype, int32_t layout, int32_t B, int32_t C_I,
                       int32_t H, int32_t W, const void* w, int32_t C_O, int32_t K,
                       const float* scale, const float* shift, const ds_groups* g, int32_t stride,
                       int32_t pad, int32_t act, const void* residual, void* y, void* ws,
                       size_t ws_bytes, void* stream);

/* Sliced depthwise 3x3 convolution (Eq. 10, one channel per group) with split
 * batch-norm and activation; output width = input width = k_in[t].  bf16 NHWC;
 * w: device bf16 [3, 3, C]; scale/shift device fp32 [n_rows, C]. */
size_t ds_slot_workspace(int32_t B);   /* workspace of ds_sliced_dwconv / ds_sliced_layernorm */
int32_t ds_sliced_dwconv(const void* x, int32_t B, int32_t C, int32_t H, int32_t W, const void* w,
                         const float* scale, const float* shift, const ds_groups* g,
                         int32_t stride, int32_t act, void* y, void* ws, size_t ws_bytes,
                         void* stream);

/* Depthwise convolution with a spatially sliced filter (Section 3.2: kernel size Eq. 11,
 * dilation Eq. 12, padding Eq. 13).  The filter is stored once as K x K taps (K odd, at most 7;
 * w: device bf16 [K, K, C]).  Group t uses the centred ksize[t] x ksize[t] block of it
 * (K - ksize[t] even), of that block every dilation[t]-th tap, applied at dilation[t] (the taps
 * keep the spacing they have in the stored filter), with pad[t] zeros on each side; its output is
 * Ho_t x Wo_t = (H + 2 pad - span) / stride + 1 with span = (ceil(ksize / dilation) - 1) dilation + 1.
 * With pad[t] = (K - 1) / 2 - (K - ksize[t]) / 2 this equals the full K x K filter with the
 * unselected taps zeroed and padding (K - 1) / 2.  Split batch-norm and activation as in
 * ds_sliced_dwconv.  x: device bf16 [B, H, W, C]; y: device bf16, sample b at
 * y + b * y_sample_stride, holding [Ho_t, Wo_t, C] packed (row stride Wo_t * C, channel stride C,
 * channels beyond k_in[t] not written); y_sample_stride >= Ho_t * Wo_t * C for every group.
 * Host struct. */
typedef struct ds_spatial {
    int32_t ksize[DS_MAX_GROUPS];
    int32_t dilation[DS_MAX_GROUPS];
    int32_t pad[DS_MAX_GROUPS];
} ds_spatial;
int32_t ds_sliced_dwconv_spatial(const void* x, int32_t B, int32_t C, int32_t H, int32_t W,
                                 const void* w, int32_t K, const float* scale, const float* shift,
                                 const ds_groups* g, const ds_spatial* sp, int32_t stride,
                                 int32_t act, void* y, int64_t y_sample_stride, void* ws,
                                 size_t ws_bytes, void* stream);

/* Global average pool and classifier with sliced input width (the "Pool + FC" row of the routing-space tables,
 * Section 5.2): logits[b, :] = W[:, :k_in[t]] . mean over the HW pixels of x[b, :, :k_in[t]] + bias for every sample b of
 * group t.  x: device bf16 [B, HW, C] (channels-last, original sample order, C = stored width); w: device bf16
 * [n_out, C]; bias: device fp32 [n_out] or NULL; logits: device fp32 [B, n_out]; the mean and the products are
 * accumulated in fp32.  ws: ds_pool_head_workspace(B, C) bytes. */
size_t ds_pool_head_workspace(int32_t B, int32_t C);
int32_t ds_pool_head(const void* x, int32_t B, int32_t HW, int32_t C, const void* w, const float* bias,
                     int32_t n_out, const ds_groups* g, float* logits, void* ws, size_t ws_bytes, void* stream);

/* 3x3 stride-2 padding-1 max-pool of the ResNet-shaped stem (Section 5.2, DS-ResNet): x device bf16 [B, H, W, C],
 * y device bf16 [B, (H - 1) / 2 + 1, (W - 1) / 2 + 1, C]; padding never wins (it counts as minus infinity). */
int32_t ds_maxpool(const void* x, int32_t B, int32_t H, int32_t W, int32_t C, void* y, void* stream);

/* LayerNorm over the k_in[t] valid features of each row with gamma[:k], beta[:k]
 * (the statistics use the valid features only).  x, y: device bf16 [B, rows, ld]. */
int32_t ds_sliced_layernorm(const void* x, int64_t x_ld, const float* gamma, const float* beta,
                            float eps, const ds_groups* g, int32_t B, int32_t rows, void* y,
                            int64_t y_ld, void* ws, size_t ws_bytes, void* stream);

/* Sliced multi-head self-attention (Eq. 16-18): Q,K,V = x[:, :d_e] . W{q,k,v}[:h*Dh, :d_e]^T + b;
 * per head j < h: softmax(Q_j K_j^T / sqrt(Dh)) V_j; y = concat . Wproj[:d_e, :h*Dh]^T + bproj
 * (+ residual).  Group t uses d_e = k_in[t] and h*Dh = k_out[t].  x, residual, y:
 * device bf16 [B, N, D_e]; wqkv: device bf16 [3, H*Dh, D_e] (Wq, Wk, Wv stacked, each
 * sliced to its own leading block); bqkv: device fp32 [3, H*Dh] or NULL; wproj:
 * device bf16 [D_e, H*Dh]; bproj: device fp32 [D_e] or NULL.  head_dim must be 32, 48
 * or 64 (DS-ViT++'s Q-K-V widths 192..384 in steps of 48 with 4..8 heads are 8 stored heads
 * of 48), N <= 224. */
size_t ds_sliced_mhsa_workspace(int32_t B, int32_t N, int32_t H, int32_t head_dim, int32_t T);
int32_t ds_sliced_mhsa(const void* x, int32_t B, int32_t N, int32_t D_e, const void* wqkv,
                       const float* bqkv, const void* wproj, const float* bproj, int32_t H,
                       int32_t head_dim, const ds_groups* g, const void* residual, void* y,
                       void* ws, size_t ws_bytes, void* stream);

/* Whole-network forward (Section 5.2 assemblies).  arch selects the graph; `ints`
 * is the host integer description and `params` the device parameter pointers, in
 * the order documented next to each DS_ARCH_* below.  images: device bf16
 * [B, 3, image, image]; route_override: device int32 [n_gates, B] or NULL;
 * logit_bias: device fp32 [n_gates, B, T] or NULL; logits: device fp32
 * [B, num_classes] in the original sample order; routes_out: device int32
 * [n_gates, B]. */
/* DS_ARCH_MBNET: MobileNetV1-shaped net, one gate after block `gate_after` (Section 5.2, DS-MBNet).
 *   ints:   image, stem_out, n_blocks, gate_after, gate_hidden, T, num_classes,
 *           n_blocks x (C_in, C_out, stride), cin[T][n_blocks], cout[T][n_blocks] (valid widths per route),
 *           optionally kfull[n_blocks], ksize[T][n_blocks] (DS-MBNet++, Eq. 11): block i stores a
 *           kfull[i] x kfull[i] depthwise filter (odd, at most 7) and route t uses its centred
 *           ksize[t][i] x ksize[t][i] block at padding (ksize - 1) / 2, so the resolution does not
 *           depend on the route; blocks before the gate use row 0
 *   params: stem.w bf16 [3*3*3][stem_out] (tap-major, input channel, then filters), stem.scale, stem.shift,
 *           per block: dw.w bf16 [k][k][C_in] (k = 3, or kfull[i]), dw.scale, dw.shift fp32 [Tb][C_in], pw.w bf16 [C_out][C_in],
 *           pw.scale, pw.shift fp32 [Tb][C_out] (Tb = 1 before the gate, T after),
 *           gate.w1 [gate_hidden][C], gate.b1, gate.w2 [T][gate_hidden], gate.b2 (fp32),
 *           fc.w bf16 [num_classes][C_last], fc.b fp32. */
#define DS_ARCH_MBNET  1
/* DS_ARCH_RESNET: bottleneck ResNet, a gate in the first block of each of 4 stages (DS-ResNet).
 *   ints:   image, stem_out, T, num_classes, widths[4], blocks[4], gate_hidden[4], mid[4][T], out[4][T],
 *           optionally nblk[4][T]: route t runs only the first nblk[s][t] (1..blocks[s]) blocks of
 *           stage s (dynamic depth, Section 3.4); its slots pass through the later blocks unchanged;
 *           after nblk optionally one flags word: bit 0 = the gate of the first stage decides for all
 *           four stages (DS-ResNet++, Section 5.2), the other gates' parameters are not read and
 *           routes_out repeats the first row
 *   params: stem.w bf16 [7*7*3][stem_out], stem.scale, stem.shift,
 *           per stage: gate.w1, gate.b1, gate.w2, gate.b2 (fp32), then per block
 *             c1.w bf16 [w][1][1][C_in], c1.scale, c1.shift fp32 [T][w],
 *             c2.w bf16 [w][3][3][w], c2.scale, c2.shift, c3.w bf16 [4w][1][1][w], c3.scale, c3.shift [T][4w],
 *             first block only: proj.w bf16 [4w][1][1][C_in], proj.scale, proj.shift,
 *           fc.w bf16 [num_classes][4*w_last], fc.b fp32. */
#define DS_ARCH_RESNET 2
/* DS_ARCH_VIT: pre-LN vision transformer, one route per image chosen before the patch embedding (DS-ViT).
 *   ints:   image, patch, embed, heads, head_dim, mlp, depth, tokens, T, num_classes,
 *           routes[T][3] = (d_e, heads, hidden), or routes[T][4] = (d_e, heads, hidden, blocks):
 *           with the fourth entry a route runs only the first `blocks` (0..depth) of the stored
 *           layers (dynamic depth, Section 3.4); the remaining layers leave its tokens untouched
 *   params: embed.w bf16 [embed][3*patch*patch], embed.b, cls bf16 [embed], pos bf16 [tokens][embed],
 *           per layer: ln1.g, ln1.b, wqkv bf16 [3][heads*head_dim][embed], bqkv fp32 [3][heads*head_dim],
 *             wproj bf16 [embed][heads*head_dim], bproj, ln2.g, ln2.b, fc1.w bf16 [mlp][embed], fc1.b,
 *             fc2.w bf16 [embed][mlp], fc2.b,
 *           ln.g, ln.b, head.w bf16 [num_classes][embed], head.b.
 *   Routes come from logit_bias (argmax) or route_override; one of them is required. */
#define DS_ARCH_VIT    3
/* DS_ARCH_VIT_STEM: DS_ARCH_VIT behind the convolutional stem of Section 3.4 (blocks [c, ds, ds, c]): a 7x7
 * stride-2 padding-3 convolution and two depthwise-separable blocks (3x3 depthwise, 1x1 pointwise), each
 * layer with folded batch-norm and ReLU, all at stem_dim channels and never sliced; the gate (Eq. 21-22)
 * pools the stem's feature map and picks the route (logit_bias and route_override optional, as for the
 * CNNs); the patch embedding is the stem's last convolution, patch x patch with stride patch and no
 * padding over that map, its filters sliced to the route's d_e.  tokens = ((image / 2) / patch)^2 + 1.
 *   ints:   image, patch, embed, heads, head_dim, mlp, depth, tokens, T, num_classes,
 *           rs (3 or 4 entries per route), stem_dim (multiple of 8, <= 64), gate_hidden, routes[T][rs]
 *   params: stem.c0.w bf16 [7*7*3][stem_dim], stem.c0.scale, stem.c0.shift fp32 [stem_dim],
 *           2 x (dw.w bf16 [3][3][C], dw.scale, dw.shift fp32 [C], pw.w bf16 [C][C], pw.scale, pw.shift),
 *           gate.w1 [gate_hidden][C], gate.b1, gate.w2 [T][gate_hidden], gate.b2 (fp32),
 *           embed.w bf16 [embed][patch][patch][C], then as DS_ARCH_VIT from embed.b on. */
#define DS_ARCH_VIT_STEM 4
typedef struct ds_net {
    int32_t arch;
    int32_t n_ints;
    const int32_t* ints;            /* host */
    int32_t n_params;
    const void* const* params;      /* host array of device pointers */
} ds_net;
size_t ds_forward_workspace(const ds_net* net, int32_t B);
int32_t ds_forward(const ds_net* net, const void* images, int32_t B, const int32_t* route_override,
                   const float* logit_bias, float* logits, int32_t* routes_out, void* ws,
                   size_t ws_bytes, void* stream);
/* ds_forward that also hands out the outputs of chosen blocks, for checking a network layer by layer against a
 * reference (Section 5.2 assemblies; a block is a depthwise-separable block of DS-MBNet, a bottleneck of DS-ResNet
 * counted over all stages, a transformer layer of DS-ViT, each numbered from 0 in execution order).  tap_blocks:
 * host int32 [n_taps] (n_taps <= 64); tap_out: host array of n_taps device buffers, bf16 [B, rows, C_stored] of that
 * block's output resolution and stored width, original sample order, channels-last; of each sample only its valid
 * slice [rows, :c_out] is written (a sample whose route skips the block is not written at all).  Everything else
 * as ds_forward, same workspace. */
int32_t ds_forward_taps(const ds_net* net, const void* images, int32_t B, const int32_t* route_override,
                        const float* logit_bias, float* logits, int32_t* routes_out, int32_t n_taps,
                        const int32_t* tap_blocks, void* const* tap_out, void* ws, size_t ws_bytes, void* stream);
/* The same forward pass with the batch run as `parts` (1..4) concurrent pieces: samples are independent (Section 3.1,
 * Eq. 1: the route and the sliced computation are per input), so the batch is cut into equal shares (rounded up to
 * a multiple of 8 samples), each share is gated, bucketed and computed on its own — the first on `stream`, the others
 * on streams the library creates on first use (up to 3 per device, default priority, kept until the process ends) —
 * and the launch ramps and tails of one share's kernels are filled by the other's.  The side streams start after the
 * work already queued on `stream` and `stream` continues after them, so to the caller the call is one piece of work
 * on `stream`.  Arguments, results and errors as ds_forward (every output is per sample, hence identical); ws needs
 * ds_forward_parts_workspace(net, B, parts) bytes (0 for parts outside 1..4).  parts = 1 is ds_forward.
 * Calls that overlap in time on one device share the side streams and are serialised by them. */
size_t ds_forward_parts_workspace(const ds_net* net, int32_t B, int32_t parts);
int32_t ds_forward_parts(const ds_net* net, const void* images, int32_t B, const int32_t* route_override,
                         const float* logit_bias, float* logits, int32_t* routes_out, void* ws,
                         size_t ws_bytes, int32_t parts, void* stream);

/* Instrumentation: while recording is on, every kernel launch is bracketed by a pair of HIP
 * events on its stream.  The event packets keep consecutive kernels from overlapping their
 * launch and drain phases (10-15 % on the batch-256 networks), so a caller that wants both a
 * throughput figure and kernel durations switches recording on for a sample of its steps only:
 * ds_profile_enable(1) resumes recording, ds_profile_enable(0) pauses it, records accumulate until
 * ds_profile_reset().  ds_profile_read waits for the recorded events and returns the summed
 * milliseconds and launch count of one kernel class: 0 grouped GEMM on linear/1x1 layers,
 * 1 grouped GEMM walking KxK taps, 2 attention, 3 depthwise conv, 4 LayerNorm, 5 stem conv,
 * 6 max-pool, 7 pool+classifier, 8 gate, 9 bucket, 10 index helpers, 11 3x3 stride-1 convolution with the
 * patch staged once, 12 short-reduction 1x1 layers (one workgroup per row tile).  ds_profile_launches gives the
 * recorded launches one by one in launch order: kinds[i] and ms[i] for i < min(*count, capacity), *count = the number
 * recorded.  Not thread-safe; host pointers. */
int32_t ds_profile_enable(int32_t on);
int32_t ds_profile_reset(void);
int32_t ds_profile_read(int32_t kind, double* total_ms, int64_t* launches);
int32_t ds_profile_launches(int32_t* kinds, float* ms, int64_t capacity, int64_t* count);

#ifdef __cplusplus
}
#endif
#endif /* DSNET_H */
