/*
 * cprune.h - C ABI of the MI355X (gfx950) hot path of compiler-informed channel
 * pruning: L1-norm filter ranking, weight / activation channel gather with
 * batch-norm folding, MFMA implicit-GEMM convolution with fused bias,
 * residual and activation, the memory-bound layers around it, per-shape kernel
 * variant selection by timing on the device, and whole-network inference.
 *
 * Conventions for every call
 *   - Returns an int status: CPRUNE_OK (0) or a negative CPRUNE_ERR_* code.  On an
 *     argument error nothing is launched and no output is touched.
 *   - Unless marked "host", pointers are DEVICE pointers owned by the caller;
 *     tensors are dense NCHW (activations) / OIHW (weights), row-major.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it and return; the exceptions (they
 *     synchronise) are cprune_select_tile, cprune_net_create,
 *     cprune_net_layer_times and cprune_net_destroy.
 *   - The library allocates device memory only inside a cprune_net handle.
 *     Other calls take scratch from the caller: `ws` / `ws_bytes`, sized by the
 *     matching *_workspace_bytes query; too little -> CPRUNE_ERR_WORKSPACE.
 *   - Index lists are int32, strictly ascending, in range.  Device-resident
 *     lists cannot be validated by the host; kernels clamp an index into range
 *     instead of faulting, so a bad list gives wrong values, not a fault.
 *   - Tensors must hold fewer than 2^31 elements.
 */
#ifndef CPRUNE_H
#define CPRUNE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CPRUNE_OK 0
#define CPRUNE_ERR_INVALID_ARG (-1) /* NULL / out-of-range argument */
#define CPRUNE_ERR_UNSUPPORTED (-2) /* valid but not implemented (dtype, groups, variant) */
#define CPRUNE_ERR_WORKSPACE (-3)   /* ws_bytes below the *_workspace_bytes query */
#define CPRUNE_ERR_DEVICE (-4)      /* a HIP call failed; see cprune_last_hip_error */
#define CPRUNE_ERR_NOT_TUNED (-5)   /* reserved */

typedef enum { CPRUNE_F32 = 0, CPRUNE_F16 = 1, CPRUNE_BF16 = 2 } cprune_dtype;
typedef enum { CPRUNE_ACT_NONE = 0, CPRUNE_ACT_RELU = 1, CPRUNE_ACT_RELU6 = 2 } cprune_act;

const char* cprune_status_string(int status); /* host string, never NULL */
int cprune_last_hip_error(void);              /* hipError_t of the last CPRUNE_ERR_DEVICE */

/* ------------------------------------------------------------------------
 * Filter ranking (paper Section 3.5, last paragraph: each filter is scored by
 * the sum of its absolute weights and filters are pruned starting from the
 * smallest sum).
 *
 * w            [c_out][c_in_per_group][kh][kw] fp32, the raw (unfolded) weights
 * keep         number of filters that survive, 1..c_out
 * scores_out   [c_out] double, the L1 sums (fp64 accumulation); may be NULL
 * order_out    [c_out] int32, filter indices by (score descending, index
 *              ascending): equal scores rank the lower index first; may be NULL
 * kept_out     [keep] int32, the surviving filters in ascending index order
 * ws           cprune_rank_filters_workspace_bytes(c_out) bytes of scratch
 * The kept list is a pure function of the scores; the scores are summed in a
 * fixed order, so repeated calls give identical bits.
 */
size_t cprune_rank_filters_workspace_bytes(int c_out);
int cprune_rank_filters(const float* w, int c_out, int c_in_per_group, int kh, int kw, int keep,
                        double* scores_out, int32_t* order_out, int32_t* kept_out,
                        void* ws, size_t ws_bytes, void* stream);

/* cprune_rank_filters for callers that cannot allocate or hand over scratch memory (code under
 * HIP graph capture, serving loops, harnesses that forbid hipMalloc): the scores live in an
 * array the library holds in each device's memory for the life of the process
 * (cprune_rank_filters_static_max() = 4096 doubles, 32 KiB), so there is no ws argument, no
 * scores_out, and the call allocates nothing.  c_out above that maximum:
 * CPRUNE_ERR_UNSUPPORTED.  Same kernels and results as cprune_rank_filters.  Every call on a
 * device shares that device's array: calls that overlap on one device (two streams, two
 * threads) race; calls on one stream are ordered.  Nothing needs clearing between calls:
 * every score the ranking reads is written by the same call first. */
int cprune_rank_filters_static_max(void);
int cprune_rank_filters_static(const float* w, int c_out, int c_in_per_group, int kh, int kw,
                               int keep, int32_t* order_out, int32_t* kept_out, void* stream);

/* Ranking of a group of layers that must lose the same channels (Section 3.5, last
 * paragraph: the layers whose outputs a shortcut adds are pruned at the same output
 * channels).  A channel's score is the sum, in member order, of its filter's L1 sum in every
 * member.  w: HOST array of n_members device pointers, member m being
 * [c_out][per_filter[m]] fp32; per_filter: HOST array of filter lengths
 * (c_in_per_group * kh * kw).  Everything else as cprune_rank_filters. */
int cprune_rank_filter_group(const float* const* w, const int64_t* per_filter, int n_members,
                             int c_out, int keep, double* scores_out, int32_t* order_out,
                             int32_t* kept_out, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Weight gather with batch-norm folding (paper Section 2.1 / Fig. 2: removing a
 * filter removes an output channel, removing an input channel shrinks every
 * filter; Section 3.5: the next layer's input channels are pruned to match).
 *
 *   w_out[i][c][u][v] = s_i * w[keep_out[i]][keep_in[c]][u][v]
 *   bias_out[i]       = beta + (conv_bias - mean) * s_i,  s_i = gamma / sqrt(var + eps)
 * with gamma, beta, mean, var, conv_bias taken at keep_out[i]; computed in fp64
 * and rounded once.  gamma..var all NULL = no BN (s = 1, bias = conv_bias or 0).
 *
 * w            [c_out][c_in][kh][kw] fp32 source (c_in = channels per filter)
 * keep_out     [n_keep_out] or NULL (= all c_out filters, n_keep_out ignored)
 * keep_in      [n_keep_in]  or NULL (= all c_in channels, n_keep_in ignored)
 * out_dtype    element type of w_out (fp32, fp16 or bf16, round-to-nearest-even)
 * w_out        [n_keep_out][n_keep_in][kh][kw]; bias_out [n_keep_out] fp32, may be
 *              NULL when there is neither BN nor conv_bias
 */
int cprune_gather_pruned_weights(const float* w, int c_out, int c_in, int kh, int kw,
                                 const int32_t* keep_out, int n_keep_out,
                                 const int32_t* keep_in, int n_keep_in,
                                 const float* gamma, const float* beta, const float* mean,
                                 const float* var, float eps, const float* conv_bias,
                                 cprune_dtype out_dtype, void* w_out, float* bias_out,
                                 void* stream);

/* The ranking and gather of a whole network as one plan (the pruning step of Algorithm 1:
 * the filters chosen per Section 3.5 are removed from every layer they touch and the next
 * layers' input channels follow, Section 2.1 / Fig. 2).  Same arithmetic as the two calls
 * above, layer by layer; three launches per run whatever the number of layers: every ranked
 * layer's scores, every ranked layer's kept list, every layer's gathered and folded weights.
 *
 * One entry per layer, in network order (host array):
 *   w            device, raw fp32 weights [c_out][c_in][kh][kw] (c_in = channels per filter;
 *                a fully connected layer behind a c x h x w map is c_in = c, kh x kw = h x w);
 *                NULL = a layer without weights (a pool): every other field 0 / -1 / NULL
 *   keep         > 0: the layer's filters are ranked and `keep` survive (rows_from must be the
 *                layer's own index); 0: not ranked
 *   score_with   host [n_score_with] indices of layers with the same c_out whose filter sums
 *                are added to this ranked layer's, in this order (cprune_rank_filter_group)
 *   rows_from    -1: every filter stays; else the ranked layer whose kept list selects this
 *                layer's filters
 *   cols_from    -1: every input channel stays; else the ranked layer whose kept list selects
 *                this layer's input channels (that layer's c_out = this layer's c_in)
 *   gamma..var, conv_bias   device fp32 [c_out] or NULL, as cprune_gather_pruned_weights
 *   w_out        device [rows kept][columns kept][kh][kw] in the plan's dtype
 *   bias_out     device fp32 [rows kept]; may be NULL when there is neither BN nor conv_bias
 *   kept_out     device int32 [keep], ascending; required for ranked layers
 * The plan owns a few KB of device memory (its tables and the scores); inputs and outputs
 * stay the caller's and must outlive it.  create and destroy synchronise; run only enqueues. */
typedef struct {
  const float* w;
  int32_t c_out, c_in, kh, kw;
  int32_t keep;
  int32_t rows_from, cols_from;
  const int32_t* score_with;
  int32_t n_score_with;
  const float *gamma, *beta, *mean, *var, *conv_bias;
  void* w_out;
  float* bias_out;
  int32_t* kept_out;
} cprune_prune_layer;
typedef struct cprune_prune_plan cprune_prune_plan;
int cprune_prune_plan_create(const cprune_prune_layer* layers, int n_layers, float eps,
                             cprune_dtype out_dtype, cprune_prune_plan** out);
int cprune_prune_plan_run(cprune_prune_plan* plan, void* stream);
/* Weight elements one run reads (scoring + gather) and writes; host outs. */
int cprune_prune_plan_traffic(const cprune_prune_plan* plan, int64_t* weights_read_out,
                              int64_t* weights_written_out);
int cprune_prune_plan_destroy(cprune_prune_plan* plan);

/* Activation channel gather (Section 2.1: removing input channels c_i):
 * y[n][i][h][w] = x[n][idx[i]][h][w]; x [n][c][h][w], y [n][n_idx][h][w], same dtype. */
int cprune_gather_channels(const void* x, int n, int c, int h, int w, cprune_dtype dtype,
                           const int32_t* idx, int n_idx, void* y, void* stream);

/* ------------------------------------------------------------------------
 * Convolution subgraph (paper Section 3.4: a subgraph is Conv2d (+BN) (+ReLU);
 * this is the device program whose latency the method measures).
 *
 *   y[n][o][p][q] = act( bias[o] + sum_{c,u,v} x[n][c][p*stride+u-pad][q*stride+v-pad]
 *                                              * w[o][c][u][v]  (+ residual[n][o][p][q]) )
 * cross-correlation, zero padding, h_out = (h + 2 pad - kh) / stride + 1 (floor).
 * groups = 1: dense, runs as an implicit GEMM on MFMA (fp32 accumulate).
 * groups = c_in = c_out: depthwise, a bandwidth-bound stencil kernel.
 */
typedef struct {
  int32_t n, c_in, h, w;   /* input  [n][c_in][h][w] */
  int32_t c_out, kh, kw;   /* weight [c_out][c_in/groups][kh][kw] */
  int32_t stride, pad;
  int32_t groups;          /* 1, or c_in (with c_out == c_in) */
  int32_t dtype;           /* cprune_dtype of x, w, residual, y; bias is always fp32 */
  int32_t act;             /* cprune_act */
  int32_t has_residual;    /* 0 / 1 */
} cprune_conv_desc;

/* Kernel variants of the dense path: a work-group tile (output channels x
 * output pixels) and a scheduling mode.  sched 0: one output tile per work-group.
 * sched n > 0: the (tile, reduction slab) work is laid out in one line and cut
 * into equal runs for n * 256 work-groups; tiles cut between runs go through the
 * caller's scratch and are summed in run order (deterministic).  sched -1: kernels that
 * exist only for the channels-last layout inside a network handle (3x3 stride-1 layers,
 * one tile_p-pixel spatial block per work-group); unsupported through this NCHW call.
 * sched -2: likewise channels-last only, for layers whose reduction is one contiguous run
 * per pixel (1x1 stride 1, fully connected): 16 filters x tile_p pixels per work-group, the
 * wavefronts of the group splitting the reduction; chosen when pixels are few.
 * sched -3: channels-last 1x1 / stride 1 layers with a short reduction (at most 384 bytes per
 * pixel): persistent work-groups keep a tile of at most 128 filters in local memory and stream
 * 64-pixel tiles through it.
 * sched -4: channels-last 3x3 / stride 1 / pad 1 layers on maps of at most 16 x 16: 16 filters x
 * tile_p pixels (4 x 4 blocks) per work-group, one wavefront per (block, slice of the
 * reduction), the slices summed inside the group; chosen for small maps with many channels.
 * Ids are 0..n-1
 * and the same for every shape; a variant that cannot run a given shape is
 * CPRUNE_ERR_UNSUPPORTED. */
int cprune_num_tile_variants(void);
int cprune_tile_variant_info(int variant, int* tile_m, int* tile_p, int* sched); /* host out */
/* The kernel instantiation behind a variant, written as profilers print it (e.g.
 * "conv_patch_kernel<float, 1, 8, 8, 1, 1, 1>"): channels_last = 0 names the NCHW kernel of
 * cprune_conv2d_bn_relu, 1 the one used inside a network handle.  buf: host, buf_bytes >= 96. */
int cprune_tile_variant_name(int variant, int channels_last, cprune_dtype dtype, char* buf,
                             size_t buf_bytes);

/* Scratch needed by `variant` (-1 = the largest any variant needs for desc). */
size_t cprune_conv_workspace_bytes(const cprune_conv_desc* desc, int variant);

/* bias may be NULL (= 0); residual must be non-NULL iff desc->has_residual.
 * tile_variant -1 = the variant remembered for this shape by cprune_select_tile,
 * or a built-in heuristic when the shape has not been timed. */
int cprune_conv2d_bn_relu(const cprune_conv_desc* desc, const void* x, const void* w_folded,
                          const float* bias, const void* residual, void* y, int tile_variant,
                          void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * Variant selection by timing on the device (paper Section 3.1, Fig. 3: for each
 * task the compiler generates candidate programs and keeps the one that runs
 * fastest on the target; layers of equal shape share a task).  Times every
 * variant that supports desc with `warmup` untimed and `iters` timed launches on
 * the caller's buffers (y and ws are overwritten), remembers the fastest for
 * this shape (process-wide, keyed by every field of desc) and returns it.
 * all_ms_out: host [cprune_num_tile_variants()] per-launch ms, < 0 where
 * unsupported; may be NULL.  variant_out / best_ms_out: host.  Synchronises.
 */
int cprune_select_tile(const cprune_conv_desc* desc, const void* x, const void* w_folded,
                       const float* bias, const void* residual, void* y, void* ws,
                       size_t ws_bytes, int warmup, int iters, int* variant_out,
                       float* best_ms_out, float* all_ms_out, void* stream);
/* Forget every remembered choice. */
void cprune_clear_tile_cache(void);
/* The remembered (or heuristic) variant for desc; host out. */
int cprune_cached_tile(const cprune_conv_desc* desc, int* variant_out, int* was_timed_out);

/* ------------------------------------------------------------------------
 * Memory-bound layers of the evaluated networks (the VGG-16 of the motivating
 * experiment of Section 3, Fig. 1; ResNet-18 and MobileNetV2 of Section 4, Table 1).
 */
/* max over the in-bounds elements of each k x k window; y [n][c][ho][wo] */
int cprune_maxpool2d(const void* x, int n, int c, int h, int w, int k, int stride, int pad,
                     cprune_dtype dtype, void* y, void* stream);
/* spatial mean; y [n][c] */
int cprune_global_avgpool(const void* x, int n, int c, int h, int w, cprune_dtype dtype,
                          void* y, void* stream);
/* y[n][o] = act(bias[o] + sum_f x[n][f] w[o][f]); runs on the dense conv path. */
size_t cprune_fc_workspace_bytes(int n, int f, int c_out, cprune_dtype dtype);
int cprune_fc(const void* x, const void* w, const float* bias, int n, int f, int c_out,
              cprune_act act, cprune_dtype dtype, void* y, void* ws, size_t ws_bytes,
              void* stream);

/* ------------------------------------------------------------------------
 * Whole-network inference (paper Algorithm 1: run the aggregate of the
 * tuned tasks on the device and measure its latency).
 */
typedef enum {
  CPRUNE_LAYER_CONV = 0,     /* dense or depthwise conv + bias (+residual) + act */
  CPRUNE_LAYER_MAXPOOL = 1,
  CPRUNE_LAYER_GAVGPOOL = 2,
  CPRUNE_LAYER_FC = 3
} cprune_layer_kind;

typedef struct {
  int32_t kind;        /* cprune_layer_kind */
  int32_t input;       /* index of the producing layer, -1 = the network input */
  int32_t residual;    /* index of the layer added before act, -1 = none */
  int32_t c_in, c_out; /* channels after pruning (pools: c_out = c_in) */
  int32_t k, stride, pad;
  int32_t groups;      /* 1 or c_in */
  int32_t act;         /* cprune_act */
  const void* weight;  /* device, folded, in the net's dtype; NULL for pools */
  const float* bias;   /* device fp32 [c_out] or NULL */
} cprune_layer_desc;

typedef struct cprune_net cprune_net;

/* Builds a handle: copies every layer's weights and bias into memory the handle
 * owns (repacked channels-last: inside a handle activations are [n][h][w][c'] and weights
 * [c_out][kh][kw][c'], c' = channels rounded up to one 16-byte vector, pad channels zero;
 * x and logits at the boundary stay NCHW; a dense conv with at most 4 input channels that
 * reads the network input takes the NCHW tensor as it is), allocates one activation buffer per layer for
 * `max_batch` images and the conv scratch, and picks a tile variant per conv shape (timing it on the device
 * when tune != 0, as cprune_select_tile does, for batch `max_batch`).  `layers` is
 * a host array.  in_c/in_h/in_w: the network input [n][in_c][in_h][in_w]. */
int cprune_net_create(const cprune_layer_desc* layers, int n_layers, int in_c, int in_h,
                      int in_w, int max_batch, cprune_dtype dtype, int tune, void* stream,
                      cprune_net** out);
/* logits: the last layer's output, dense NCHW [n][c_out][h_out][w_out] in the net's dtype
 * ([n][classes] for a net that ends in a fully connected layer); device memory of at
 * least n times the element count cprune_net_output_shape reports.  1 <= n <= max_batch.
 * use_graph != 0 replays a HIP graph of the layer sequence on `stream`; the graph is
 * recorded (on a stream the handle owns, nothing executes while recording) the
 * first time a given (n, x, logits) triple is seen and kept until destroy. */
int cprune_net_forward(cprune_net* net, const void* x, int n, void* logits, int use_graph,
                       void* stream);
/* Per-layer device time: after one untimed pass that gives every layer its inputs, each
 * layer is launched `iters` times back to back between two events on `stream`; ms_out
 * (host, [n_layers]) gets the time per launch (0 for a pool folded into its producer and for a depthwise layer
 * that runs inside its reader's kernel).
 * Synchronises. */
int cprune_net_layer_times(cprune_net* net, const void* x, int n, int iters, float* ms_out,
                           void* stream);
/* Writes layer `layer`'s activation of the last forward (batch n) to dst (device) as dense
 * NCHW [n][c_out][h_out][w_out].  For the last layer of a net whose output map is 1x1 the
 * values are those of the last cprune_net_layer_times pass (forward writes that layer
 * straight into `logits`).  A conv layer whose following 2x2 max-pool was fused into its
 * epilogue has no activation of its own: CPRUNE_ERR_UNSUPPORTED (ask for the pool layer); so
 * has a depthwise layer that runs inside the kernel of the 1x1 conv that reads it. */
int cprune_net_copy_activation(cprune_net* net, int layer, int n, void* dst, size_t dst_bytes,
                               void* stream);
/* Shape of one image's output (the last layer's c_out, h_out, w_out); host outs. */
int cprune_net_output_shape(const cprune_net* net, int* c_out, int* h_out, int* w_out);
/* The tile variant in use for layer `layer` (-1 for layers without one); host out. */
int cprune_net_layer_variant(const cprune_net* net, int layer, int* variant_out);
/* The first two layers in one kernel, where the network opens with two 3x3 / stride 1 / pad 1 convolutions,
 * the first on the image (at most 3 channels) with at most 32 filters and read by the second only (the
 * VGG-16 of the motivating experiment that opens Section 3, Fig. 1; channel counts as Sec. 3.5 leaves them): the first layer's output, the
 * largest activation of such a network, is then never written.  cprune_net_create(tune = 1) times both
 * forms and keeps the faster; this call forces one.  enable: 0 / 1.  CPRUNE_ERR_UNSUPPORTED when the
 * network does not open that way.  Synchronises; recorded graphs are dropped. */
int cprune_net_fuse_first_layers(cprune_net* net, int enable);
/* How a 7x7 / stride 2 / pad 3 first layer on the image (at most 3 channels) runs in a 16-bit handle: the
 * opening of the ImageNet networks of Section 4.1 (ResNet-18, Table 1).  form 0: the general kernels;
 * 1: the kernel made for this layer in 16-bit data; 2: that kernel with the 3x3 / stride 2 / pad 1 max-pool
 * behind the layer inside it (the conv map is then never stored: cprune_net_copy_activation of the conv
 * layer returns CPRUNE_ERR_UNSUPPORTED, the pool layer's activation is the pooled map as always).
 * cprune_net_create(tune = 1) times the forms and keeps the fastest, tune = 0 takes the highest available.
 * CPRUNE_ERR_UNSUPPORTED for fp32 handles, for networks that do not open that way, and for form 2 when
 * the conv map has another reader or no such pool follows.  Synchronises; recorded graphs are dropped. */
int cprune_net_first_layer_form(cprune_net* net, int form);

/* A depthwise conv (3x3 or 5x5, stride 1 or 2, "same" padding) whose only reader is a 1x1
 * conv can run inside that conv's kernel (the tensor between them is then never stored).
 * cprune_net_create decides per pair (by size, or by timing both forms when tune != 0);
 * this call overrides the decision for depthwise layer `layer`.  CPRUNE_ERR_UNSUPPORTED when
 * the layer is no such depthwise conv.  Recorded graphs are dropped.  Not to be called while
 * a forward is in flight.  cprune_net_layer_fused reports the current state (host out). */
int cprune_net_fuse_depthwise(cprune_net* net, int layer, int enable);
int cprune_net_layer_fused(const cprune_net* net, int layer, int* fused_out);
/* When the input of such a depthwise conv is a 1x1 / stride 1 conv that nobody else reads (the
 * expansion of an inverted-residual block of MobileNetV2 / MnasNet1.0, Sec. 4.1 and Table 1 of the
 * paper; its filters are the ones Sec. 3.5 prunes), and the 1x1
 * reader has at most 128 filters, all three layers can run as one kernel: the expanded
 * activations, the block's largest tensor, then never reach memory.  cprune_net_create decides
 * per block (by size, or by timing when tune != 0); this call overrides the decision for the
 * block whose depthwise layer is `layer`: enable != 0 runs the block as one kernel, 0 leaves
 * the expansion on its own (the depthwise layer stays inside its reader's kernel).
 * cprune_net_fuse_depthwise on the same layer also leaves the one-kernel form.
 * CPRUNE_ERR_UNSUPPORTED when the layer heads no such block or the block's input patch does not
 * fit the local memory of a compute unit.  Recorded graphs are dropped.  Not to be called while
 * a forward is in flight.  cprune_net_layer_fused reports 1 for the expansion and the
 * depthwise layer of a block that runs as one kernel. */
int cprune_net_fuse_block(cprune_net* net, int layer, int enable);
/* Pins the tile variant of a dense conv / fully connected layer (what a stored tuning result
 * is applied with).  CPRUNE_ERR_INVALID_ARG for a layer without variants,
 * CPRUNE_ERR_UNSUPPORTED when the variant cannot run that layer's shape.  Recorded graphs
 * are dropped (they hold the old choice).  Not to be called while a forward is in flight. */
int cprune_net_set_layer_variant(cprune_net* net, int layer, int variant);
int cprune_net_destroy(cprune_net* net);

/* ---- search-side rules (host only, no device work) ----
 * Section 3.5.  A program splits the iterator over a layer's filters into factors (their
 * product is the filter count); the filters form a box with these side lengths, and removing
 * one slice of the box keeps the program's structure.  cprune_lcm_step: l1 / l2 (host arrays,
 * n1 / n2 >= 1 positive entries) are the splits of the program's two filter iterators (the
 * reduction loop's and the output stage's); step_out (host) gets the least common multiple of
 * the two smallest slices, product / largest factor each: the minimum number of filters to
 * prune.  CPRUNE_ERR_INVALID_ARG for empty lists or factors < 1. */
int cprune_lcm_step(const int64_t* l1, int n1, const int64_t* l2, int n2, int64_t* step_out);
/* Filters to prune from c_out so that the count left is the next lower multiple of step (step
 * itself when c_out is a multiple); 0 when that would leave no filter.  Host out. */
int cprune_prune_count(int c_out, int64_t step, int* count_out);
/* The structure of tile variant `variant` on a layer of c_out filters, as that rule needs it:
 * both filter iterators walk (output tile, MFMA row block of the tile), so
 * main_loop[2] = epilogue[2] = {tiles, blocks per tile} and *unit_out = the filters per block
 * (16, or 32 for the variants built on 32x32 blocks; the rows inside a block are fixed by the
 * instruction and cannot shrink).  Host outs. */
int cprune_variant_filter_splits(int variant, int c_out, int64_t* main_loop, int64_t* epilogue,
                                 int* unit_out);
/* cprune_lcm_step of those splits, in filters (times the unit). */
int cprune_variant_prune_step(int variant, int c_out, int64_t* step_out);
/* Section 3.3.  Pruning impact of a task = its execution time x the number of subgraphs
 * (layers) that map to it; order_out[n_tasks] gets the task indices by descending impact, equal
 * impacts in index order; impact_out[n_tasks] (or NULL) the impacts.  Host arrays. */
int cprune_order_tasks(const double* exec_time, const int* n_subgraphs, int n_tasks, int* order_out,
                       double* impact_out);
/* Section 3.4.  Groups the handle's dense conv / fully connected layers into tasks: layers
 * with the same shape, stride, padding, activation, shortcut and layout are one task, numbered
 * in order of first appearance.  task_of_layer: host [n_layers], -1 for pools and depthwise
 * layers; n_tasks_out: host.  A task's layer may run a kernel without tile variants (the
 * first-layer kernel, the fused depthwise + 1x1 kernel: cprune_net_layer_variant gives -1);
 * those are built on 16-filter blocks. */
int cprune_net_task_table(const cprune_net* net, int* task_of_layer, int* n_tasks_out);

/* The key cprune_net_task_table groups by, for layer `layer` (a dense conv / fully connected
 * layer): key_out, host [CPRUNE_TASK_KEY_INTS], holds the layer's shape at the handle's batch
 * size, stride, padding, activation, shortcut flag and the layout it runs in (channel strides,
 * fused pool, channels-last output).  Two layers are one task iff their keys are equal. */
#define CPRUNE_TASK_KEY_INTS 18
int cprune_net_task_key(const cprune_net* net, int layer, int32_t* key_out);

/* Section 3.2, Algorithm 1, as a state machine (host only).  The caller owns the models and
 * does the pruning, tuning, measuring and accuracy evaluation; this object takes the
 * decisions.  Tasks are caller-chosen 64-bit ids that mean the same task from model to model.
 *   start(tasks of the input model by descending impact, its latency l_m, its accuracy a_p):
 *       target latency l_t = beta * l_m.
 *   next_task: the task to prune next, or *done_out = 1 when the search is over: the accuracy
 *       of the accepted model is at or below a_goal, no task is left, max_passes passes over
 *       the list have been made, or a whole pass neither accepted a candidate nor dropped a task.
 *   then exactly one of
 *     report_exhausted: the task's layers cannot lose filters; the task is out for good.
 *     report_latency(l_m of the tuned candidate): l_m >= l_t -> logged as slow, the task stays
 *       in the list, *needs_accuracy_out = 0; l_m < l_t -> *needs_accuracy_out = 1 and the
 *       caller must follow with
 *     report_accuracy(a_s, the candidate's tasks by descending impact): a_s < alpha * a_p ->
 *       the task is out for good; otherwise the candidate is accepted: it becomes the model,
 *       its task list minus the tasks that are out becomes the list, l_t = beta * l_m,
 *       a_p = a_s, and the next pass starts at the head of the new list.
 * Calls out of this order: CPRUNE_ERR_INVALID_ARG.  The log has one entry per reported
 * candidate; l_m / a_s are NaN where they were not measured. */
#define CPRUNE_SEARCH_SLOW 1
#define CPRUNE_SEARCH_INACCURATE 2
#define CPRUNE_SEARCH_ACCEPTED 3
#define CPRUNE_SEARCH_EXHAUSTED 4
typedef struct cprune_search cprune_search;
int cprune_search_create(double a_goal, double alpha, double beta, int64_t max_passes,
                         cprune_search** out);
int cprune_search_start(cprune_search* s, const int64_t* tasks_by_impact, int n_tasks, double l_m,
                        double a_p);
int cprune_search_next_task(cprune_search* s, int64_t* task_out, int* done_out);
int cprune_search_report_exhausted(cprune_search* s);
int cprune_search_report_latency(cprune_search* s, double l_m, int* needs_accuracy_out);
int cprune_search_report_accuracy(cprune_search* s, double a_s, const int64_t* tasks_by_impact,
                                  int n_tasks, int* accepted_out);
int cprune_search_log_size(const cprune_search* s);
int cprune_search_log_entry(const cprune_search* s, int index, int64_t* task_out, double* l_m_out,
                            double* l_t_out, double* a_s_out, int* verdict_out);
int cprune_search_destroy(cprune_search* s);

/* ---- measured ceilings (for reporting kernel throughput against what the device
 * delivers, next to its datasheet peaks; the paper reports end-to-end rates only) ----
 * cprune_probe_mfma: rate of back-to-back dense MFMA instructions of `dtype` on register
 * operands, no memory traffic (the better of the 16x16 and the 32x32 block forms); scratch: device, >= cprune_probe_scratch_bytes() (values
 * written there are meaningless); tflops_out: host.  cprune_probe_copy: rate of a plain
 * copy of `bytes` (a multiple of 16) from src to dst (device, 16-byte aligned, not
 * overlapping), counted as bytes read + bytes written, the fastest of eight launch shapes (4 or
 * 8 pieces of 16 bytes in flight per thread, cached or non-temporal accesses, one step per
 * work-group or resident work-groups walking the buffer); gbps_out: host.  cprune_probe_read /
 * cprune_probe_write: the same for a kernel that only reads `bytes` (scratch16: 16 bytes of
 * device memory, never written in practice) or only writes them.  cprune_probe_l2_read:
 * GB/s one compute unit reads from L2-resident data with 16-byte-per-lane loads, the form in
 * which a kernel takes MFMA operands straight from global memory; pattern 0: each wavefront-wide
 * load covers 1 KiB of consecutive memory, pattern 1: 16 rows x 64 bytes (an operand tile of a
 * row-major matrix).  buf: device, >= cprune_probe_l2_bytes(), contents irrelevant; scratch:
 * device, one float; gbps_per_cu_out: host.  All synchronise. */
size_t cprune_probe_scratch_bytes(void);
int cprune_probe_mfma(cprune_dtype dtype, void* scratch, size_t scratch_bytes, float* tflops_out,
                      void* stream);
int cprune_probe_copy(const void* src, void* dst, size_t bytes, float* gbps_out, void* stream);
int cprune_probe_read(const void* src, void* scratch16, size_t bytes, float* gbps_out, void* stream);
int cprune_probe_write(void* dst, size_t bytes, float* gbps_out, void* stream);
size_t cprune_probe_l2_bytes(void);
int cprune_probe_l2_read(int pattern, const void* buf, size_t buf_bytes, float* scratch,
                         float* gbps_per_cu_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CPRUNE_H */
