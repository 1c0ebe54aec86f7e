/*
 * dp_step.h -- C ABI of the MI355X (gfx950) private gradient step of DPSGD.
 *
 * One call to dp_step performs items 2-3 of the DPSGD procedure enumerated in
 * Section 1 of the paper (arxiv 2010.09063) for one minibatch:
 *   2(a) per-example gradient g_i of the example's own loss, for every layer;
 *   2(b) clip: g_i <- g_i * min(1, C / ||g_i||_2), one L2 norm over all parameters;
 *   3    sum the clipped gradients over the batch and add N(0, sigma^2 C^2 I).
 * Drawing the minibatch (item 1) and the parameter update (item 4) stay with the
 * caller.  The per-example gradients never leave the library and are mostly
 * never formed: dense layers use the norm identity ||a (x) delta|| = ||a|| ||delta||
 * (Section 1, the fully-connected per-example norm trick), convolutions on small
 * planes take the norm from Gram matrices, the other convolution / recurrent
 * layers contract each example's activations with its backprops tile by tile
 * and reduce the squares in the kernel; the clipped sum is the contraction
 * A^T diag(s) Delta.  Only where writing and re-reading an example's gradient is
 * cheaper than contracting it again (large planes, long sequences) does the
 * workspace hold a [batch][layer parameters] block, summed with the clip
 * factors afterwards.  Pad-1 3x3 convolutions (Section 2.1) may be evaluated in
 * the minimal-filtering form (fewer multiplies, the same sums up to fp32
 * rounding); results are held to the same tolerance either way.
 *
 * Pointers marked "device" are HIP device memory owned by the caller (the
 * library never frees them and keeps no reference after the call's stream
 * work); pointers marked "host" are ordinary host memory.  All functions return
 * DP_OK (0) or a negative dp_status; no C++ exception crosses this boundary.
 * After an error the contents of out_grad are unspecified.
 */
#ifndef DP_STEP_H
#define DP_STEP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dp_ctx dp_ctx; /* opaque; owned by the library */

typedef enum {
  DP_OK = 0,
  DP_EINVAL = -1, /* null pointer, bad shape, batch > max_batch, C <= 0, sigma < 0, NaN */
  DP_ENOMEM = -2, /* workspace allocation failed */
  DP_EHIP = -3,   /* a HIP runtime call failed; see dp_step_strerror */
  DP_EUNSUPPORTED = -4, /* layer sequence the kernels do not cover */
  DP_ETOOBIG = -5       /* dp_step_dense1_static: sizes beyond its fixed scratch */
} dp_status;

typedef enum {
  DP_DENSE = 0,     /* z = a W + b,   W[in_features][out_features] row-major, b[out_features] */
  DP_CONV2D = 1,    /* cross-correlation, zero padding, W[out_ch][in_ch][kh][kw], b[out_ch]   */
  DP_MAXPOOL2D = 2, /* window kh x kw, stride, no padding; gradient goes to the first maximum */
  DP_EMBEDDING = 3, /* E[vocab][embed_dim]; input int32 token ids [B, seq_len]                */
  DP_LSTM_LAST = 4, /* one-layer LSTM, returns the last hidden state; W_ih[in_features][4H],
                       W_hh[H][4H], b[4H]; 4H axis ordered i, f, g, o; h_0 = c_0 = 0          */
  DP_SEQ_MEAN = 5,  /* mean over the seq_len step vectors of an embedding's or a DP_LSTM_SEQ's output
                       (the embedding and LSTM networks of the paper's Appendix B); no parameters,
                       no fields used                                                          */
  DP_LSTM_SEQ = 6,  /* DP_LSTM_LAST's layer, but the output is every hidden state, [seq_len][H] (the
                       LSTM network of Appendix B); must be followed by DP_SEQ_MEAN              */
  DP_AVGPOOL2D = 7  /* mean over kh x kw windows, stride, no padding (the CIFAR10 network of Appendix B);
                       a window covering the whole plane is the global average pool.  It may be the
                       last layer when it leaves n_classes values, which are then the logits     */
} dp_layer_kind;

typedef enum { DP_ACT_NONE = 0, DP_ACT_RELU = 1, DP_ACT_TANH = 2 } dp_act;

typedef struct {
  int kind;                                 /* dp_layer_kind                       */
  int act;                                  /* dp_act, applied to dense / conv out */
  int in_features, out_features;            /* dense; lstm: input width, (unused)  */
  int in_ch, out_ch, kh, kw, stride, pad;   /* conv; pool uses kh, kw, stride      */
  int vocab, embed_dim;                     /* embedding                           */
  int hidden;                               /* lstm                                */
} dp_layer_desc;

typedef struct {
  int n_layers;
  const dp_layer_desc *layers; /* host; read during dp_step_init only                    */
  int in_c, in_h, in_w;        /* image input NCHW (a feature vector is in_c x 1 x 1)    */
  int seq_len;                 /* > 0: the input is int32 token ids [B, seq_len]         */
  int n_classes;               /* width of the last layer (dense without activation, or an average pool); loss =
                                  softmax cross-entropy of its output */
} dp_model_desc;

/*
 * dp_step_init -- fixes every shape, allocates all workspace for batches up to
 * max_batch and returns a context (the static-shape specialisation that Section
 * 2.2, "Just-In-Time Compilation", credits for buffer reuse: shapes are known
 * before the first step so nothing is allocated afterwards).
 *   model      host; copied.
 *   hip_stream a hipStream_t (NULL = the default stream); every later call
 *              enqueues its work there.  Init itself returns with the workspace
 *              ready for a step enqueued on that stream.
 *   out        host; receives the context.
 * Flat parameter layout: layers in order, each weight tensor then its bias, in
 * the layouts named at dp_layer_kind.
 */
int dp_step_init(const dp_model_desc *model, int max_batch, void *hip_stream, dp_ctx **out);

/*
 * Route switches (utility, no passage of the paper): every field 0 is the plan the library picks by itself.  A
 * non-zero field keeps one family of kernels out (or forces one in) for tests and A/B measurements; the results
 * are the same to rounding whichever route runs.  Read once by dp_step_init_ex; a context never changes its plan.
 */
typedef struct {
  int generic_conv;               /* 3x3 stride-1 convolutions on the generic tiled contraction                   */
  int no_minimal_filtering;       /* no kernel of the F(2x2,3x3) / F(3x3,2x2) family                              */
  int no_minimal_filtering_wgrad; /* only that family's weight-gradient kernels off                               */
  int minimal_filtering_all;      /* its forward / backward-data kernels for every eligible shape                 */
  int no_pool_fusion;             /* 2x2 / stride-2 pools as launches of their own, not in the conv epilogue      */
  int no_gram;                    /* small-plane convolution norms by the per-example contraction                 */
  int no_stored_gradients;        /* never store per-example gradients: the clipped sum repeats the contraction   */
  int no_columns;                 /* strided backward-data by the gathering contraction                           */
  int no_specialised_waves;       /* weight gradient of wide layers on the single-buffer kernel                   */
  int specialised_waves_all;      /* ... or the staging / multiplying wave split for every width                  */
  int conv_min_blocks;            /* grid the direct forward kernel narrows its tiles for (0: 512)                */
  int gemm_plain_tiles;           /* tile choice of the generic contraction without the padding-waste rule        */
  int no_fused_dense;             /* one- / two-dense-layer models and dense two-layer heads on the generic kernels */
  int no_fused_cnn;               /* the small MNIST-shaped CNN layer by layer instead of in one launch            */
  int no_lstm_wgrad;              /* the LSTM's per-example weight gradient on the generic tiled contraction       */
  int no_rows_gemm;               /* the LSTM's input projection / input gradient on the generic tiled contraction */
  int no_single_bucket;           /* the embedding's counting sort as three launches, whatever the batch           */
  int no_small_gemm;              /* two-layer networks: both batch-wide products on the split-K contraction, not
                                     on the kernel that splits K inside the workgroup                               */
  int no_resident_weights;        /* minimal-filtering form, 32 -> (at most) 32 channels: the per-group kernel instead of
                                     the persistent one that keeps the transformed weights in registers              */
  int no_side_stream;             /* the embedding's counting sort in line on the caller's stream instead of beside the
                                     forward pass on a stream of the library's own                                 */
  int no_first_layer_kernel;      /* an RGB first layer's forward pass on the generic direct kernel                  */
} dp_plan_options;

/* dp_step_init with route switches; options == NULL is dp_step_init. */
int dp_step_init_ex(const dp_model_desc *model, int max_batch, void *hip_stream, const dp_plan_options *options,
                    dp_ctx **out);

/* Number of fp32 parameters P of the model (0 if ctx is NULL).  Utility, no passage. */
size_t dp_step_num_params(const dp_ctx *ctx);

/* Bytes of device workspace the context holds (Section 4 discusses memory as what bounds the batch size). */
size_t dp_step_workspace_bytes(const dp_ctx *ctx);

/*
 * dp_step_validate -- debug check of the integer inputs, which dp_step itself trusts: counts the labels outside
 * [0, n_classes) and, for token models, the ids outside [0, vocab).  Utility, no passage.
 *   x, y    device, as for dp_step (x is read only when the model takes token ids)
 *   n_bad   host; receives the count (0 = the batch is safe to pass to dp_step)
 * Synchronises the context's stream.
 */
int dp_step_validate(dp_ctx *ctx, const void *x, const int32_t *y, int batch, int *n_bad);

/*
 * dp_step -- the private step (Section 1, DPSGD items 2-3).
 *   params   device fp32[P]
 *   x        device fp32[batch, in_c, in_h, in_w] or int32[batch, seq_len]
 *   y        device int32[batch], class ids in [0, n_classes)
 *   batch    0 <= batch <= max_batch (0 yields pure noise)
 *   C        clip norm, > 0; +INFINITY disables clipping (then sigma must be 0)
 *   sigma    noise multiplier, >= 0; 0 adds exactly nothing
 *   seed     key of the Philox4x32-10 stream; coordinate j takes lane j%4 of block
 *            j/4, counter (block lo, block hi, 0, 0); uniforms are
 *            ((r >> 9) + 1/2) 2^-23, two Box-Muller pairs per block
 *   out_grad device fp32[P] = sum_i g_i min(1, C/||g_i||) + sigma C z   (a sum, not a mean)
 * Asynchronous: work is enqueued on the context's stream; no host sync, no
 * allocation.  Token ids and labels out of range are undefined behaviour.
 */
int dp_step(dp_ctx *ctx, const float *params, const void *x, const int32_t *y, int batch, float C, float sigma,
            uint64_t seed, float *out_grad);

/*
 * dp_step_sgd -- dp_step followed by the parameter update of the same procedure (Section 1, DPSGD
 * item 4), fused into the final write:   params[j] -= (lr / batch) * (clipped_sum[j] + sigma*C*z_j).
 * (An extension: the step proper ends with the noised sum; dividing by the batch size and updating
 * otherwise stay with the caller.)
 *   params     device, [num_params], read by the step and UPDATED IN PLACE by its last kernel.
 *   lr         learning rate; the aggregate is a sum over the batch, so the step uses lr / batch.
 *   out_grad   device, [num_params] or NULL: where given, also receives the noised sum as dp_step writes it.
 *   batch      1 .. max_batch.  Other arguments, ownership and errors as for dp_step.
 */
int dp_step_sgd(dp_ctx *ctx, float *params, const void *x, const int32_t *y, int batch, float C, float sigma,
                uint64_t seed, float lr, float *out_grad);

/*
 * dp_step_sample_indices -- the minibatch draw of the procedure (Section 1, DPSGD item 1; the paper leaves the
 * draw open): `batch` indices drawn independently and uniformly from [0, n_examples), with replacement.  Index k
 * is (word k%4 of the Philox4x32-10 block with key `seed` and counter (k/4, 0, 1, 0)) * n_examples >> 32; the
 * third counter word keeps these blocks apart from the noise stream of the same seed.
 *   indices    device int32[batch]; enqueued on hip_stream (NULL = the default stream); 1 <= n_examples < 2^31.
 */
int dp_step_sample_indices(uint64_t seed, int64_t n_examples, int batch, int32_t *indices, void *hip_stream);

/*
 * dp_step_loop -- `steps` iterations of the whole procedure (Section 1, DPSGD items 1-4) on a dataset resident in
 * device memory, with no host work between the steps but kernel launches.  Step t (t = 0 ...) uses seed0 + t for
 * its draw and its noise: draw `batch` indices (dp_step_sample_indices), gather those examples, take the private
 * step on them and update:  params -= (lr / batch) * (sum_i clip(g_i) + sigma*C*z).
 *   params           device fp32[P], updated in place after every step
 *   data_x, data_y   device; fp32[n_examples, in_c, in_h, in_w] or int32[n_examples, seq_len]; int32[n_examples]
 *   batch            1 .. max_batch of the context
 * The first call on a context allocates room for one drawn minibatch (freed with the context); later calls
 * allocate nothing.  Asynchronous like dp_step.  (An extension beyond the step proper, as dp_step_sgd is.)
 */
int dp_step_loop(dp_ctx *ctx, float *params, const void *data_x, const int32_t *data_y, int64_t n_examples, int steps,
                 int batch, float C, float sigma, uint64_t seed0, float lr);

/*
 * dp_step_nonprivate -- the ordinary summed gradient sum_i g_i with the same
 * forward / backward kernels and no norms, clipping or noise (the comparator of
 * the paper's private / non-private runtime ratio, Table 1).
 */
int dp_step_nonprivate(dp_ctx *ctx, const float *params, const void *x, const int32_t *y, int batch,
                       float *out_grad);

/*
 * dp_step_dense1_static -- dp_step for a model that is ONE dense layer (softmax regression: logits = x W + b),
 * for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  It needs no context and calls no allocating routine: its scratch (partial clipped sums and clip
 * factors) is a fixed 8 MiB array in the library's device image, one copy per GPU for the life of the process.
 *   params     device fp32[(in_features + 1) * n_classes]: W[in_features][n_classes] row-major, then b
 *   x, y       device fp32[batch, in_features], int32[batch]
 *   norms_out  device fp32[batch] or NULL: receives the unclipped per-example norms
 *   hip_stream a hipStream_t (NULL = the default stream) the two launches are enqueued on
 *   C, sigma, seed, out_grad: as for dp_step; results equal dp_step's on the same model to rounding.
 * Limits: in_features <= 1023, n_classes <= 15, in_features * (n_classes rounded up to 4, 10 or
 * 15, + 4) <= 14800, batch <= 65536; beyond
 * them DP_ETOOBIG and nothing is launched.
 * Every call on one GPU uses that GPU's one scratch array: calls that overlap in time on one GPU (two streams,
 * two threads) race on it; serialise them.  Nothing in the array needs clearing between calls.
 */
int dp_step_dense1_static(const float *params, const float *x, const int32_t *y, int batch, int in_features,
                          int n_classes, float C, float sigma, uint64_t seed, float *out_grad, float *norms_out,
                          void *hip_stream);

/*
 * dp_step_last_norms -- copies the unclipped per-example norms ||g_i|| of the
 * most recent dp_step into norms_out (device fp32[batch of that step]);
 * enqueued on the context's stream.  Test hook for the clipping invariant (Section 1, item 2b:
 * after clipping no example's gradient is longer than C).
 */
int dp_step_last_norms(dp_ctx *ctx, float *norms_out);

/*
 * Per-kernel timing (utility, no passage).  With profiling on, every kernel launch of later steps is
 * bracketed by HIP events on the context's stream.  dp_step_profile_read
 * synchronises the stream and returns, for up to `cap` distinct kernel labels
 * in launch order: the label (pointer into the context, valid until free), the
 * number of launches since the last reset and the summed milliseconds.
 * Returns the number of labels (or a negative dp_status).
 */
int dp_step_profile(dp_ctx *ctx, int enable);
int dp_step_profile_read(dp_ctx *ctx, int cap, const char **labels, int *launches, float *total_ms, int reset);

/*
 * dp_step_describe_plan -- which kernel family each parameter layer was planned on, as text
 * "<layer>:fwd=..,bwd=..,norm=..,sum=..;" ("mf32"/"mf64"/"mf": minimal-filtering form, 16 multiplies where the
 * direct form has 36; "gram"; "+store"/"weighted": stored per-example gradients).  Utility, no passage; the
 * benchmark uses it to price each launch by the multiplies its route really issues.
 *   buf, cap   host buffer; DP_EINVAL if the text does not fit.
 */
int dp_step_describe_plan(const dp_ctx *ctx, char *buf, size_t cap);

/*
 * dp_step_ceiling -- measured reference points for roofline figures (utility, no passage).  what = 0: a plain
 * device copy of 256 MiB, GB/s read + written; 1: a register-only v_mfma_f32_32x32x2_f32 loop on every CU,
 * TFLOP/s; 2: microseconds per launch of an empty kernel, 1000 launches back to back on the stream.  Allocates
 * and frees its own buffers and synchronises; *value (host) receives the figure.
 */
int dp_step_ceiling(int what, void *hip_stream, double *value);

/* Static description of a status code, plus the last HIP error text for DP_EHIP.  Utility, no passage. */
const char *dp_step_strerror(int code);

/* Releases the context and its workspace (NULL is a no-op).  Utility, no passage. */
void dp_step_free(dp_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* DP_STEP_H */
