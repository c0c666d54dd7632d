/*
 * gati.h - C ABI of the learned-cache lookup library for AMD MI355X (gfx950).
 *
 * A learned cache sits after one hidden layer of a base DNN.  Its interface is that of
 * any cache: given the hidden layer's output it returns a prediction when it hits
 * (paper, Section 2.3 "Towards Learned Caches").  It is made of two small networks run in
 * sequence (Section 3, "Learned Cache Design"): a predictor that maps the hidden
 * layer output to a class distribution, and a selector that decides whether that
 * prediction may be served as a hit.  Hits leave the batch; misses continue on the
 * base model and meet the next layer's cache (Section 1; Appendix A.1, effective
 * cache-hit rate).
 *
 * This library is that lookup for a whole batch of in-flight requests at one layer,
 * plus the stable compaction of the misses that feeds the next layer:
 *
 *   pooled[c]  = mean over the spatial / token axis of the activation   (pooling predictor,
 *                                                                         Section 3 table of
 *                                                                         predictor architectures)
 *   hidden     = relu(W1 pooled + b1)                                    (hidden layer, ReLU)
 *   logits     = W2 hidden + b2,  prob = softmax(logits),  class = argmax
 *   score      = ws . [pooled ; prob] + bs,  confidence = 1/(1+exp(-score))   (selector)
 *   hit        = confidence > threshold
 *   misses     = ids whose hit flag is 0, in their incoming order
 *
 * All pointers named "device" are HIP device pointers valid on the device that was
 * current when the cache was created; "host" pointers are ordinary host memory.  The
 * library never frees or keeps caller buffers.  Every call that takes a stream only
 * enqueues work on it and returns; nothing synchronises the device and nothing is
 * allocated after gati_cache_create (gati_trainer_create).  No function throws or aborts: errors come back
 * as a gati_status_t and leave the outputs untouched (argument errors are detected on
 * the host before anything is launched).
 */
#ifndef GATI_H
#define GATI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gati_cache gati_cache_t; /* opaque, owned by the library */

typedef enum {
    GATI_OK = 0,
    GATI_ERR_INVALID_ARG = 1, /* null required pointer, bad enum, non-positive size, n_max out of range */
    GATI_ERR_UNSUPPORTED = 2, /* a valid request this build has no kernel for */
    GATI_ERR_OOM = 3,         /* device or host allocation failed in gati_cache_create */
    GATI_ERR_DEVICE = 4       /* a HIP call failed (launch, copy, wrong device) */
} gati_status_t;

typedef enum { GATI_F32 = 0, GATI_BF16 = 1 } gati_dtype_t;

typedef enum {
    GATI_LAYOUT_NCS = 0, /* [n, C, S]: channel-major, S = H*W contiguous (NCHW feature maps) */
    GATI_LAYOUT_NSC = 1  /* [n, S, C]: token-major / channels-last, C contiguous              */
} gati_layout_t;

/* How a hit is decided.
 *   GATI_SEL_LINEAR   the selector network: logistic of an affine map over [pooled ; prob]
 *   GATI_SEL_SOFTMAX  no selector network: confidence = largest class probability, the
 *                     softmax-threshold baseline the paper compares against (Appendix,
 *                     "Decoupling prediction and selection"); ws and bs are ignored
 *   GATI_SEL_HIDDEN   the selector network with one hidden layer (Section 3, "Selector Network
 *                     Design"): g = relu(Ws [features ; prob] + cs), confidence =
 *                     logistic(vs . g + bs).  selector_hidden units, 1..1024.  The first layer is
 *                     a matrix product like the predictor's: in a GATI_BF16 cache Ws, its operands
 *                     and g are rounded to bf16; the second layer is fp32.  ws is ignored.        */
typedef enum { GATI_SEL_LINEAR = 0, GATI_SEL_SOFTMAX = 1, GATI_SEL_HIDDEN = 2 } gati_selector_t;

/* Which predictor network the cache holds (paper, Section 3, table of predictor architectures).
 *   GATI_PRED_GAP_MLP  global average pool -> FC(C->H) -> ReLU -> FC(H->K): the fully connected
 *                      topology applied to the globally pooled features
 *   GATI_PRED_POOL_FC  the paper's Pool(h): adaptive average pool of the in_h x in_w feature map to
 *                      out_h x out_w (window i of an axis covers [floor(i*in/out), ceil((i+1)*in/out)),
 *                      the PyTorch rule), ReLU, then one FC over the F = C*out_h*out_w features
 *                      (feature order [c][oy][ox]).  Needs S = in_h*in_w; position y*in_w + x of the map
 *                      is element s of the row in either layout (channels-last maps take a plain
 *                      kernel, channel-major ones the tiled one).  H, W1 and b1 are unused; W2 is
 *                      [K, F] and ws is [F + K].
 *   GATI_PRED_FC_MLP   the paper's FC(h): the activation row flattened in storage order (D = C*S
 *                      values) -> FC(D->H) -> ReLU -> FC(H->K).  W1 is [H, D]; the selector reads
 *                      [hidden ; prob], so ws is [H + K]; the "pooled" features reported by
 *                      gati_cache_pool are the H hidden activations.  Rows whose length D is a
 *                      multiple of 64 run on the matrix cores (activation pointer 16-byte aligned);
 *                      other lengths take a plain kernel.
 *   GATI_PRED_CONV_FC  the paper's Conv(k,s): convolution of the C x in_h x in_w map with H filters of
 *                      conv_k x conv_k, stride conv_s, no padding, ReLU, then one FC over the
 *                      F = H*oh*ow hidden values, oh = (in_h - conv_k)/conv_s + 1 (feature order
 *                      [filter][oy][ox]).  Needs S = in_h*in_w (either layout; channels-last maps take a
 *                      plain kernel).  W1 is
 *                      [H, C, conv_k, conv_k], b1 [H], W2 [K, F], ws [F + K].  H <= 64, conv_k <= 15
 *                      (GATI_ERR_UNSUPPORTED otherwise).                                            */
typedef enum { GATI_PRED_GAP_MLP = 0, GATI_PRED_POOL_FC = 1, GATI_PRED_FC_MLP = 2, GATI_PRED_CONV_FC = 3 } gati_predictor_t;

/* Shape of one learned cache (Section 3: predictor Input -> Hidden(h) -> Output, selector).
 *   C, S       activation channels and reduced length (pool extent = all of S)
 *   H, K       predictor hidden width and number of classes
 *   act_dtype  element type of the activation tensor.  It also fixes the arithmetic of the
 *              two FC layers: GATI_F32 -> fp32 operands; GATI_BF16 -> W1, W2 and the FC
 *              operands (pooled, hidden) rounded to bf16 (nearest even), fp32 accumulation.
 *              Pooling, biases, softmax, selector and sigmoid are fp32 in both.
 *   threshold  tau; a row is a hit iff confidence > tau (strictly)
 *   max_rows   largest n_max any later call may pass (sizes the library's workspace)
 *   selector   how the hit flag is decided, see gati_selector_t
 *   predictor  which predictor network and its in/out map sizes, see gati_predictor_t          */
typedef struct {
    int32_t C, S, H, K;
    gati_dtype_t act_dtype;
    gati_layout_t layout;
    float threshold;
    int32_t max_rows;
    gati_selector_t selector;
    gati_predictor_t predictor;
    int32_t in_h, in_w, out_h, out_w; /* GATI_PRED_POOL_FC (all four); GATI_PRED_CONV_FC (in_h, in_w) */
    int32_t selector_hidden;          /* GATI_SEL_HIDDEN only: units in the selector's hidden layer */
    int32_t conv_k, conv_s;           /* GATI_PRED_CONV_FC only: filter size and stride */
} gati_cache_desc_t;

/* Weights, HOST pointers, fp32, row-major [out, in].  Copied (and converted) by
 * gati_cache_create; the caller may free them as soon as it returns. */
typedef struct {
    const float *W1; /* [H, C]                                                    */
    const float *b1; /* [H]                                                       */
    const float *W2; /* [K, H]                                                    */
    const float *b2; /* [K]                                                       */
    const float *ws; /* [C + K]: weights of the pooled features first, then of the class probabilities;
                        may be NULL for GATI_SEL_SOFTMAX and GATI_SEL_HIDDEN, which do not read it */
    float bs;        /* selector bias (GATI_SEL_HIDDEN: bias of its second layer)  */
    /* GATI_SEL_HIDDEN only (may be NULL otherwise); F = number of features, as for ws: */
    const float *Ws; /* [selector_hidden, F + K]: features first, then class probabilities */
    const float *cs; /* [selector_hidden] first-layer bias                        */
    const float *vs; /* [selector_hidden] second-layer weights                    */
} gati_cache_weights_t;

/* Build a cache on the current HIP device: uploads the weights in the library's private
 * layout and allocates a workspace for max_rows rows.  *out is set only on GATI_OK. */
gati_status_t gati_cache_create(const gati_cache_desc_t *desc, const gati_cache_weights_t *weights,
                                gati_cache_t **out);

/* Free everything the cache owns.  The caller must have finished (synchronised) all work
 * that uses it.  NULL is GATI_OK. */
gati_status_t gati_cache_destroy(gati_cache_t *cache);

/* Replace every weight of an existing cache with a new set of the same shapes (Section 5,
 * "Retraining Learned Caches": the adaptation service periodically retrains predictor and
 * selector and swaps them in; gati_trainer_* below runs the retraining steps).  Host fp32
 * arrays as for gati_cache_create; repacked and copied before the call returns.  The call
 * waits for all work on the device first, so lookups enqueued earlier use the old weights and
 * lookups issued afterwards the new ones; no allocation takes place.  The threshold is kept. */
gati_status_t gati_cache_set_weights(gati_cache_t *cache, const gati_cache_weights_t *weights);

/* Replace the selector bias and threshold of an existing cache (host scalars).  They travel to the
 * device as kernel arguments, so the change holds for calls enqueued after this one; launches
 * already recorded in a captured HIP graph keep the values they were captured with (re-capture
 * to change them). */
gati_status_t gati_cache_set_selector(gati_cache_t *cache, float bs, float threshold);

/* One lookup per active row (Section 3: prediction operation, then selection operation).
 *
 *   act         device; the layer's activation tensor.  Row r starts at act + r*C*S*elem.
 *   row_index   device [n] int32 or NULL.  Active row i reads activation row row_index[i]
 *               (NULL: row i).  Entries must address rows that exist in act.
 *   n_max       host upper bound on the number of active rows, 0 <= n_max <= max_rows.
 *   n_dev       device int32 scalar holding the true count, or NULL for n = n_max.  The
 *               kernels use min(max(*n_dev,0), n_max), so a previous layer's miss count can
 *               feed this call without a host round trip.
 *   pred_class  device [n_max] int32   argmax of the logits, lowest index on ties
 *   confidence  device [n_max] float   selector confidence
 *   hit         device [n_max] uint8   1 = hit, 0 = miss
 *   logits      device [n_max, K] float or NULL to skip writing them
 *   stream      hipStream_t (NULL = the default stream)
 *
 * Outputs at indices >= n are left untouched.  n = 0 is GATI_OK and writes nothing.
 * Calls on the same cache must not overlap in time (they share its workspace). */
gati_status_t gati_cache_lookup(gati_cache_t *cache, const void *act, const int32_t *row_index,
                                int32_t n_max, const int32_t *n_dev,
                                int32_t *pred_class, float *confidence, uint8_t *hit,
                                float *logits, void *stream);

/* The pooling step alone (pooling predictor, Section 3): pooled[i, c] = mean over s of the
 * activation of active row i, fp32.  pooled is device [n_max, F] with F = C (or the
 * C*out_h*out_w ReLU'd window means of GATI_PRED_POOL_FC).  Same row_index / n_max /
 * n_dev meaning as gati_cache_lookup. */
gati_status_t gati_cache_pool(gati_cache_t *cache, const void *act, const int32_t *row_index,
                              int32_t n_max, const int32_t *n_dev, float *pooled, void *stream);

/* Misses continue to the next layer (Section 1: a request that misses keeps running on
 * the base model): ids_out = [ids_in[i] for i < n if hit[i] == 0], order preserved;
 * *n_miss_dev = number written.
 *
 *   hit         device [n_max] uint8 (any non-zero byte is a hit)
 *   ids_in      device [n_max] int32 or NULL for the identity list 0..n-1
 *   n_max,n_dev as above (cache->max_rows bounds n_max when cache is not NULL; cache may be
 *               NULL, the call needs no cache state)
 *   ids_out     device [n_max] int32; must not alias ids_in
 *   n_miss_dev  device int32 scalar; may alias n_dev (it is read before it is written)
 *
 * Lists of up to 4096 entries are compacted by one workgroup in one launch.  Longer lists take two
 * launches over many workgroups that share a 4 KB table of per-span miss counts in device memory;
 * the library allocates that table (hipMalloc) the first time a device sees n_max > 4096 and keeps
 * it until the process ends, so such calls must not overlap in time on one device, and the first
 * of them must not be issued under stream capture. */
gati_status_t gati_compact_misses(gati_cache_t *cache, const uint8_t *hit, const int32_t *ids_in,
                                  int32_t n_max, const int32_t *n_dev,
                                  int32_t *ids_out, int32_t *n_miss_dev, void *stream);

/* gati_compact_misses for callers that cannot allocate device memory at all: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results; the
 * table of per-span miss counts lives in a fixed array inside the library's code object (4 KB per
 * GPU, present from load until the process ends), so no call ever allocates or frees anything.
 * n_max above GATI_COMPACT_STATIC_MAX_ROWS is GATI_ERR_UNSUPPORTED.  Every call on a GPU uses that
 * GPU's one array: calls with n_max > 4096 that overlap in time on one GPU (two streams, two
 * threads) race and give wrong lists; calls on one stream are safe.  Nothing needs clearing between
 * calls: each call writes every table entry it later reads. */
#define GATI_COMPACT_STATIC_MAX_ROWS (1 << 22)
gati_status_t gati_compact_misses_static(gati_cache_t *cache, const uint8_t *hit, const int32_t *ids_in,
                                         int32_t n_max, const int32_t *n_dev,
                                         int32_t *ids_out, int32_t *n_miss_dev, void *stream);

/* gati_cache_lookup followed by gati_compact_misses on its hit flags, as one call: the last
 * kernel of the lookup also compacts (Section 1 / Appendix A.1: only the misses of one
 * layer's cache reach the next layer's).  Arguments as in the two calls above; ids_out and
 * n_miss_dev are required; outputs are identical to calling the two entry points in turn. */
gati_status_t gati_cache_lookup_compact(gati_cache_t *cache, const void *act, const int32_t *row_index,
                                        int32_t n_max, const int32_t *n_dev,
                                        int32_t *pred_class, float *confidence, uint8_t *hit,
                                        float *logits, const int32_t *ids_in,
                                        int32_t *ids_out, int32_t *n_miss_dev, void *stream);

/* Static, never-NULL description of a status code. */
const char *gati_status_string(gati_status_t status);

/* Name of the pooling kernel variant the cache dispatches to ("ncs_wave", "ncs_segw",
 * "ncs_seg", "nsc_unit", "nsc_vec", "generic", "ncs_adaptive", "adaptive_generic", "fc_flat", "fc_flat_generic", "conv_mfma",
 * "conv_generic"); static string, for reports and profiles. */
const char *gati_cache_pool_variant(const gati_cache_t *cache);

/* ---------------------------------------------------------------------------------------------
 * Retraining (Section 3, "Training Learned Caches"; Section 5, "Retraining Learned Caches":
 * predictor and selector are retrained periodically on recently served inputs, for which the
 * base DNN's output is known, and the new weights replace the old ones).  A trainer holds fp32
 * master weights on the device and runs SGD steps on them; gati_trainer_get_weights +
 * gati_cache_set_weights move the result into a serving cache.
 *
 * The paper names the ingredients of the two losses (true labels and the base DNN's class distribution
 * for the predictor; a heavier penalty on selector false positives) and prints no formula: the target
 * t, L_pred and L_sel below are THIS LIBRARY'S READING of Section 3, "Training Learned Caches", with
 * alpha and fp_weight as parameters because the paper gives no values.
 *
 * One step on a batch of n samples, all arithmetic in fp32:
 *   p        pooled features of the sample (what gati_cache_pool writes)
 *   h        = relu(W1 p + b1),  z = W2 h + b2,  q = softmax(z)
 *   target   t = (1 - alpha) onehot(label) + alpha Y          Y: the base DNN's class distribution
 *   L_pred   = -(1/n) sum_i sum_k t_ik log q_ik               (reading of the distillation-style loss)
 *   G_i      = [argmax_k z_ik == argmax_k Y_ik], lowest index on ties   (selector ground truth)
 *   c_i      = 1/(1 + exp(-(ws . [p_i ; q_i] + bs)))
 *   L_sel    = -(1/n) sum_i [ G_i log c_i + fp_weight (1 - G_i) log(1 - c_i) ]
 *                                                              (false positives cost fp_weight times more)
 *   every weight theta <- theta - lr dL/dtheta, with L_pred for W1, b1, W2, b2 and L_sel for ws, bs;
 *   the selector sees q as data (L_sel has no gradient into the predictor), and uses the q and
 *   the G of before the update.
 * With GATI_SEL_HIDDEN (Section 3, "Selector Network Design": the selector has one hidden layer) the
 * selector is g_i = relu(Ws [p_i ; q_i] + cs), c_i = 1/(1 + exp(-(vs . g_i + bs))) with the same loss;
 * its gradients reach Ws, cs, vs and bs through the ReLU, never q.
 * With GATI_PRED_POOL_FC (the paper's Pool(h)) there is no hidden layer: p are the C*out_h*out_w ReLU'd
 * window means gati_cache_pool writes for such a cache, z = W2 p + b2, and W1, b1 are not used (NULL).
 * With GATI_PRED_FC_MLP (the paper's FC(h)) the input rows are the flattened activation (D = C*S values,
 * as fp32), W1 is [H, D], and the selector reads [h ; q] -- the hidden layer and the class distribution,
 * as the lookup does -- both as data: L_sel sends no gradient into the predictor.
 * With GATI_PRED_CONV_FC (the paper's Conv(k,s)) the input rows are the channel-major map (C*in_h*in_w
 * values, as fp32), W1 is [H, C, conv_k, conv_k] (H filters), h = relu(conv(x, W1, stride conv_s) + b1)
 * flattened [filter][oy][ox], W2 is [K, F] and the selector reads [h ; q] (F + K inputs).
 * With GATI_SEL_SOFTMAX (no selector network) only the predictor is trained: L_sel = 0, ws and bs are not
 * used and gati_trainer_get_weights leaves them alone (ws may be NULL).
 * act_dtype, layout and threshold of the descriptor are ignored; S, in_h, in_w, conv_k, conv_s matter for
 * the predictors that name them above.                                                             */
typedef struct gati_trainer gati_trainer_t; /* opaque, owned by the library */

typedef struct {
    float lr;        /* learning rate, >= 0 (Section 7 uses 0.002)          */
    float alpha;     /* weight of the base DNN's distribution in the target, in [0, 1] */
    float fp_weight; /* penalty factor of selector false positives, >= 0   */
} gati_train_params_t;

/* Build a trainer on the current HIP device from host fp32 weights (as for gati_cache_create)
 * with a workspace for desc->max_rows samples per step.  *out is set only on GATI_OK. */
gati_status_t gati_trainer_create(const gati_cache_desc_t *desc, const gati_cache_weights_t *weights,
                                  gati_trainer_t **out);

/* Free everything the trainer owns; the caller has synchronised its work.  NULL is GATI_OK. */
gati_status_t gati_trainer_destroy(gati_trainer_t *trainer);

/* Enqueue one SGD step on `stream`.
 *   pooled      device [n, ld_pooled] fp32, ld_pooled >= F: row i holds sample i's F input values (F = C;
 *               C*out_h*out_w for GATI_PRED_POOL_FC; C*S for GATI_PRED_FC_MLP and GATI_PRED_CONV_FC)
 *   n           host count, 0 <= n <= max_rows (0: nothing happens)
 *   labels      device [n] int32 true class, in [0, K)
 *   teacher     device [n, ld_teacher] fp32, ld_teacher >= K: the base DNN's class probabilities
 *   losses      device [2] fp32 or NULL: L_pred and L_sel of the batch under the weights of
 *               BEFORE the update
 * Nothing is allocated and nothing synchronises.  Steps on one trainer must not overlap in time
 * (they share its workspace); results do not depend on anything but the arguments. */
gati_status_t gati_trainer_step(gati_trainer_t *trainer, const float *pooled, int32_t ld_pooled, int32_t n,
                                const int32_t *labels, const float *teacher, int32_t ld_teacher,
                                const gati_train_params_t *params, float *losses, void *stream);

/* Copy the current weights to HOST arrays W1 [H, C], b1 [H], W2 [K, H], b2 [K], ws [C + K] and
 * *bs, after waiting for all work on the device; shapes as gati_cache_create takes them for the
 * trainer's predictor (FC(h): W1 [H, C*S], ws [H + K]; Conv(k,s): W1 [H, C, k, k], W2 [K, F],
 * ws [F + K]).  A trainer with a hidden-layer selector or without a selector network has no ws
 * (NULL is accepted there); the hidden-layer selector comes from gati_trainer_get_hidden_selector.
 * A GATI_PRED_POOL_FC trainer has no W1, b1 (NULL accepted); its W2 is [K, F] and ws [F + K]. */
gati_status_t gati_trainer_get_weights(gati_trainer_t *trainer, float *W1, float *b1, float *W2, float *b2,
                                       float *ws, float *bs);

/* The hidden-layer selector's weights to HOST arrays Ws [selector_hidden, C + K], cs and vs
 * [selector_hidden]; GATI_ERR_UNSUPPORTED for a trainer with the linear selector. */
gati_status_t gati_trainer_get_hidden_selector(gati_trainer_t *trainer, float *Ws, float *cs, float *vs);

/* A second handle on the same cache for concurrent use: the fork shares the weights, tables and selector
 * scalars of `cache` (Section 5: one deployed predictor / selector per layer) and has a workspace of its
 * own, so lookups through the fork may overlap in time with lookups through `cache` or through other
 * forks, e.g. on another stream - calls through ONE handle still may not overlap, since they share that
 * handle's workspace.  Weights and the selector change only through the cache that was created
 * (gati_cache_set_weights, gati_cache_set_selector and gati_cache_load_trainer return
 * GATI_ERR_INVALID_ARG for a fork) and are then seen by every fork, under the ordering rules of those
 * calls.  Allocates the workspace (GATI_ERR_OOM if that fails) and waits for the device once; must be
 * called with the cache's device current.  A fork is destroyed with gati_cache_destroy; destroying a cache
 * that still has forks returns GATI_ERR_INVALID_ARG and destroys nothing.  Forking and destroying handles of
 * one cache from several host threads at once is not supported. */
gati_status_t gati_cache_fork(gati_cache_t *cache, gati_cache_t **fork);

/* Put a trainer's current weights into a serving cache without leaving the device (Section 5: the
 * retrained predictor and selector replace the old ones while serving goes on).  Kernels on `stream`
 * repack the trainer's fp32 master weights into the cache's own layouts (bf16 caches round to nearest
 * even, as gati_cache_create does), so the swap is ordered with whatever else is enqueued on that
 * stream: retraining steps enqueued before it are included, lookups enqueued before it on the same
 * stream see the old weights and lookups enqueued after it the new ones.  Nothing is allocated and
 * other streams are not waited for.  With a selector network the call then waits for `stream` itself
 * (not for the device) to read back one scalar, the selector bias, which reaches the lookup kernels as
 * an argument.  Cache and trainer must have been created on the same device for the same predictor,
 * selector mode and shapes (GATI_ERR_INVALID_ARG otherwise).  The caller keeps lookups on OTHER streams
 * away from the cache until the stream has passed the swap. */
gati_status_t gati_cache_load_trainer(gati_cache_t *cache, gati_trainer_t *trainer, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GATI_H */
