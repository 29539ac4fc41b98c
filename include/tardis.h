/*
 * libtardis -- partially-linear feed-forward network for one AMD MI355X (gfx950).
 *
 * The method (arXiv 2501.10054, "Accelerating Large Language Models through
 * Partially Linear Feed-Forward Network") replaces each FFN neuron's activation
 * by a line a_j*z + c_j inside a calibrated input range [lo_j, hi_j), folds
 * W2*diag(a)*W1 into one d x d matrix W' with bias b', and at run time computes
 * y = W'x + b', asks a cheap predictor which neurons leave their range, and
 * repairs exactly those neurons with the original weights and activation.
 *
 * Orientation.  The paper writes row vectors, FFN(x) = sigma(x W1) W2 with W1 of
 * size d x h.  This interface uses the transposed, Linear-layer layout:
 *
 *     W1 : h x d row-major  (row j    = neuron j's input weights)
 *     W2 : d x h row-major  (column j = neuron j's output weights)
 *     FFN(x) = W2 * sigma(W1 x + b1) + b2
 *
 * so the paper's folded matrix C is W'^T and its slope/intercept (a, b) are
 * (a_j, c_j) here.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE memory owned by the caller, contiguous,
 *     row-major, 16-byte aligned, unless a parameter says "host".
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Online calls only enqueue work: they never synchronise the host and never
 *     allocate.  Offline calls (calibrate, fold) allocate and free temporaries
 *     and may synchronise.
 *   - Errors are reported by return code only.  Arguments are validated before
 *     anything is launched; an asynchronous GPU fault surfaces at the caller's
 *     next synchronisation.  One stream at a time may use a handle.
 *   - Ranges are half open: a neuron is "in range" iff lo_j <= z_j < hi_j.
 *   - Handles are checked against the library's table of live layers: NULL, a
 *     pointer this library did not hand out, or a destroyed handle gives
 *     TARDIS_ERR_STATE (never a dereference).  If an online call returns
 *     TARDIS_ERR_HIP (a launch failed half way) the handle's working memory is in
 *     an unknown state: every later online call on it returns TARDIS_ERR_STATE;
 *     destroy it and fold again.
 */
#ifndef TARDIS_H
#define TARDIS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TARDIS_VERSION 1

typedef struct tardis_layer_s* tardis_handle_t; /* opaque: one folded FFN layer */

typedef enum {
    TARDIS_OK = 0,
    TARDIS_ERR_INVALID_ARG = 1, /* NULL where data is required, bad enum, misaligned */
    TARDIS_ERR_SHAPE = 2,       /* non-positive or unsupported sizes */
    TARDIS_ERR_DTYPE = 3,       /* dtype not supported by this call */
    TARDIS_ERR_STATE = 4,       /* handle not usable for this call */
    TARDIS_ERR_OOM = 5,         /* device allocation failed */
    TARDIS_ERR_HIP = 6          /* any other HIP runtime error */
} tardis_status_t;

typedef enum {
    TARDIS_ACT_GELU_ERF = 0, /* z * Phi(z) */
    TARDIS_ACT_GELU_TANH = 1,
    TARDIS_ACT_RELU = 2,
    TARDIS_ACT_IDENTITY = 3
} tardis_act_t;

typedef enum {
    TARDIS_F32 = 0,
    TARDIS_BF16 = 1,
    TARDIS_FP8_E4M3 = 2 /* storage of the folded matrix only (tardis_fold_opts.folded_dtype) */
} tardis_dtype_t;

/* One FFN layer (Sec. "Opportunity": FFN(x) = sigma(x W1) W2, here transposed
 * and with the optional biases the paper omits for presentation).
 * `dtype` is the storage type of W1, W2, b1, b2 and of the tokens x and
 * outputs y of the online calls. */
typedef struct {
    int64_t d;       /* model width  (>= 1) */
    int64_t h;       /* hidden width (>= 1) */
    int32_t dtype;   /* tardis_dtype_t */
    int32_t act;     /* tardis_act_t   */
    const void* W1;  /* h x d */
    const void* b1;  /* h, or NULL for zero */
    const void* W2;  /* d x h */
    const void* b2;  /* d, or NULL for zero */
} tardis_ffn_desc;

typedef struct {
    int32_t sketch_bits;   /* predictor code width: 8, or 4, 3, 2 (grouped, see tardis_fold) */
    int32_t folded_dtype;  /* storage of W': desc.dtype, or for a bf16 layer TARDIS_FP8_E4M3 (Sec. "Discussion":
                              the method composes with weight compression): every row of W' gets the
                              smallest power-of-two scale 2^e with max|row| / 2^e <= 448 and its elements
                              are rounded to 8-bit floats (1 sign, 4 exponent bits with bias 7, 3 mantissa
                              bits, no infinities; ties to even) in that scale.  One- and two-token calls
                              stream the 8-bit rows (half the bytes of W'); every other path multiplies a
                              bf16 copy holding the same numbers.  Three mantissa bits move an element by
                              up to 2^-4 of itself: y is then about 3e-2 (relative L2) away from the exact
                              folded result - outside the 1e-2 this library otherwise keeps, which is
                              why it is an option */
    int64_t max_batch;     /* largest n accepted by the batched online calls (1 .. 4096; longer prompts are
                              the caller's to cut); from 65 on the layer
                              also holds scratch for the prompt path, about n * (5 d + 10 h) bytes */
    int32_t deterministic; /* 0, or 1: results that are bit-identical from run to run.  Every online call on
                              the layer then runs as groups of up to 16 tokens whose repair is accumulated
                              in counted fixed-point words (integer adds commute; a word's unit comes from
                              a bound, computed at fold time, on what an output can receive), flagged lists
                              are processed in ascending order, and nothing is summed in an order that
                              depends on timing.  Needs a bf16 layer with d = 1024, 2048 or 4096
                              (TARDIS_ERR_SHAPE otherwise); calls with more than 16 tokens are slower
                              than on a layer folded without it. */
    float margin;          /* 0 <= margin < 0.5: the predictor tests against each neuron's range narrowed by
                              this fraction of its width at either end, lo + margin (hi - lo) <= z' < hi -
                              margin (hi - lo); more neurons are flagged (and repaired exactly), fewer
                              out-of-range ones are missed by a coarse sketch.  0: the range itself. */
} tardis_fold_opts;

/* ---------------------------------------------------------------- offline */

/* Range selection and linear fit (Sec. "Insights", Insight 2, and Sec.
 * "Non-linear Function Approximation": a range holding a portion t of each
 * neuron's calibration inputs, then a least-squares line through the activation
 * on that range).  For every neuron j: z_ij = W1[j].x_i + b1_j over the n_cal
 * calibration tokens; lo_j, hi_j = the (1-t)/2 and (1+t)/2 quantiles (linear
 * interpolation between order statistics); a_j, c_j = ordinary least squares of
 * sigma(z) on z over the samples with lo_j <= z < hi_j (slope 0 and the mean of
 * sigma if fewer than two distinct samples).
 *
 *   X_cal     n_cal x d tokens, desc->dtype.   1 <= n_cal <= 32768.
 *   coverage  the in-range portion t in (0, 1], used for every neuron when
 *             coverage_per_neuron is NULL.
 *   coverage_per_neuron  optional device array of h per-neuron portions.
 *   lo, hi, a, c  device float arrays of length h, written by the call.
 * Synchronises the stream before returning (temporaries are freed). */
tardis_status_t tardis_calibrate(const tardis_ffn_desc* desc, const void* X_cal, int64_t n_cal,
                                 float coverage, const float* coverage_per_neuron,
                                 float* lo, float* hi, float* a, float* c, void* stream);

/* As tardis_calibrate, with the range of every neuron found by the greedy search
 * of Algorithm 1 (its inner loop; Sec. "Non-linear Function Approximation",
 * "Range Searching") instead of central quantiles: the range starts empty at the
 * centroid of the neuron's calibration inputs (mode of a Gaussian kernel density
 * estimate, bandwidth 1.06 std n^(-1/5), evaluated at 256 equally spaced points
 * from the smallest to the largest sample) and grows by `step` at a time, to the
 * left or to the right, whichever candidate range is approximated by its own
 * least-squares line with the smaller sum of |sigma(z) - (a z + c)| over its
 * samples (the right one on equality), until it holds the portion t of the
 * samples.  A side whose end lies beyond every sample is not grown further, so
 * the search ends after at most (max z - min z) / step + 2 steps; a call in which
 * some neuron would need more than 4096 steps (a step far below the spread of
 * that neuron's inputs) returns TARDIS_ERR_INVALID_ARG and its outputs are not
 * to be used.  The layer-level and
 * neuron-level threshold assignment of Algorithm 1 is not part of this call:
 * pass its result through coverage_per_neuron.
 *   step   range increment s > 0, in units of the pre-activation.
 *   1 <= n_cal <= 8192.  Other arguments and behaviour as tardis_calibrate. */
tardis_status_t tardis_calibrate_search(const tardis_ffn_desc* desc, const void* X_cal, int64_t n_cal,
                                        float coverage, const float* coverage_per_neuron, float step,
                                        float* lo, float* hi, float* a, float* c, void* stream);

/* The two estimate_error steps of Algorithm 1 (Sec. "Non-linear Function
 * Approximation", "Adaptive Thresholding"): the empirical error of a layer whose
 * neurons are approximated on the given ranges by the given lines, over the
 * calibration tokens.  Per neuron
 *     E_n = sum_x err_n(x),   err_n(x) = |sigma(z_n) - (a_n z_n + c_n)| * ||W2[:, n]||_2
 * for the inputs with lo_n <= z_n < hi_n (the L2 distance between the neuron's
 * exact and approximated contribution to the output; zero outside the range),
 * and for the layer the sum over its neurons.
 *   lo, hi, a, c   device float arrays of length h (from a calibration call).
 *   err_neurons    h floats, written.    err_layer  one float, written; may be NULL.
 * 1 <= n_cal <= 32768.  Synchronises the stream before returning. */
tardis_status_t tardis_estimate_errors(const tardis_ffn_desc* desc, const void* X_cal, int64_t n_cal,
                                       const float* lo, const float* hi, const float* a, const float* c,
                                       float* err_neurons, float* err_layer, void* stream);

/* error_aware_threshold of Algorithm 1: thresholds (in-range portions) for n items -
 * the layers of a model, or the neurons of a layer - from their errors,
 *     minimise sum_i err_i t_i   subject to   sum_i t_i = t * n,  t_min <= t_i <= t_max.
 * The paper prints the objective and the equality only; without bounds the
 * programme has no minimum, so the caller supplies them (0 <= t_min <= t <= t_max
 * <= 1, else TARDIS_ERR_INVALID_ARG).  The items of largest error get t_min, the
 * others t_max, at most one item in between takes the rest of the budget; among
 * equal errors the lower index counts as the larger.  Feed the result to the
 * coverage_per_neuron argument of a calibration call (neurons), or use one entry
 * per layer as that layer's t.
 *   err    n device floats (finite, >= 0).   t_out  n device floats, written.
 * Stream-ordered; does not synchronise. */
tardis_status_t tardis_assign_thresholds(const float* err, int64_t n, float t, float t_min, float t_max,
                                         float* t_out, void* stream);

/* Constant folding and predictor construction (Sec. "Constant Folded Matrix
 * Generation" and Sec. "Predictor Generation").  Builds
 *     W' = W2 diag(a) W1            (d x d, stored in desc->dtype, rounded once)
 *     b' = W2 (c + a*b1) + b2       (d, fp32)
 * and the predictor: an int8 round-to-nearest per-row symmetric code Q of W1
 * (s_j = max_k|W1[j,k]|/127, q_jk = rint(W1[j,k]/s_j)) with the range bounds in
 * code units, tlo_j = fp32((lo_j-b1_j)/s_j), thi_j = fp32((hi_j-b1_j)/s_j).
 * With opts->sketch_bits = 4 the code is grouped instead (the paper's predictor is
 * a low-bit quantised W1; this is its round-to-nearest form with 4-bit codes): each
 * row is cut into groups G of 32 consecutive columns (the last may be shorter),
 *     g_jG = max_{k in G}|W1[j,k]|,  s_j = max_G g_jG / (7*15),
 *     m_jG = ceil(g_jG / (7 s_j)) clamped to [1,15],
 *     q_jk = rint(W1[j,k] / (m_jG s_j)) clamped to [-7,7],
 * all in fp64 (sketch_bits = 3 and 2: the same with 3 and 1 in place of 7, i.e.
 * codes in [-3, 3] and [-1, 1]; this build keeps them in 4-bit slots, so they cost
 * the bytes of the 4-bit sketch - they are there to measure what narrower codes do
 * to the flags, Sec. "Predictor Size"), and the predictor uses the integer code Q_jk = m_jG q_jk (|Q| <= 105)
 * exactly as it uses the 8-bit code; tlo, thi as above with this s_j.  Storage is
 * 4 bits per weight plus one multiplier per group where the decode kernel reads the
 * packed form (bf16, d = 2048 or 4096), one byte per weight elsewhere; a layer
 * folded for more than 17 tokens per call keeps both, and its calls with 4 to 17
 * tokens read the one-byte form (same integers, faster there).
 *
 * W1, b1, b2 are BORROWED: they must stay valid and unchanged until
 * tardis_destroy (the repair step reads W1 in place).  W2 is copied into a
 * neuron-major h x d transpose owned by the handle and may be released.
 * lo, hi, a, c (device, length h) are copied.  All working memory of the online
 * calls, sized by opts->max_batch, is allocated here.  opts may be NULL
 * (sketch_bits 8, folded_dtype = desc->dtype, max_batch 1).
 * Synchronises the stream before returning. */
tardis_status_t tardis_fold(const tardis_ffn_desc* desc, const float* lo, const float* hi,
                            const float* a, const float* c, const tardis_fold_opts* opts,
                            void* stream, tardis_handle_t* out);

/* ----------------------------------------------------------------- online */

/* One token through the folded layer (Sec. "Inference Runtime"): speculative
 * result W'x + b', predictor pass, and for every flagged neuron j the repair
 *     z_j = W1[j].x + b1_j,  y += (sigma(z_j) - (a_j z_j + c_j)) * W2[:, j].
 * Every flagged neuron is repaired whether or not its exact z_j is in range.
 * The predictor: m = max|x_k|, e = floor(log2 m) - 6, xq_k = clamp(rint(x_k /
 * 2^e), -127, 127); acc_j = sum_k q_jk xq_k (int32); v_j = fp32(acc_j) * 2^e;
 * neuron j is flagged unless tlo_j <= v_j < thi_j.  x with a non-finite entry
 * gives unspecified (but memory-safe) results.
 *   x  d values, desc dtype.   y  d values, desc dtype.  x and y must not alias. */
tardis_status_t tardis_ffn_forward(tardis_handle_t L, const void* x, void* y, void* stream);

/* n tokens (1 <= n <= max_batch), strictly per token: token t is repaired only
 * for the neurons its own predictor pass flagged.  x, y: n x d.
 * How the tokens are processed depends on n (groups of up to 16 tokens per
 * launch; passes of up to 64; from 65 tokens four dense matrix products, as the
 * paper's remark on prompt processing suggests) and never on their values; the
 * masks are the same bits on every path, y agrees to rounding. */
tardis_status_t tardis_ffn_forward_batched(tardis_handle_t L, const void* x, int64_t n, void* y,
                                           void* stream);

/* tardis_ffn_forward_batched for callers that cannot allocate or let a library hold
 * per-handle working memory for them: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The call allocates nothing: the
 * accumulators, completion counters, flagged-neuron records and speculative rows of
 * the decode kernels live in one static device array of the library (about 3.9 MiB
 * on every GPU the library runs on, held until the process ends) instead of the
 * handle's buffers.  Same kernels, same results: masks bit for bit, y to rounding.
 *   n         1 .. 16 tokens.  x, y: n x d, bf16.
 *   mask_out  optional, n x ceil(h/32) words as in tardis_get_last_outliers (the
 *             handle's own record of its last call is NOT updated by this call).
 * Limits: a bf16 layer the single-launch decode kernels serve (d = 1024, 2048 or
 * 4096), h <= 16384; anything else returns TARDIS_ERR_SHAPE (TARDIS_ERR_STATE for a
 * layer without those kernels).  Every call on one GPU shares the one array: calls
 * that overlap in time on the same GPU (two streams, two threads) race; calls on one
 * stream, or otherwise ordered, are safe, and each call clears what it needs zeroed
 * itself. */
tardis_status_t tardis_ffn_forward_static(tardis_handle_t L, const void* x, int64_t n, void* y,
                                          uint32_t* mask_out, void* stream);

/* A stack of folded layers of equal width d and dtype (FFN blocks chained
 * without attention; the glue is this library's choice, the paper has none):
 *     x_0 = x,  y_l = layer_l(x_l),  x_{l+1} = y_l / sqrt(mean(y_l^2) + 1e-6)
 * per token, unit gain, no residual; the normalised activation is rounded to
 * the layer dtype.  y receives the last layer's (un-normalised) output.
 * `layers` is a HOST array of n_layers distinct handles; each layer's predictor
 * output stays readable through tardis_get_last_outliers on its handle.
 * 1 <= n <= every layer's max_batch.  x, y: n x d.
 * One launch per layer by default.  Layers folded with the environment
 * variable TARDIS_STACK_FUSED=1 run a one-token call (bf16, d in {1024, 2048,
 * 4096}, 2..64 layers, not under stream capture) as ONE resident launch whose
 * blocks wait for one another with a bounded number of polls; should a wait
 * ever run out, y is filled with NaNs and the layers are re-armed (results of
 * that call are lost, the handles stay usable).  Same results up to summation
 * order; =2 returns TARDIS_ERR_SHAPE where that launch cannot serve the call
 * instead of falling back. */
tardis_status_t tardis_stack_forward(const tardis_handle_t* layers, int32_t n_layers, const void* x,
                                     int64_t n, void* y, void* stream);

/* A hint, not a computation (nothing in the paper; it only moves memory traffic
 * in time): `next` is the layer whose online call follows L's, as in a model
 * whose layers run in a fixed order.  One- and two-token calls on L then spend
 * the end of their kernel - when most of the chip has finished and the memory
 * system idles - requesting the first predictor rows of `next`, which the next
 * call finds in cache (about 8 % per layer at d = 4096, ffn = 16384).  Results
 * are unchanged.  next may be L itself (the same layer is called again);
 * next = NULL clears the hint; a hint to a layer that has been
 * destroyed since, or of another shape, is ignored.  tardis_stack_forward sets
 * it by itself for the duration of the call.  A HIP graph captured from a
 * hinted call keeps the address it was captured with: like a graph of a
 * destroyed layer's own call, it must not be replayed once `next` is destroyed. */
tardis_status_t tardis_set_next_layer(tardis_handle_t L, tardis_handle_t next);

/* The unmodified FFN, y = W2 sigma(W1 x + b1) + b2, on the same streaming
 * kernels: the dense baseline the folded path is measured against (from 65
 * tokens on, two matrix-core products, as for the folded path's prompts).
 * 1 <= n <= max_batch.  x, y: n x d. */
tardis_status_t tardis_dense_forward(tardis_handle_t L, const void* x, int64_t n, void* y,
                                     void* stream);

/* ------------------------------------------------------------- inspection */

/* Copies of the folded state (stream-ordered).  Wp: d x d in desc dtype; bp: d
 * floats.  Either may be NULL. */
tardis_status_t tardis_get_folded(tardis_handle_t L, void* Wp, float* bp, void* stream);

/* Q: h x d int8, the integer codes the predictor multiplies with (for a 4-bit
 * sketch the products m_jG q_jk); tlo, thi: h floats.  Any may be NULL. */
tardis_status_t tardis_get_predictor_state(tardis_handle_t L, int8_t* Q, float* tlo, float* thi,
                                           void* stream);

/* Group multipliers of a 4-bit sketch: M is h x ceil(d/32) bytes, M[j][G] = m_jG.
 * TARDIS_ERR_STATE for a layer folded with an 8-bit sketch (4-, 3- and 2-bit sketches have them). */
tardis_status_t tardis_get_sketch_groups(tardis_handle_t L, uint8_t* M, void* stream);

/* Predictor output of the most recent online call on this handle, for its n
 * tokens (stream-ordered copies into caller buffers; any may be NULL):
 *   mask    n x ceil(h/32) words; bit (j%32) of word j/32 set iff neuron j flagged
 *   counts  n ints, flagged neurons per token
 *   list    n x h ints; row t holds token t's flagged indices in its first
 *           counts[t] slots, in unspecified order (the mask is canonical)
 * n must equal the token count of that call. */
tardis_status_t tardis_get_last_outliers(tardis_handle_t L, int64_t n, uint32_t* mask,
                                         int32_t* counts, int32_t* list, void* stream);

/* The union over the n tokens of the most recent online call: the neurons flagged
 * by at least one of them - what a batch has to fetch of the original weights
 * (Sec. "Inference Runtime", memory footprint; the batched-decode figures report
 * it).  Computed on the device, stream-ordered; either output may be NULL.
 *   union_mask   ceil(h/32) words, bit layout as in tardis_get_last_outliers
 *   union_count  one int (device memory): the number of set bits
 * n must equal the token count of that call. */
tardis_status_t tardis_get_last_union(tardis_handle_t L, int64_t n, uint32_t* union_mask,
                                      int32_t* union_count, void* stream);

/* The normalised activation this layer handed to the next one in the most
 * recent tardis_stack_forward (n x d, layer dtype; stream-ordered copy).  Only
 * meaningful for a layer that was not last in that stack. */
tardis_status_t tardis_get_handover(tardis_handle_t L, int64_t n, void* out, void* stream);

/* Frees everything the handle owns.  The caller must have synchronised every
 * stream that used it.  NULL is accepted; a pointer that is not a live handle
 * (destroyed before, or never made here) returns TARDIS_ERR_STATE. */
tardis_status_t tardis_destroy(tardis_handle_t L);

/* Static, NUL-terminated description of a status code (host). */
const char* tardis_status_string(tardis_status_t s);

/* TARDIS_VERSION the library was built with. */
int32_t tardis_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TARDIS_H */
