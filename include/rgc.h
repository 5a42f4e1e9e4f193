/* rgc.h -- C ABI of the MI355X (gfx950) Residual Gradient Compression library.
 *
 * The library implements, on ONE GPU, the per-iteration hot path of RedSync's Residual
 * Gradient Compression (arXiv 1808.04357):
 *
 *   compress   (Algorithm 1, inner loop over layers):  V += G;  Masks = select(V, D);
 *              message = compress(V . Masks);  V = V . (1 - Masks)
 *   decompress (Section 2.3, last paragraph before the cost model): the N gathered sparse
 *              messages are added into a dense array.
 *
 * Every function returns an int status (RGC_OK = 0, negative = error) unless stated; no C++
 * exception crosses this boundary.  All tensor and message pointers are DEVICE pointers into
 * memory owned by the caller (hipMalloc / a PyTorch-ROCm tensor); descriptor arrays
 * (rgc_layer[], rgc_msg[], pointer and size arrays) are HOST memory and are copied before
 * the call returns.  Work is enqueued on the caller's HIP stream; nothing synchronises the
 * stream or the device.  The context owns only scratch memory and speed hints: results never
 * depend on what an earlier call left in it.
 * A context serves one call at a time: the calls made on it must be ordered on the device (one
 * stream, or streams the caller has ordered with events) and come from one host thread at a
 * time, because they share its scratch.  Different contexts are independent of each other and
 * may be used from different streams and threads concurrently.
 * Stream capture: the first call that shows a context a new list of layers (or of messages)
 * allocates device tables and uploads them; a repeated call with the same descriptors only
 * launches kernels (rgc_message_means, rgc_clip_coefficient and rgc_compress_layers_threshold
 * also allocate a scratch array on their first use, and so does rgc_compress_layers for layers
 * that select more than about 2 % of their elements or more than 2^20 entries).  After one eager call of the same function
 * with the same descriptors, rgc_compress_layers (and its _scaled and _threshold forms),
 * rgc_message_means, rgc_clip_coefficient and rgc_decompress_accumulate may therefore be
 * recorded into a HIP graph on a capturing stream and replayed: all that changes
 * from step to step (residual, velocity, hints, per-layer state) is device memory.  The calls
 * that copy results to the host (rgc_last_error, rgc_decompress_status and the diagnostics of
 * rgc_diag.h) are not for capture.
 */
#ifndef RGC_H_
#define RGC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------------------- */
#define RGC_OK       0
#define RGC_EINVAL  (-1) /* null pointer, n < 1, n >= 2^31, k < 1, k > n, negative count,
                            unknown flag bit, too many layers/workers for the context     */
#define RGC_ENOMEM  (-2) /* scratch sized at rgc_create is too small for this call, or an
                            allocation failed in rgc_create                                */
#define RGC_EHIP    (-3) /* a HIP runtime call failed; rgc_strerror gives its text         */
#define RGC_EINTERNAL (-4) /* a kernel reported an inconsistency (a bug; results invalid)  */

/* ---- flags -------------------------------------------------------------------------- */
/* rgc_compress_layers, rgc_compress_layers_scaled */
#define RGC_NO_MOMENTUM_MASK 0x1u /* keep the velocity u of sent entries (default clears it) */
#define RGC_NO_HINTS         0x2u /* ignore and do not update the per-layer speed hints:
                                     every layer takes the hint-free multi-pass path        */
#define RGC_NESTEROV         0x4u /* momentum correction in its Nesterov form (see below)    */
#define RGC_SELECT_LARGEST   0x100u /* the communication-set is the k LARGEST elements (see below) */
#define RGC_SELECT_SMALLEST  0x200u /* ... the k SMALLEST elements; at most one of the two     */
/* rgc_compress_layers_threshold: RGC_NO_MOMENTUM_MASK, RGC_NESTEROV and */
#define RGC_THRESHOLD_SEARCH 0x400u /* search the thresholds (Algorithm 3) instead of reusing them */
/* rgc_decompress_accumulate: exactly one of the first two */
#define RGC_OVERWRITE        0x10u /* dense = acc * scale                                   */
#define RGC_ADD_TO_DST       0x20u /* dense = dense + acc * scale (two roundings, no fma)   */
#define RGC_ONE_VALUE        0x80u /* with either of the two: every message's val points to ONE float
                                      that all its entries carry (quantized messages, Section 2.2) */
#define RGC_VALIDATE         0x40u /* with either of the two: also check the messages on the
                                      device (see rgc_decompress_status)                    */
/* bits of the status word of rgc_decompress_status */
#define RGC_STATUS_INDEX_RANGE 0x1u /* some message holds an index outside [0, n) of its layer */
#define RGC_STATUS_INDEX_ORDER 0x2u /* some message's indices are not strictly ascending       */

typedef struct rgc_ctx rgc_ctx; /* opaque */

/* One layer of a compression call (host struct holding device pointers).
 * Section 2, Algorithm 1: G_j is `grad`, V_j is `residual`; Section 2.5 names the
 * momentum-corrected variant, whose velocity is `momentum`.  Tensors are flat, contiguous
 * fp32; only 4-byte alignment is required (16-byte aligned tensors take the fast loads). */
typedef struct {
  const float* grad;      /* [n] read only                                                  */
  float*       residual;  /* [n] in/out: V on entry, masked V + G (or V + u) on return      */
  float*       momentum;  /* [n] in/out velocity u, or NULL for the plain variant           */
  int64_t      n;         /* 1 <= n < 2^31                                                  */
  int32_t      k;         /* 1 <= k <= n, number of entries to send (rgc_k_for_density)     */
  int32_t*     out_idx;   /* [k] layer-local 0-based indices, strictly ascending            */
  float*       out_val;   /* [k] out_val[j] = accumulated value at out_idx[j], sign kept    */
  int32_t*     out_count; /* [1] device word, receives k: the message's length element
                             (Section 2.3: a message starts with an element that gives its length) */
} rgc_layer;

/* One (worker, layer) message handed to decompression: `count` entries, `idx` strictly
 * ascending and < n of that layer (what rgc_compress_layers emits).  count is a host value. */
typedef struct {
  const int32_t* idx;
  const float*   val;
  int32_t        count;
} rgc_msg;

/* Create a context on HIP device `device_id` able to handle calls whose layers hold at most
 * `max_total_elems` elements in total, in at most `max_layers` layers.  Allocates all scratch
 * once (about 0.51 byte per element plus 80 KiB per layer); later compression calls allocate
 * device memory only when they see a layer list (pointers, sizes) not seen recently.
 * Decompression grows its own tables on first use and when a call needs more.
 * Errors: RGC_EINVAL (null out, sizes < 1), RGC_ENOMEM, RGC_EHIP. */
int rgc_create(rgc_ctx** out, int device_id, int64_t max_total_elems, int32_t max_layers);

/* Free everything the context owns.  The caller must have synchronised the streams it used. */
int rgc_destroy(rgc_ctx* ctx);

/* k = max(1, ceil(n * density_ppm / 1e6)) clipped to n, in integer arithmetic (Section 2.1
 * uses density 0.1 % = 1000 ppm; n = 1,048,576 gives 1049).  Returns 0 for n < 1. */
int32_t rgc_k_for_density(int64_t n, uint32_t density_ppm);

/* Compression step of Algorithm 1 for `num_layers` independent layers, batched.
 * For each layer:  a = residual + grad            (plain)
 *              or  u = fma(momentum, u, grad) with one rounding; a = residual + u
 *   the k entries of largest |a| are selected exactly (order of the IEEE bit pattern with the
 *   sign cleared; equal magnitudes: lowest index first; NaN above Inf above finite);
 *   out_idx/out_val/out_count receive them in ascending index order;
 *   residual = +0.0f at the selected entries and a elsewhere; the velocity is cleared at the
 *   selected entries too unless RGC_NO_MOMENTUM_MASK.
 * `momentum` (the factor m) is used only by layers whose momentum pointer is non-NULL.
 * Tensors of different layers, and the tensors of one layer, must not overlap.
 * The first call for a layer set (and any call whose cached threshold hint turns out
 * unusable) takes several passes over the data; later calls take one.  The result is the
 * same bit for bit either way.
 * Errors (nothing is enqueued, no buffer is modified): RGC_EINVAL, RGC_ENOMEM, RGC_EHIP. */
int rgc_compress_layers(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers,
                        float momentum, uint32_t flags, void* hip_stream);

/* rgc_compress_layers with every gradient element multiplied first by *grad_scale, a float in
 * DEVICE memory read when the kernel runs (one rounding: g' = fl(scale * g)); NULL = no scaling.
 * This is how the coefficient of local gradient clipping (Section 2.4) enters the accumulate.
 * With RGC_NESTEROV (either entry point) the layers that have a velocity use the Nesterov form
 * of the momentum correction that Section 2.5 names (rule of the DGC paper it defers to):
 *   u = m * (u + g),  a = (V + u) + g,  every operation rounded on its own, left to right. */
int rgc_compress_layers_scaled(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers,
                               float momentum, const float* grad_scale, uint32_t flags,
                               void* hip_stream);

/* Alternating Signs Quantization (Section 2.2): in one iteration the communication-set of a layer
 * is its k largest elements, in the next its k smallest, and the message carries the k indices and
 * ONE value, the average of the k elements.  Here it is three pieces:
 *  - selection: rgc_compress_layers(_scaled) with RGC_SELECT_LARGEST or RGC_SELECT_SMALLEST (the
 *    caller alternates them): the k largest (smallest) elements of the accumulated tensor BY VALUE,
 *    sign included, equal values to the lowest index, +0 and -0 being equal; the paper expects
 *    them to be all positive (negative), and a layer with fewer than k such elements goes on with
 *    its zeros and then the elements of the other sign closest to zero.  NaNs rank by bit pattern
 *    (sign bit clear: above +Inf; set: below -Inf).  Everything else (indices ascending, out_val =
 *    the k accumulated values, masking of residual and velocity) is as in the plain call.  The
 *    speed hints of the three selection modes are kept apart; a layer short of elements of the
 *    expected sign has none and takes the multi-pass path on every call.
 *  - rgc_message_means: means[l] = average of layer l's out_val[0 .. *out_count): the sum of the
 *    values rounded ONCE to fp64 (nearest even; no order of additions enters), divided by the count
 *    in fp64 and rounded to fp32.  A NaN, or infinities of both signs, among the values give NaN,
 *    infinities of one sign that infinity.  `means` is DEVICE memory, num_layers floats.  A length
 *    word above the layer's k (possible only after rgc_compress_layers_threshold, whose messages this
 *    call is not meant for) is read as k.  The
 *    message of layer l is then (count, out_idx, means[l]); layers the caller does not want
 *    quantized (the paper leaves the output layer alone) simply keep their out_val.
 *  - decompression: rgc_decompress_accumulate with RGC_ONE_VALUE takes such messages (val -> the
 *    message's one float).
 * Errors (nothing enqueued): RGC_EINVAL (also both selection flags at once), RGC_ENOMEM, RGC_EHIP. */
int rgc_message_means(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers, float* means,
                      void* hip_stream);

/* rgc_message_means for callers that cannot allocate device or pinned memory when they call: code
 * under HIP stream capture, tight serving loops, harnesses that forbid hipMalloc.  It takes no context
 * and calls no allocating routine, on its first call as little as later; its partial sums live in a
 * static array of the library's code object (1.44 MiB, one copy per GPU, held until the process ends).
 * It runs on the CURRENT HIP device.  values[l] / counts[l]: DEVICE pointers to message l's values and
 * to its length word (what rgc_compress_layers wrote as out_val / out_count); capacity[l]: how many
 * values the buffer holds (the layer's k; a larger length word is read as capacity[l]); the three
 * arrays themselves are HOST memory and are copied into the kernel arguments before the call returns.
 * means: DEVICE, num_layers floats.  Same arithmetic and so the same bits as rgc_message_means on
 * the same messages.
 * Limit: num_layers <= RGC_NOALLOC_MAX_LAYERS, else RGC_ENOMEM (nothing enqueued).
 * All calls on one GPU share that GPU's array: calls that overlap there (two streams, two threads)
 * race; order them on one stream or with events.  Nothing in the array needs to be cleared between calls.
 * Errors (nothing enqueued): RGC_EINVAL, RGC_ENOMEM, RGC_EHIP. */
#define RGC_NOALLOC_MAX_LAYERS 64
int rgc_message_means_noalloc(const float* const* values, const int32_t* const* counts,
                              const int32_t* capacity, int32_t num_layers, float* means,
                              void* hip_stream);

/* The compression step with threshold binary search selection (Section 2.1, Algorithm 3) in place
 * of the exact top-k: the communication-set of a layer is EVERY element of the accumulated tensor
 * whose magnitude exceeds the layer's threshold, so the message length varies.
 *  - With RGC_THRESHOLD_SEARCH the thresholds are searched first, per layer, as Algorithm 3 does:
 *      mean = mean |a|, max = max |a|; l = 0, r = 1;
 *      while r - l > 2^-10: ratio = l + (r - l)/2; t = mean + ratio * (max - mean);
 *                           nnz = #{|a| > t};  k < nnz < 2k: stop;  nnz <= k: r = ratio;  else l = ratio
 *    (the listing's second branch as its text means it; its epsilon, not given, is 2^-10; mean from an
 *    fp64 sum rounded to fp32, everything else in fp32, each operation rounded; if no count falls
 *    between k and 2k the last threshold tried is used), and thresholds[l] receives the result.
 *  - Without the flag thresholds[l] is applied as given: the sampled variant of the same section,
 *    which searches once and reuses the threshold for the next few iterations; the caller keeps the
 *    schedule (the paper's interval is 5).
 * thresholds: DEVICE memory, num_layers floats, read and (with the flag) written when the kernels
 * run.  nnz: DEVICE memory, num_layers int32, or NULL: receives the number of elements above the
 * threshold.  layers[l].k is the k of the search; out_idx and out_val must hold 2 * k entries
 * (k <= 2^30).  *out_count = min(nnz, 2k): if more than 2k elements exceed the threshold (possible
 * with a reused threshold or a search that found no count between k and 2k) the first 2k of them in
 * index order are sent and the others stay in the residual.  Indices ascending, values, masking of
 * residual and velocity, momentum correction (momentum, RGC_NESTEROV, RGC_NO_MOMENTUM_MASK) as in
 * rgc_compress_layers, grad_scale (DEVICE, or NULL) as in rgc_compress_layers_scaled: the paper
 * clips the gradients of its recurrent models, whose large layers are the ones it selects this
 * way.  Inputs must be finite.  Shares the context's scratch with the other calls
 * (one at a time per context) and leaves the speed hints of rgc_compress_layers alone.
 * Errors (nothing enqueued): RGC_EINVAL, RGC_ENOMEM, RGC_EHIP. */
int rgc_compress_layers_threshold(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers,
                                  float momentum, const float* grad_scale, float* thresholds,
                                  int32_t* nnz, uint32_t flags, void* hip_stream);

/* Local gradient clipping (Section 2.4: the gradients of all layers are clipped by their common
 * norm before they are added to the residuals; with N workers the clipping threshold shrinks by the
 * factor sqrt(N)).
 * Enqueues two small kernels that read layers[l].grad of every layer (only grad and n are used) and
 * store  c = norm > t ? t / norm : 1,  t = max_norm / sqrt(num_workers),  norm = the L2 norm over
 * all elements of all layers (the squares are exact in fp64, their sum is rounded to fp64 ONCE, so
 * no order of additions enters; an infinite element gives c = 0, a NaN gives c = 1), into
 * *coefficient, a float in DEVICE memory, for rgc_compress_layers_scaled to use on the same stream.
 * Errors (nothing enqueued): RGC_EINVAL (also max_norm <= 0, num_workers < 1), RGC_ENOMEM, RGC_EHIP. */
int rgc_clip_coefficient(rgc_ctx* ctx, const rgc_layer* layers, int32_t num_layers, float max_norm,
                         int32_t num_workers, float* coefficient, void* hip_stream);

/* Decompression of Section 2.3 for `num_layers` dense buffers and `num_workers` workers.
 * msgs is worker-major: msgs[w * num_layers + l] is worker w's message for layer l.
 * For every layer l and element i:  acc = +0;  for w = 0 .. num_workers-1 in this order:
 * acc += val (fp32) for the entry of worker w with idx == i, if any;  then
 *   RGC_OVERWRITE : dense[l][i] = acc * scale        (every element is written)
 *   RGC_ADD_TO_DST: dense[l][i] = dense[l][i] + acc * scale
 * The summation order is fixed, so the result does not depend on scheduling.
 * dense: host array of num_layers device pointers; n: host array of their lengths.
 * Precondition: each message's idx strictly ascending and < n[l] (what compression emits, and
 * what an Allgather of such messages holds: Section 2.3).  It is not checked unless flags
 * carries RGC_VALIDATE; a message that violates it never makes the kernels leave the buffers
 * they were given, but the dense result is then unspecified.
 * Errors (nothing enqueued): RGC_EINVAL, RGC_ENOMEM, RGC_EHIP. */
int rgc_decompress_accumulate(rgc_ctx* ctx, const rgc_msg* msgs, int32_t num_workers,
                              int32_t num_layers, float* const* dense, const int64_t* n,
                              float scale, uint32_t flags, void* hip_stream);

/* What the RGC_VALIDATE checks of the decompression calls enqueued so far have found: waits for
 * `hip_stream`, stores the OR of their RGC_STATUS_* bits into *out_status (host memory; 0 = all
 * messages met the precondition) and clears the word.  Errors: RGC_EINVAL, RGC_EHIP. */
int rgc_decompress_status(rgc_ctx* ctx, uint32_t* out_status, void* hip_stream);

/* Forget every cached threshold hint, so that the next call behaves like a first call (never changes
 * results). */
int rgc_reset_hints(rgc_ctx* ctx);

/* Whether a kernel of any compression call enqueued so far has reported an internal inconsistency (a
 * candidate list and its histogram that disagree, a message that came out shorter than k: a bug in the
 * library, after which results are invalid).  Waits for `hip_stream`, copies one word.  Returns RGC_OK,
 * RGC_EINTERNAL (it stays set until the context is destroyed), RGC_EINVAL or RGC_EHIP. */
int rgc_last_error(rgc_ctx* ctx, void* hip_stream);

/* Text for a status code; for RGC_EHIP the text of the last HIP error seen by this thread. */
const char* rgc_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* RGC_H_ */
