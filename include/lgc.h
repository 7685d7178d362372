/*
 * liblgc — per-node compression hot path of Learned Gradient Compression (LGC)
 * for AMD MI355X (gfx950).  C ABI; no C++ or framework types cross it.
 *
 * The calls follow the state and the steps of the paper's Alg. 1 / Alg. 2
 * (per-node loop of the parameter-server and ring-allreduce variants):
 *
 *   g       fresh gradient of this iteration            (grad Loss)
 *   v       accumulated gradient / residual             (g_acc, g_l)
 *   u       momentum buffer of the momentum correction  (Sec. V-A, last paragraph)
 *   vals    the selected values g~ in ascending index order, idx their positions
 *   latent  E_c(g~), rec = D_c(latent)                   (Sec. IV)
 *   dense   the averaged reconstructed gradient          (Sec. V-B)
 *
 * Conventions (all entry points)
 *  - Every data pointer is a DEVICE pointer owned by the caller, fp32 or uint32,
 *    contiguous.  The library keeps no pointer after a call returns (the
 *    autoencoder handle copies its weights when it is created).
 *    The arrays of one call must not overlap each other (nor the nodes' rows
 *    of one array: stride >= n); what an entry point reads and what it
 *    writes is stated with it.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work: they never synchronise the stream and never read
 *    results back to the host.  Outputs are valid once the stream has drained.
 *  - Several simulated nodes are handled in one call: `batch` nodes whose
 *    arrays start `stride` ELEMENTS apart (node b uses base + b*stride;
 *    stride >= n).  batch = 1 is the single-node form.
 *  - A context owns only scratch memory.  One context serves one stream at a
 *    time and is not thread-safe; calls on one context that overlap race.
 *    Different contexts may work on different streams at the same time, any
 *    number of them.  In one kernel of the library blocks wait for other
 *    blocks (the exact selection in one launch: the fall-back of a node whose
 *    sampled threshold failed, and exact selection of mid-sized inputs): a
 *    block there only ever waits for work that was handed out, earlier, to a
 *    block that is already running, so the waits end whatever else shares the
 *    device; they are bounded all the same (an expired wait gives invalid
 *    outputs, a non-zero error count in lgc_stats and LGC_EDEVICE, never a hang).
 *  - No call between lgc_create / lgc_reserve and lgc_destroy allocates or
 *    frees device memory or synchronises (lgc_stats and lgc_profile_read, which
 *    read back, aside), and none uses a memset: the calls can be recorded into
 *    a HIP graph (stream capture).  The
 *    selection calls alternate between two sets of scratch state from call
 *    to call, so a graph that is replayed must hold an EVEN number of
 *    selection calls (lgc_topk, lgc_accumulate_topk and their per-layer forms)
 *    per context.
 *  - Argument errors are detected on the host before anything is launched and
 *    reported as LGC_EINVAL (null pointer, n == 0, n >= 2^31, k > n, k, n or
 *    batch beyond what the context was created for, stride < n, pointers not
 *    4-byte aligned).  k == 0 is valid: nothing is selected.
 *  - No exceptions cross the boundary.  lgc_last_error gives a message for the
 *    last failing call on that context (or, with NULL, of the calling thread).
 */
#ifndef LGC_H
#define LGC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lgc_ctx lgc_ctx; /* opaque: scratch for selection and autoencoder */
typedef struct lgc_ae lgc_ae;   /* opaque: autoencoder description + device copy of its weights */

typedef enum {
    LGC_OK = 0,
    LGC_EINVAL = 1,  /* bad argument; nothing was launched */
    LGC_ENOMEM = 2,  /* host or device allocation failed */
    LGC_EHIP = 3,    /* a HIP runtime call failed */
    LGC_EDEVICE = 4  /* a kernel reported an internal failure (see lgc_stats) */
} lgc_status;

/* Create a context on HIP device `device` able to handle up to max_n elements
 * per node, max_k selected values per node and max_batch nodes per call.
 * Allocates all selection scratch here (device memory, a few tens of MB at the
 * largest benchmark shape); nothing else allocates on the selection path. */
lgc_status lgc_create(lgc_ctx **out, int device, uint64_t max_n, uint64_t max_k, int max_batch);
void lgc_destroy(lgc_ctx *ctx);
const char *lgc_last_error(const lgc_ctx *ctx);
const char *lgc_status_string(lgc_status s);

/*
 * a1. Local accumulation with momentum correction — Alg. 1 / Alg. 2, first
 * line of the layer loop (g_l = grad + g_acc), with the DGC-style momentum
 * correction that Sec. V-A refers to:
 *        u <- momentum*u + g ;  v <- v + u        (in place, elementwise)
 * Three separate fp32 roundings per element, never a fused multiply-add;
 * denormals are kept.  momentum = 0 gives the paper's line exactly.
 * A NaN operand, or Inf - Inf, gives a NaN; the sign and the payload of that
 * NaN are not specified (processors differ in which operand's they pass on and
 * in the NaN they generate).  Every result that is not a NaN is bit-exact.
 * g, u, v: [batch][stride] device fp32, n valid elements per node.
 */
lgc_status lgc_accumulate(lgc_ctx *ctx, const float *g, float *u, float *v, uint64_t n, int batch,
                          uint64_t stride, float momentum, void *stream);

/*
 * a2. Exact top-k magnitude selection with residual update — Alg. 1 / Alg. 2:
 * threshold, mask, g~ = mask.*g_l, g_acc keeps the rest.  Exactly k positions
 * per node are selected (Sec. V-A fixes the size of g~): order positions by
 * (|v| descending, index ascending) on the key bits(v) & 0x7fffffff and take
 * the first k.  The key orders every fp32 value: -0 equals +0, NaNs lie above
 * Inf and order among themselves by their payload bits.  Outputs per node b:
 *   out_idx [b*k .. b*k+k)  the selected positions, ascending
 *   out_vals[b*k .. b*k+k)  v at those positions (bit-exact, sign kept)
 * then v <- +0 at the selected positions, and u <- +0 there too (momentum
 * factor masking) unless u is NULL.  Every other element of v, u is untouched.
 * The threshold is found on the device; nothing returns to the host.
 */
lgc_status lgc_topk(lgc_ctx *ctx, float *v, float *u /* nullable */, uint64_t n, int batch,
                    uint64_t stride, uint64_t k, float *out_vals, uint32_t *out_idx, void *stream);

/* a1 + a2 in one pass over g, u, v.  Defined as lgc_accumulate followed by
 * lgc_topk; the results are bit-identical to that pair. */
lgc_status lgc_accumulate_topk(lgc_ctx *ctx, const float *g, float *u, float *v, uint64_t n,
                               int batch, uint64_t stride, float momentum, uint64_t k,
                               float *out_vals, uint32_t *out_idx, void *stream);

/*
 * lgc_accumulate_topk for callers that cannot allocate device memory and cannot
 * hold a context that did: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results bit for bit as
 * lgc_accumulate_topk, but no lgc_ctx: the selection scratch (candidate bitmap,
 * row counts, candidate list, histograms) is a fixed array of
 * LGC_STATIC_SCRATCH_BYTES in the library's device image, which every GPU
 * that runs the library holds until the process ends.  The call allocates and
 * frees nothing, on the device or through the HIP runtime, and never
 * synchronises.  The first call on a device looks the array's address up once.
 *  - Limit: the scratch a context for exactly (n, k, batch) would need must fit
 *    the array: about batch * (n / 8 + 12 * (1.5 k + 9 sqrt(k n / 65536)) + 1 MB)
 *    bytes, e.g. 4 nodes x 25.6 M elements with k = 25 600, or one node of
 *    2^27 elements with k = 2^17.  Larger inputs are rejected with LGC_EINVAL
 *    (the message names the sizes); use a context for them.
 *  - All calls on one GPU share that GPU's array: calls that overlap in time
 *    on one GPU (different streams or threads) race.  The array keeps the last
 *    call's contents; every call clears what it needs at zero with a fill
 *    kernel of its own (no memset), so any number of calls may be recorded
 *    into one HIP graph.
 *  - `device` is the HIP device the pointers live on.  lgc_last_error(NULL)
 *    gives the message of a failing call.  The counters of lgc_stats are not
 *    available through this entry point.
 */
#define LGC_STATIC_SCRATCH_BYTES (32u << 20)
lgc_status lgc_accumulate_topk_static(int device, const float *g, float *u, float *v, uint64_t n, int batch,
                                      uint64_t stride, float momentum, uint64_t k, float *out_vals,
                                      uint32_t *out_idx, void *stream);

/*
 * Autoencoder description — Sec. IV-C, Tables I and II: a stack of 1-D
 * convolutions (encoder) and 1-D transposed convolutions (decoder).
 * Each layer has kernel size 1 or 3, stride 1 or 2 and padding (ksize-1)/2, so
 * a stride-2 layer maps length L to ceil(L/2) (encoder) and back to exactly
 * the length its encoder counterpart consumed (decoder; the two stacks must
 * hold the same number of stride-2 layers).  Leaky-ReLU with `slope`
 * (0 = ReLU) follows every layer except the last of each stack.
 * enc[0].c_in = 1 and dec[n_dec-1].c_out = 1: the input is one node's vector
 * of k selected values.  dec[0].c_in = enc[n_enc-1].c_out.  Consecutive layers
 * must agree in channels, except that the last decoder layer, if it has stride
 * 1, may take one channel more than the layer before it produces: that makes
 * the decoder of the parameter-server pattern (see lgc_decode_innovation).
 * Weights (device pointers, read and COPIED during this call, which
 * synchronises the device once):
 *   enc_w[l]: [c_out][c_in][ksize]   enc_b[l]: [c_out]
 *   dec_w[l]: [c_in][c_out][ksize]   dec_b[l]: [c_out]
 */
typedef struct {
    int32_t c_in, c_out, ksize, stride;
} lgc_layer;

lgc_status lgc_ae_create(lgc_ae **out, int device, int n_enc, const lgc_layer *enc, int n_dec,
                         const lgc_layer *dec, float slope, const float *const *enc_w,
                         const float *const *enc_b, const float *const *dec_w,
                         const float *const *dec_b);
void lgc_ae_destroy(lgc_ae *ae);
/* Floats per node in the latent for an input of k values: C_latent * L_latent. */
uint64_t lgc_latent_len(const lgc_ae *ae, uint64_t k);

/* a3. Encoder g^c = E_c(g~) (Sec. IV, Table I).  vals: [batch][k];
 * latent: [batch][C_latent][L_latent] (channel-major per node).
 * fp32 arithmetic with fp32 accumulation.  k == 0 is a no-op.
 * Stacks other than two kernel-3 / stride-2 layers of up to 16 channels keep
 * their intermediate tensors in the context's activation scratch, which must
 * have been reserved (lgc_reserve); the call itself never allocates. */
lgc_status lgc_encode(lgc_ctx *ctx, const lgc_ae *ae, const float *vals, uint64_t k, int batch,
                      float *latent, void *stream);

/* a4. Decoder g^rec = D_c(latent) (Sec. IV, Table II).  rec: [batch][k]. */
lgc_status lgc_decode(lgc_ctx *ctx, const lgc_ae *ae, const float *latent, uint64_t k, int batch,
                      float *rec, void *stream);

/*
 * a5. Placement and node average — Sec. V-B, g^rec = (1/K) sum_k g_k^rec
 * written back at the selected positions:
 *        dense[idx[b][j]] <- dense[idx[b][j]] + scale*vals[b][j]
 * for nodes b = 0..batch-1 applied strictly in that order (product and sum
 * rounded separately).  Within one node idx must be strictly ascending (which
 * lgc_topk's output is); across nodes positions may repeat.  vals, idx:
 * [batch][k]; dense: [n], normally zero-filled by the caller beforehand.  An
 * index >= n is skipped and counted as a device error (lgc_stats); so is,
 * for batch > 1, a position that is not above its predecessor (the result is
 * then unspecified at positions that several nodes hold).
 */
lgc_status lgc_scatter(lgc_ctx *ctx, const float *vals, const uint32_t *idx, uint64_t k, int batch,
                       float scale, float *dense, uint64_t n, void *stream);

/* ---- per-layer selection (Sec. V-A; layer loop of Alg. 1 / Alg. 2) ---- */

/*
 * The paper selects per layer: the flat vector is the concatenation of the
 * layers' gradients, layer l keeps its own mu_l = alpha/100 * n_l largest
 * magnitudes, and the kept values of all layers are concatenated in layer
 * order.  A segment plan describes the layers once (the model does not change
 * between iterations):
 *   offsets: HOST array [n_seg + 1], offsets[0] = 0 < ... < offsets[n_seg] = n
 *            (segment l is [offsets[l], offsets[l+1]), none empty)
 *   ks:      HOST array [n_seg], ks[l] <= n_l values kept in segment l (0 allowed)
 * Both are read during the call only.  The plan lives on `device`.
 */
typedef struct lgc_segments lgc_segments;
lgc_status lgc_segments_create(lgc_segments **out, int device, uint64_t n, uint64_t n_seg,
                               const uint64_t *offsets, const uint64_t *ks);
void lgc_segments_destroy(lgc_segments *seg);
uint64_t lgc_segments_total_k(const lgc_segments *seg); /* sum of ks: outputs per node */

/*
 * Per-layer exact top-k with residual update.  Every segment is selected
 * exactly like the flat vector in lgc_topk (same key, same tie rule, exactly
 * ks[l] positions).  Outputs per node b, K = lgc_segments_total_k(seg):
 *   out_idx [b*K ..)  positions in the flat numbering: segment 0's (ascending),
 *                     then segment 1's, ... — ascending overall
 *   out_vals[b*K ..)  v at those positions, bit-exact
 * then v <- +0 and (unless u is NULL) u <- +0 there.  n is the plan's n; it and
 * K must fit the context (max_n, max_k).  The scratch for the plan must have
 * been reserved (lgc_reserve); the call itself never allocates.
 */
lgc_status lgc_topk_segmented(lgc_ctx *ctx, const lgc_segments *seg, float *v, float *u /* nullable */,
                              int batch, uint64_t stride, float *out_vals, uint32_t *out_idx, void *stream);

/* lgc_accumulate followed by lgc_topk_segmented, in one pass over g, u, v;
 * bit-identical to that pair. */
lgc_status lgc_accumulate_topk_segmented(lgc_ctx *ctx, const lgc_segments *seg, const float *g, float *u,
                                         float *v, int batch, uint64_t stride, float momentum,
                                         float *out_vals, uint32_t *out_idx, void *stream);

/* ---- parameter-server pattern: innovation component (Alg. 1, Sec. IV-C, Sec. V-B) ---- */

/*
 * Innovation component g~^I — Alg. 1 (threshold_inv, mask_inv, g~^I = g~ .*
 * mask_inv): a vector of the size of g~ holding the top-magnitude values of g~
 * and +0 elsewhere.  Alg. 1 forms it inside the layer loop, so it is taken per
 * segment of g~: `seg` is a plan over the vector of selected values (n = its
 * length, offsets = where each layer's values start, ks = values kept per
 * layer; one segment covering everything gives the flat form).  Key and tie
 * rule as in lgc_topk; exactly ks[l] values are kept per segment.
 * vals: [batch][n], not modified;  out: [batch][n], must not alias vals.
 * One block works on one segment of one node, which suits the paper's layers;
 * a single segment of millions of values is correct but slow.
 */
lgc_status lgc_innovation(lgc_ctx *ctx, const lgc_segments *seg, const float *vals, int batch, float *out,
                          void *stream);

/*
 * Decoder of the parameter-server pattern, g^rec = D_c(g^c, g~^I) — Sec. IV-C:
 * before the final layer the intermediate representation (length k) is
 * concatenated with the innovation component as one more channel, appended
 * last.  The autoencoder must have been created with a decoder whose last
 * layer has stride 1 and c_in = (c_out of the layer before) + 1; lgc_decode
 * rejects such an autoencoder and this call rejects any other.
 * innov: [batch][k] (lgc_innovation's output);  rec: [batch][k].
 */
lgc_status lgc_decode_innovation(lgc_ctx *ctx, const lgc_ae *ae, const float *latent, const float *innov,
                                 uint64_t k, int batch, float *rec, void *stream);

/* ---- ring-allreduce pattern (Sec. V-A, Sec. V-C, Alg. 2) ---- */

/*
 * Values at positions another node selected — Sec. V-A: under ring-allreduce
 * one node selects and shares its positions; every other node builds its g~
 * from the same positions, and the mask / residual lines of Alg. 2 apply with
 * that mask.  For every node b and j < k:
 *        out_vals[b][j] = v[b][idx[j]] ;  v[b][idx[j]] = +0 ;  u[b][idx[j]] = +0
 * idx: [k] device uint32, ONE list shared by all `batch` nodes, distinct
 * (lgc_topk's out_idx of the selecting node); u may be NULL.  A position >= n
 * yields 0 and is counted as a device error (lgc_stats).
 */
lgc_status lgc_gather(lgc_ctx *ctx, float *v, float *u /* nullable */, uint64_t n, int batch,
                      uint64_t stride, const uint32_t *idx, uint64_t k, float *out_vals, void *stream);

/* lgc_accumulate (a1) followed by lgc_gather: the whole per-iteration work of a
 * node that does not select (one streaming pass, no selection at all). */
lgc_status lgc_accumulate_gather(lgc_ctx *ctx, const float *g, float *u, float *v, uint64_t n, int batch,
                                 uint64_t stride, float momentum, const uint32_t *idx, uint64_t k,
                                 float *out_vals, void *stream);

/*
 * Average of the nodes' compressed representations — Alg. 2 / Sec. V-C,
 * g^avg = (1/K) sum_k g^c_k:
 *        out[i] = (..((0 + scale*x[0][i]) + scale*x[1][i]) + ..) + scale*x[batch-1][i]
 * every product and sum rounded to fp32 on its own, nodes in order (the same
 * convention as lgc_scatter).  x: [batch][len]; out: [len], may not alias x.
 */
lgc_status lgc_average(lgc_ctx *ctx, const float *x, uint64_t len, int batch, float scale, float *out,
                       void *stream);

/* ---- reservation ---- */

/*
 * Reserves, ahead of the hot path, the scratch that lgc_create cannot size:
 *   ae  (nullable): the activation buffers lgc_encode / lgc_decode /
 *        lgc_decode_innovation need with this autoencoder for inputs of up to
 *        k values per node and up to `batch` nodes (the largest intermediate
 *        tensor of either stack, twice; nothing for stacks that run as one
 *        launch);
 *   seg (nullable): the per-layer thresholds and the candidate list of
 *        lgc_topk_segmented / lgc_accumulate_topk_segmented with this plan.
 * A later reservation only ever grows the buffers, so one call per
 * autoencoder and plan in use covers them all.  May allocate and, when it
 * replaces a smaller buffer, synchronises the device first.  Without the
 * reservation the calls named above return LGC_EINVAL and say so.
 */
lgc_status lgc_reserve(lgc_ctx *ctx, const lgc_ae *ae /* nullable */, uint64_t k, int batch,
                       const lgc_segments *seg /* nullable */);

/* ---- diagnostics (never needed on the hot path) ---- */

/* LGC_OPT_SELECT_PATH: how lgc_topk / lgc_accumulate_topk select (the results
 * are the same whichever way):
 *   0 = automatic (default): the sampled-threshold fast path with the exact
 *       radix path as on-device fall-back; once the library has seen
 *       selections fall back, it takes the exact path outright for some
 *       selections of the context before it tries the fast path again: 1
 *       after the first fall-back, twice as many after each further one, 64
 *       at most, and from 1 again once the fast path has served a selection.
 *       It sees the outcomes without any synchronisation: each selection
 *       stores its number to one of two pinned host words, which the host
 *       reads when it queues the next selection, so the switch comes some
 *       calls late when the host runs ahead of the device, and a recorded
 *       HIP graph keeps the choice made when it was recorded.
 *   1 = always the exact radix path.
 *   2 = always the fast path first, whatever happened before.
 * What the switch is for: where very many magnitudes are equal around the k-th
 * largest, as in quantised gradients, no threshold separates about k elements,
 * and reaching the exact path through the failed fast path costs more than
 * taking it outright (4 nodes x 25.6 M elements of seven distinct values:
 * 1.31 ms against 0.96 ms per accumulate + top-k).
 * LGC_OPT_PROFILE: 1 = time the streaming kernel launches of lgc_accumulate /
 * lgc_topk / lgc_accumulate_topk, their per-layer forms and lgc_accumulate_gather
 * with HIP events (read by lgc_profile_read): the first launch of a call stamps
 * a start event, the last one a stop event; no other packet enters the queue.
 * Leave it off while a stream is being captured into a HIP graph.
 * LGC_OPT_CARRY_THRESHOLD (default 1): the fast path of lgc_topk /
 * lgc_accumulate_topk (and, layer by layer, of their per-layer forms, for the
 * layers long enough to be sampled) needs a threshold with a few more than k
 * elements above it before its pass over the vector.  It samples the vector for one; with this
 * option on it may instead take one worked out on the device from the exact
 * k-th magnitudes of the context's last selections (Alg. 1 / Alg. 2 run
 * every iteration on the same residuals, whose k-th magnitude moves smoothly):
 * their trend continued by one step, lowered by a margin: what the last
 * selection's own candidate count says holds half as many candidates again as
 * k (per layer: twice k_l), or four times the recent distance between the
 * k-th magnitudes and what the two selections before them predicted, if that
 * is more.  The threshold is offered only if the margin is expected to flag
 * no more candidates than the list has room for, after four selections in a
 * row, and only to the next selection of the context with the same n and k
 * (per layer: the same plan).  Results do
 * not depend on it: a threshold that turns out too high or too low sends that
 * node to the exact path, as after a bad sample, and doubles the number of
 * selections in a row (4 at first, 128 at most) that must be on record before
 * the next offer.  0 = always sample.  The
 * record is kept and judged on the device, by the selections themselves (any
 * other kind of selection on the context, exact or per-layer, leaves it
 * empty), so it works the same in a replayed HIP graph.  Setting the option
 * synchronises the device and empties the record. */
typedef enum { LGC_OPT_SELECT_PATH = 0, LGC_OPT_PROFILE = 1, LGC_OPT_CARRY_THRESHOLD = 2 } lgc_option;
lgc_status lgc_set_option(lgc_ctx *ctx, lgc_option opt, int64_t value);

/* Synchronises the device and reports, summed since the last call of
 * lgc_stats: selections served by the fast path, selections that fell back
 * to the exact path on the device (one selection = one node in lgc_topk /
 * lgc_accumulate_topk, one sampled layer of one node in the per-layer calls),
 * and the device-side error count (bounded waits that expired; positions out
 * of range or out of order in lgc_scatter / lgc_gather).  Returns LGC_EDEVICE
 * if errors != 0. */
lgc_status lgc_stats(lgc_ctx *ctx, uint64_t *fast, uint64_t *fallback, uint64_t *errors);

/* Synchronises and reports the selections (nodes) since the last call of this
 * function whose candidate threshold was carried over from earlier selections
 * instead of sampled (see LGC_OPT_CARRY_THRESHOLD). */
lgc_status lgc_stats_carried(lgc_ctx *ctx, uint64_t *carried);

/* Synchronises, then returns the summed duration (ms) and the number of
 * bracketed calls since the last read (a call's streaming work may be several
 * launches: large inputs are streamed in shares of about 2 GB). */
lgc_status lgc_profile_read(lgc_ctx *ctx, double *total_ms, uint64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* LGC_H */
