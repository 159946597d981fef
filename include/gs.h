/*
 * gs.h -- C ABI of the MI355X (gfx950) per-layer optimizer step.
 *
 * The step is the one GreedySnake's vertical schedule produces once per layer
 * (arxiv 2512.17570): the layer's k micro-batch gradients are accumulated in full precision
 * (Sec. 2.1 "Gradient accumulation"; Sec. 3.4), the global L2 norm of the accumulated
 * gradient is reduced for clipping (Sec. 2.1 "Pipelined optimizer step"), and an element-wise
 * Adam(W) update is applied to the three full-precision states of every weight -- master
 * parameter, momentum, variance (Sec. 2.2) -- after which the master parameter is converted
 * to low precision to refresh the working parameter (Sec. 2.2, step (4) of the optimizer
 * figure).  Because the update is element-wise it may be applied to any contiguous range:
 * in full, split into an immediate part and a deferred part (delay ratio alpha, Sec. 4.4),
 * or chunk by chunk over states that live in host memory (Sec. 2.2 chunk loop; Sec. 4.3).
 *
 * Conventions for every entry point
 *   - Plain C types only.  "device" pointers are HIP device addresses, "host" pointers are
 *     ordinary process addresses, "pinned host" pointers come from gs_pinned_alloc (or any
 *     hipHostMalloc).  `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *   - bf16 tensors are arrays of uint16_t holding the upper half of an IEEE binary32.
 *   - Element indices are int64_t.  Ranges are half-open [begin,end); begin == end is a
 *     no-op that returns GS_OK.  begin/end need no alignment.  Every array argument is
 *     indexed by the same absolute element index i in [begin,end); element 0 of each array
 *     must be 16-byte aligned and the arrays must hold at least `end` elements.  Only
 *     elements in [begin,end) are read or written.
 *   - The caller owns all tensors and workspaces.  Pointer tables (`grads`) are host arrays
 *     copied by value at call time; they may be freed as soon as the call returns.
 *   - All device work is enqueued on `stream` and the call returns without waiting.
 *   - Every argument is validated before the first HIP call; a rejected call has touched
 *     nothing.  Functions return a gs_status; nothing throws or aborts.
 *   - Device work runs on the current HIP device; pointers, streams and contexts passed to a
 *     call must belong to it.  The stateless entry points may be called from several host threads
 *     at once; a gs_stream_ctx or gs_tier_ctx must be used by one thread at a time.
 *   - Input and output arrays of one call must not overlap each other, except where a call
 *     states that an output may be its own input.
 *   - Results do not depend on how a range is partitioned: applying the step to [a,b) and
 *     then to [b,c) gives bit-identical p, m, v, w to applying it to [a,c) (Sec. 6.5 requires
 *     results that are reproducible across partition ratios).
 */
#ifndef GS_H
#define GS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GS_OK = 0,
    GS_ERR_INVALID_ARG = -1, /* null pointer, bad range, k out of [1,GS_MAX_K], bad hyper-parameter, misalignment */
    GS_ERR_WORKSPACE = -2,   /* workspace missing or smaller than gs_sqnorm_workspace_bytes() */
    GS_ERR_HIP = -3,         /* a HIP runtime call failed; see gs_last_hip_error() */
    GS_ERR_NOMEM = -4,       /* host or device allocation failed */
    GS_ERR_IO = -5,          /* a file read or write of the file tier failed; see gs_tier_ctx_error() */
    GS_ERR_TOO_LARGE = -6    /* range longer than the fixed scratch array of gs_grad_sqnorm_noalloc covers */
} gs_status;

/* Largest number of micro-batch gradient buffers one call accepts. */
#define GS_MAX_K 32

/*
 * Hyper-parameters of one AdamW step.  The paper names the optimizer (Adam, three fp32
 * states per weight, Sec. 2.2) but prints no arithmetic; the update implemented is
 *     g  = c * sum_j grad_j                         (fp32 sum, j ascending, no 1/k)
 *     m' = beta1*m + (1-beta1)*g
 *     v' = beta2*v + (1-beta2)*g*g
 *     p' = p*(1 - lr*weight_decay) - (lr/(1-beta1^t)) * m' / (sqrt(v')/sqrt(1-beta2^t) + eps)
 *     w  = bf16_round_to_nearest_even(p')
 * with t = step.  Requirements: lr >= 0, 0 <= beta1 < 1, 0 <= beta2 < 1, eps >= 0,
 * weight_decay >= 0, all finite; step >= 1.  max_grad_norm <= 0 disables clipping.
 * Both halves of a split step use the same hparams (same t).
 */
typedef struct {
    float lr;
    float beta1;
    float beta2;
    float eps;
    float weight_decay;
    float max_grad_norm;
    int32_t step;
} gs_adamw_hparams;

/* ------------------------------------------------------------------------------------------
 * Gradient norm (Sec. 2.1: clipping needs the global L2 norm over all gradients, so the
 * optimizer waits for it).
 * ------------------------------------------------------------------------------------------ */

/* Bytes of device workspace the norm-reducing calls need at least; a constant independent of n
 * and k (about 2 MB). */
size_t gs_sqnorm_workspace_bytes(void);

/* Workspace size with which gs_grad_accum_sqnorm, gs_accum_adamw_spec and gs_accum_add (with a
 * norm) run in their fastest shape on a range of `range_elems` elements (one partial per
 * 256-element tile: about range_elems/32 bytes; never less than gs_sqnorm_workspace_bytes()).  Those calls accept any
 * workspace of at least the minimum size and pick the shape that fits; results do not depend on
 * it beyond fp64 summation order.  gs_grad_sqnorm itself gains nothing from a larger workspace. */
size_t gs_sqnorm_workspace_bytes_for(int64_t range_elems);

/*
 * S = sum over i in [begin,end) of a_i^2, where a_i = sum_{j<k} float(grads[j][i]) is the
 * fp32 accumulation of the k bf16 micro-batch gradients (j ascending).  Squares and the
 * reduction are carried in fp64.  The result is deterministic for given arguments.
 *   grads        host array of k device pointers (bf16, each >= end elements)
 *   d_sqnorm     device double; receives S (accumulate == 0) or *d_sqnorm + S (accumulate != 0),
 *                so a caller can build the global norm over several layers or ranges
 *   d_workspace  device buffer of at least gs_sqnorm_workspace_bytes() bytes, 8-byte aligned;
 *                contents need no initialisation and are clobbered.  Calls that share a
 *                workspace must be ordered on one stream.
 * begin == end writes 0 (or leaves *d_sqnorm unchanged when accumulating).
 */
gs_status gs_grad_sqnorm(const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                         double *d_sqnorm, int accumulate,
                         void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * gs_grad_sqnorm for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels,
 * same arguments minus the workspace, same value bit for bit as gs_grad_sqnorm with a workspace of
 * gs_sqnorm_workspace_bytes() bytes; the workgroup partials live in a fixed device array of the
 * library's own (2 098 176 bytes, held by every GPU the library runs on until the process ends).
 * The call makes no hipMalloc/hipFree and uses no allocating library routine.
 *   - end - begin may be at most GS_NOALLOC_MAX_ELEMS; a longer range is GS_ERR_TOO_LARGE and
 *     nothing is enqueued (split it and accumulate).
 *   - The first call on a device looks up that device's copy of the array (one runtime query,
 *     kept afterwards); make that call outside stream capture.
 *   - All calls on one GPU share the one array, which keeps the last call's partials: nothing in
 *     it needs clearing (each launch overwrites what it later reads), but calls that overlap in
 *     time on one GPU -- different streams, different host threads -- race on it.  Order them on
 *     one stream, or use gs_grad_sqnorm with a workspace per stream.
 */
#define GS_NOALLOC_MAX_ELEMS ((int64_t)1 << 33)
gs_status gs_grad_sqnorm_noalloc(const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                                 double *d_sqnorm, int accumulate, void *stream);

/* ------------------------------------------------------------------------------------------
 * Fused accumulate + clip + AdamW + bf16 emit (Sec. 2.1 gradient accumulation in full
 * precision; Sec. 2.2 optimizer step over a parameter chunk; Sec. 4.4 partial update of
 * (1-alpha) / alpha of a layer).
 * ------------------------------------------------------------------------------------------ */

/*
 * Applies the update documented at gs_adamw_hparams to every element of [begin,end).
 *   p, m, v   device fp32, updated in place
 *   w_bf16    device bf16, written (never read)
 *   grads     host array of k device pointers to bf16 gradient buffers, read only.  The fp32
 *             sum of the k buffers lives in registers only; no accumulation buffer exists.
 *   d_sqnorm  device double holding the TOTAL squared gradient norm (all layers / ranges that
 *             are clipped together), as produced by gs_grad_sqnorm; read on the device when
 *             the kernel runs, so no host synchronisation is needed between the two calls.
 *             The clip coefficient is c = min(1, max_grad_norm / (sqrt(S) + 1e-6)).
 *             NULL, or hp->max_grad_norm <= 0, means c = 1.
 * Non-finite gradients propagate by IEEE rules into the states they touch; a NaN norm gives
 * c = 1 and an infinite norm c = 0.  Callers that want to skip such a step read *d_sqnorm.
 * Weight-decay exclusion (biases, LayerNorm) is done by calling per range with
 * weight_decay = 0.
 */
gs_status gs_accum_adamw(float *p, float *m, float *v, uint16_t *w_bf16,
                         const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                         const gs_adamw_hparams *hp, const double *d_sqnorm, void *stream);

/* ------------------------------------------------------------------------------------------
 * Staged two-pass variant (same results, fewer bytes when k > 4).  The paper keeps a layer's
 * gradients accumulated in ONE full-precision GPU buffer (Sec. 1 footnote; Sec. 3.4; Sec. 6.2
 * notes that such gradient buffers are resident in GPU memory); the global-norm dependency (Sec. 2.1) forces two passes over
 * the gradients anyway, so the first pass can leave that fp32 sum behind and the second pass reads
 * 4 bytes per parameter instead of 2k:  (2k+4) + 30 bytes per parameter in total instead of
 * 2k + (2k+26).
 * ------------------------------------------------------------------------------------------ */

/*
 * gs_grad_sqnorm that also writes acc_f32[i] = a_i (the fp32 sum of the k bf16 gradients, j
 * ascending) for i in [begin,end).  acc_f32: device fp32, >= end elements, 16-byte aligned, caller
 * owned.  All other arguments and the value left in *d_sqnorm are exactly those of gs_grad_sqnorm.
 */
gs_status gs_grad_accum_sqnorm(const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                               float *acc_f32, double *d_sqnorm, int accumulate,
                               void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Accumulate as you go (Sec. 3.4, Sec. 4.3: each micro-batch's backward adds its gradient into
 * the layer's full-precision buffer on the GPU).  For i in [begin,end):
 *     acc_f32[i] = (first ? +0 : acc_f32[i]) + widen(grad_bf16[i])
 * so k calls in micro-batch order (first != 0 on the first only) leave exactly the sum that
 * gs_grad_accum_sqnorm writes for the same k buffers.
 *   acc_f32    device fp32, >= end elements, 16-byte aligned; with first != 0 its old contents
 *              are ignored (no clearing pass needed).
 *   grad_bf16  device bf16 bit patterns, >= end elements, 16-byte aligned, read only.
 *   d_sqnorm   NULL, or device fp64 scalar that receives the squared L2 norm of the UPDATED
 *              acc over [begin,end) (normally asked for on the last micro-batch only);
 *              accumulate as in gs_grad_sqnorm.  With NULL the workspace arguments are ignored;
 *              otherwise they follow gs_grad_sqnorm's rules.
 * Asynchronous on `stream`; elements outside [begin,end) are not touched.
 */
gs_status gs_accum_add(float *acc_f32, const uint16_t *grad_bf16, int first, int64_t begin, int64_t end,
                       double *d_sqnorm, int accumulate,
                       void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Squared L2 norm of a finished accumulation buffer: S = sum over i in [begin,end) of acc_f32[i]^2,
 * squares and reduction in fp64 -- for a buffer whose norm was not taken by the call that
 * finished it (e.g. a shard that came back from a reduction across devices).  Arguments as for
 * gs_grad_sqnorm with the fp32 buffer (device, >= end elements, 16-byte aligned, read only) in
 * place of the k gradient buffers.
 */
gs_status gs_acc_sqnorm(const float *acc_f32, int64_t begin, int64_t end, double *d_sqnorm, int accumulate,
                        void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * gs_accum_adamw with the gradient sum taken from acc_f32 (as written by gs_grad_accum_sqnorm)
 * instead of k bf16 buffers.  p, m, v, w come out bit-identical to gs_accum_adamw on the
 * same gradients, and the same partition independence holds.
 */
gs_status gs_adamw_from_acc(float *p, float *m, float *v, uint16_t *w_bf16, const float *acc_f32,
                            int64_t begin, int64_t end, const gs_adamw_hparams *hp,
                            const double *d_sqnorm, void *stream);

/* ------------------------------------------------------------------------------------------
 * Speculative single-pass step.  Sec. 2.1 of the paper points at prior work that takes the
 * optimizer step before the global gradient norm is known, because clipping rarely changes the
 * gradients; the step then does not have to wait for the whole backward pass, and the gradients
 * are read once (2k+26 bytes per parameter in total instead of 2k + 2k+26).  Undoing a wrong
 * guess needs the old states, so these entry points are out of place.
 * ------------------------------------------------------------------------------------------ */

/*
 * Out-of-place form of gs_accum_adamw: states are read from p, m, v and written to p_out,
 * m_out, v_out (device fp32, >= end elements, 16-byte aligned).  Each output may be exactly its
 * own input (then this is gs_accum_adamw) or must not overlap it; anything else is rejected.
 */
gs_status gs_accum_adamw_oop(const float *p, const float *m, const float *v,
                             float *p_out, float *m_out, float *v_out, uint16_t *w_bf16,
                             const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                             const gs_adamw_hparams *hp, const double *d_sqnorm, void *stream);

/*
 * The step with clip coefficient 1 (hp->max_grad_norm is not applied), written out of place,
 * while the squared norm S of the same accumulated gradients over [begin,end) is reduced into
 * *d_sqnorm (= S, or += S when accumulate != 0; same value as gs_grad_sqnorm up to fp64
 * summation order).  Workspace as for gs_grad_sqnorm.  Protocol: run it over every range that is
 * clipped together, accumulating S; read S back; if gs_clip_coefficient(S, max_grad_norm) == 1
 * the outputs are the new states (swap the buffers); otherwise redo the ranges with
 * gs_accum_adamw_oop from the untouched inputs and the finished *d_sqnorm.
 */
gs_status gs_accum_adamw_spec(const float *p, const float *m, const float *v,
                              float *p_out, float *m_out, float *v_out, uint16_t *w_bf16,
                              const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                              const gs_adamw_hparams *hp, double *d_sqnorm, int accumulate,
                              void *d_workspace, size_t workspace_bytes, void *stream);

/* Host-side copy of the clip coefficient the kernels derive from a total squared norm:
 * min(1, max_grad_norm / ((float)sqrt(S) + 1e-6)); 1 when max_grad_norm <= 0.  No HIP call. */
float gs_clip_coefficient(double sqnorm_total, float max_grad_norm);

/* ------------------------------------------------------------------------------------------
 * Compute-unit budget for the deferred part (Sec. 4.4: the delayed fraction of the optimizer
 * step runs concurrently with the next iteration's forward pass and only has to finish before
 * its layer executes).  A bandwidth-bound step that fills every CU slows a concurrent GEMM far
 * more than it is slowed itself; a stream confined to a subset of the CUs leaves the rest of the
 * chip, and part of the memory system, to the forward pass.
 * ------------------------------------------------------------------------------------------ */

/*
 * Creates a HIP stream (default priority) whose kernels run on at most `num_cus` compute units
 * (the lowest-numbered ones; CUs/16 <= num_cus <= CUs of the current device, i.e. 16..256 on
 * MI355X: the mask is spread over the chip's eight dies, and masks that leave a die with fewer
 * than two CUs have not been validated, so they are refused with GS_ERR_INVALID_ARG).  *stream
 * receives a hipStream_t to pass as the `stream` argument of the calls above.  Destroy with
 * gs_cu_stream_destroy after the work on it has finished.
 */
gs_status gs_cu_stream_create(void **stream, int num_cus);
gs_status gs_cu_stream_destroy(void *stream);

/*
 * The deferred part of each layer's step as a schedule with per-layer deadlines (Sec. 4.4: the
 * delayed alpha share of a layer's update runs during the next iteration's forward pass and has to
 * be finished before that layer executes).  A context owns one stream -- confined to `num_cus`
 * compute units as from gs_cu_stream_create, or unconfined with num_cus = 0 -- on which the
 * deferred ranges run in the order they are handed over, and one event per layer
 * (0 <= layer < max_layers <= 65536).
 *   gs_defer_layer_step   gs_accum_adamw over [begin,end) of the layer (same arguments, same bits),
 *                         enqueued on the context's stream behind whatever `producer_stream` holds
 *                         at the call (gradients, the norm scalar); then the layer's event is
 *                         recorded.  The same hp (same t), d_sqnorm and gradient buffers as the
 *                         immediate part; the buffers must stay untouched until the layer is done.
 *   gs_defer_wait_layer   the deadline: work enqueued on `consumer_stream` after this call -- the
 *                         layer's forward, or whatever overwrites its gradient buffers -- starts
 *                         only when the layer's latest deferred step has finished.  A layer with
 *                         nothing deferred costs nothing.  Device-side wait; the host does not block.
 *   gs_defer_layer_done   1 if the layer's latest deferred step has finished (or none was enqueued),
 *                         0 if it is still pending, -1 on error.  Never blocks.
 *   gs_defer_ctx_sync     blocks until everything enqueued on the context has finished.
 *   gs_defer_ctx_stream   the context's hipStream_t (owned by the context), e.g. for a caller that wants
 *                         to check that it runs beside its own streams: the runtime multiplexes streams
 *                         onto a few hardware queues, and two streams on one queue take turns.
 * One calling thread at a time per context; all calls with the device current on which it was made.
 */
typedef struct gs_defer_ctx gs_defer_ctx;
gs_status gs_defer_ctx_create(gs_defer_ctx **out, int max_layers, int num_cus);
gs_status gs_defer_ctx_destroy(gs_defer_ctx *ctx); /* waits for pending work, frees everything */
gs_status gs_defer_layer_step(gs_defer_ctx *ctx, int layer, float *p, float *m, float *v, uint16_t *w_bf16,
                              const uint16_t *const *grads, int k, int64_t begin, int64_t end,
                              const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream);
gs_status gs_defer_wait_layer(gs_defer_ctx *ctx, int layer, void *consumer_stream);
int gs_defer_layer_done(gs_defer_ctx *ctx, int layer);
gs_status gs_defer_ctx_sync(gs_defer_ctx *ctx);
void *gs_defer_ctx_stream(gs_defer_ctx *ctx);

/* ------------------------------------------------------------------------------------------
 * Step for states that live in pinned host memory (Sec. 2.2: for each parameter chunk, load
 * gradients + master parameters + optimizer states, step, write back; Sec. 4.3 the optimizer
 * stages of the backward pipeline -- here the slow link is host<->device PCIe instead of
 * SSD<->host).  A context fixes how the states cross the link: staged through device memory by
 * the copy path (gs_stream_ctx_create), or touched in place by the kernel
 * (gs_stream_ctx_create_inplace).  gs_stream_layer_step is the same call for both and gives
 * the same bits.
 * ------------------------------------------------------------------------------------------ */

typedef struct gs_stream_ctx gs_stream_ctx;

/*
 * Staged: the context owns an upload stream, a compute stream, a download stream, `slots`
 * (2..64) staging slots of 3 x chunk_elems fp32 in device memory (chunk_elems in [1, 2^34]) and
 * the events that order them; gs_stream_layer_step walks the layer in chunks -- chunk c+1 is
 * uploaded with hipMemcpyAsync while the kernel updates chunk c in its slot and chunk c-1 is
 * copied back.  Costs no CU time beyond the short kernel per chunk and measured 48 GB/s each way
 * at its best, but how fast a copy runs is up to the runtime (copy path per copy, hardware queue
 * per stream).  GS_ERR_NOMEM if the slots cannot be allocated.
 */
gs_status gs_stream_ctx_create(gs_stream_ctx **out, int64_t chunk_elems, int slots);

/*
 * What a staged context found when it was created.  The pipeline of Sec. 4.3 only pays if upload,
 * kernel and download run at the same time, but the runtime may put two of the context's three
 * streams on one hardware queue, where they take turns (upload and download on one queue, or the
 * kernel's wait for the next upload holding back the previous download: half the rate either way).
 * gs_stream_ctx_create therefore checks each pair -- a burst of copies on one stream, a 4 KB copy
 * on the other that has to finish while the burst is still running -- and swaps a colliding stream
 * for a fresh one (up to nine times).  Returns 1 if all three ran side by side in the end, 0 if a
 * pair still took turns, -1 if the check was skipped (slots under 1 MB, in-place context) or ctx
 * is NULL.  No HIP call.
 */
int gs_stream_ctx_copies_overlap(const gs_stream_ctx *ctx);

/*
 * In place: the context owns one stream, and the step kernel runs on the pinned host arrays
 * themselves -- each wave loads its tile of p, m, v over the link, updates it and stores it
 * back.  Nothing is staged in device memory and no copy engine is used: 44-45 GB/s each way,
 * whatever else the process does with copies and streams.  num_cus = 0: an ordinary stream;
 * num_cus > 0: a stream confined to that many compute units, as from gs_cu_stream_create (the
 * link, not the CU count, bounds this step: 16 CUs sustain the full rate and leave the rest of
 * the GPU to other work).  num_cus < 0, or outside gs_cu_stream_create's range when positive, is
 * GS_ERR_INVALID_ARG.
 */
gs_status gs_stream_ctx_create_inplace(gs_stream_ctx **out, int num_cus);
gs_status gs_stream_ctx_destroy(gs_stream_ctx *ctx); /* waits for pending work, frees everything */

/*
 * Applies the same update as gs_accum_adamw to all n elements of a layer whose p, m, v are in
 * PINNED host memory, updating them in place: chunk by chunk through the context's staging
 * slots, or by the kernel itself if the context is from gs_stream_ctx_create_inplace.
 * Results are bit-identical to gs_accum_adamw on a device copy of the same states, in both
 * modes and for every chunk size.
 *   h_p, h_m, h_v   pinned host fp32 (device-accessible, as hipHostMalloc / gs_pinned_alloc
 *                   give it), n elements each, updated in place; 4-byte aligned for a
 *                   staged context, 16-byte aligned for an in-place one.  An in-place context
 *                   asks the runtime about the first and last element of each array and
 *                   returns GS_ERR_INVALID_ARG unless both are page-locked host memory mapped
 *                   at the same address on the device (pageable memory under a kernel would
 *                   fault the GPU)
 *   d_w_bf16        device bf16, n elements, written
 *   d_grads         host array of k device pointers (bf16, n elements each)
 *   d_sqnorm        as for gs_accum_adamw (device double or NULL)
 *   producer_stream stream on which the gradients and *d_sqnorm were produced; work already
 *                   enqueued there is waited for before the kernel (NULL = null stream)
 * The call enqueues the work and returns; host buffers must stay untouched until
 * gs_stream_ctx_sync.  Several layers may be enqueued back to back on one context.  Must be
 * called with the device current on which the context was created (else GS_ERR_INVALID_ARG).
 */
gs_status gs_stream_layer_step(gs_stream_ctx *ctx, float *h_p, float *h_m, float *h_v,
                               uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k, int64_t n,
                               const gs_adamw_hparams *hp, const double *d_sqnorm,
                               void *producer_stream);

/*
 * The same over [begin,end) only (0 <= begin <= end; the arrays hold at least `end` elements and
 * are indexed from the layer's element 0, as everywhere): the split step of Sec. 4.4 on
 * host-resident states -- the immediate part now, the deferred part later, on the same or another
 * context; [0,s) followed by [s,n) leaves bit for bit what gs_stream_layer_step leaves.
 */
gs_status gs_stream_layer_step_range(gs_stream_ctx *ctx, float *h_p, float *h_m, float *h_v,
                                     uint16_t *d_w_bf16, const uint16_t *const *d_grads, int k,
                                     int64_t begin, int64_t end,
                                     const gs_adamw_hparams *hp, const double *d_sqnorm,
                                     void *producer_stream);

/* Blocks until everything enqueued on the context has finished (the host arrays hold the new states). */
gs_status gs_stream_ctx_sync(gs_stream_ctx *ctx);

/* ------------------------------------------------------------------------------------------
 * Three-tier step: file (SSD) <-> pinned host <-> device.  The paper keeps optimizer states on
 * SSD and pipelines, per layer, states SSD->CPU | step | states CPU->SSD (Sec. 4.3), with a
 * storage ratio deciding which share of the states stays in CPU memory instead (Sec. 4.5).
 * A layer's fp32 p, m, v are split at element n_host: [0,n_host) in pinned host memory,
 * [n_host,n) in three files.  n_host = n is gs_stream_layer_step; n_host = 0 keeps everything
 * in the files.
 * ------------------------------------------------------------------------------------------ */

typedef struct gs_tier_ctx gs_tier_ctx;

typedef struct {
    float *h_p, *h_m, *h_v;            /* pinned host fp32, 16-byte aligned, elements [0,n_host), checked like
                                          gs_stream_layer_step's in-place arrays; may be NULL if n_host == 0 */
    int64_t n_host;                    /* 0 <= n_host <= n */
    int fd_p, fd_m, fd_v;              /* open descriptors (read+write); ignored if n_host == n */
    int64_t off_p, off_m, off_v;       /* byte offset of element n_host in each file; element i >= n_host
                                          is the float at off + 4*(i - n_host) */
} gs_tier_layer;

/*
 * Creates a context: a gs_stream_ctx (num_cus as for gs_stream_ctx_create_inplace), `slots` (2..64) bounce
 * slots of 3 x chunk_elems fp32 in pinned host memory (each array starts on a 4 KB boundary), one
 * reader and one writer thread.  chunk_elems in [1, 2^34].  GS_ERR_NOMEM if the pinned memory
 * cannot be had.
 */
gs_status gs_tier_ctx_create(gs_tier_ctx **out, int64_t chunk_elems, int slots, int num_cus);

/*
 * Applies the same update as gs_accum_adamw to all n elements of the layer described by *L.
 * The host share is stepped in place like gs_stream_layer_step, in launches of chunk_elems.  The
 * file share is walked in chunks of chunk_elems, interleaved with those launches: the context's
 * reader thread reads p/m/v of a chunk into a bounce slot (waiting, if need be, until the writer
 * has released that slot) and enqueues the kernel in place on the slot; the writer thread writes
 * the slot back to the same file offsets once the kernel has finished.
 * The call itself does no I/O and never waits for any: it checks its arguments, records an event
 * on producer_stream (the step runs after whatever that stream holds at this moment), copies *L,
 * *hp and the k gradient pointers, queues the layer behind earlier ones and returns.  Host
 * arrays, files, gradients and d_w_bf16 must stay valid and untouched until gs_tier_ctx_sync;
 * L, hp and the d_grads table itself may go at once.  A range of a layer's file share must not
 * be queued twice without a gs_tier_ctx_sync in between (the second read could overtake the
 * first write-back).
 * Results are bit-identical to gs_accum_adamw on a device copy of the same states, for every
 * n_host and chunk size.  Other arguments as for gs_stream_layer_step.  The files must hold the
 * whole range (a short file is GS_ERR_IO, reported like every I/O failure: see below).  Descriptors opened with O_DIRECT are recognised
 * (fcntl): their transfers go through ordinary page-aligned memory of the bounce slots' size
 * (allocated on first use) and one extra host copy, because the kernel cannot do direct I/O on
 * page-locked memory that the GPU driver maps; offsets, n_host*4, chunk_elems*4 and (n-n_host)*4
 * then have to be multiples of the device's block size.  The descriptors are not closed.
 * One calling thread at a time per context.  Reads, writes and enqueues fail on the context's
 * own threads, after the call that queued them has returned GS_OK: the first such failure makes
 * the context failed for good -- layers still queued are dropped, gs_tier_ctx_sync and every
 * later call return that status, gs_tier_ctx_error its text.
 */
gs_status gs_tier_layer_step(gs_tier_ctx *ctx, const gs_tier_layer *L, uint16_t *d_w_bf16,
                             const uint16_t *const *d_grads, int k, int64_t n,
                             const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream);

/* The same over [begin,end) of the layer only (0 <= begin <= end <= n): whatever part of the range
 * lies in the host share is stepped in place, whatever part lies in the file share goes through
 * the bounce slots.  Split at any point, the two calls leave bit for bit what the whole call leaves. */
gs_status gs_tier_layer_step_range(gs_tier_ctx *ctx, const gs_tier_layer *L, uint16_t *d_w_bf16,
                                   const uint16_t *const *d_grads, int k, int64_t n, int64_t begin, int64_t end,
                                   const gs_adamw_hparams *hp, const double *d_sqnorm, void *producer_stream);

/* Blocks until every enqueued chunk has been computed and written back to its host array or file
 * (the page cache counts as written; fsync is the caller's call). */
gs_status gs_tier_ctx_sync(gs_tier_ctx *ctx);
gs_status gs_tier_ctx_destroy(gs_tier_ctx *ctx); /* syncs, stops both threads, frees everything */
/* Text of the context's first failure ("" if none), e.g. "pwrite(m): No space left on device", or,
 * for a HIP call that failed on one of the context's threads, what was being done followed by the
 * runtime's message (gs_last_hip_error is per thread and would not show it).  The pointer is valid until the calling thread's next call of this function. */
const char *gs_tier_ctx_error(gs_tier_ctx *ctx);

/* Page-locked host memory without power-of-two padding (Sec. 5 notes that a framework's
 * pinned allocator may round each buffer up to a power of two; host-resident optimizer
 * states of tens of GB cannot afford that).  Returns NULL on failure. */
void *gs_pinned_alloc(size_t bytes);
void gs_pinned_free(void *ptr);

/* ------------------------------------------------------------------------------------------ */
const char *gs_strerror(gs_status s);
/* Text of the last HIP error seen by the calling thread ("" if none). */
const char *gs_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* GS_H */
