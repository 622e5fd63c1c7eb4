/* ptchunk — the chunk-based model-state hot path of ProTrain-style memory
 * management, for one AMD MI355X (gfx950).
 *
 * Model states (16-bit parameters, 16-bit gradients, fp32 master weights, fp32
 * momentum, fp32 variance: 16 bytes per parameter — paper, Introduction) are held
 * in fixed-size flat CHUNKS (paper, "Hierarchical Chunk Management for Model
 * States").  A prefix of the chunks is PERSISTENT: resident in GPU memory and
 * updated there; the remaining chunks live in pinned host memory and pass through
 * pre-allocated device chunk buffers when they are needed (same section; three
 * buffers = prefetch / execute / offload, "Analysis of Searched Configurations").
 * The parameter update is Adam in fp32 under mixed precision (Background;
 * Appendix A.1, "Modeling Runtime").  The paper defines neither gradient clipping
 * nor loss scaling nor the Adam variant; this library fixes them as: global
 * L2-norm clipping with coefficient min(1, c/(norm+1e-6)); AdamW (decoupled decay,
 * bias correction, eps added after the square root); dynamic loss scaling with
 * skip-on-non-finite.
 *
 * One optimizer step is the call sequence
 *     pt_chunk_pack_grads      gradients -> gradient chunks (+ per-chunk sum of squares, non-finite flag)
 *     pt_chunk_grad_sqnorm     (optional recompute from chunks) + finalize: global norm, found_inf
 *     pt_chunk_stream_step     host-resident chunks: H2D -> update -> D2H on side streams  (optional)
 *     pt_chunk_adamw_step      GPU-resident chunks, one launch
 *     pt_step_end              joins the side streams, advances the step counter / loss scale
 * Everything is enqueued asynchronously; nothing in these five calls allocates or
 * synchronises with the host (one exception, stated at pt_chunk_adamw_step).
 *
 * CONVENTIONS
 *  - Plain C ABI.  Every function returns a pt_status (PT_OK == 0) and never
 *    throws or aborts; pt_last_error(ctx) gives the text of the last failure.
 *  - "device" pointers are HIP device addresses on the device that was current
 *    at pt_ctx_create; "host" pointers are ordinary process memory; "pinned"
 *    pointers are host memory from hipHostMalloc (or torch pin_memory).
 *  - The CALLER owns all chunk memory (device and pinned) and the compute stream.
 *    The library borrows pointers for the duration of the enqueued work.  The
 *    context owns only its scratch (partials, device scalars, pointer tables),
 *    its side streams and events, and the device chunk buffers of the streamed
 *    path.
 *  - Sizes and offsets are in ELEMENTS.  chunk_elems must be a multiple of 8.
 *    Every chunk base pointer must be 16-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  The calls of one
 *    step work on the context's shared scratch in call order: give them one stream, or make
 *    each call's stream wait (event) for the previous call's.  The tiny scalar kernels of a call
 *    (per-chunk sums, the final norm) may be enqueued later, by the next call of the step that
 *    needs them and on THAT call's stream - which is behind the earlier call under this rule.
 *  - A context is not thread-safe; use one per optimizer instance.
 */
#ifndef PTCHUNK_H
#define PTCHUNK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pt_ctx pt_ctx;
typedef struct pt_pack_plan pt_pack_plan;

typedef enum {
  PT_OK = 0,
  PT_ERR_INVALID_ARG = 1, /* NULL pointer, zero size, range outside the context's chunks ... */
  PT_ERR_ALIGNMENT = 2,   /* chunk_elems not a multiple of 8, chunk base not 16-byte aligned */
  PT_ERR_HIP = 3,         /* a HIP runtime call failed; text in pt_last_error */
  PT_ERR_STATE = 4,       /* call out of order (update before the norm was finalized ...) */
  PT_ERR_UNSUPPORTED = 5,
  PT_ERR_NOMEM = 6
} pt_status;

typedef enum { PT_BF16 = 0, PT_FP16 = 1 } pt_dtype;

/* One contiguous run of one tensor inside one chunk. */
typedef struct {
  const void* src;    /* device: first element of the tensor (16-bit elements)         */
  uint64_t src_off;   /* first element of the run within the tensor                     */
  uint64_t len;       /* elements in the run (> 0)                                      */
  uint64_t chunk_off; /* first element of the run within the chunk                      */
  uint32_t chunk;     /* destination chunk index                                        */
  uint32_t tensor;    /* index of the tensor the run belongs to (filled by pt_layout_dense) */
} pt_segment;

/* Hyper-parameters of one update, in fp64 (the device derives its fp32 constants
 * from these in fp64 and rounds once).  max_norm <= 0 disables clipping. */
typedef struct {
  double lr, beta1, beta2, eps, weight_decay, max_norm;
} pt_hparams;

/* Dynamic loss scaling.  Typical: init_scale 65536, growth 2, backoff 0.5,
 * growth_interval 2000.  The scale never drops below 1. */
typedef struct {
  double init_scale, growth, backoff;
  int32_t growth_interval;
  int32_t reserved;
} pt_scaler_cfg;

/* Scalars of the step in flight (after finalize) or of the last step. */
typedef struct {
  double sqnorm;      /* sum over all chunks of (g / loss_scale)^2                     */
  double norm;        /* sqrt(sqnorm)                                                    */
  double clip_coef;   /* min(1, max_norm/(norm+1e-6)); valid once an update call ran     */
  double loss_scale;  /* scale in force for this step                                    */
  float grad_mult;    /* float(clip_coef / loss_scale): what the update kernel multiplies g by */
  int32_t found_inf;  /* 1 if any gradient word is +-inf or NaN: the step is skipped     */
  int32_t step;       /* number of APPLIED updates so far (not advanced by a skipped step) */
  int32_t good_steps; /* consecutive finite steps since the last scale change            */
} pt_step_report;

/* The nine fp32 constants the update kernel used in the last update call:
 * beta1, beta2, 1-beta1, 1-beta2, 1-lr*wd, lr/(1-beta1^t), 1/sqrt(1-beta2^t), eps, grad_mult. */
typedef struct {
  float c[9];
  int32_t skip;
} pt_update_consts;

const char* pt_version(void);
const char* pt_status_string(int status);
/* Text of the last failure on this context ("" if none).  ctx may be NULL: then
 * the text of the last failure of a call that had no context (pt_ctx_create). */
const char* pt_last_error(const pt_ctx* ctx);

/* ---- context ------------------------------------------------------------------
 * Creates a context for n_chunks chunks of chunk_elems elements each, on the
 * current HIP device.  Allocates the scratch (a few MB) and synchronises; not a hot
 * call.  scaler == NULL: loss scale fixed at 1 (the bf16 configurations).
 * A non-finite gradient skips the step in either case. */
int pt_ctx_create(pt_ctx** out, int dtype, uint64_t chunk_elems, uint32_t n_chunks,
                  const pt_scaler_cfg* scaler);
int pt_ctx_destroy(pt_ctx* ctx);

/* Overwrites the step counter / loss-scale state (resume).  Enqueued on stream. */
int pt_ctx_set_state(pt_ctx* ctx, int32_t step, double loss_scale, int32_t good_steps, void* stream);

/* Weight-decay groups.  The listed runs (chunk, chunk_off, len of each segment; src is ignored)
 * are kept OUT of the weight decay in every later update of this context - resident, streamed
 * or host-side: their decay factor is 1 instead of 1 - lr*wd (biases and normalisation gains in
 * common practice; the paper does not speak of weight decay).  Replaces any earlier list;
 * n_segs == 0 clears it.  Allocates and synchronises the device: an init-time call. */
int pt_ctx_set_no_decay(pt_ctx* ctx, const pt_segment* segs, uint32_t n_segs);

/* Options (host state only, take effect at the next call).  Launch shape - none of these
 * changes a result bit:
 *   "adamw_grid"    workgroups of the update kernel; 0 = the library's default
 *   "adamw_threads" workgroup size of the update kernel: 256, 512, or 0 = the library chooses by launch size (default)
 *   "adamw_unroll"  4-element units a lane loads before it computes: 1, 2, 4 or 8
 *   "adamw_nt"      non-temporal hints on the update's loads and stores: 1 = always, 0 = never, 2 = the library
 *                   chooses by launch size (default): none while the launch's state fits the 256 MB Infinity Cache
 *   "pack_tile_elems"  elements one workgroup of pack/unpack moves; read by pt_pack_plan_create
 *   "stream_test_reject"  for tests of pt_stream_reserve: its trial of the copy streams rejects that many
 *                   stream pairs (0..5) whatever it measures, so that the replacement runs
 *   "stream_test_unhealthy"  for tests: 1 = the next look at a finished streamed step finds it serialised
 *                   whatever it measured, so that the replacement of the side streams runs
 * Gradient storage (variants of the path; the paper's gradients are the 16-bit array):
 *   "grad_fp32"     1 = the gradient chunks of this context hold fp32 (micro-batches accumulated
 *                   by pt_chunk_accum_grads): every `grad` / `h_grad` argument of the norm, the
 *                   resident, streamed and host-side update then points to chunk_elems floats,
 *                   and pt_chunk_pack_grads is refused.  Choose before pt_stream_reserve (the
 *                   chunk buffers grow to 18 bytes per element; PT_ERR_STATE afterwards) and
 *                   before pt_pack_plan_create (plans are tiled for the kernel they feed).
 *   "adamw_zero_grads"  1 = pt_chunk_adamw_step overwrites every gradient element it has read
 *                   with zero (for callers whose backward pass adds into the chunks).  A skipped
 *                   step zeroes them too: the non-finite value that caused the skip must not stay
 *                   in the sums, or every later step would be skipped as well.  The streamed and
 *                   host-side updates never write gradients: their host copies are overwritten by
 *                   the next offload. */
int pt_ctx_set_option(pt_ctx* ctx, const char* name, int64_t value);

/* ---- layout (host, integer only) ---------------------------------------------------
 * Dense layout: the tensors are concatenated in the order given and cut every
 * chunk_elems elements; a tensor may straddle a chunk boundary; only the tail of
 * the last chunk is padding.  Writes up to `cap` segments (src = NULL, to be
 * filled by the caller from `tensor`), the number of segments and of chunks.
 * With out == NULL only the counts are computed.  Zero-sized tensors produce no
 * segment. */
int pt_layout_dense(const uint64_t* tensor_elems, uint32_t n_tensors, uint64_t chunk_elems,
                    pt_segment* out, uint32_t cap, uint32_t* n_segments, uint32_t* n_chunks);

/* Paper-faithful layout (paper, Appendix B.1 "Chunk Organization and Size Search"): the tensors
 * are given in execution order, each once (a parameter shared between layers at its first
 * occurrence); a tensor is never split between chunks; consecutive tensors with the same
 * tensor_group id (one transformer block) are kept in one chunk whenever the block fits an
 * empty chunk, else they are placed one by one; tensors with PT_NO_GROUP (or tensor_group ==
 * NULL) stand alone.  A piece that does not fit the rest of the current chunk opens the next
 * chunk, the rest stays unused ("memory waste").  Every tensor starts at a multiple of 8
 * elements of its chunk.  Outputs as pt_layout_dense, one segment per non-empty tensor, plus
 * waste_elems = n_chunks * chunk_elems - sum of the sizes (may be NULL).  A tensor larger than a
 * chunk is PT_ERR_INVALID_ARG. */
#define PT_NO_GROUP 0xffffffffu
int pt_layout_grouped(const uint64_t* tensor_elems, const uint32_t* tensor_group, uint32_t n_tensors,
                      uint64_t chunk_elems, pt_segment* out, uint32_t cap, uint32_t* n_segments,
                      uint32_t* n_chunks, uint64_t* waste_elems);

/* The order in which the tensors go into pt_layout_grouped (same passage: parameters are organised by
 * execution order, and a parameter that several layers share counts at its first occurrence).
 * uses: n_uses tensor indices (each < n_tensors) in the order the forward pass touches them; an index may
 * repeat.  order: n_tensors entries, written with the tensors in the order of their first use, followed by
 * the tensors the trace never names, in declaration order (the paper does not place those).
 * PT_ERR_INVALID_ARG for an index out of range or a NULL array that is needed.  Host only. */
int pt_layout_execution_order(const uint32_t* uses, uint32_t n_uses, uint32_t n_tensors, uint32_t* order);

/* Chunk-size search of the same passage: simulates pt_layout_grouped for the candidate sizes
 * S_min, S_min + step, ... <= S_min + span, where S_min = max(largest tensor, min_chunk_elems)
 * rounded up to step_elems, and returns the size of least waste (ties: the smaller size).  The
 * paper states neither the grid nor the tie rule; span 2^25 and step 2^20 elements reproduce the
 * chunk counts of its Table 4 (12 for the 32-block GPT-2 1B, 49 for the 48-block GPT-2 10B). */
int pt_chunk_size_search(const uint64_t* tensor_elems, const uint32_t* tensor_group, uint32_t n_tensors,
                         uint64_t min_chunk_elems, uint64_t span_elems, uint64_t step_elems,
                         uint64_t* best_chunk_elems, uint32_t* n_chunks, uint64_t* waste_elems);

/* ---- pack plan -----------------------------------------------------------------------
 * Validates a segment table against the context (ranges inside chunks, no two
 * segments overlapping in a chunk), cuts it into tiles and uploads the tile list.
 * Allocates and synchronises: do it once, outside the step.  The plan records the
 * src pointers; build a new plan when the gradient tensors move.
 * segs: host array.  n_segs may be 0 (the plan then does nothing). */
int pt_pack_plan_create(pt_ctx* ctx, const pt_segment* segs, uint32_t n_segs, pt_pack_plan** out);
int pt_pack_plan_destroy(pt_pack_plan* plan);

/* ---- the hot calls -------------------------------------------------------------------- */

/* Gradients land in chunks (paper: gradients are one of the model states grouped
 * into chunks; "Hierarchical Chunk Management for Model States").
 * Copies every segment's 16-bit words, unchanged, into grad_chunks[seg.chunk] at
 * chunk_off; fused with it, for every chunk the plan touches: the fp64 sum of
 * (g/loss_scale)^2 over the segments' elements and a flag "some word is +-inf or
 * NaN", left in the context for pt_chunk_grad_sqnorm(..., NULL, ...).
 * Words of the chunk that no segment covers (padding) are not written.
 * grad_chunks: host array of ctx.n_chunks device pointers (entries of chunks the
 * plan does not touch may be NULL).
 * PT_ERR_STATE if another plan has packed into one of this plan's chunks since the last
 * pt_step_end (the chunk's sum would be this plan's share only): one plan per chunk and step. */
int pt_chunk_pack_grads(pt_ctx* ctx, const pt_pack_plan* plan, void* const* grad_chunks, void* stream);

/* Gradient accumulation over micro-batches (a variant; needs option "grad_fp32").  For every
 * element of every segment of the plan: acc = decode(src word) if `overwrite` (first
 * micro-batch), else acc = acc + decode(src word), one binary32 addition.  acc_chunks: host
 * array of ctx.n_chunks device pointers to chunk_elems floats each (16-byte aligned; entries
 * of chunks the plan does not touch may be NULL); elements no segment covers are not written.
 * take_norm != 0 (the last micro-batch): as pt_chunk_pack_grads, leaves per chunk the fp64 sum of
 * (acc/loss_scale)^2 and the non-finite flag of the ACCUMULATED values in the context, for
 * pt_chunk_grad_sqnorm(..., NULL, ...); with take_norm == 0 the context keeps its old partials. */
int pt_chunk_accum_grads(pt_ctx* ctx, const pt_pack_plan* plan, float* const* acc_chunks, int overwrite,
                         int take_norm, void* stream);

/* Inverse copy: chunk words -> the segments' tensors (e.g. updated 16-bit
 * parameters back to the model's tensors; round-trip tests).  The segments' src
 * pointers are written through. */
int pt_chunk_unpack(pt_ctx* ctx, const pt_pack_plan* plan, const void* const* chunks, void* stream);

/* Global gradient norm (not in the paper; the global L2 norm of the unscaled
 * gradients, fp64 accumulation in a fixed order, bitwise reproducible run to run).
 * grad_chunks != NULL: recomputes the per-chunk sum of squares and non-finite
 *   flag of chunks [first_chunk, first_chunk+n_chunks) from the whole chunk
 *   (padding is zero and adds nothing).  grad_chunks is a host array indexed by
 *   absolute chunk number; only that range is read.
 * grad_chunks == NULL: keeps the per-chunk values left by pt_chunk_pack_grads
 *   (or by an earlier call: a chunk that was reduced on the GPU before it was
 *   offloaded keeps its value).
 * finalize != 0: sums the per-chunk values of ALL chunks of the context in chunk
 *   order into sqnorm / norm / found_inf (device scalars) and opens the step for
 *   the update calls.
 *   PT_FINALIZE_STRICT (1): every chunk must have got its value in THIS step, i.e. since
 *     the last pt_step_end, from a pack or accumulate plan that touches it or from a
 *     recompute; otherwise PT_ERR_STATE - a chunk nobody reduced would enter the norm with
 *     last step's sum and last step's non-finite flag.
 *   PT_FINALIZE_CARRY (2): chunks without a value from this step keep their old one (a
 *     gradient chunk that was reduced before it was offloaded and has not changed since).
 *   A chunk keeps the value of the LAST call that reduced it: pack all of a chunk's
 *   gradients with one plan per step.  pt_chunk_pack_grads refuses (PT_ERR_STATE) a plan that
 *   touches a chunk another plan has packed in this step - the first plan's share would drop
 *   out of the norm - unless the chunk was recomputed in between.
 *   PT_ERR_STATE while a streamed update is still open (pt_step_end closes it). */
#define PT_FINALIZE_STRICT 1
#define PT_FINALIZE_CARRY 2
int pt_chunk_grad_sqnorm(pt_ctx* ctx, const void* const* grad_chunks, uint32_t first_chunk,
                         uint32_t n_chunks, int finalize, void* stream);

/* The global gradient norm for callers that cannot allocate: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Computes what pt_chunk_grad_sqnorm(grad_chunks, 0,
 * n_chunks, finalize) computes - same kernels, same fixed reduction order, the same bits - without a
 * context: the block partials and per-chunk sums live in a file-scope device array of the library
 * (6.05 MiB per GPU, held until the process ends) instead of memory a context allocated.  Calls no
 * hipMalloc / hipFree and no allocating routine; enqueues three kernels on `stream` and returns.
 *   grad_arena       device: n_chunks gradient chunks of chunk_elems 16-bit words each, back to back
 *                    (chunk c starts at element c * chunk_elems); 16-byte aligned; read only
 *   dtype            PT_BF16 or PT_FP16 (how the words decode)
 *   loss_scale       every value is divided by it before it is squared (1 for unscaled gradients)
 *   out_sqnorm_norm  device, two doubles written by the last kernel: [0] = sum of (g/loss_scale)^2,
 *                    [1] = its square root
 *   out_found_inf    device, one int32 written by the last kernel: 1 if any word is +-inf or NaN
 * Limits: n_chunks <= 4096 and n_chunks * ceil(chunk_elems / 32768) <= 2^19 (2^34 elements when chunks
 * are multiples of 32768: the LLaMA-7B and -13B states fit); beyond that PT_ERR_UNSUPPORTED, nothing is
 * launched.  Errors have no context: their text is pt_last_error(NULL) of the calling thread.
 * All calls on one GPU share the one scratch array: calls that overlap in time on one GPU (two
 * streams, two threads) race; order them.  The array keeps the last call's contents; every launch
 * overwrites all the entries the next launch reads, so nothing needs clearing.  The array's device
 * address is looked up once per device (hipGetSymbolAddress), by pt_ctx_create or by the first call
 * of this function on that device - make that first call outside a graph capture. */
int pt_chunk_grad_sqnorm_noalloc(const void* grad_arena, int dtype, uint64_t chunk_elems, uint32_t n_chunks,
                                 double loss_scale, double* out_sqnorm_norm, int32_t* out_found_inf, void* stream);

/* Update of GPU-resident ("persistent") chunks (paper: persistent chunks reside
 * on the GPU and are updated there; Appendix A.1 T_GPU_OPTIM).  For every element
 * of chunks [first_chunk, first_chunk+n_chunks), padding included:
 *     g  = decode(grad) * grad_mult                 grad_mult = clip_coef / loss_scale
 *     m  = beta1 m + (1-beta1) g
 *     v  = beta2 v + (1-beta2) g^2
 *     w  = w (1 - lr wd) - lr/(1-beta1^t) * m / (sqrt(v)/sqrt(1-beta2^t) + eps)
 *     param16 = round-to-nearest-even(w)
 * in fp32 with correctly rounded operations, t = applied updates so far + 1.
 * If the step's found_inf is set nothing is written.  One kernel launch covers
 * all n_chunks chunks.
 * grad/master/m/v/param16: host arrays of n_chunks device pointers (entry i is
 * chunk first_chunk+i).  The context keeps a device copy of these tables; when a
 * call presents pointers that differ from the copy, the table is re-uploaded
 * after a hipStreamSynchronize(stream) — the only host synchronisation of a hot
 * call, and it happens on the first call and whenever chunks move.
 * Requires a finalized norm in this step (else PT_ERR_STATE). */
int pt_chunk_adamw_step(pt_ctx* ctx, const pt_hparams* hp, uint32_t first_chunk, uint32_t n_chunks,
                        const void* const* grad, float* const* master, float* const* m,
                        float* const* v, void* const* param16, void* stream);

/* Device chunk buffers for the streamed path (paper: pre-allocated chunk buffers
 * for non-persistent chunks).  Allocates n_slots buffers of 16 bytes x chunk_elems,
 * three side streams and the events.  n_slots >= 2.  Not a hot call.
 * The side streams it keeps are the second three it makes (the first three are given up once the others
 * exist): the first streams a process makes were measured to share hardware queues with the caller's
 * stream, later ones to find queues of their own.
 * With chunk buffers of 32 MiB or more it also makes the first copies of the upload and the offload stream
 * itself, side by side (a stream keeps the copy engine of its first copy, and two streams that took the same
 * one carry one direction of the link at a time), then measures one copy up, one down and both at once
 * through the first buffer and a pinned scratch; a pair that does not overlap is replaced, up to five times.  Skipped when the scratch (at most 128 MiB, kept until the context goes) cannot be pinned. */
int pt_stream_reserve(pt_ctx* ctx, uint32_t n_slots);

/* Outcome of that test: duplex_tested 0 = not run; duplex_ok 1 = upload and offload overlapped; attempts =
 * stream pairs tried (1 = the first pair overlapped); rebuilds = times pt_chunk_stream_step has replaced the
 * side streams since (see there).  Any pointer may be NULL.  Host only. */
int pt_stream_status(const pt_ctx* ctx, int32_t* duplex_tested, int32_t* duplex_ok, int32_t* attempts,
                     int32_t* rebuilds);

/* Update of host-resident ("non-persistent") chunks through the chunk buffers
 * (paper: non-persistent chunks are offloaded to CPU memory and moved over the
 * CPU-GPU link, "Hierarchical Chunk Management for Model States"; upload/offload
 * terms of Appendix A.1).  For chunk i of the range, slot = i mod n_slots:
 *     upload stream : wait slot free; H2D grad(2B) + master, m, v (12B) per element
 *     compute stream: wait upload;    the same update kernel on the slot
 *     offload stream: wait kernel;    D2H master, m, v (12B) + param16 (2B); slot free
 * so that uploads, kernels and offloads of neighbouring chunks overlap, and all
 * of it overlaps whatever the caller enqueues on `stream` afterwards (typically
 * pt_chunk_adamw_step for the resident chunks).  `stream` is only used to order
 * the side streams after the work already enqueued on it (the finalized norm);
 * pt_step_end(ctx, stream) joins them back.  Results are bit-identical to
 * pt_chunk_adamw_step on the same data.  If the step is skipped the uploads and
 * offloads still run: master, m and v come back unchanged and param16 comes back
 * as round-to-nearest-even(master), which is what it held if it was produced by
 * this library or initialised from the master weights.
 * h_*: host arrays of n_chunks PINNED pointers (entry i is chunk first_chunk+i).
 * Requires pt_stream_reserve and a finalized norm in this step.
 * The upload and offload streams want hardware queues of their own: in a process that holds many other
 * streams (HIP maps streams onto GPU_MAX_HW_QUEUES hardware queues, 4 by default) the two directions can
 * end up behind each other, and the link then carries one direction at a time.  pt_stream_reserve checks
 * single copies for that; and each call here first reads two timed events that bracketed the previous
 * streamed step (if they are done: it never waits): a step that moved less than 0.65 of the link's
 * one-direction rate had its directions behind each other, and the call then replaces the three side
 * streams by new ones before it enqueues anything (at most four times per context; pt_stream_status).
 * That one call tries the new streams out and synchronises the device; every other call only enqueues. */
int pt_chunk_stream_step(pt_ctx* ctx, const pt_hparams* hp, uint32_t first_chunk, uint32_t n_chunks,
                         const void* const* h_grad, float* const* h_master, float* const* h_m,
                         float* const* h_v, void* const* h_param16, void* stream);

/* Update of host-resident chunks ON THE HOST: the paper's own placement (CPU Adam for
 * non-persistent chunks, running concurrently with GPU work; "Hierarchical Chunk Management for
 * Model States", Appendix A.1 T_CPU_OPTIM).  Same arithmetic and the same nine fp32 constants
 * as pt_chunk_adamw_step - the scalar kernel of the step leaves them in pinned host memory as
 * well, and the call waits for the event behind that kernel only, not for bulk work queued after
 * it - so results are bit-identical to the device paths.  BLOCKING: returns when n_threads host threads (this one
 * included) have updated master, m, v and param16 of chunks [first_chunk, first_chunk+n_chunks)
 * in place.  Queue pt_chunk_adamw_step for the resident chunks first and the two run side by
 * side.  h_*: host arrays of n_chunks host pointers (pinned or not).  A skipped step leaves the
 * arrays untouched.  Requires a finalized norm in this step. */
int pt_chunk_host_adamw_step(pt_ctx* ctx, const pt_hparams* hp, uint32_t first_chunk, uint32_t n_chunks,
                             const void* const* h_grad, float* const* h_master, float* const* h_m,
                             float* const* h_v, void* const* h_param16, uint32_t n_threads, void* stream);

/* Closes the step: makes `stream` wait for the side streams of a streamed update,
 * then on the device: found_inf ? (loss_scale = max(loss_scale*backoff, 1),
 * good_steps = 0) : (step += 1, good_steps += 1, and loss_scale *= growth when
 * good_steps reaches growth_interval).  Without a scaler only the counter moves. */
int pt_step_end(pt_ctx* ctx, void* stream);

/* ---- read-back (these synchronise `stream`) ----------------------------------------- */
int pt_step_report_read(pt_ctx* ctx, pt_step_report* out, void* stream);
int pt_update_consts_read(pt_ctx* ctx, pt_update_consts* out, void* stream);

/* ---- test hook ------------------------------------------------------------------------
 * Opens the step with the given scalars instead of a computed norm: the update
 * kernel multiplies gradients by exactly `grad_mult` (no clipping on top) and
 * skips if found_inf != 0.  For kernel-isolated tests. */
int pt_step_override(pt_ctx* ctx, float grad_mult, int32_t found_inf, void* stream);

/* ---- OPTIM-phase cost model (host only) -------------------------------------------------
 * The paper's runtime model restricted to the optimizer phase (Appendix A.1, Eq. 2: the part
 * that runs on the GPU and the part that does not run side by side, the longer one decides;
 * both are "modeled based on parameter size") and its model-state memory term (Appendix A.2:
 * M_persist * n_persist + M_buffer * n_buffer, here 16 bytes per element each).  Times are
 * linear in the number of elements, with coefficients the caller measured (bench.py --model):
 *   resident part   t = gpu_s_fixed  + gpu_s_per_elem  * n_persist * chunk_elems      (pack + update)
 *   streamed part   t = link_s_fixed + link_s_per_elem * rest                         (PT_OPTIM_STREAM)
 *   host-side part  t = host_s_fixed + host_s_per_elem * rest                         (PT_OPTIM_HOST)
 *   step            t = first + max(beside, other) [+ stream_contention * min(beside, other) when streaming:
 *                       the slot kernels and DMA engines share HBM with the resident update]
 *                   where first = gpu_serial_share * resident is the resident work that comes before the gradient
 *                   norm is final (pack and reduction) and beside = resident - first: under global-norm clipping
 *                   the other part cannot start earlier.  gpu_serial_share = 0 gives the paper's plain max.
 * A part over zero elements costs nothing; with every chunk resident the step is the resident part. */
typedef enum { PT_OPTIM_STREAM = 0, PT_OPTIM_HOST = 1 } pt_optim_mode;
typedef struct {
  double gpu_s_fixed, gpu_s_per_elem;
  double link_s_fixed, link_s_per_elem;
  double host_s_fixed, host_s_per_elem;
  double stream_contention;
  double gpu_serial_share;   /* in [0, 1] */
} pt_optim_rates;
typedef struct {
  uint32_t n_persist;  /* resident chunks: the first n_persist of the model (prefix rule)   */
  uint32_t n_slots;    /* chunk buffers counted in hbm_bytes (0 when everything is resident) */
  int32_t mode;
  int32_t reserved;
  double t_step, t_gpu, t_other; /* predicted seconds */
  uint64_t hbm_bytes;  /* 16 * chunk_elems * (n_persist + n_slots)                           */
} pt_optim_choice;

int pt_optim_predict(const pt_optim_rates* rates, uint64_t chunk_elems, uint32_t n_chunks, uint32_t n_persist,
                     int mode, double* t_gpu, double* t_other, double* t_step);
/* Exhaustive scan of n_persist in [0, n_chunks] under 16*chunk_elems*(n_persist + buffers) <=
 * hbm_budget_bytes; least predicted step time wins, ties go to the smaller footprint.
 * PT_ERR_INVALID_ARG if not even the chunk buffers fit. */
int pt_optim_choose(const pt_optim_rates* rates, uint64_t chunk_elems, uint32_t n_chunks,
                    uint64_t hbm_budget_bytes, int mode, uint32_t n_slots, pt_optim_choice* out);

/* ---- measurement aid ----------------------------------------------------------------
 * A plain device-to-device streaming copy of `bytes` bytes (16-byte aligned pointers
 * and size): the known-size kernel against which hardware traffic counters and the
 * attainable HBM rate of a box are calibrated.  Not part of the optimizer path. */
int pt_calib_copy(void* dst, const void* src, uint64_t bytes, void* stream);

/* The update's own memory access pattern with the arithmetic taken out: over chunks
 * [first_chunk, first_chunk+n_chunks), with the pointers the last pt_chunk_adamw_step on them left in
 * the context (PT_ERR_STATE if there was none) and the same launch shape, reads gradient, master,
 * momentum and variance (14 bytes per element) and writes master, momentum and variance back as read and
 * param16 re-derived from the master weight (14 bytes): the state keeps its values.  What it attains is
 * the ceiling the memory system sets for this mix of four read and four write streams on this placement.
 * 16-bit gradient chunks, no no-decay runs.  Not part of the optimizer path. */
int pt_calib_adamw_pattern(pt_ctx* ctx, uint32_t first_chunk, uint32_t n_chunks, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PTCHUNK_H */
