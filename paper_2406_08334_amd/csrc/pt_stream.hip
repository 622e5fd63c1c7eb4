// Streamed update of host-resident chunks through a ring of device chunk
// buffers: upload, update and offload run on three side streams ordered by
// events, so that H2D(i+1), the kernel of chunk i and D2H(i-1) overlap each other
// and whatever the caller runs on its own stream.
//
// Link-bound: 14 bytes up and 14 bytes down per element over the host link
// against 28 bytes of HBM traffic in the kernel.
#include <chrono>
#include <vector>

#include "pt_common.h"

// One device chunk buffer ("slot"), 16 bytes per element (18 with fp32 gradient chunks):
//   [ master S*4 | m S*4 | v S*4 | grad S*2 or S*4 | param16 S*2 ]
static inline size_t grad_bytes(const pt_ctx* c) { return c->grad_f32 ? 4 : 2; }
static inline size_t slot_bytes(const pt_ctx* c) { return (14 + grad_bytes(c)) * size_t(c->S); }
static inline char* slot_master(const pt_ctx* c, uint32_t s) { return (char*)c->slot_mem[s]; }
static inline char* slot_m(const pt_ctx* c, uint32_t s) { return (char*)c->slot_mem[s] + 4 * c->S; }
static inline char* slot_v(const pt_ctx* c, uint32_t s) { return (char*)c->slot_mem[s] + 8 * c->S; }
static inline char* slot_grad(const pt_ctx* c, uint32_t s) { return (char*)c->slot_mem[s] + 12 * c->S; }
static inline char* slot_p16(const pt_ctx* c, uint32_t s) { return (char*)c->slot_mem[s] + (12 + grad_bytes(c)) * c->S; }

static int reserve_slots(pt_ctx* ctx, uint32_t n_slots);
static int duplex_self_test(pt_ctx* ctx);
static int replace_side_streams(pt_ctx* ctx, bool new_comp, std::vector<hipStream_t>& retired);

// Gives back whatever a reservation (failed or complete) has created, so that the call can be repeated.
void pt_stream_release(pt_ctx* ctx) {
  if (ctx->s_up) { (void)hipStreamDestroy(ctx->s_up); ctx->s_up = nullptr; }
  if (ctx->s_comp) { (void)hipStreamDestroy(ctx->s_comp); ctx->s_comp = nullptr; }
  if (ctx->s_down) { (void)hipStreamDestroy(ctx->s_down); ctx->s_down = nullptr; }
  if (ctx->ev_fork) { (void)hipEventDestroy(ctx->ev_fork); ctx->ev_fork = nullptr; }
  if (ctx->ev_t0) { (void)hipEventDestroy(ctx->ev_t0); ctx->ev_t0 = nullptr; }
  if (ctx->ev_t1) { (void)hipEventDestroy(ctx->ev_t1); ctx->ev_t1 = nullptr; }
  ctx->health_pending = false;
  if (ctx->h_trial) { (void)hipHostFree(ctx->h_trial); ctx->h_trial = nullptr; }
  for (uint32_t s = 0; s < PT_MAX_SLOTS; ++s) {
    if (ctx->ev_up[s]) { (void)hipEventDestroy(ctx->ev_up[s]); ctx->ev_up[s] = nullptr; }
    if (ctx->ev_k[s]) { (void)hipEventDestroy(ctx->ev_k[s]); ctx->ev_k[s] = nullptr; }
    if (ctx->ev_down[s]) { (void)hipEventDestroy(ctx->ev_down[s]); ctx->ev_down[s] = nullptr; }
    if (ctx->slot_mem[s]) { (void)hipFree(ctx->slot_mem[s]); ctx->slot_mem[s] = nullptr; }
  }
}

extern "C" int pt_stream_reserve(pt_ctx* ctx, uint32_t n_slots) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (n_slots < 2 || n_slots > PT_MAX_SLOTS)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_stream_reserve: n_slots must be in [2, %u]", PT_MAX_SLOTS);
  if (ctx->n_slots) return pt_fail(ctx, PT_ERR_STATE, "pt_stream_reserve: chunk buffers already reserved");
  const int rc = reserve_slots(ctx, n_slots);
  if (rc != PT_OK) pt_stream_release(ctx);   // the error text set by the failing step stays
  return rc;
}

static int reserve_slots(pt_ctx* ctx, uint32_t n_slots) {
  // upload, compute, offload: three streams created one after the other, each wants a hardware queue of
  // its own (copies in the two directions overlap only then)
  PT_HIP(ctx, hipStreamCreateWithFlags(&ctx->s_up, hipStreamNonBlocking));
  PT_HIP(ctx, hipStreamCreateWithFlags(&ctx->s_comp, hipStreamNonBlocking));
  PT_HIP(ctx, hipStreamCreateWithFlags(&ctx->s_down, hipStreamNonBlocking));
  PT_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming));
  PT_HIP(ctx, hipEventCreate(&ctx->ev_t0));
  PT_HIP(ctx, hipEventCreate(&ctx->ev_t1));
  for (uint32_t s = 0; s < n_slots; ++s) {
    PT_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_up[s], hipEventDisableTiming));
    PT_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_k[s], hipEventDisableTiming));
    PT_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_down[s], hipEventDisableTiming));
    hipError_t e = hipMalloc(&ctx->slot_mem[s], slot_bytes(ctx));
    if (e != hipSuccess)
      return pt_fail(ctx, e == hipErrorOutOfMemory ? PT_ERR_NOMEM : PT_ERR_HIP,
                     "pt_stream_reserve: hipMalloc of chunk buffer %u (%llu bytes) failed: %s", s,
                     (unsigned long long)slot_bytes(ctx), hipGetErrorString(e));
    // the buffer's five arrays become column C+s of the pointer table
    const void* p;
    int rc;
    p = slot_grad(ctx, s);
    if ((rc = pt_table_bind(ctx, ROW_GRAD, ctx->C + s, 1, &p, false, nullptr, nullptr)) != PT_OK) return rc;
    p = slot_master(ctx, s);
    if ((rc = pt_table_bind(ctx, ROW_MASTER, ctx->C + s, 1, &p, false, nullptr, nullptr)) != PT_OK) return rc;
    p = slot_m(ctx, s);
    if ((rc = pt_table_bind(ctx, ROW_M, ctx->C + s, 1, &p, false, nullptr, nullptr)) != PT_OK) return rc;
    p = slot_v(ctx, s);
    if ((rc = pt_table_bind(ctx, ROW_V, ctx->C + s, 1, &p, false, nullptr, nullptr)) != PT_OK) return rc;
    p = slot_p16(ctx, s);
    if ((rc = pt_table_bind(ctx, ROW_P16, ctx->C + s, 1, &p, false, nullptr, nullptr)) != PT_OK) return rc;
  }
  PT_HIP(ctx, hipDeviceSynchronize());
  // The three streams made above are given up again for three made while they still exist.  Measured with
  // one program in fresh processes: with the first three, 2-3 runs of 8 had the step's two directions behind
  // each other (782 ms for 24 chunks) and 4-5 of 8 had the uploads wait for the caller's resident update
  // (511 ms); with their replacements 10 of 10 ran clean (481 ms) - the first streams a process makes share
  // hardware queues with the caller's stream, later ones find queues of their own.
  int rc;
  {
    std::vector<hipStream_t> retired;
    if ((rc = replace_side_streams(ctx, true, retired)) != PT_OK) return rc;
    for (hipStream_t s : retired) (void)hipStreamDestroy(s);
  }
  rc = duplex_self_test(ctx);
  if (rc != PT_OK) return rc;
  ctx->n_slots = n_slots;
  return PT_OK;
}

// Upload and offload must run side by side.  HIP maps streams onto a few hardware queues
// (GPU_MAX_HW_QUEUES, four by default) and copies onto copy engines, by rules a process cannot steer, and
// two things were measured to go wrong on MI355X (ROCm 7.2):
//  * the FIRST copies decide the engines: a stream keeps the engine it took for its first copy; one whose
//    first copy is issued while the engines are idle takes the engine of the stream before it, and the two
//    then carry one direction of the link at a time (both at once take 0.999 of the added-up times, against
//    0.588 for streams whose first copies ran side by side);
//  * in some processes - two or three of eight runs of one program - a whole step runs with the two
//    directions largely behind each other (28.9 instead of 46.8 GB/s per direction) although single copies
//    on the same streams overlap: streams share hardware queues there, and an event wait of one stalls the
//    copies of another.  Offloading by a copy kernel instead of the copy engine does not escape it (24 GB/s
//    in such a process).
// What the library does about it: the reservation makes the two streams' first copies itself - one up, one
// down, issued together, through the first chunk buffer and a pinned scratch it keeps - and measures a copy
// up, a copy down and both at once, replacing a pair that does not overlap (a few times at most); and every
// streamed step is bracketed by two timed events, which the next pt_chunk_stream_step reads (once they are
// done: no waiting): a step that moved less than 0.65 of the link's one-direction rate (healthy 0.80-0.85,
// serialised 0.5) makes it replace the three side streams by new ones before it enqueues anything, up to
// PT_MAX_STREAM_REBUILDS times.  Skipped for small chunk buffers (nothing to measure) and when the scratch
// cannot be pinned.  pt_stream_status tells the outcome.
constexpr uint32_t PT_MAX_STREAM_REBUILDS = 4;

// seconds for (up ? one copy up) and (down ? one copy down) of T bytes, issued together; the least of three
static bool trial_copies(pt_ctx* ctx, size_t T, bool up, bool down, double* sec, int* rc) {
  char* h = (char*)ctx->h_trial;
  char* d = (char*)ctx->slot_mem[0];
  double best = 1e30;
  for (int rep = 0; rep < 3; ++rep) {
    hipError_t e = hipSuccess;
    const auto t0 = std::chrono::steady_clock::now();
    if (up) e = hipMemcpyAsync(d, h, T, hipMemcpyHostToDevice, ctx->s_up);
    if (e == hipSuccess && down) e = hipMemcpyAsync(h + T, d + T, T, hipMemcpyDeviceToHost, ctx->s_down);
    if (e == hipSuccess && up) e = hipStreamSynchronize(ctx->s_up);
    if (e == hipSuccess && down) e = hipStreamSynchronize(ctx->s_down);
    if (e != hipSuccess) {
      *rc = pt_fail(ctx, PT_ERR_HIP, "trial copies of the side streams failed: %s", hipGetErrorString(e));
      return false;
    }
    best = std::min(best, std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count());
  }
  *sec = best;
  return true;
}

// New upload and offload streams (new_comp: a new compute stream too), created while the old ones are still
// alive so that they do not simply take the old ones' places; `retired` receives the old ones.
static int replace_side_streams(pt_ctx* ctx, bool new_comp, std::vector<hipStream_t>& retired) {
  hipStream_t up = nullptr, comp = nullptr, down = nullptr;
  hipError_t e = hipStreamCreateWithFlags(&up, hipStreamNonBlocking);
  if (e == hipSuccess && new_comp) e = hipStreamCreateWithFlags(&comp, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&down, hipStreamNonBlocking);
  if (e != hipSuccess) {
    if (up) (void)hipStreamDestroy(up);
    if (comp) (void)hipStreamDestroy(comp);
    if (down) (void)hipStreamDestroy(down);
    return pt_fail(ctx, PT_ERR_HIP, "hipStreamCreateWithFlags failed while replacing the side streams: %s", hipGetErrorString(e));
  }
  retired.push_back(ctx->s_up); retired.push_back(ctx->s_down);
  ctx->s_up = up; ctx->s_down = down;
  if (new_comp) { retired.push_back(ctx->s_comp); ctx->s_comp = comp; }
  return PT_OK;
}

// Primes the current pair (first copies side by side), then measures it; replaces and repeats while it does
// not overlap.  The side streams must be idle.
static int duplex_self_test(pt_ctx* ctx) {
  ctx->duplex_tested = false; ctx->duplex_ok = false; ctx->duplex_attempts = 0;
  const size_t T = std::min<size_t>(size_t(64) << 20, (slot_bytes(ctx) / 2) & ~size_t(4095));
  if (T < (size_t(16) << 20)) return PT_OK;
  if (!ctx->h_trial) {
    if (hipHostMalloc(&ctx->h_trial, 2 * T, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();          // the caller has pinned what there is: go without the test
      ctx->h_trial = nullptr;
      return PT_OK;
    }
    std::memset(ctx->h_trial, 0, 2 * T);
  }
  std::vector<hipStream_t> retired;
  int rc = PT_OK;
  double warm;
  trial_copies(ctx, T, true, true, &warm, &rc);       // the two streams' first copies, side by side
  for (uint32_t attempt = 1; rc == PT_OK && attempt <= 6; ++attempt) {
    double t_up, t_down, t_both;
    if (!trial_copies(ctx, T, true, false, &t_up, &rc) || !trial_copies(ctx, T, false, true, &t_down, &rc) ||
        !trial_copies(ctx, T, true, true, &t_both, &rc))
      break;
    ctx->duplex_tested = true;
    ctx->duplex_attempts = attempt;
    ctx->link_one_dir_Bps = double(T) / std::max(t_up, t_down);
    // overlapped copies take about 0.6 of the two times added up, copies behind each other all of it
    ctx->duplex_ok = t_both <= 0.8 * (t_up + t_down) && attempt > ctx->opt_duplex_reject;
    if (ctx->duplex_ok || attempt == 6) break;
    if ((rc = replace_side_streams(ctx, false, retired)) != PT_OK) break;
    trial_copies(ctx, T, true, true, &warm, &rc);     // the new streams' first copies run side by side
  }
  for (hipStream_t s : retired) (void)hipStreamDestroy(s);
  (void)hipDeviceSynchronize();
  return rc;
}

extern "C" int pt_stream_status(const pt_ctx* ctx, int32_t* duplex_tested, int32_t* duplex_ok, int32_t* attempts,
                                int32_t* rebuilds) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (duplex_tested) *duplex_tested = ctx->duplex_tested ? 1 : 0;
  if (duplex_ok) *duplex_ok = ctx->duplex_ok ? 1 : 0;
  if (attempts) *attempts = int32_t(ctx->duplex_attempts);
  if (rebuilds) *rebuilds = int32_t(ctx->stream_rebuilds);
  return PT_OK;
}

// Reads the verdict on the last streamed step, if it is in, and replaces the side streams after a serialised one.
static int look_at_last_step(pt_ctx* ctx) {
  if (!ctx->health_pending) return PT_OK;
  if (hipEventQuery(ctx->ev_t1) != hipSuccess) {
    (void)hipGetLastError();      // "not ready" is no error of this call: the step is looked at next time
    return PT_OK;
  }
  ctx->health_pending = false;
  float ms = 0.0f;
  if (hipEventElapsedTime(&ms, ctx->ev_t0, ctx->ev_t1) != hipSuccess || !(ms > 0.0f) || !(ctx->link_one_dir_Bps > 0.0)) {
    (void)hipGetLastError();
    return PT_OK;
  }
  const double rate = double(ctx->health_bytes) / (double(ms) * 1e-3);
  const bool serialised = ctx->health_chunks >= 6 && rate < 0.65 * ctx->link_one_dir_Bps;
  if (!(serialised || ctx->opt_force_unhealthy) || ctx->stream_rebuilds >= PT_MAX_STREAM_REBUILDS) return PT_OK;
  ctx->opt_force_unhealthy = 0;
  // ev_t1 is done, so everything the side streams were given has run: they are idle
  std::vector<hipStream_t> retired;
  int rc = replace_side_streams(ctx, true, retired);
  if (rc != PT_OK) return rc;
  for (hipStream_t s : retired) (void)hipStreamDestroy(s);
  ctx->stream_rebuilds += 1;
  return duplex_self_test(ctx);
}

extern "C" int pt_chunk_stream_step(pt_ctx* ctx, const pt_hparams* hp, uint32_t first_chunk, uint32_t n_chunks,
                                    const void* const* h_grad, float* const* h_master, float* const* h_m,
                                    float* const* h_v, void* const* h_param16, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (!hp) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_stream_step: hp is NULL");
  if (uint64_t(first_chunk) + n_chunks > ctx->C)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_stream_step: chunks [%u, %u) outside the context's %u chunks",
                   first_chunk, first_chunk + n_chunks, ctx->C);
  if (n_chunks && (!h_grad || !h_master || !h_m || !h_v || !h_param16))
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_stream_step: NULL pointer array");
  if (!ctx->n_slots) return pt_fail(ctx, PT_ERR_STATE, "pt_chunk_stream_step: call pt_stream_reserve first");
  if (!ctx->norm_finalized)
    return pt_fail(ctx, PT_ERR_STATE, "pt_chunk_stream_step: no finalized gradient norm in this step");
  for (uint32_t i = 0; i < n_chunks; ++i)
    if (!h_grad[i] || !h_master[i] || !h_m[i] || !h_v[i] || !h_param16[i])
      return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_stream_step: NULL host pointer for chunk %u", first_chunk + i);
  if (n_chunks == 0) return PT_OK;

  int rc = look_at_last_step(ctx);
  if (rc != PT_OK) return rc;
  rc = pt_prepare_consts(ctx, hp, st);
  if (rc != PT_OK) return rc;
  // side streams start after everything already enqueued on the caller's stream
  PT_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
  PT_HIP(ctx, hipStreamWaitEvent(ctx->s_up, ctx->ev_fork, 0));
  PT_HIP(ctx, hipStreamWaitEvent(ctx->s_comp, ctx->ev_fork, 0));
  // bracket the step with two timed events, unless the last bracket has not been read yet
  const bool watch = ctx->duplex_tested && !ctx->health_pending;
  if (watch) PT_HIP(ctx, hipEventRecord(ctx->ev_t0, ctx->s_up));

  const size_t S = ctx->S;
  for (uint32_t i = 0; i < n_chunks; ++i) {
    const uint32_t s = i % ctx->n_slots;
    // upload: the slot must have been offloaded by its previous tenant
    if (ctx->slot_used[s]) PT_HIP(ctx, hipStreamWaitEvent(ctx->s_up, ctx->ev_down[s], 0));
    PT_HIP(ctx, hipMemcpyAsync(slot_grad(ctx, s), h_grad[i], grad_bytes(ctx) * S, hipMemcpyHostToDevice, ctx->s_up));
    PT_HIP(ctx, hipMemcpyAsync(slot_master(ctx, s), h_master[i], 4 * S, hipMemcpyHostToDevice, ctx->s_up));
    PT_HIP(ctx, hipMemcpyAsync(slot_m(ctx, s), h_m[i], 4 * S, hipMemcpyHostToDevice, ctx->s_up));
    PT_HIP(ctx, hipMemcpyAsync(slot_v(ctx, s), h_v[i], 4 * S, hipMemcpyHostToDevice, ctx->s_up));
    PT_HIP(ctx, hipEventRecord(ctx->ev_up[s], ctx->s_up));
    // update on the slot
    PT_HIP(ctx, hipStreamWaitEvent(ctx->s_comp, ctx->ev_up[s], 0));
    if ((rc = pt_launch_adamw(ctx, ctx->C + s, 1, ctx->s_comp, true, first_chunk + i, false)) != PT_OK) return rc;
    PT_HIP(ctx, hipEventRecord(ctx->ev_k[s], ctx->s_comp));
    // offload
    PT_HIP(ctx, hipStreamWaitEvent(ctx->s_down, ctx->ev_k[s], 0));
    PT_HIP(ctx, hipMemcpyAsync(h_master[i], slot_master(ctx, s), 4 * S, hipMemcpyDeviceToHost, ctx->s_down));
    PT_HIP(ctx, hipMemcpyAsync(h_m[i], slot_m(ctx, s), 4 * S, hipMemcpyDeviceToHost, ctx->s_down));
    PT_HIP(ctx, hipMemcpyAsync(h_v[i], slot_v(ctx, s), 4 * S, hipMemcpyDeviceToHost, ctx->s_down));
    PT_HIP(ctx, hipMemcpyAsync(h_param16[i], slot_p16(ctx, s), 2 * S, hipMemcpyDeviceToHost, ctx->s_down));
    PT_HIP(ctx, hipEventRecord(ctx->ev_down[s], ctx->s_down));
    ctx->slot_used[s] = true;
    ctx->last_slot = s;
    ctx->stream_pending = true;
  }
  if (watch) {
    PT_HIP(ctx, hipEventRecord(ctx->ev_t1, ctx->s_down));
    ctx->health_pending = true;
    ctx->health_bytes = uint64_t(14) * S * n_chunks;
    ctx->health_chunks = n_chunks;
  }
  return PT_OK;
}
