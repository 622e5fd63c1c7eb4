// Streamed update of host-resident chunks through a ring of device chunk
// buffers: upload, update and offload run on three side streams ordered by
// events, so that H2D(i+1), the kernel of chunk i and D2H(i-1) overlap each other
// and whatever the caller runs on its own stream.
//
// Link-bound: 14 bytes up and 14 bytes down per element over the host link
// against 28 bytes of HBM traffic in the kernel.
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

// Gives back whatever a reservation (failed or complete) has created, so that the call can be repeated.
void pt_stream_release(pt_ctx* ctx) {
  if (ctx->s_up) { (void)hipStreamDestroy(ctx->s_up); ctx->s_up = nullptr; }
  if (ctx->s_comp) { (void)hipStreamDestroy(ctx->s_comp); ctx->s_comp = nullptr; }
  if (ctx->s_down) { (void)hipStreamDestroy(ctx->s_down); ctx->s_down = nullptr; }
  if (ctx->ev_fork) { (void)hipEventDestroy(ctx->ev_fork); ctx->ev_fork = nullptr; }
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
  ctx->n_slots = n_slots;
  return PT_OK;
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

  int rc = pt_prepare_consts(ctx, hp, st);
  if (rc != PT_OK) return rc;
  // side streams start after everything already enqueued on the caller's stream
  PT_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
  PT_HIP(ctx, hipStreamWaitEvent(ctx->s_up, ctx->ev_fork, 0));
  PT_HIP(ctx, hipStreamWaitEvent(ctx->s_comp, ctx->ev_fork, 0));

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
  return PT_OK;
}
