// Host-side update of host-resident chunks: the paper's own placement of the update of
// non-persistent chunks ("CPU Adam" running concurrently with GPU work; Hierarchical Chunk
// Management for Model States; Appendix A.1, T_CPU_OPTIM).  Host threads walk the pinned
// master / momentum / variance arrays in place, so nothing but the 16-bit gradients and
// parameters ever needs to cross the CPU-GPU link.
//
// Same fp32 operation sequence as the device kernel, driven by the same nine fp32
// constants (read back from the device once per step), so host-updated and
// device-updated chunks are bit-identical.  The loops, the grain queue and the thread pool
// are plain host C++ in pt_host_update.h; this file is the entry point around them.
#include "pt_common.h"
#include "pt_host_update.h"

#pragma clang fp contract(off)

void pt_host_pool_destroy(pt_ctx* ctx) {
  delete ctx->host_pool;
  ctx->host_pool = nullptr;
}

extern "C" int pt_chunk_host_adamw_step(pt_ctx* ctx, const pt_hparams* hp, uint32_t first_chunk, uint32_t n_chunks,
                                        const void* const* h_grad, float* const* h_master, float* const* h_m,
                                        float* const* h_v, void* const* h_param16, uint32_t n_threads,
                                        void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (!hp) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_host_adamw_step: hp is NULL");
  if (uint64_t(first_chunk) + n_chunks > ctx->C)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_host_adamw_step: chunks [%u, %u) outside the context's %u chunks",
                   first_chunk, first_chunk + n_chunks, ctx->C);
  if (n_chunks && (!h_grad || !h_master || !h_m || !h_v || !h_param16))
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_host_adamw_step: NULL pointer array");
  if (n_threads == 0 || n_threads > 1024)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_host_adamw_step: n_threads must be in [1, 1024]");
  if (!ctx->norm_finalized)
    return pt_fail(ctx, PT_ERR_STATE, "pt_chunk_host_adamw_step: no finalized gradient norm in this step");
  for (uint32_t i = 0; i < n_chunks; ++i)
    if (!h_grad[i] || !h_master[i] || !h_m[i] || !h_v[i] || !h_param16[i])
      return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_host_adamw_step: NULL host pointer for chunk %u", first_chunk + i);
  if (n_chunks == 0) return PT_OK;

  // The step's constants come from the device, so that host and device updates use the same
  // bits.  Only the scalar kernels are waited for, not the bulk work queued behind them.
  int rc = pt_prepare_consts(ctx, hp, st);
  if (rc != PT_OK) return rc;
  // ev_scalar was recorded right behind the scalar kernel of this step (pt_prepare_consts), which left a copy
  // of the scalars in pinned host memory: waiting for that event is all it takes - no stream of the library's
  // own, whose copy could end up behind the resident update in a shared hardware queue
  PT_HIP(ctx, hipEventSynchronize(ctx->ev_scalar));
  PtDevState hs;
  std::memcpy(&hs, ctx->h_state, sizeof hs);
  if (hs.skip) return PT_OK;                     // skipped step: the host arrays stay as they are
  pt_host::Job job;
  job.k = pt_host::Consts{hs.c[0], hs.c[1], hs.c[2], hs.c[3], hs.c[4], hs.c[5], hs.c[6], hs.c[7], hs.c[8]};
  job.dtype_fp16 = ctx->dtype == PT_FP16;
  job.grad_f32 = ctx->grad_f32;
  job.S = ctx->S;
  job.first_chunk = first_chunk;
  job.n_chunks = n_chunks;
  job.h_grad = h_grad; job.h_master = h_master; job.h_m = h_m; job.h_v = h_v; job.h_param16 = h_param16;
  if (!ctx->h_nd_begin.empty()) { job.nd_begin = ctx->h_nd_begin.data(); job.nd_ranges = ctx->h_nd_ranges.data(); }
  // The workers belong to the context and sleep between steps; they are (re)started only when the
  // caller asks for another thread count.  This thread works along, so the pool holds n_threads - 1.
  return pt_guarded(ctx, "pt_chunk_host_adamw_step", [&] {
    if (!ctx->host_pool || ctx->host_pool_threads != n_threads) {
      delete ctx->host_pool;
      ctx->host_pool = nullptr;
      ctx->host_pool = new pt_host::Pool(n_threads - 1);
      ctx->host_pool_threads = n_threads;
    }
    ctx->host_pool->run(job);
    return int(PT_OK);
  });
}
