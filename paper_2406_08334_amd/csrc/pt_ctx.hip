// Context, error plumbing, pointer tables, host-side layout builder and the
// single-thread scalar kernels (state set / override / step end).
#include "pt_common.h"

#include <algorithm>

static thread_local std::string g_noctx_error;

int pt_fail(pt_ctx* ctx, int status, const char* fmt, ...) noexcept {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  try {
    if (ctx) ctx->err = buf; else g_noctx_error = buf;
  } catch (...) {
    // no memory even for the text: the status code still says what happened
  }
  return status;
}

// ---- scalar kernels ------------------------------------------------------------------

__global__ void k_init_state(PtDevState* st, double loss_scale, double growth, double backoff,
                             int32_t growth_interval, int32_t scaler_enabled) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  st->sqnorm = 0.0; st->norm = 0.0; st->clip_coef = 1.0;
  st->loss_scale = loss_scale; st->growth = growth; st->backoff = backoff;
  st->found_inf = 0; st->step = 0; st->good_steps = 0;
  st->growth_interval = growth_interval; st->scaler_enabled = scaler_enabled;
  st->override_active = 0; st->override_grad_mult = 1.0f;
  for (int i = 0; i < 9; ++i) st->c[i] = 0.0f;
  st->skip = 0;
}

__global__ void k_set_state(PtDevState* st, int32_t step, double loss_scale, int32_t good_steps) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  st->step = step; st->loss_scale = loss_scale; st->good_steps = good_steps;
}

__global__ void k_override(PtDevState* st, float grad_mult, int32_t found_inf) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  st->override_active = 1; st->override_grad_mult = grad_mult; st->found_inf = found_inf;
  st->sqnorm = 0.0; st->norm = 0.0;
}

// Loss-scale machine and step counter (dynamic loss scaling with skip on
// non-finite gradients; the counter does not move on a skipped step).
__global__ void k_step_end(PtDevState* st) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  if (st->found_inf) {
    if (st->scaler_enabled) {
      double s = st->loss_scale * st->backoff;
      st->loss_scale = s > 1.0 ? s : 1.0;
      st->good_steps = 0;
    }
  } else {
    st->step += 1;
    if (st->scaler_enabled) {
      st->good_steps += 1;
      if (st->good_steps >= st->growth_interval) {
        st->loss_scale = st->loss_scale * st->growth;
        st->good_steps = 0;
      }
    }
  }
  st->override_active = 0;
}

// ---- public: misc -------------------------------------------------------------------------

extern "C" const char* pt_version(void) { return "ptchunk 0.1 (gfx950)"; }

extern "C" const char* pt_status_string(int s) {
  switch (s) {
    case PT_OK: return "PT_OK";
    case PT_ERR_INVALID_ARG: return "PT_ERR_INVALID_ARG";
    case PT_ERR_ALIGNMENT: return "PT_ERR_ALIGNMENT";
    case PT_ERR_HIP: return "PT_ERR_HIP";
    case PT_ERR_STATE: return "PT_ERR_STATE";
    case PT_ERR_UNSUPPORTED: return "PT_ERR_UNSUPPORTED";
    case PT_ERR_NOMEM: return "PT_ERR_NOMEM";
    default: return "PT_ERR_UNKNOWN";
  }
}

extern "C" const char* pt_last_error(const pt_ctx* ctx) {
  return ctx ? ctx->err.c_str() : g_noctx_error.c_str();
}

// ---- public: context ----------------------------------------------------------------------

static void ctx_free_all(pt_ctx* ctx) {
  pt_host_pool_destroy(ctx);
  pt_stream_release(ctx);
  if (ctx->ev_scalar) (void)hipEventDestroy(ctx->ev_scalar);
  if (ctx->h_state) (void)hipHostFree(ctx->h_state);
  if (ctx->d_nd_begin) (void)hipFree(ctx->d_nd_begin);
  if (ctx->d_nd_ranges) (void)hipFree(ctx->d_nd_ranges);
  if (ctx->d_state) (void)hipFree(ctx->d_state);
  if (ctx->d_table) (void)hipFree(ctx->d_table);
  if (ctx->d_chunk_sq) (void)hipFree(ctx->d_chunk_sq);
  if (ctx->d_chunk_flag) (void)hipFree(ctx->d_chunk_flag);
  if (ctx->d_norm_part) (void)hipFree(ctx->d_norm_part);
  if (ctx->d_norm_flag) (void)hipFree(ctx->d_norm_flag);
}

static int ctx_alloc(pt_ctx* ctx, const pt_scaler_cfg* sc) {
  PT_HIP(ctx, hipGetDevice(&ctx->device));
  if (int rc = pt_static_scratch_setup(nullptr); rc != PT_OK) return pt_fail(ctx, rc, "%s", pt_last_error(nullptr));
  PT_HIP(ctx, hipMalloc(&ctx->d_state, sizeof(PtDevState)));
  size_t tab_bytes = size_t(N_ROWS) * ctx->table_cols * sizeof(uint64_t);
  PT_HIP(ctx, hipMalloc(&ctx->d_table, tab_bytes));
  PT_HIP(ctx, hipMemset(ctx->d_table, 0, tab_bytes));
  ctx->h_table.assign(size_t(N_ROWS) * ctx->table_cols, 0);
  ctx->chunk_fresh.assign(ctx->C, 0);
  ctx->chunk_packed_by.assign(ctx->C, 0);
  PT_HIP(ctx, hipMalloc(&ctx->d_chunk_sq, ctx->C * sizeof(double)));
  PT_HIP(ctx, hipMemset(ctx->d_chunk_sq, 0, ctx->C * sizeof(double)));
  PT_HIP(ctx, hipMalloc(&ctx->d_chunk_flag, ctx->C * sizeof(uint32_t)));
  PT_HIP(ctx, hipMemset(ctx->d_chunk_flag, 0, ctx->C * sizeof(uint32_t)));
  size_t np = size_t(ctx->C) * ctx->norm_blocks;
  PT_HIP(ctx, hipMalloc(&ctx->d_norm_part, np * sizeof(double)));
  PT_HIP(ctx, hipMalloc(&ctx->d_norm_flag, np * sizeof(uint32_t)));
  PT_HIP(ctx, hipEventCreateWithFlags(&ctx->ev_scalar, hipEventDisableTiming));
  PT_HIP(ctx, hipHostMalloc((void**)&ctx->h_state, sizeof(PtDevState), hipHostMallocDefault));
  std::memset(ctx->h_state, 0, sizeof(PtDevState));
  PT_HIP(ctx, hipHostGetDevicePointer((void**)&ctx->h_state_dev, ctx->h_state, 0));
  double init = sc ? sc->init_scale : 1.0;
  hipLaunchKernelGGL(k_init_state, dim3(1), dim3(1), 0, nullptr, ctx->d_state, init,
                     sc ? sc->growth : 1.0, sc ? sc->backoff : 1.0,
                     sc ? sc->growth_interval : 0, sc ? 1 : 0);
  PT_LAUNCH_CHECK(ctx, "k_init_state");
  PT_HIP(ctx, hipDeviceSynchronize());
  return PT_OK;
}

extern "C" int pt_ctx_create(pt_ctx** out, int dtype, uint64_t chunk_elems, uint32_t n_chunks,
                             const pt_scaler_cfg* scaler) {
  if (!out) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_ctx_create: out is NULL");
  *out = nullptr;
  if (dtype != PT_BF16 && dtype != PT_FP16)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_ctx_create: dtype %d is neither PT_BF16 nor PT_FP16", dtype);
  if (chunk_elems == 0 || n_chunks == 0)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_ctx_create: chunk_elems and n_chunks must be > 0");
  if (chunk_elems % 8 != 0)
    return pt_fail(nullptr, PT_ERR_ALIGNMENT, "pt_ctx_create: chunk_elems %llu is not a multiple of 8",
                   (unsigned long long)chunk_elems);
  if (chunk_elems > (uint64_t(1) << 40) || n_chunks > 60000)
    return pt_fail(nullptr, PT_ERR_UNSUPPORTED, "pt_ctx_create: chunk_elems > 2^40 or n_chunks > 60000");
  if (scaler) {
    if (!(scaler->init_scale >= 1.0) || !(scaler->growth >= 1.0) || !(scaler->backoff > 0.0) ||
        !(scaler->backoff <= 1.0) || scaler->growth_interval < 1)
      return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_ctx_create: scaler needs init_scale >= 1, growth >= 1, "
                     "0 < backoff <= 1, growth_interval >= 1");
  }
  pt_ctx* ctx = new (std::nothrow) pt_ctx();
  if (!ctx) return pt_fail(nullptr, PT_ERR_NOMEM, "pt_ctx_create: out of host memory");
  ctx->dtype = dtype;
  ctx->S = chunk_elems;
  ctx->C = n_chunks;
  ctx->norm_blocks = uint32_t((chunk_elems + PT_NORM_BLOCK_ELEMS - 1) / PT_NORM_BLOCK_ELEMS);
  ctx->table_cols = n_chunks + PT_MAX_SLOTS;
  ctx->scaler = scaler != nullptr;
  int rc = pt_guarded(ctx, "pt_ctx_create", [&] { return ctx_alloc(ctx, scaler); });
  if (rc != PT_OK) {
    try { g_noctx_error = ctx->err; } catch (...) {}
    ctx_free_all(ctx);
    delete ctx;
    return rc;
  }
  *out = ctx;
  return PT_OK;
}

extern "C" int pt_ctx_destroy(pt_ctx* ctx) {
  if (!ctx) return PT_OK;
  (void)hipDeviceSynchronize();
  ctx_free_all(ctx);
  delete ctx;
  return PT_OK;
}

extern "C" int pt_ctx_set_state(pt_ctx* ctx, int32_t step, double loss_scale, int32_t good_steps,
                                void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (step < 0 || good_steps < 0 || !(loss_scale >= 1.0))
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_ctx_set_state: step, good_steps >= 0 and loss_scale >= 1 required");
  if (!ctx->scaler && loss_scale != 1.0)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_ctx_set_state: context has no scaler, loss_scale must be 1");
  if (int rc = pt_flush_pending(ctx, (hipStream_t)stream); rc != PT_OK) return rc;
  hipLaunchKernelGGL(k_set_state, dim3(1), dim3(1), 0, (hipStream_t)stream, ctx->d_state, step,
                     loss_scale, good_steps);
  PT_LAUNCH_CHECK(ctx, "k_set_state");
  return PT_OK;
}

extern "C" int pt_ctx_set_option(pt_ctx* ctx, const char* name, int64_t value) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (!name) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_ctx_set_option: name is NULL");
  if (std::strcmp(name, "adamw_grid") == 0) {
    if (value < 0 || value > (1 << 20)) return pt_fail(ctx, PT_ERR_INVALID_ARG, "adamw_grid must be in [0, 2^20]");
    ctx->opt_adamw_grid = uint32_t(value);
    return PT_OK;
  }
  if (std::strcmp(name, "adamw_unroll") == 0) {
    if (value != 1 && value != 2 && value != 4 && value != 8)
      return pt_fail(ctx, PT_ERR_INVALID_ARG, "adamw_unroll must be 1, 2, 4 or 8");
    ctx->opt_adamw_unroll = uint32_t(value);
    return PT_OK;
  }
  if (std::strcmp(name, "adamw_threads") == 0) {
    if (value != 0 && value != 256 && value != 512) return pt_fail(ctx, PT_ERR_INVALID_ARG, "adamw_threads must be 0, 256 or 512");
    ctx->opt_adamw_threads = uint32_t(value);
    return PT_OK;
  }
  if (std::strcmp(name, "stream_test_unhealthy") == 0) {
    ctx->opt_force_unhealthy = value != 0;
    return PT_OK;
  }
  if (std::strcmp(name, "stream_test_reject") == 0) {
    if (value < 0 || value > 5) return pt_fail(ctx, PT_ERR_INVALID_ARG, "stream_test_reject must be in [0, 5]");
    ctx->opt_duplex_reject = uint32_t(value);
    return PT_OK;
  }
  if (std::strcmp(name, "pack_tile_elems") == 0) {
    if (value < 1024 || value > (1 << 26)) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pack_tile_elems must be in [1024, 2^26]");
    ctx->opt_pack_tile_elems = uint32_t(value);
    return PT_OK;
  }
  if (std::strcmp(name, "adamw_nt") == 0) {
    if (value < 0 || value > 2) return pt_fail(ctx, PT_ERR_INVALID_ARG, "adamw_nt must be 0, 1 or 2");
    ctx->opt_adamw_nt = uint32_t(value);
    return PT_OK;
  }
  if (std::strcmp(name, "adamw_zero_grads") == 0) {
    ctx->opt_zero_grads = value != 0;
    return PT_OK;
  }
  if (std::strcmp(name, "grad_fp32") == 0) {
    if (ctx->n_slots && (value != 0) != ctx->grad_f32)
      return pt_fail(ctx, PT_ERR_STATE, "grad_fp32 must be chosen before pt_stream_reserve (the chunk buffers are sized by it)");
    ctx->grad_f32 = value != 0;
    ctx->norm_finalized = false;
    return PT_OK;
  }
  return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_ctx_set_option: unknown option '%s'", name);
}

static int set_no_decay(pt_ctx* ctx, const pt_segment* segs, uint32_t n_segs);

extern "C" int pt_ctx_set_no_decay(pt_ctx* ctx, const pt_segment* segs, uint32_t n_segs) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (!segs && n_segs) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_ctx_set_no_decay: segs is NULL");
  return pt_guarded(ctx, "pt_ctx_set_no_decay", [&] { return set_no_decay(ctx, segs, n_segs); });
}

static int set_no_decay(pt_ctx* ctx, const pt_segment* segs, uint32_t n_segs) {
  // per chunk: sort, merge touching ranges
  std::vector<std::vector<std::pair<uint64_t, uint64_t>>> per(ctx->C);
  for (uint32_t i = 0; i < n_segs; ++i) {
    const pt_segment& s = segs[i];
    if (s.len == 0) continue;
    if (s.chunk >= ctx->C || s.chunk_off >= ctx->S || s.len > ctx->S - s.chunk_off)
      return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_ctx_set_no_decay: segment %u lies outside the context's chunks", i);
    per[s.chunk].push_back({s.chunk_off, s.chunk_off + s.len});
  }
  std::vector<uint32_t> begin(size_t(ctx->C) + 1, 0);
  std::vector<uint64_t> ranges;
  for (uint32_t c = 0; c < ctx->C; ++c) {
    auto& v = per[c];
    std::sort(v.begin(), v.end());
    size_t first = ranges.size() / 2;
    for (auto& r : v) {
      if (ranges.size() / 2 > first && r.first <= ranges.back()) {
        if (r.second > ranges.back()) ranges.back() = r.second;
      } else {
        ranges.push_back(r.first);
        ranges.push_back(r.second);
      }
    }
    begin[c + 1] = uint32_t(ranges.size() / 2);
  }
  (void)hipDeviceSynchronize();          // kernels in flight may still read the old ranges
  if (ctx->d_nd_begin) { (void)hipFree(ctx->d_nd_begin); ctx->d_nd_begin = nullptr; }
  if (ctx->d_nd_ranges) { (void)hipFree(ctx->d_nd_ranges); ctx->d_nd_ranges = nullptr; }
  ctx->h_nd_begin.clear();
  ctx->h_nd_ranges.clear();
  if (ranges.empty()) return PT_OK;      // nothing kept out of the decay: the unmasked kernel runs
  PT_HIP(ctx, hipMalloc(&ctx->d_nd_ranges, ranges.size() * sizeof(uint64_t)));
  PT_HIP(ctx, hipMemcpy(ctx->d_nd_ranges, ranges.data(), ranges.size() * sizeof(uint64_t), hipMemcpyHostToDevice));
  PT_HIP(ctx, hipMalloc(&ctx->d_nd_begin, begin.size() * sizeof(uint32_t)));
  PT_HIP(ctx, hipMemcpy(ctx->d_nd_begin, begin.data(), begin.size() * sizeof(uint32_t), hipMemcpyHostToDevice));
  ctx->h_nd_begin = std::move(begin);
  ctx->h_nd_ranges = std::move(ranges);
  return PT_OK;
}

extern "C" int pt_step_override(pt_ctx* ctx, float grad_mult, int32_t found_inf, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (ctx->stream_pending)
    return pt_fail(ctx, PT_ERR_STATE, "pt_step_override: a streamed update is still open (its kernels read the step's "
                   "scalars); close the step with pt_step_end first");
  if (int rc = pt_flush_pending(ctx, (hipStream_t)stream); rc != PT_OK) return rc;   // a computed norm, if any, comes first
  hipLaunchKernelGGL(k_override, dim3(1), dim3(1), 0, (hipStream_t)stream, ctx->d_state, grad_mult,
                     found_inf ? 1 : 0);
  PT_LAUNCH_CHECK(ctx, "k_override");
  ctx->norm_finalized = true;
  ctx->prepared = false;
  return PT_OK;
}

extern "C" int pt_step_end(pt_ctx* ctx, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (ctx->stream_pending) {
    // offloads complete in order on one stream: the last one recorded covers them all
    PT_HIP(ctx, hipStreamWaitEvent(st, ctx->ev_down[ctx->last_slot], 0));
    ctx->stream_pending = false;
  }
  if (int rc = pt_flush_pending(ctx, st); rc != PT_OK) return rc;     // a step without an update still needs its found_inf
  hipLaunchKernelGGL(k_step_end, dim3(1), dim3(1), 0, st, ctx->d_state);
  PT_LAUNCH_CHECK(ctx, "k_step_end");
  ctx->norm_finalized = false;
  ctx->prepared = false;
  std::fill(ctx->chunk_fresh.begin(), ctx->chunk_fresh.end(), uint8_t(0));   // the next step needs new partial sums
  std::fill(ctx->chunk_packed_by.begin(), ctx->chunk_packed_by.end(), uint64_t(0));
  return PT_OK;
}

extern "C" int pt_step_report_read(pt_ctx* ctx, pt_step_report* out, void* stream) {
  if (!ctx || !out) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_step_report_read: NULL argument");
  if (int rc = pt_flush_pending(ctx, (hipStream_t)stream); rc != PT_OK) return rc;
  PtDevState h;
  PT_HIP(ctx, hipMemcpyAsync(&h, ctx->d_state, sizeof h, hipMemcpyDeviceToHost, (hipStream_t)stream));
  PT_HIP(ctx, hipStreamSynchronize((hipStream_t)stream));
  out->sqnorm = h.sqnorm; out->norm = h.norm; out->clip_coef = h.clip_coef;
  out->loss_scale = h.loss_scale; out->grad_mult = h.c[8]; out->found_inf = h.found_inf;
  out->step = h.step; out->good_steps = h.good_steps;
  return PT_OK;
}

extern "C" int pt_update_consts_read(pt_ctx* ctx, pt_update_consts* out, void* stream) {
  if (!ctx || !out) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_update_consts_read: NULL argument");
  if (int rc = pt_flush_pending(ctx, (hipStream_t)stream); rc != PT_OK) return rc;
  PtDevState h;
  PT_HIP(ctx, hipMemcpyAsync(&h, ctx->d_state, sizeof h, hipMemcpyDeviceToHost, (hipStream_t)stream));
  PT_HIP(ctx, hipStreamSynchronize((hipStream_t)stream));
  for (int i = 0; i < 9; ++i) out->c[i] = h.c[i];
  out->skip = h.skip;
  return PT_OK;
}

// ---- pointer table -------------------------------------------------------------------------

int pt_table_bind(pt_ctx* ctx, int row, uint32_t first, uint32_t n, const void* const* ptrs,
                  bool allow_null, hipStream_t stream, bool* changed) {
  uint64_t* h = ctx->h_table.data() + size_t(row) * ctx->table_cols + first;
  bool diff = false;
  for (uint32_t i = 0; i < n; ++i) {
    uint64_t p = (uint64_t)(uintptr_t)ptrs[i];
    if (!p && !allow_null) return pt_fail(ctx, PT_ERR_INVALID_ARG, "chunk pointer %u of row %d is NULL", first + i, row);
    if (p & 15) return pt_fail(ctx, PT_ERR_ALIGNMENT, "chunk pointer %u of row %d is not 16-byte aligned", first + i, row);
    if (h[i] != p) diff = true;
  }
  if (diff) {
    // Work already enqueued may still read the old entries: drain it first.  The host shadow takes
    // the new pointers only once the device table holds them, so a failed upload is retried by the
    // next call instead of being taken for done.
    PT_HIP(ctx, hipStreamSynchronize(stream));
    PT_HIP(ctx, hipMemcpy(ctx->d_table + size_t(row) * ctx->table_cols + first, ptrs, n * sizeof(uint64_t),
                          hipMemcpyHostToDevice));
    for (uint32_t i = 0; i < n; ++i) h[i] = (uint64_t)(uintptr_t)ptrs[i];
  }
  if (changed) *changed = diff;
  return PT_OK;
}

// ---- layout -----------------------------------------------------------------------------------

extern "C" int pt_layout_dense(const uint64_t* tensor_elems, uint32_t n_tensors, uint64_t chunk_elems,
                               pt_segment* out, uint32_t cap, uint32_t* n_segments, uint32_t* n_chunks) {
  if ((!tensor_elems && n_tensors) || !n_segments || !n_chunks)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_dense: NULL argument");
  if (chunk_elems == 0) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_dense: chunk_elems is 0");
  if (chunk_elems % 8 != 0)
    return pt_fail(nullptr, PT_ERR_ALIGNMENT, "pt_layout_dense: chunk_elems is not a multiple of 8");
  uint64_t pos = 0;       // global element offset
  uint64_t nseg = 0;
  for (uint32_t t = 0; t < n_tensors; ++t) {
    uint64_t left = tensor_elems[t], off = 0;
    if (pos + left < pos) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_dense: total size overflows");
    while (left) {
      uint64_t c = pos / chunk_elems, in = pos % chunk_elems;
      uint64_t run = chunk_elems - in < left ? chunk_elems - in : left;
      if (c > 0xfffffffeull) return pt_fail(nullptr, PT_ERR_UNSUPPORTED, "pt_layout_dense: too many chunks");
      if (out) {
        if (nseg >= cap) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_dense: cap %u too small", cap);
        pt_segment& s = out[nseg];
        s.src = nullptr; s.src_off = off; s.len = run; s.chunk_off = in; s.chunk = uint32_t(c); s.tensor = t;
      }
      ++nseg; pos += run; off += run; left -= run;
    }
  }
  if (nseg > 0xffffffffull) return pt_fail(nullptr, PT_ERR_UNSUPPORTED, "pt_layout_dense: too many segments");
  *n_segments = uint32_t(nseg);
  *n_chunks = uint32_t((pos + chunk_elems - 1) / chunk_elems);
  return PT_OK;
}

// ---- paper-faithful layout: no tensor split, transformer blocks kept together -----------------
// (Appendix B.1 of the paper, "Chunk Organization and Size Search".)

namespace {

constexpr uint64_t LAYOUT_ALIGN = 8;   // elements: every tensor starts on a 16-byte boundary of its chunk

inline uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// End offset after placing tensors [lo, hi) back to back from `start` (empty tensors take no room).
uint64_t span_of(const uint64_t* elems, uint32_t lo, uint32_t hi, uint64_t start) {
  uint64_t off = start;
  for (uint32_t t = lo; t < hi; ++t)
    if (elems[t]) off = round_up(off, LAYOUT_ALIGN) + elems[t];
  return off;
}

// Places every tensor; returns false if a tensor is larger than a chunk.  out may be NULL.
bool place_grouped(const uint64_t* elems, const uint32_t* group, uint32_t n, uint64_t S, pt_segment* out,
                   uint64_t cap, uint64_t* n_seg, uint64_t* n_chunks, bool* cap_hit) {
  uint64_t chunk = 0, off = 0, segs = 0;
  bool any = false;
  *cap_hit = false;
  uint32_t i = 0;
  while (i < n) {
    uint32_t j = i + 1;
    if (group && group[i] != PT_NO_GROUP)
      while (j < n && group[j] == group[i]) ++j;
    const bool together = span_of(elems, i, j, 0) <= S;       // the run fits an empty chunk: keep it whole
    uint32_t lo = i;
    while (lo < j) {
      const uint32_t hi = together ? j : lo + 1;
      uint64_t total = 0;
      for (uint32_t t = lo; t < hi; ++t) total += elems[t];
      if (total) {
        if (span_of(elems, lo, hi, 0) > S) return false;
        if (span_of(elems, lo, hi, off) > S) { ++chunk; off = 0; }
        for (uint32_t t = lo; t < hi; ++t) {
          if (!elems[t]) continue;
          off = round_up(off, LAYOUT_ALIGN);
          if (out) {
            if (segs >= cap) { *cap_hit = true; return true; }
            pt_segment& s = out[segs];
            s.src = nullptr; s.src_off = 0; s.len = elems[t]; s.chunk_off = off; s.chunk = uint32_t(chunk); s.tensor = t;
          }
          ++segs;
          off += elems[t];
          any = true;
        }
      }
      lo = hi;
    }
    i = j;
  }
  *n_seg = segs;
  *n_chunks = any ? chunk + 1 : 0;
  return true;
}

}  // namespace

extern "C" int pt_layout_execution_order(const uint32_t* uses, uint32_t n_uses, uint32_t n_tensors, uint32_t* order) {
  if ((n_uses && !uses) || (n_tensors && !order))
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_execution_order: NULL pointer");
  for (uint32_t k = 0; k < n_uses; ++k)
    if (uses[k] >= n_tensors)
      return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_execution_order: use %u names tensor %u of %u", k, uses[k],
                     n_tensors);
  return pt_guarded(nullptr, "pt_layout_execution_order", [&] {
    // one walk over the trace: a tensor takes the next place the first time it is met
    std::vector<uint8_t> placed(n_tensors, 0);
    uint32_t n = 0;
    for (uint32_t k = 0; k < n_uses; ++k)
      if (!placed[uses[k]]) { placed[uses[k]] = 1; order[n++] = uses[k]; }
    for (uint32_t t = 0; t < n_tensors; ++t)
      if (!placed[t]) order[n++] = t;
    return int(PT_OK);
  });
}

extern "C" int pt_layout_grouped(const uint64_t* tensor_elems, const uint32_t* tensor_group, uint32_t n_tensors,
                                 uint64_t chunk_elems, pt_segment* out, uint32_t cap, uint32_t* n_segments,
                                 uint32_t* n_chunks, uint64_t* waste_elems) {
  if ((!tensor_elems && n_tensors) || !n_segments || !n_chunks)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_grouped: NULL argument");
  if (chunk_elems == 0) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_grouped: chunk_elems is 0");
  if (chunk_elems % 8 != 0) return pt_fail(nullptr, PT_ERR_ALIGNMENT, "pt_layout_grouped: chunk_elems is not a multiple of 8");
  uint64_t nseg = 0, nch = 0, total = 0;
  for (uint32_t t = 0; t < n_tensors; ++t) total += tensor_elems[t];
  bool cap_hit = false;
  if (!place_grouped(tensor_elems, tensor_group, n_tensors, chunk_elems, out, cap, &nseg, &nch, &cap_hit))
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_grouped: a tensor is larger than a chunk of %llu elements",
                   (unsigned long long)chunk_elems);
  if (cap_hit) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_layout_grouped: cap %u too small", cap);
  if (nch > 0xfffffffeull) return pt_fail(nullptr, PT_ERR_UNSUPPORTED, "pt_layout_grouped: too many chunks");
  *n_segments = uint32_t(nseg);
  *n_chunks = uint32_t(nch);
  if (waste_elems) *waste_elems = nch * chunk_elems - total;
  return PT_OK;
}

extern "C" int pt_chunk_size_search(const uint64_t* tensor_elems, const uint32_t* tensor_group, uint32_t n_tensors,
                                    uint64_t min_chunk_elems, uint64_t span_elems, uint64_t step_elems,
                                    uint64_t* best_chunk_elems, uint32_t* n_chunks, uint64_t* waste_elems) {
  if ((!tensor_elems && n_tensors) || !best_chunk_elems)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_chunk_size_search: NULL argument");
  if (step_elems == 0 || step_elems % 8 != 0)
    return pt_fail(nullptr, PT_ERR_ALIGNMENT, "pt_chunk_size_search: step_elems must be a positive multiple of 8");
  uint64_t biggest = 1, total = 0;
  for (uint32_t t = 0; t < n_tensors; ++t) { total += tensor_elems[t]; if (tensor_elems[t] > biggest) biggest = tensor_elems[t]; }
  const uint64_t s_min = round_up(biggest > min_chunk_elems ? biggest : min_chunk_elems, step_elems);
  if (span_elems / step_elems > 10000000ull)
    return pt_fail(nullptr, PT_ERR_UNSUPPORTED, "pt_chunk_size_search: more than 10^7 candidates");
  bool found = false;
  uint64_t best_S = 0, best_waste = 0, best_chunks = 0;
  for (uint64_t S = s_min; S <= s_min + span_elems; S += step_elems) {
    uint64_t nseg = 0, nch = 0;
    bool cap_hit = false;
    if (!place_grouped(tensor_elems, tensor_group, n_tensors, S, nullptr, 0, &nseg, &nch, &cap_hit)) continue;
    const uint64_t waste = nch * S - total;
    if (!found || waste < best_waste) { found = true; best_S = S; best_waste = waste; best_chunks = nch; }
  }
  if (!found) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_chunk_size_search: no feasible chunk size on the grid");
  *best_chunk_elems = best_S;
  if (n_chunks) *n_chunks = uint32_t(best_chunks);
  if (waste_elems) *waste_elems = best_waste;
  return PT_OK;
}

// ---- measurement aid: a plain streaming copy ----------------------------------------------------

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256) k_calib_copy(u32x4_t* __restrict__ dst, const u32x4_t* __restrict__ src,
                                                    uint64_t n_vec) {
  const uint64_t stride = uint64_t(gridDim.x) * 256 * 4;
  for (uint64_t i = uint64_t(blockIdx.x) * 256 * 4 + threadIdx.x; i < n_vec; i += stride) {
    u32x4_t q[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (i + r * 256 < n_vec) q[r] = __builtin_nontemporal_load(src + i + r * 256);
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (i + r * 256 < n_vec) __builtin_nontemporal_store(q[r], dst + i + r * 256);
  }
}

extern "C" int pt_calib_copy(void* dst, const void* src, uint64_t bytes, void* stream) {
  if (!dst || !src) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_calib_copy: NULL pointer");
  if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | bytes) & 15)
    return pt_fail(nullptr, PT_ERR_ALIGNMENT, "pt_calib_copy: pointers and size must be multiples of 16");
  if (bytes == 0) return PT_OK;
  uint64_t n_vec = bytes / 16;
  uint64_t blocks = (n_vec + 1023) / 1024;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(k_calib_copy, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream,
                     (u32x4_t*)dst, (const u32x4_t*)src, n_vec);
  if (hipGetLastError() != hipSuccess) return pt_fail(nullptr, PT_ERR_HIP, "pt_calib_copy: launch failed");
  return PT_OK;
}
