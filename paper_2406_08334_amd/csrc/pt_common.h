// Internal declarations shared by the translation units of libptchunk.so.
// Not part of the public boundary (that is include/ptchunk.h).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "ptchunk.h"

// Device (global) address space qualifier for pointers rebuilt from integer addresses: the
// compiler then emits global_* memory instructions instead of flat_* ones.
#define PT_GLOBAL __attribute__((address_space(1)))

// ---- device-resident scalars of a context ---------------------------------------
// One instance per context, in device memory.  Written only by the single-thread
// scalar kernels; read (uniformly) by the bulk kernels.
struct PtDevState {
  double sqnorm;
  double norm;
  double clip_coef;
  double loss_scale;
  double growth;
  double backoff;
  int32_t found_inf;
  int32_t step;          // applied updates so far
  int32_t good_steps;
  int32_t growth_interval;
  int32_t scaler_enabled;
  int32_t override_active;
  float override_grad_mult;
  // constants of the update in flight (see pt_update_consts)
  float c[9];
  int32_t skip;
};

// Rows of the per-context device pointer table.  Each row has n_chunks + n_slots
// entries; entries [n_chunks, n_chunks + n_slots) are the device chunk buffers
// of the streamed path.
enum PtRow : int {
  ROW_GRAD = 0,
  ROW_MASTER = 1,
  ROW_M = 2,
  ROW_V = 3,
  ROW_P16 = 4,
  ROW_PACK = 5,    // gradient chunks as seen by pack / sqnorm
  ROW_UNPACK = 6,  // source chunks of unpack
  N_ROWS = 7
};

constexpr uint32_t PT_MAX_SLOTS = 8;
constexpr uint32_t PT_ADAMW_MIN_GRID = 16384;      // default grid of the update kernel: max(this, tiles / 3)
constexpr uint32_t PT_ADAMW_DEFAULT_UNROLL = 4;
constexpr uint32_t PT_NORM_BLOCK_ELEMS = 32768;  // elements one block of the norm kernel reduces
constexpr uint32_t PT_PACK_TILE_ELEMS = 8192;    // chunk-space tile of the pack kernel (one 4-vector batch per lane)

struct PtTile {        // one block of work of the pack / unpack kernels
  uint64_t tensor_addr;  // byte address of the first element on the tensor side
  uint64_t chunk_off;    // first element on the chunk side
  uint32_t chunk;
  uint32_t len;          // 1 .. tile size of the plan
};

struct pt_pack_plan {
  pt_ctx* ctx = nullptr;
  uint32_t n_tiles = 0;
  PtTile* d_tiles = nullptr;
  uint32_t* d_chunk_tile_begin = nullptr;  // n_chunks + 1 entries (tiles sorted by chunk)
  double* d_tile_sq = nullptr;
  uint32_t* d_tile_flag = nullptr;
  uint64_t total_elems = 0;
  uint64_t id = 0;                         // never reused within a context (a destroyed plan's address may be)
  std::vector<uint32_t> touched;           // chunks that own at least one tile
};

namespace pt_host { class Pool; }

// A per-chunk reduction of partial sums that has been put off (see pt_norm.hip).
struct PtPendingReduce {
  bool active = false;
  const double* part = nullptr;
  const uint32_t* flag = nullptr;
  const uint32_t* tile_begin = nullptr;
  uint32_t first = 0, n = 0, per_chunk = 0;
  hipStream_t stream = nullptr;          // where it was asked for (used if the plan goes away first)
  const pt_pack_plan* plan = nullptr;    // owner of part / flag / tile_begin
};

struct pt_ctx {
  int device = 0;
  int dtype = PT_BF16;
  uint64_t S = 0;          // chunk_elems
  uint32_t C = 0;          // n_chunks
  uint32_t norm_blocks = 0;  // blocks per chunk of the norm kernel
  uint32_t table_cols = 0;   // C + PT_MAX_SLOTS
  // launch-shape options (pt_ctx_set_option)
  uint32_t opt_adamw_grid = 0;      // workgroups of the update kernel; 0 = max(PT_ADAMW_MIN_GRID, tiles / 3)
  uint32_t opt_adamw_unroll = PT_ADAMW_DEFAULT_UNROLL;  // 4-element units per lane per tile: 1, 2, 4 or 8
  uint32_t opt_adamw_threads = 0;   // workgroup size of the update kernel: 256, 512, or 0 = by launch size (pt_adamw_threads)
  uint32_t opt_adamw_nt = 2;        // non-temporal hints on the update's loads and stores: 0 no, 1 yes, 2 = by launch size (pt_adamw_nt)
  uint32_t opt_pack_tile_elems = PT_PACK_TILE_ELEMS;  // read when a pack plan is created
  bool scaler = false;
  bool grad_f32 = false;            // gradient chunks hold fp32 (accumulated micro-batches), option "grad_fp32"
  uint32_t opt_zero_grads = 0;      // pt_chunk_adamw_step zeroes the gradient chunks it has read

  PtDevState* d_state = nullptr;
  uint64_t* d_table = nullptr;          // [N_ROWS][table_cols]
  std::vector<uint64_t> h_table;        // host shadow of d_table
  double* d_chunk_sq = nullptr;         // [C]
  uint32_t* d_chunk_flag = nullptr;     // [C]
  double* d_norm_part = nullptr;        // [C * norm_blocks]
  uint32_t* d_norm_flag = nullptr;      // [C * norm_blocks]

  // host-side step bookkeeping
  std::vector<uint64_t> chunk_packed_by;   // [C] id of the pack plan whose partial sum is the chunk's value in this step, 0 = none
  uint64_t plan_ids = 0;
  std::vector<uint8_t> chunk_fresh;     // [C] 1 = the chunk's sum of squares was taken in this step (since pt_step_end)
  bool norm_finalized = false;
  bool prepared = false;
  PtPendingReduce pend_reduce;          // scalar work put off to be fused into one launch (pt_norm.hip)
  bool pend_finalize = false;
  pt_hparams prepared_hp{};

  // streamed path
  uint32_t n_slots = 0;
  void* slot_mem[PT_MAX_SLOTS] = {};
  hipStream_t s_up = nullptr, s_comp = nullptr, s_down = nullptr;
  hipEvent_t ev_fork = nullptr;
  hipEvent_t ev_up[PT_MAX_SLOTS] = {}, ev_k[PT_MAX_SLOTS] = {}, ev_down[PT_MAX_SLOTS] = {};
  // outcome of the duplex self-test of pt_stream_reserve: tested (the chunk buffers were large enough and the
  // scratch could be pinned), ok (upload and offload overlapped), offload streams tried
  uint32_t opt_force_unhealthy = 0;     // tests: the next look at a finished step finds it serialised whatever it measured
  uint32_t stream_rebuilds = 0;         // times the side streams were replaced after a serialised step
  void* h_trial = nullptr;              // pinned scratch of the trial copies (kept while chunk buffers are reserved)
  double link_one_dir_Bps = 0.0;        // one-direction rate of the link, from the reservation's trial copies
  hipEvent_t ev_t0 = nullptr, ev_t1 = nullptr;   // first upload may start / last offload done (timed)
  bool health_pending = false;
  uint64_t health_bytes = 0;            // bytes per direction of the step the two events bracket
  uint32_t health_chunks = 0;
  uint32_t opt_duplex_reject = 0;       // the self-test rejects that many offload streams whatever it measures (tests)
  bool duplex_tested = false, duplex_ok = false;
  uint32_t duplex_attempts = 0;
  bool slot_used[PT_MAX_SLOTS] = {};
  bool stream_pending = false;
  uint32_t last_slot = 0;

  // weight-decay groups: per chunk, sorted disjoint element ranges kept out of the decay
  uint32_t* d_nd_begin = nullptr;        // [C + 1] indices into d_nd_ranges (NULL: no ranges set)
  uint64_t* d_nd_ranges = nullptr;       // pairs (lo, hi)
  std::vector<uint32_t> h_nd_begin;
  std::vector<uint64_t> h_nd_ranges;

  // host-side update: a side stream and a pinned landing buffer for the step's scalars
  PtDevState* h_state_dev = nullptr;    // h_state as the device addresses it (the scalar kernels mirror the state there)
  hipEvent_t ev_scalar = nullptr;
  PtDevState* h_state = nullptr;
  pt_host::Pool* host_pool = nullptr;   // worker threads of the host-side update, started on first use
  uint32_t host_pool_threads = 0;       // n_threads the pool was built for

  std::string err;
};

// ---- error plumbing ----------------------------------------------------------------
int pt_fail(pt_ctx* ctx, int status, const char* fmt, ...) noexcept;

// Runs the body of an entry point that allocates host memory; a C++ exception becomes a status
// code, so that nothing is ever thrown across the C boundary.
template <class F>
inline int pt_guarded(pt_ctx* ctx, const char* who, F&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return pt_fail(ctx, PT_ERR_NOMEM, "%s: out of host memory", who);
  } catch (...) {
    return pt_fail(ctx, PT_ERR_UNSUPPORTED, "%s: unexpected C++ exception", who);
  }
}

#define PT_HIP(ctx, call)                                                              \
  do {                                                                                 \
    hipError_t e__ = (call);                                                           \
    if (e__ != hipSuccess)                                                             \
      return pt_fail((ctx), PT_ERR_HIP, "%s failed: %s (%s:%d)", #call,                \
                     hipGetErrorString(e__), __FILE__, __LINE__);                      \
  } while (0)

#define PT_LAUNCH_CHECK(ctx, name)                                                     \
  do {                                                                                 \
    hipError_t e__ = hipGetLastError();                                                \
    if (e__ != hipSuccess)                                                             \
      return pt_fail((ctx), PT_ERR_HIP, "launch of %s failed: %s", (name),             \
                     hipGetErrorString(e__));                                          \
  } while (0)

// ---- fixed-order block reduction (device) --------------------------------------------
// Sum of `acc` and OR of `flag` over a workgroup of 256 threads, in a fixed order: a 64-lane
// shuffle tree per wave, then the four waves one after the other through LDS.  No atomics, so a
// result does not depend on timing.  The result is valid in thread 0 only.  Every kernel that
// leaves a partial sum of squares (pack, accumulate, the standalone norm, the per-chunk sums)
// reduces through this one function, so their partials are interchangeable bit for bit.
constexpr int PT_REDUCE_THREADS = 256;

__device__ __forceinline__ void pt_block_sum(double& acc, uint32_t& flag) {
  __shared__ double s_sum[PT_REDUCE_THREADS / 64];
  __shared__ uint32_t s_flag[PT_REDUCE_THREADS / 64];
  double w = acc;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) w += __shfl_down(w, off, 64);
  const uint32_t f = __any(flag != 0) ? 1u : 0u;
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
  if (lane == 0) { s_sum[wid] = w; s_flag[wid] = f; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = s_sum[0];
    uint32_t g = s_flag[0];
#pragma unroll
    for (int i = 1; i < PT_REDUCE_THREADS / 64; ++i) { t += s_sum[i]; g |= s_flag[i]; }
    acc = t; flag = g;
  }
}

// ---- helpers implemented in pt_ctx.hip ---------------------------------------------
// Makes rows[r][first .. first+n) of the device pointer table equal to ptrs[0..n);
// re-uploads (after synchronising `stream`) only when something changed.
// allow_null: NULL entries are accepted (and stored as 0).
int pt_table_bind(pt_ctx* ctx, int row, uint32_t first, uint32_t n, const void* const* ptrs,
                  bool allow_null, hipStream_t stream, bool* changed);
inline const uint64_t* pt_row(const pt_ctx* ctx, int row) {
  return ctx->d_table + size_t(row) * ctx->table_cols;
}

// ---- implemented in pt_adamw.hip ------------------------------------------------------
// recast_on_skip: on a skipped step rewrite param16 = RNE(master) instead of doing nothing.
// mask_chunk0: chunk index (for the no-decay ranges) of table column first_col.
// zero_grads: overwrite the gradient chunks with zeros once read (resident chunks only).
// Workgroup size for an update launch over n_cols chunks: the option if set, else 512 for launches of 2^28
// elements or more (measured equal or up to 1 % faster there) and 256 for small ones (launch-bound: more, smaller
// workgroups start sooner).
inline uint32_t pt_adamw_threads(const pt_ctx* ctx, uint32_t n_cols) {
  if (ctx->opt_adamw_threads) return ctx->opt_adamw_threads;
  return ctx->S * uint64_t(n_cols) >= (uint64_t(1) << 28) ? 512u : 256u;
}
// Non-temporal hints for an update launch over n_cols chunks: the option if set, else by the state the launch
// touches (16 bytes per element).  A state that fits the 256 MB Infinity Cache is re-read from it step after
// step, and hints that keep it out of the cache cost 10 % there (21.4 against 22.7 us for 64 MiB, 71 against 80 us
// for 256 MiB); beyond it the streams have no reuse and the hints gain 4-10 % (120 against 133 us for 384 MiB).
inline bool pt_adamw_nt(const pt_ctx* ctx, uint32_t n_cols) {
  if (ctx->opt_adamw_nt != 2) return ctx->opt_adamw_nt != 0;
  return 16 * ctx->S * uint64_t(n_cols) > (uint64_t(256) << 20);
}
int pt_launch_adamw(pt_ctx* ctx, uint32_t first_col, uint32_t n_cols, hipStream_t stream, bool recast_on_skip,
                    uint32_t mask_chunk0, bool zero_grads);

// ---- implemented in pt_stream.hip ----------------------------------------------------------
// Destroys the streamed path's streams and events and frees its chunk buffers (no-op when none).
void pt_stream_release(pt_ctx* ctx);

// ---- implemented in pt_host.hip ------------------------------------------------------------
// Stops and joins the context's worker threads (no-op when there are none).
void pt_host_pool_destroy(pt_ctx* ctx);

// ---- implemented in pt_norm.hip ---------------------------------------------------------
// Looks up (once per device) the device address of the file-scope scratch array that
// pt_chunk_grad_sqnorm_noalloc works in; out may be NULL.  Called by pt_ctx_create, so that a process
// with a context never pays the lookup inside a hot call.
int pt_static_scratch_setup(void** out);
// Sums per-block partials into per-chunk values.  uniform mode (tile_begin == NULL):
// chunk first+i owns partials [i*per_chunk, (i+1)*per_chunk).  With a plan whose n_touched chunks and
// n_partials partial sums are few, the reduction is put off and runs inside the launch that finalizes
// the norm (plan == NULL: always at once).
int pt_launch_chunk_reduce(pt_ctx* ctx, const double* part, const uint32_t* flag,
                           const uint32_t* tile_begin, uint32_t first, uint32_t n,
                           uint32_t per_chunk, hipStream_t stream, const pt_pack_plan* plan, uint32_t n_partials,
                           uint32_t n_touched);
// Launches, on `stream`, whatever scalar work of the step has been put off (per-chunk reduction, finalize).
// Every call that reads the step's scalars or replaces what is pending goes through this first.
int pt_flush_pending(pt_ctx* ctx, hipStream_t stream);
// Derives this step's update constants from `hp` if that has not happened yet - in one launch together
// with any pending reduction and finalize.
int pt_prepare_consts(pt_ctx* ctx, const pt_hparams* hp, hipStream_t stream);
