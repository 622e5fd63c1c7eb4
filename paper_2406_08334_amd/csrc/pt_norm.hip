// Global gradient norm: per-block fp64 partial sums of squares over gradient
// chunks, a fixed-order per-chunk reduction, and the finalize step.
//
// HBM-bound: 2 bytes read per element.  Each lane issues 16-byte loads that are
// contiguous across the wavefront (1 KiB per wave instruction), converts every
// 16-bit word to fp64 and accumulates squares in fp64 (two 16-bit significands
// multiply exactly, so only the additions round).  Reduction order is fixed:
// lane-serial, then a 64-lane shuffle tree, then the four waves through LDS, then
// one slot per block - no atomics, so results are bitwise reproducible.
#include "pt_common.h"

#include <hip/hip_fp16.h>

#include <mutex>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int NB_THREADS = PT_REDUCE_THREADS;

template <int DT>
__device__ __forceinline__ double word_to_f64(uint32_t w16) {
  if (DT == PT_BF16) {
    return (double)__uint_as_float(w16 << 16);
  } else {
    __half_raw r; r.x = (unsigned short)w16;
    return (double)__half2float(__half(r));
  }
}

template <int DT>
__device__ __forceinline__ uint32_t pair_nonfinite(uint32_t two_words) {
  // exponent field all ones in either half
  constexpr uint32_t E = DT == PT_BF16 ? 0x7f80u : 0x7c00u;
  uint32_t lo = two_words & E, hi = (two_words >> 16) & E;
  return (lo == E) | (hi == E);
}

template <int DT>
__device__ __forceinline__ void accum_vec(const u32x4& q, double inv_scale, double& a0, double& a1,
                                          uint32_t& flag) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    double x0 = word_to_f64<DT>(w[k] & 0xffffu) * inv_scale;
    double x1 = word_to_f64<DT>(w[k] >> 16) * inv_scale;
    a0 = fma(x0, x0, a0);
    a1 = fma(x1, x1, a1);
    flag |= pair_nonfinite<DT>(w[k]);
  }
}

// One block's share of a chunk: the fp64 sum of (g/scale)^2 and the non-finite flag over elements
// [b*PT_NORM_BLOCK_ELEMS, min(S, (b+1)*PT_NORM_BLOCK_ELEMS)) of the chunk at `base`; valid in thread 0.
template <int DT>
__device__ __forceinline__ void sqnorm_block(const PT_GLOBAL u32x4* base, uint64_t S, uint32_t b, double inv_scale,
                                             double& acc, uint32_t& flag) {
  const uint64_t vec_total = S / 8;
  const uint64_t v0 = uint64_t(b) * (PT_NORM_BLOCK_ELEMS / 8);
  uint64_t v1 = v0 + PT_NORM_BLOCK_ELEMS / 8;
  if (v1 > vec_total) v1 = vec_total;
  double a0 = 0.0, a1 = 0.0;
  flag = 0;
  uint64_t v = v0 + threadIdx.x;
  // four independent 16-byte loads in flight per lane
  for (; v + 3 * NB_THREADS < v1; v += 4 * NB_THREADS) {
    u32x4 q0 = __builtin_nontemporal_load(base + v);
    u32x4 q1 = __builtin_nontemporal_load(base + v + NB_THREADS);
    u32x4 q2 = __builtin_nontemporal_load(base + v + 2 * NB_THREADS);
    u32x4 q3 = __builtin_nontemporal_load(base + v + 3 * NB_THREADS);
    accum_vec<DT>(q0, inv_scale, a0, a1, flag);
    accum_vec<DT>(q1, inv_scale, a0, a1, flag);
    accum_vec<DT>(q2, inv_scale, a0, a1, flag);
    accum_vec<DT>(q3, inv_scale, a0, a1, flag);
  }
  for (; v < v1; v += NB_THREADS) {
    u32x4 q = __builtin_nontemporal_load(base + v);
    accum_vec<DT>(q, inv_scale, a0, a1, flag);
  }
  acc = a0 + a1;
  pt_block_sum(acc, flag);
}

// grid = (norm_blocks, n_chunks).  Block (b, i) reduces its share of chunk first+i, whose base
// pointer comes from the context's pointer table.
template <int DT>
__global__ void __launch_bounds__(NB_THREADS)
k_sqnorm(const uint64_t* __restrict__ grad_row, uint32_t first, uint64_t S,
         const PtDevState* __restrict__ st, double* __restrict__ part, uint32_t* __restrict__ flagout) {
  const uint32_t b = blockIdx.x, i = blockIdx.y;
  const PT_GLOBAL u32x4* base = (const PT_GLOBAL u32x4*)(grad_row[first + i]);   // global_* loads
  double acc;
  uint32_t flag;
  sqnorm_block<DT>(base, S, b, 1.0 / st->loss_scale, acc, flag);
  if (threadIdx.x == 0) {
    size_t slot = size_t(i) * gridDim.x + b;
    part[slot] = acc;
    flagout[slot] = flag;
  }
}

// The same reduction over fp32 gradient chunks (accumulated micro-batches): 4 bytes read per
// element, every value widened to fp64 before it is scaled and squared.
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void accum_vec_f32(const f32x4& q, double inv_scale, double& a0, double& a1,
                                              uint32_t& flag) {
#pragma unroll
  for (int k = 0; k < 4; k += 2) {
    double x0 = (double)q[k] * inv_scale;
    double x1 = (double)q[k + 1] * inv_scale;
    a0 = fma(x0, x0, a0);
    a1 = fma(x1, x1, a1);
    flag |= uint32_t((__float_as_uint(q[k]) & 0x7f800000u) == 0x7f800000u) |
            uint32_t((__float_as_uint(q[k + 1]) & 0x7f800000u) == 0x7f800000u);
  }
}

__global__ void __launch_bounds__(NB_THREADS)
k_sqnorm_f32(const uint64_t* __restrict__ grad_row, uint32_t first, uint64_t S,
             const PtDevState* __restrict__ st, double* __restrict__ part, uint32_t* __restrict__ flagout) {
  const uint32_t b = blockIdx.x, i = blockIdx.y;
  const PT_GLOBAL f32x4* base = (const PT_GLOBAL f32x4*)(grad_row[first + i]);
  const uint64_t vec_total = S / 4;
  const uint64_t v0 = uint64_t(b) * (PT_NORM_BLOCK_ELEMS / 4);
  uint64_t v1 = v0 + PT_NORM_BLOCK_ELEMS / 4;
  if (v1 > vec_total) v1 = vec_total;
  const double inv_scale = 1.0 / st->loss_scale;
  double a0 = 0.0, a1 = 0.0;
  uint32_t flag = 0;
  uint64_t v = v0 + threadIdx.x;
  for (; v + 3 * NB_THREADS < v1; v += 4 * NB_THREADS) {
    f32x4 q0 = __builtin_nontemporal_load(base + v);
    f32x4 q1 = __builtin_nontemporal_load(base + v + NB_THREADS);
    f32x4 q2 = __builtin_nontemporal_load(base + v + 2 * NB_THREADS);
    f32x4 q3 = __builtin_nontemporal_load(base + v + 3 * NB_THREADS);
    accum_vec_f32(q0, inv_scale, a0, a1, flag);
    accum_vec_f32(q1, inv_scale, a0, a1, flag);
    accum_vec_f32(q2, inv_scale, a0, a1, flag);
    accum_vec_f32(q3, inv_scale, a0, a1, flag);
  }
  for (; v < v1; v += NB_THREADS) {
    f32x4 q = __builtin_nontemporal_load(base + v);
    accum_vec_f32(q, inv_scale, a0, a1, flag);
  }
  double acc = a0 + a1;
  pt_block_sum(acc, flag);
  if (threadIdx.x == 0) {
    size_t slot = size_t(i) * gridDim.x + b;
    part[slot] = acc;
    flagout[slot] = flag;
  }
}

// One block per chunk: sums that chunk's partials (lane-strided serial sums, then
// the fixed block tree).  tile_begin == NULL: chunk first+i owns
// [i*per_chunk, (i+1)*per_chunk); otherwise [tile_begin[c], tile_begin[c+1]) and a
// chunk with an empty range keeps its previous value.
__global__ void __launch_bounds__(NB_THREADS)
k_chunk_reduce(const double* __restrict__ part, const uint32_t* __restrict__ flag,
               const uint32_t* __restrict__ tile_begin, uint32_t first, uint32_t per_chunk,
               double* __restrict__ chunk_sq, uint32_t* __restrict__ chunk_flag) {
  const uint32_t i = blockIdx.x, c = first + i;
  uint32_t lo, hi;
  if (tile_begin) { lo = tile_begin[c]; hi = tile_begin[c + 1]; if (lo == hi) return; }
  else { lo = i * per_chunk; hi = lo + per_chunk; }
  double acc = 0.0;
  uint32_t f = 0;
  for (uint32_t k = lo + threadIdx.x; k < hi; k += NB_THREADS) { acc += part[k]; f |= flag[k]; }
  pt_block_sum(acc, f);
  if (threadIdx.x == 0) { chunk_sq[c] = acc; chunk_flag[c] = f; }
}

// Sums the per-chunk values of all chunks in chunk order (single thread: C is a
// few hundred at most) and publishes the step's scalars.
__device__ __forceinline__ void finalize_body(const double* chunk_sq, const uint32_t* chunk_flag, uint32_t C, PtDevState* st) {
  double t = 0.0;
  uint32_t f = 0;
  for (uint32_t c = 0; c < C; ++c) { t += chunk_sq[c]; f |= chunk_flag[c]; }
  st->sqnorm = t;
  st->norm = sqrt(t);
  st->found_inf = f ? 1 : 0;
  st->override_active = 0;
}

__global__ void k_finalize(const double* chunk_sq, const uint32_t* chunk_flag, uint32_t C, PtDevState* st) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  finalize_body(chunk_sq, chunk_flag, C, st);
}

// Derives the nine fp32 constants of this update from the fp64 hyper-parameters
// and the step's device scalars (Adam bias correction with t = applied updates
// + 1; clip coefficient min(1, c/(norm+1e-6)); unscale by the loss scale).
__device__ __forceinline__ void prepare_body(PtDevState* st, const pt_hparams& hp) {
  const double t = double(st->step + 1);
  double clip = 1.0;
  float gm;
  if (st->override_active) {
    gm = st->override_grad_mult;
  } else {
    if (hp.max_norm > 0.0) {
      double c = hp.max_norm / (st->norm + 1e-6);
      clip = c < 1.0 ? c : 1.0;
    }
    gm = float(clip / st->loss_scale);
  }
  st->clip_coef = clip;
  st->c[0] = float(hp.beta1);
  st->c[1] = float(hp.beta2);
  st->c[2] = float(1.0 - hp.beta1);
  st->c[3] = float(1.0 - hp.beta2);
  st->c[4] = float(1.0 - hp.lr * hp.weight_decay);
  st->c[5] = float(hp.lr / (1.0 - pow(hp.beta1, t)));
  st->c[6] = float(1.0 / sqrt(1.0 - pow(hp.beta2, t)));
  st->c[7] = float(hp.eps);
  st->c[8] = gm;
  st->skip = st->found_inf ? 1 : 0;
}

// `mirror`: a copy of the step's scalars in pinned host memory that the device addresses directly.  The
// host-side update reads its constants there after waiting for the event behind this kernel - no stream, no
// copy, nothing that could queue up behind the resident update.
__global__ void k_prepare(PtDevState* st, pt_hparams hp, PtDevState* mirror) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  prepare_body(st, hp);
  *mirror = *st;
  __threadfence_system();
}

// The scalar work of a step in ONE launch, for small states where launches are what a step costs:
// one block walks the chunks one after the other - each chunk's partial sums reduced exactly as
// k_chunk_reduce does it - then its thread 0 sums the chunks (k_finalize) and derives the update's
// constants (k_prepare).  Same operations in the same order as the three separate kernels.
//   n_reduce == 0: no per-chunk reduction (already done);  do_finalize == 0: the norm is already final.
__global__ void __launch_bounds__(NB_THREADS)
k_reduce_finalize_prepare(const double* __restrict__ part, const uint32_t* __restrict__ flag,
                          const uint32_t* __restrict__ tile_begin, uint32_t first, uint32_t n_reduce, uint32_t per_chunk,
                          double* chunk_sq, uint32_t* chunk_flag, uint32_t C, PtDevState* st, pt_hparams hp,
                          int do_finalize, int do_prepare, PtDevState* mirror) {
  for (uint32_t i = 0; i < n_reduce; ++i) {
    const uint32_t c = first + i;
    uint32_t lo, hi;
    if (tile_begin) { lo = tile_begin[c]; hi = tile_begin[c + 1]; if (lo == hi) continue; }
    else { lo = i * per_chunk; hi = lo + per_chunk; }
    double acc = 0.0;
    uint32_t f = 0;
    for (uint32_t k = lo + threadIdx.x; k < hi; k += NB_THREADS) { acc += part[k]; f |= flag[k]; }
    pt_block_sum(acc, f);
    if (threadIdx.x == 0) { chunk_sq[c] = acc; chunk_flag[c] = f; }
    __syncthreads();                 // the reduction's LDS slots are reused by the next chunk
  }
  if (threadIdx.x != 0) return;
  // thread 0 wrote every per-chunk value of this launch itself; the others come from earlier kernels
  if (do_finalize) finalize_body(chunk_sq, chunk_flag, C, st);
  if (do_prepare) {
    prepare_body(st, hp);
    *mirror = *st;
    __threadfence_system();
  }
}

}  // namespace

// ---- scalar work of a step: launched at once, or deferred and fused -------------------------
//
// A step's scalar kernels (per-chunk reduction of the partial sums, finalize, prepare) are tiny;
// for a small state their launches are most of the step.  So the finalize is always deferred to
// the first call that needs its result - normally the update, which then derives its constants in
// the same launch - and the per-chunk reduction of a pack / accumulate plan is deferred with it
// when the plan is small enough for one block to walk (PT_FUSE_MAX_CHUNKS chunks,
// PT_FUSE_MAX_PARTIALS partial sums).  Every call that reads or replaces what is pending flushes it
// first (pt_flush_pending): results and their order are those of the separate kernels.

constexpr uint32_t PT_FUSE_MAX_CHUNKS = 8;
constexpr uint32_t PT_FUSE_MAX_PARTIALS = 16384;

static int launch_reduce_now(pt_ctx* ctx, const PtPendingReduce& r, hipStream_t stream) {
  if (r.n == 0) return PT_OK;
  hipLaunchKernelGGL(k_chunk_reduce, dim3(r.n), dim3(NB_THREADS), 0, stream, r.part, r.flag, r.tile_begin,
                     r.first, r.per_chunk, ctx->d_chunk_sq, ctx->d_chunk_flag);
  PT_LAUNCH_CHECK(ctx, "k_chunk_reduce");
  return PT_OK;
}

int pt_flush_pending(pt_ctx* ctx, hipStream_t stream) {
  if (ctx->pend_reduce.active) {
    ctx->pend_reduce.active = false;
    int rc = launch_reduce_now(ctx, ctx->pend_reduce, stream);
    if (rc != PT_OK) return rc;
  }
  if (ctx->pend_finalize) {
    ctx->pend_finalize = false;
    hipLaunchKernelGGL(k_finalize, dim3(1), dim3(64), 0, stream, ctx->d_chunk_sq, ctx->d_chunk_flag, ctx->C, ctx->d_state);
    PT_LAUNCH_CHECK(ctx, "k_finalize");
  }
  return PT_OK;
}

int pt_launch_chunk_reduce(pt_ctx* ctx, const double* part, const uint32_t* flag,
                           const uint32_t* tile_begin, uint32_t first, uint32_t n,
                           uint32_t per_chunk, hipStream_t stream, const pt_pack_plan* plan, uint32_t n_partials,
                           uint32_t n_touched) {
  if (n == 0) return PT_OK;
  // whatever is pending comes first: a later reduction of the same chunk replaces an earlier one
  int rc = pt_flush_pending(ctx, stream);
  if (rc != PT_OK) return rc;
  PtPendingReduce r{true, part, flag, tile_begin, first, n, per_chunk, stream, plan};
  if (plan && n_touched <= PT_FUSE_MAX_CHUNKS && n <= 64 && n_partials <= PT_FUSE_MAX_PARTIALS) {
    ctx->pend_reduce = r;            // runs inside the launch that finalizes the norm
    return PT_OK;
  }
  return launch_reduce_now(ctx, r, stream);
}

int pt_prepare_consts(pt_ctx* ctx, const pt_hparams* hp, hipStream_t stream) {
  if (ctx->prepared) {
    if (std::memcmp(&ctx->prepared_hp, hp, sizeof *hp) == 0) return PT_OK;
    if (ctx->stream_pending)
      return pt_fail(ctx, PT_ERR_STATE, "hyper-parameters changed while a streamed update of this step is in flight");
  }
  if (ctx->pend_reduce.active || ctx->pend_finalize) {
    const PtPendingReduce r = ctx->pend_reduce;
    const bool red = r.active;
    hipLaunchKernelGGL(k_reduce_finalize_prepare, dim3(1), dim3(NB_THREADS), 0, stream, red ? r.part : nullptr,
                       red ? r.flag : nullptr, red ? r.tile_begin : nullptr, red ? r.first : 0u, red ? r.n : 0u,
                       red ? r.per_chunk : 0u, ctx->d_chunk_sq, ctx->d_chunk_flag, ctx->C, ctx->d_state, *hp,
                       ctx->pend_finalize ? 1 : 0, 1, ctx->h_state_dev);
    PT_LAUNCH_CHECK(ctx, "k_reduce_finalize_prepare");
    ctx->pend_reduce.active = false;
    ctx->pend_finalize = false;
  } else {
    hipLaunchKernelGGL(k_prepare, dim3(1), dim3(1), 0, stream, ctx->d_state, *hp, ctx->h_state_dev);
    PT_LAUNCH_CHECK(ctx, "k_prepare");
  }
  PT_HIP(ctx, hipEventRecord(ctx->ev_scalar, stream));   // lets the host-side update read the scalars early
  ctx->prepared = true;
  ctx->prepared_hp = *hp;
  return PT_OK;
}

extern "C" int pt_chunk_grad_sqnorm(pt_ctx* ctx, const void* const* grad_chunks, uint32_t first_chunk,
                                    uint32_t n_chunks, int finalize, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (uint64_t(first_chunk) + n_chunks > ctx->C)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_grad_sqnorm: chunks [%u, %u) outside the context's %u chunks",
                   first_chunk, first_chunk + n_chunks, ctx->C);
  if (finalize < 0 || finalize > PT_FINALIZE_CARRY)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_grad_sqnorm: finalize must be 0, PT_FINALIZE_STRICT or PT_FINALIZE_CARRY");
  if (grad_chunks && n_chunks) {
    int rc = pt_table_bind(ctx, ROW_PACK, first_chunk, n_chunks, grad_chunks + first_chunk, false, st, nullptr);
    if (rc != PT_OK) return rc;
    dim3 grid(ctx->norm_blocks, n_chunks);
    if (ctx->grad_f32)
      hipLaunchKernelGGL(k_sqnorm_f32, grid, dim3(NB_THREADS), 0, st, pt_row(ctx, ROW_PACK), first_chunk,
                         ctx->S, ctx->d_state, ctx->d_norm_part, ctx->d_norm_flag);
    else if (ctx->dtype == PT_BF16)
      hipLaunchKernelGGL(k_sqnorm<PT_BF16>, grid, dim3(NB_THREADS), 0, st, pt_row(ctx, ROW_PACK), first_chunk,
                         ctx->S, ctx->d_state, ctx->d_norm_part, ctx->d_norm_flag);
    else
      hipLaunchKernelGGL(k_sqnorm<PT_FP16>, grid, dim3(NB_THREADS), 0, st, pt_row(ctx, ROW_PACK), first_chunk,
                         ctx->S, ctx->d_state, ctx->d_norm_part, ctx->d_norm_flag);
    PT_LAUNCH_CHECK(ctx, "k_sqnorm");
    int rc2 = pt_launch_chunk_reduce(ctx, ctx->d_norm_part, ctx->d_norm_flag, nullptr, first_chunk, n_chunks,
                                     ctx->norm_blocks, st, nullptr, 0, n_chunks);
    if (rc2 != PT_OK) return rc2;
    // a recompute covers the whole chunk: whatever plan packed it, its value is complete now
    for (uint32_t c = first_chunk; c < first_chunk + n_chunks; ++c) { ctx->chunk_fresh[c] = 1; ctx->chunk_packed_by[c] = 0; }
  }
  if (finalize) {
    if (ctx->stream_pending)
      return pt_fail(ctx, PT_ERR_STATE, "pt_chunk_grad_sqnorm: a streamed update is still open (its kernels read the "
                     "step's scalars); close the step with pt_step_end first");
    if (finalize != PT_FINALIZE_CARRY) {
      for (uint32_t c = 0; c < ctx->C; ++c)
        if (!ctx->chunk_fresh[c])
          return pt_fail(ctx, PT_ERR_STATE, "pt_chunk_grad_sqnorm: chunk %u has no sum of squares from this step (nothing "
                         "packed, accumulated or recomputed for it since the last pt_step_end); its old value would enter "
                         "the norm - finalize with PT_FINALIZE_CARRY if that is meant", c);
    }
    // The sum over the chunks runs with the first call that needs it: the update (in the launch that
    // derives its constants), a read-back, or pt_step_end.
    ctx->pend_finalize = true;
    ctx->norm_finalized = true;
    ctx->prepared = false;
  }
  return PT_OK;
}

// ---- the norm for callers that cannot allocate -------------------------------------------------
// Same kernels and the same reduction order as pt_chunk_grad_sqnorm(grad_chunks, ..., finalize), but
// without a context: the block partials and per-chunk sums live in one file-scope device array
// instead of memory a context allocated, and the gradient chunks are addressed as one arena.

namespace {

constexpr uint32_t PT_STATIC_MAX_PARTIALS = 1u << 19;   // blocks of PT_NORM_BLOCK_ELEMS elements: 2^34 elements
constexpr uint32_t PT_STATIC_MAX_CHUNKS = 4096;
constexpr int PT_STATIC_MAX_DEVICES = 64;

struct PtStaticScratch {
  double part[PT_STATIC_MAX_PARTIALS];
  uint32_t flag[PT_STATIC_MAX_PARTIALS];
  double chunk_sq[PT_STATIC_MAX_CHUNKS];
  uint32_t chunk_flag[PT_STATIC_MAX_CHUNKS];
};

}  // namespace

// 6.05 MiB per GPU the library runs on, held until the process ends.  In host code this name is only a
// stand-in for the symbol: the device address comes from hipGetSymbolAddress (scratch_of_current_device).
static __device__ __align__(256) unsigned char scratch[sizeof(PtStaticScratch)];

namespace {

// As k_sqnorm, for chunks that lie back to back in one arena; the loss scale comes by value.
template <int DT>
__global__ void __launch_bounds__(NB_THREADS)
k_sqnorm_arena(const void* __restrict__ arena, uint64_t S, double loss_scale, double* __restrict__ part,
               uint32_t* __restrict__ flagout) {
  const uint32_t b = blockIdx.x, i = blockIdx.y;
  const PT_GLOBAL u32x4* base = (const PT_GLOBAL u32x4*)((uint64_t)(uintptr_t)arena + 2ull * S * i);
  double acc;
  uint32_t flag;
  sqnorm_block<DT>(base, S, b, 1.0 / loss_scale, acc, flag);
  if (threadIdx.x == 0) {
    size_t slot = size_t(i) * gridDim.x + b;
    part[slot] = acc;
    flagout[slot] = flag;
  }
}

// As k_finalize, into the caller's outputs.
__global__ void k_finalize_out(const double* __restrict__ chunk_sq, const uint32_t* __restrict__ chunk_flag,
                               uint32_t C, double* __restrict__ out_sq_norm, int32_t* __restrict__ out_found_inf) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double t = 0.0;
  uint32_t f = 0;
  for (uint32_t c = 0; c < C; ++c) { t += chunk_sq[c]; f |= chunk_flag[c]; }
  out_sq_norm[0] = t;
  out_sq_norm[1] = sqrt(t);
  *out_found_inf = f ? 1 : 0;
}

std::mutex g_scratch_mutex;
void* g_scratch_addr[PT_STATIC_MAX_DEVICES] = {};

}  // namespace

// Device address of `scratch` on the current device, looked up once per device (every GPU holds its
// own copy of the array at its own address).
int pt_static_scratch_setup(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return pt_fail(nullptr, PT_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= PT_STATIC_MAX_DEVICES)
    return pt_fail(nullptr, PT_ERR_UNSUPPORTED, "device %d: at most %d devices are supported", dev, PT_STATIC_MAX_DEVICES);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return pt_fail(nullptr, PT_ERR_HIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_addr[dev] = p;
  }
  if (out) *out = g_scratch_addr[dev];
  return PT_OK;
}

extern "C" int pt_chunk_grad_sqnorm_noalloc(const void* grad_arena, int dtype, uint64_t chunk_elems, uint32_t n_chunks,
                                            double loss_scale, double* out_sqnorm_norm, int32_t* out_found_inf,
                                            void* stream) {
  if (!grad_arena || !out_sqnorm_norm || !out_found_inf)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_chunk_grad_sqnorm_noalloc: NULL pointer");
  if (dtype != PT_BF16 && dtype != PT_FP16)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_chunk_grad_sqnorm_noalloc: dtype %d is neither PT_BF16 nor PT_FP16", dtype);
  if (chunk_elems == 0 || n_chunks == 0)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_chunk_grad_sqnorm_noalloc: chunk_elems and n_chunks must be > 0");
  if (chunk_elems % 8 != 0 || (reinterpret_cast<uintptr_t>(grad_arena) & 15u))
    return pt_fail(nullptr, PT_ERR_ALIGNMENT,
                   "pt_chunk_grad_sqnorm_noalloc: chunk_elems must be a multiple of 8 and the arena 16-byte aligned");
  if ((reinterpret_cast<uintptr_t>(out_sqnorm_norm) & 7u) || (reinterpret_cast<uintptr_t>(out_found_inf) & 3u))
    return pt_fail(nullptr, PT_ERR_ALIGNMENT, "pt_chunk_grad_sqnorm_noalloc: misaligned output pointer");
  if (!(loss_scale >= 1.0) || !(loss_scale <= 1.8446744073709552e19))
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_chunk_grad_sqnorm_noalloc: loss_scale must be in [1, 2^64]");
  const uint64_t blocks_per_chunk = (chunk_elems + PT_NORM_BLOCK_ELEMS - 1) / PT_NORM_BLOCK_ELEMS;
  if (n_chunks > PT_STATIC_MAX_CHUNKS || blocks_per_chunk * n_chunks > PT_STATIC_MAX_PARTIALS)
    return pt_fail(nullptr, PT_ERR_UNSUPPORTED,
                   "pt_chunk_grad_sqnorm_noalloc: %u chunks of %llu elements exceed the static scratch (at most %u chunks "
                   "and %u blocks of %u elements, i.e. 2^34 elements); use pt_chunk_grad_sqnorm with a context",
                   n_chunks, (unsigned long long)chunk_elems, PT_STATIC_MAX_CHUNKS, PT_STATIC_MAX_PARTIALS,
                   PT_NORM_BLOCK_ELEMS);
  void* base = nullptr;
  int rc = pt_static_scratch_setup(&base);
  if (rc != PT_OK) return rc;
  // every address below derives from the looked-up device address, never from the array's name
  PtStaticScratch* sc = static_cast<PtStaticScratch*>(base);
  hipStream_t st = (hipStream_t)stream;
  dim3 grid((uint32_t)blocks_per_chunk, n_chunks);
  // Nothing here has to start at zero: each launch writes every partial and per-chunk slot that the
  // next one reads (n_chunks * blocks_per_chunk partials, n_chunks sums), so stale contents of an
  // earlier, larger call are never read.
  if (dtype == PT_BF16)
    hipLaunchKernelGGL(k_sqnorm_arena<PT_BF16>, grid, dim3(NB_THREADS), 0, st, grad_arena, chunk_elems, loss_scale,
                       sc->part, sc->flag);
  else
    hipLaunchKernelGGL(k_sqnorm_arena<PT_FP16>, grid, dim3(NB_THREADS), 0, st, grad_arena, chunk_elems, loss_scale,
                       sc->part, sc->flag);
  if (hipGetLastError() != hipSuccess) return pt_fail(nullptr, PT_ERR_HIP, "pt_chunk_grad_sqnorm_noalloc: launch of k_sqnorm_arena failed");
  hipLaunchKernelGGL(k_chunk_reduce, dim3(n_chunks), dim3(NB_THREADS), 0, st, sc->part, sc->flag,
                     (const uint32_t*)nullptr, 0u, (uint32_t)blocks_per_chunk, sc->chunk_sq, sc->chunk_flag);
  if (hipGetLastError() != hipSuccess) return pt_fail(nullptr, PT_ERR_HIP, "pt_chunk_grad_sqnorm_noalloc: launch of k_chunk_reduce failed");
  hipLaunchKernelGGL(k_finalize_out, dim3(1), dim3(64), 0, st, sc->chunk_sq, sc->chunk_flag, n_chunks, out_sqnorm_norm,
                     out_found_inf);
  if (hipGetLastError() != hipSuccess) return pt_fail(nullptr, PT_ERR_HIP, "pt_chunk_grad_sqnorm_noalloc: launch of k_finalize_out failed");
  return PT_OK;
}
