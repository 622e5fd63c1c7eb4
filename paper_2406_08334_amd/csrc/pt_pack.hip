// Pack gradients into chunks (and the inverse copy), one block per tile of a
// precomputed work list, fused with the per-tile sum of squares and the
// non-finite scan.
//
// HBM-bound: 2 bytes read + 2 bytes written per element.  Tiles are cut in
// CHUNK space at multiples of the tile size (PT_PACK_TILE_ELEMS by default), so many tiny tensors and a few
// huge ones give equally sized blocks.  Words are moved as 16-bit integers,
// never through a float.  The 16-byte vector body is aligned on the destination;
// when source and destination are not congruent modulo 16 bytes the source side
// falls back to 16-bit loads (the transformer shapes used here are congruent).
#include "pt_common.h"

#include <hip/hip_fp16.h>

#include <algorithm>
#include <memory>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int PK_THREADS = PT_REDUCE_THREADS;

template <int DT>
__device__ __forceinline__ double word_sq(uint32_t w16, double inv_scale) {
  double x;
  if (DT == PT_BF16) {
    x = (double)__uint_as_float(w16 << 16);
  } else {
    __half_raw r; r.x = (unsigned short)w16;
    x = (double)__half2float(__half(r));
  }
  x *= inv_scale;
  return x * x;
}

template <int DT>
__device__ __forceinline__ uint32_t word_nonfinite(uint32_t w16) {
  constexpr uint32_t E = DT == PT_BF16 ? 0x7f80u : 0x7c00u;
  return (w16 & E) == E;
}

template <int DT>
__device__ __forceinline__ void accum_vec(const u32x4& q, double inv_scale, double& a0, double& a1,
                                          uint32_t& flag) {
  const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    a0 += word_sq<DT>(w[k] & 0xffffu, inv_scale);
    a1 += word_sq<DT>(w[k] >> 16, inv_scale);
    flag |= word_nonfinite<DT>(w[k] & 0xffffu) | word_nonfinite<DT>(w[k] >> 16);
  }
}

__device__ __forceinline__ u32x4 load_vec_unaligned16(const PT_GLOBAL uint16_t* s) {
  // eight 16-bit loads: the source is only 2-byte aligned relative to the destination
  u32x4 q;
  q.x = uint32_t(s[0]) | (uint32_t(s[1]) << 16);
  q.y = uint32_t(s[2]) | (uint32_t(s[3]) << 16);
  q.z = uint32_t(s[4]) | (uint32_t(s[5]) << 16);
  q.w = uint32_t(s[6]) | (uint32_t(s[7]) << 16);
  return q;
}

// DIR 0: tensor -> chunk with sum of squares and non-finite scan (pack).
// DIR 1: chunk -> tensor (unpack), no reduction.
template <int DT, int DIR>
__global__ void __launch_bounds__(PK_THREADS)
k_pack(const PtTile* __restrict__ tiles, const uint64_t* __restrict__ chunk_row,
       const PtDevState* __restrict__ st, double* __restrict__ tile_sq, uint32_t* __restrict__ tile_flag) {
  const PtTile t = tiles[blockIdx.x];
  // both sides are device (global) memory: typed so, to get global_* instead of flat_* accesses
  PT_GLOBAL uint16_t* chunk_side = (PT_GLOBAL uint16_t*)(chunk_row[t.chunk]) + t.chunk_off;
  PT_GLOBAL uint16_t* tensor_side = (PT_GLOBAL uint16_t*)(t.tensor_addr);
  const PT_GLOBAL uint16_t* src = DIR == 0 ? tensor_side : chunk_side;
  PT_GLOBAL uint16_t* dst = DIR == 0 ? chunk_side : tensor_side;
  const uint32_t len = t.len;

  // elements before the destination reaches a 16-byte boundary
  uint32_t head = uint32_t(((16u - (uint32_t((uintptr_t)dst) & 15u)) & 15u) >> 1);
  if (head > len) head = len;
  const uint32_t nvec = (len - head) / 8;
  const uint32_t tail0 = head + nvec * 8;

  const double inv_scale = DIR == 0 ? 1.0 / st->loss_scale : 1.0;
  double a0 = 0.0, a1 = 0.0;
  uint32_t flag = 0;

  // head and tail: at most 7 elements each, one lane per element
  if (threadIdx.x < head) {
    uint16_t w = src[threadIdx.x];
    dst[threadIdx.x] = w;
    if (DIR == 0) { a0 += word_sq<DT>(w, inv_scale); flag |= word_nonfinite<DT>(w); }
  }
  if (threadIdx.x >= 64 && threadIdx.x - 64 < len - tail0) {
    uint32_t e = tail0 + (threadIdx.x - 64);
    uint16_t w = src[e];
    dst[e] = w;
    if (DIR == 0) { a1 += word_sq<DT>(w, inv_scale); flag |= word_nonfinite<DT>(w); }
  }

  const PT_GLOBAL uint16_t* sb = src + head;
  PT_GLOBAL u32x4* db = (PT_GLOBAL u32x4*)(dst + head);
  if (((uintptr_t)sb & 15u) == 0) {
    const PT_GLOBAL u32x4* sv = (const PT_GLOBAL u32x4*)sb;
    uint32_t i = threadIdx.x;
    for (; i + 3 * PK_THREADS < nvec; i += 4 * PK_THREADS) {
      u32x4 q0 = __builtin_nontemporal_load(sv + i);
      u32x4 q1 = __builtin_nontemporal_load(sv + i + PK_THREADS);
      u32x4 q2 = __builtin_nontemporal_load(sv + i + 2 * PK_THREADS);
      u32x4 q3 = __builtin_nontemporal_load(sv + i + 3 * PK_THREADS);
      __builtin_nontemporal_store(q0, db + i);
      __builtin_nontemporal_store(q1, db + i + PK_THREADS);
      __builtin_nontemporal_store(q2, db + i + 2 * PK_THREADS);
      __builtin_nontemporal_store(q3, db + i + 3 * PK_THREADS);
      if (DIR == 0) {
        accum_vec<DT>(q0, inv_scale, a0, a1, flag);
        accum_vec<DT>(q1, inv_scale, a0, a1, flag);
        accum_vec<DT>(q2, inv_scale, a0, a1, flag);
        accum_vec<DT>(q3, inv_scale, a0, a1, flag);
      }
    }
    for (; i < nvec; i += PK_THREADS) {
      u32x4 q = __builtin_nontemporal_load(sv + i);
      __builtin_nontemporal_store(q, db + i);
      if (DIR == 0) accum_vec<DT>(q, inv_scale, a0, a1, flag);
    }
  } else {
    for (uint32_t i = threadIdx.x; i < nvec; i += PK_THREADS) {
      u32x4 q = load_vec_unaligned16(sb + size_t(i) * 8);
      db[i] = q;
      if (DIR == 0) accum_vec<DT>(q, inv_scale, a0, a1, flag);
    }
  }

  if (DIR == 0) {
    double acc = a0 + a1;
    pt_block_sum(acc, flag);
    if (threadIdx.x == 0) {
      tile_sq[blockIdx.x] = acc;
      tile_flag[blockIdx.x] = flag;
    }
  }
}

}  // namespace

// ---- plan ----------------------------------------------------------------------------------

static void plan_free(pt_pack_plan* p) {
  if (p->d_tiles) (void)hipFree(p->d_tiles);
  if (p->d_chunk_tile_begin) (void)hipFree(p->d_chunk_tile_begin);
  if (p->d_tile_sq) (void)hipFree(p->d_tile_sq);
  if (p->d_tile_flag) (void)hipFree(p->d_tile_flag);
}

static int plan_create(pt_ctx* ctx, const pt_segment* segs, uint32_t n_segs, pt_pack_plan** out);

extern "C" int pt_pack_plan_create(pt_ctx* ctx, const pt_segment* segs, uint32_t n_segs, pt_pack_plan** out) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (!out || (!segs && n_segs)) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_pack_plan_create: NULL argument");
  *out = nullptr;
  return pt_guarded(ctx, "pt_pack_plan_create", [&] { return plan_create(ctx, segs, n_segs, out); });
}

static int plan_create(pt_ctx* ctx, const pt_segment* segs, uint32_t n_segs, pt_pack_plan** out) {
  // validate: inside chunks, sources present and 2-byte aligned, no overlap inside a chunk
  std::vector<uint32_t> order(n_segs);
  for (uint32_t i = 0; i < n_segs; ++i) {
    const pt_segment& s = segs[i];
    if (!s.src) return pt_fail(ctx, PT_ERR_INVALID_ARG, "segment %u: src is NULL", i);
    if (reinterpret_cast<uintptr_t>(s.src) & 1u) return pt_fail(ctx, PT_ERR_ALIGNMENT, "segment %u: src is not 2-byte aligned", i);
    if (s.len == 0) return pt_fail(ctx, PT_ERR_INVALID_ARG, "segment %u: len is 0", i);
    if (s.chunk >= ctx->C) return pt_fail(ctx, PT_ERR_INVALID_ARG, "segment %u: chunk %u outside the context's %u chunks", i, s.chunk, ctx->C);
    if (s.chunk_off >= ctx->S || s.len > ctx->S - s.chunk_off)
      return pt_fail(ctx, PT_ERR_INVALID_ARG, "segment %u: [%llu, +%llu) overruns the chunk of %llu elements", i,
                     (unsigned long long)s.chunk_off, (unsigned long long)s.len, (unsigned long long)ctx->S);
    order[i] = i;
  }
  std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
    if (segs[a].chunk != segs[b].chunk) return segs[a].chunk < segs[b].chunk;
    return segs[a].chunk_off < segs[b].chunk_off;
  });
  for (uint32_t k = 1; k < n_segs; ++k) {
    const pt_segment& p = segs[order[k - 1]];
    const pt_segment& q = segs[order[k]];
    if (p.chunk == q.chunk && p.chunk_off + p.len > q.chunk_off)
      return pt_fail(ctx, PT_ERR_INVALID_ARG, "segments %u and %u overlap in chunk %u", order[k - 1], order[k], p.chunk);
  }
  // cut into tiles at multiples of the tile size in chunk space
  // With fp32 gradient chunks the plan feeds the accumulate kernel, which moves 2.5 times the
  // bytes per element: half the tile gives it the same short-lived workgroups (measured best).
  const uint64_t tile_elems = ctx->grad_f32 ? std::max<uint64_t>(1024, ctx->opt_pack_tile_elems / 2)
                                            : ctx->opt_pack_tile_elems;
  std::vector<PtTile> tiles;
  std::vector<uint32_t> begin(size_t(ctx->C) + 1, 0);
  uint64_t total = 0;
  for (uint32_t k = 0; k < n_segs; ++k) {
    const pt_segment& s = segs[order[k]];
    uint64_t done = 0;
    while (done < s.len) {
      uint64_t coff = s.chunk_off + done;
      uint64_t room = tile_elems - (coff % tile_elems);
      uint64_t run = std::min<uint64_t>(room, s.len - done);
      PtTile t;
      t.tensor_addr = uint64_t(reinterpret_cast<uintptr_t>(s.src)) + 2 * (s.src_off + done);
      t.chunk_off = coff; t.chunk = s.chunk; t.len = uint32_t(run);
      tiles.push_back(t);
      begin[s.chunk + 1] += 1;
      done += run;
    }
    total += s.len;
  }
  if (tiles.size() > 0x7fffffffull) return pt_fail(ctx, PT_ERR_UNSUPPORTED, "pt_pack_plan_create: too many tiles");
  for (uint32_t c = 0; c < ctx->C; ++c) begin[c + 1] += begin[c];

  pt_pack_plan* p = new (std::nothrow) pt_pack_plan();
  if (!p) return pt_fail(ctx, PT_ERR_NOMEM, "pt_pack_plan_create: out of host memory");
  std::unique_ptr<pt_pack_plan> hold(p);            // freed on every early return and on an exception
  p->ctx = ctx; p->n_tiles = uint32_t(tiles.size()); p->total_elems = total;
  p->id = ++ctx->plan_ids;
  for (uint32_t c = 0; c < ctx->C; ++c)
    if (begin[c + 1] > begin[c]) p->touched.push_back(c);
  auto bail = [&](hipError_t e, const char* what) {
    plan_free(p);
    p->d_tiles = nullptr; p->d_chunk_tile_begin = nullptr; p->d_tile_sq = nullptr; p->d_tile_flag = nullptr;
    return pt_fail(ctx, PT_ERR_HIP, "pt_pack_plan_create: %s failed: %s", what, hipGetErrorString(e));
  };
  hipError_t e;
  size_t nt = std::max<size_t>(tiles.size(), 1);
  if ((e = hipMalloc(&p->d_tiles, nt * sizeof(PtTile))) != hipSuccess) return bail(e, "hipMalloc(tiles)");
  if ((e = hipMalloc(&p->d_chunk_tile_begin, begin.size() * sizeof(uint32_t))) != hipSuccess) return bail(e, "hipMalloc(begin)");
  if ((e = hipMalloc(&p->d_tile_sq, nt * sizeof(double))) != hipSuccess) return bail(e, "hipMalloc(tile_sq)");
  if ((e = hipMalloc(&p->d_tile_flag, nt * sizeof(uint32_t))) != hipSuccess) return bail(e, "hipMalloc(tile_flag)");
  if (!tiles.empty() &&
      (e = hipMemcpy(p->d_tiles, tiles.data(), tiles.size() * sizeof(PtTile), hipMemcpyHostToDevice)) != hipSuccess)
    return bail(e, "hipMemcpy(tiles)");
  if ((e = hipMemcpy(p->d_chunk_tile_begin, begin.data(), begin.size() * sizeof(uint32_t), hipMemcpyHostToDevice)) != hipSuccess)
    return bail(e, "hipMemcpy(begin)");
  *out = hold.release();
  return PT_OK;
}

extern "C" int pt_pack_plan_destroy(pt_pack_plan* plan) {
  if (!plan) return PT_OK;
  // a reduction of this plan's partial sums that was put off runs now, before they are freed
  if (plan->ctx && plan->ctx->pend_reduce.active && plan->ctx->pend_reduce.plan == plan)
    (void)pt_flush_pending(plan->ctx, plan->ctx->pend_reduce.stream);
  (void)hipDeviceSynchronize();
  if (plan->ctx)      // a plan that no longer exists does not stand in another plan's way
    for (uint32_t c : plan->touched)
      if (plan->ctx->chunk_packed_by[c] == plan->id) plan->ctx->chunk_packed_by[c] = 0;
  plan_free(plan);
  delete plan;
  return PT_OK;
}

// ---- hot calls --------------------------------------------------------------------------------

template <int DIR>
static int run_pack(pt_ctx* ctx, const pt_pack_plan* plan, const void* const* chunks, int row, hipStream_t st,
                    const char* who) {
  if (!plan || !chunks) return pt_fail(ctx, PT_ERR_INVALID_ARG, "%s: NULL argument", who);
  if (plan->ctx != ctx) return pt_fail(ctx, PT_ERR_INVALID_ARG, "%s: plan belongs to another context", who);
  int rc = pt_table_bind(ctx, row, 0, ctx->C, chunks, true, st, nullptr);
  if (rc != PT_OK) return rc;
  if (plan->n_tiles == 0) return PT_OK;
  // every chunk the plan touches needs a pointer (NULL is legal only for untouched chunks)
  const uint64_t* h = ctx->h_table.data() + size_t(row) * ctx->table_cols;
  for (uint32_t c : plan->touched)
    if (!h[c]) return pt_fail(ctx, PT_ERR_INVALID_ARG, "%s: chunk %u is used by the plan but its pointer is NULL", who, c);
  if (DIR == 0) {
    // A chunk's sum of squares is the partial of the LAST plan that packed into it: a second plan on the same
    // chunk in one step would silently drop the first plan's share from the norm.
    for (uint32_t c : plan->touched)
      if (ctx->chunk_packed_by[c] && ctx->chunk_packed_by[c] != plan->id)
        return pt_fail(ctx, PT_ERR_STATE, "%s: chunk %u already holds the gradients of another plan of this step; its sum of "
                       "squares would be replaced, not added to - pack a chunk with one plan per step (or recompute the "
                       "norm from the chunks with pt_chunk_grad_sqnorm(grad_chunks, ...) before packing again)", who, c);
  }
  dim3 grid(plan->n_tiles);
  // The inverse copy has no arithmetic to pace it; measured on MI355X it runs 15 % faster with three
  // workgroups per compute unit than with the eight that fit (4.24 against 4.96 ms for 6.7e9 elements).
  // Unused dynamic LDS (52 KiB of the unit's 160) sets that limit.  Pack itself is indifferent to it.
  const size_t lds = DIR == 1 ? 53248 : 0;
  if (ctx->dtype == PT_BF16)
    hipLaunchKernelGGL((k_pack<PT_BF16, DIR>), grid, dim3(PK_THREADS), lds, st, plan->d_tiles, pt_row(ctx, row),
                       ctx->d_state, plan->d_tile_sq, plan->d_tile_flag);
  else
    hipLaunchKernelGGL((k_pack<PT_FP16, DIR>), grid, dim3(PK_THREADS), lds, st, plan->d_tiles, pt_row(ctx, row),
                       ctx->d_state, plan->d_tile_sq, plan->d_tile_flag);
  PT_LAUNCH_CHECK(ctx, who);
  if (DIR == 0) {
    rc = pt_launch_chunk_reduce(ctx, plan->d_tile_sq, plan->d_tile_flag, plan->d_chunk_tile_begin, 0, ctx->C, 0, st, plan,
                                plan->n_tiles, uint32_t(plan->touched.size()));
    if (rc != PT_OK) return rc;
    for (uint32_t c : plan->touched) { ctx->chunk_fresh[c] = 1; ctx->chunk_packed_by[c] = plan->id; }
  }
  return PT_OK;
}

extern "C" int pt_chunk_pack_grads(pt_ctx* ctx, const pt_pack_plan* plan, void* const* grad_chunks, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (ctx->grad_f32)
    return pt_fail(ctx, PT_ERR_STATE, "pt_chunk_pack_grads: this context holds fp32 gradient chunks; use pt_chunk_accum_grads");
  return run_pack<0>(ctx, plan, (const void* const*)grad_chunks, ROW_PACK, (hipStream_t)stream, "pt_chunk_pack_grads");
}

extern "C" int pt_chunk_unpack(pt_ctx* ctx, const pt_pack_plan* plan, const void* const* chunks, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  return run_pack<1>(ctx, plan, chunks, ROW_UNPACK, (hipStream_t)stream, "pt_chunk_unpack");
}
