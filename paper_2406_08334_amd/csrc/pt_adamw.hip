// Fused mixed-precision AdamW over chunks: one launch covers every chunk of a
// range through the context's device pointer table.
//
// HBM-bound: per element 14 bytes read (g16, w, m, v) and 14 written (w, m, v,
// p16); 16 read with fp32 gradient chunks, and 2 or 4 more written when the gradients are
// zeroed on the way out.  Work unit = 4 consecutive elements per lane: one 16-byte access per fp32
// array and one 8-byte access per 16-bit array, so that every wave instruction
// touches one contiguous 1 KiB (fp32) or 512 B (16-bit) span.  UNROLL units per
// lane are loaded before the first is used, to keep enough bytes in flight.
// Arithmetic: the fp32 operation sequence below with correctly rounded *, fma,
// sqrt and / (this file is compiled with contraction off and without fast-math).
#include "pt_common.h"

#include <hip/hip_fp16.h>

#pragma clang fp contract(off)

namespace {

// workgroup size of the update kernel: 512 (default; measured 0.6-1.4 % faster than 256 on MI355X) or 256

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
// Chunk arrays are device (global) memory: typed as such so that loads and stores are
// global_* instructions instead of flat_* ones.
typedef PT_GLOBAL f32x4* gf32x4_ptr;
typedef PT_GLOBAL u32x2* gu32x2_ptr;
typedef const PT_GLOBAL f32x4* cgf32x4_ptr;
typedef const PT_GLOBAL u32x2* cgu32x2_ptr;

// NT: non-temporal hints (every byte is touched once per step).
template <bool NT, class P>
__device__ __forceinline__ auto ld_stream(P p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT, class T, class P>
__device__ __forceinline__ void st_stream(T v, P p) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

template <int DT>
__device__ __forceinline__ float decode16(uint32_t w16) {
  if (DT == PT_BF16) {
    return __uint_as_float(w16 << 16);
  } else {
    __half_raw r; r.x = (unsigned short)w16;
    return __half2float(__half(r));
  }
}

template <int DT>
__device__ __forceinline__ uint32_t encode16(float x) {
  if (DT == PT_BF16) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;  // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;                    // round to nearest, ties to even
  } else {
    // The recast rounds the STORED fp32 master weight.  Without this barrier the compiler
    // folds the producing fma and the conversion into one mixed-precision fma that rounds
    // the exact result straight to fp16, which can differ from RNE16(RNE32(.)) by one ulp.
    asm volatile("" : "+v"(x));
    __half_raw r = __half_raw(__float2half_rn(x));
    return (uint32_t)r.x;
  }
}

struct Consts { float b1, b2, omb1, omb2, decay, step_size, rsb2, eps, gm; };

// Four gradient elements as they sit in a gradient chunk: four 16-bit words, or four floats
// when the chunk accumulates micro-batches in fp32.
template <bool GF32> struct GradUnit { typedef u32x2 vec; };
template <> struct GradUnit<true> { typedef f32x4 vec; };

template <int DT, bool GF32>
__device__ __forceinline__ void decode_unit(const typename GradUnit<GF32>::vec& q, float (&g)[4]) {
  if constexpr (GF32) {
    g[0] = q[0]; g[1] = q[1]; g[2] = q[2]; g[3] = q[3];
  } else {
    g[0] = decode16<DT>(q.x & 0xffffu); g[1] = decode16<DT>(q.x >> 16);
    g[2] = decode16<DT>(q.y & 0xffffu); g[3] = decode16<DT>(q.y >> 16);
  }
}

// dk: decay factor of each of the four elements (k.decay, or 1 for elements kept out of the decay)
template <int DT, bool GF32>
__device__ __forceinline__ void update_unit(const Consts& k, const float (&dk)[4],
                                            const typename GradUnit<GF32>::vec& gq, f32x4& w, f32x4& m,
                                            f32x4& v, u32x2& p2) {
  float gv[4];
  decode_unit<DT, GF32>(gq, gv);
  uint32_t pw[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    // one correctly rounded binary32 operation per line; contraction is off for this file
    float g = gv[j] * k.gm;
    float t1 = k.omb1 * g;
    float mn = __builtin_fmaf(k.b1, m[j], t1);
    float t2 = k.omb2 * g;
    t2 = t2 * g;
    float vn = __builtin_fmaf(k.b2, v[j], t2);
    float d = __builtin_fmaf(__builtin_sqrtf(vn), k.rsb2, k.eps);
    float u = mn / d;
    float t3 = w[j] * dk[j];
    float wn = __builtin_fmaf(-k.step_size, u, t3);
    m[j] = mn; v[j] = vn; w[j] = wn;
    pw[j] = encode16<DT>(wn);
  }
  p2.x = pw[0] | (pw[1] << 16);
  p2.y = pw[2] | (pw[3] << 16);
}

// One flat index space of tiles (256 x UNROLL units of 4 elements) over all chunks of
// the launch: tile T belongs to chunk T / tiles_per_chunk.  Block b takes tiles
// b, b + gridDim.x, ...  With the default grid (a third of the tiles) a block's two or three
// tiles lie a third of the launch apart, in different chunks, so the five base pointers are
// re-read from the table for nearly every tile (five uniform loads against 28 KiB or more of
// traffic per tile); a small grid keeps consecutive tiles in one chunk and skips the re-read.
//
// MASKED: some element ranges of some chunks are kept out of the weight decay (sorted,
// disjoint ranges per chunk: nd_begin[c] .. nd_begin[c+1] index pairs (lo, hi) in nd_ranges).
// A tile that no range touches, or that lies inside one range, runs the same vector path with
// one decay factor; only tiles cut by a range edge take the element-wise path.
//
// GF32: the gradient chunks hold fp32 (accumulated micro-batches) instead of 16-bit words.
// zero_grads: every gradient element is overwritten with zero once it has been read (for
// callers whose backward pass adds into the chunk); a skipped step zeroes them as well (store-only
// pass), so that the non-finite value that caused the skip does not stay in the sums.
template <int AW_THREADS, int DT, int UNROLL, bool NT, bool MASKED, bool GF32>
__global__ void __launch_bounds__(AW_THREADS)
k_adamw(const uint64_t* __restrict__ table, uint32_t table_cols, uint32_t first_col, uint32_t n_cols,
        uint64_t S, uint32_t tiles_per_chunk, const PtDevState* __restrict__ st, int recast_on_skip,
        const uint32_t* __restrict__ nd_begin, const uint64_t* __restrict__ nd_ranges, uint32_t mask_chunk0,
        int zero_grads) {
  typedef typename GradUnit<GF32>::vec gvec;
  typedef PT_GLOBAL gvec* g_ptr;
  constexpr uint32_t TILE_UNITS = AW_THREADS * UNROLL;
  const gvec gzero = {};
  const uint64_t units = S / 4;
  const uint32_t total_tiles = tiles_per_chunk * n_cols;
  if (st->skip) {
    // Skipped step: nothing changes.  A chunk buffer of the streamed path is offloaded in
    // full afterwards and its param16 array was never uploaded, so it is refilled from the
    // untouched master weights (param16 == RNE(master) is the invariant of every update).
    if (recast_on_skip) {
      for (uint32_t T = blockIdx.x; T < total_tiles; T += gridDim.x) {
        const uint32_t ci = T / tiles_per_chunk, tile = T - ci * tiles_per_chunk;
        cgf32x4_ptr wq = (cgf32x4_ptr)(table[size_t(ROW_MASTER) * table_cols + first_col + ci]);
        gu32x2_ptr pq = (gu32x2_ptr)(table[size_t(ROW_P16) * table_cols + first_col + ci]);
        const uint64_t u_end = min(units, (uint64_t(tile) + 1) * TILE_UNITS);
        for (uint64_t u = uint64_t(tile) * TILE_UNITS + threadIdx.x; u < u_end; u += AW_THREADS) {
          f32x4 w = wq[u];
          u32x2 p;
          p.x = encode16<DT>(w[0]) | (encode16<DT>(w[1]) << 16);
          p.y = encode16<DT>(w[2]) | (encode16<DT>(w[3]) << 16);
          pq[u] = p;
        }
      }
    }
    // The gradients are zeroed on a skipped step too: a caller whose backward pass ADDS into the
    // chunks would otherwise carry the inf/NaN that caused the skip into every later sum.
    if (zero_grads) {
      for (uint32_t T = blockIdx.x; T < total_tiles; T += gridDim.x) {
        const uint32_t ci = T / tiles_per_chunk, tile = T - ci * tiles_per_chunk;
        g_ptr gq = (g_ptr)(table[size_t(ROW_GRAD) * table_cols + first_col + ci]);
        const uint64_t u_end = min(units, (uint64_t(tile) + 1) * TILE_UNITS);
        for (uint64_t u = uint64_t(tile) * TILE_UNITS + threadIdx.x; u < u_end; u += AW_THREADS)
          st_stream<NT>(gzero, gq + u);
      }
    }
    return;
  }
  Consts k;
  k.b1 = st->c[0]; k.b2 = st->c[1]; k.omb1 = st->c[2]; k.omb2 = st->c[3]; k.decay = st->c[4];
  k.step_size = st->c[5]; k.rsb2 = st->c[6]; k.eps = st->c[7]; k.gm = st->c[8];

  uint32_t cur = 0xffffffffu;
  g_ptr gp = nullptr;
  gf32x4_ptr wp = nullptr, mp = nullptr, vp = nullptr;
  gu32x2_ptr pp = nullptr;
  for (uint32_t T = blockIdx.x; T < total_tiles; T += gridDim.x) {
    const uint32_t ci = T / tiles_per_chunk, tile = T - ci * tiles_per_chunk;
    if (ci != cur) {
      cur = ci;
      const uint32_t col = first_col + ci;
      gp = (g_ptr)(table[size_t(ROW_GRAD) * table_cols + col]);
      wp = (gf32x4_ptr)(table[size_t(ROW_MASTER) * table_cols + col]);
      mp = (gf32x4_ptr)(table[size_t(ROW_M) * table_cols + col]);
      vp = (gf32x4_ptr)(table[size_t(ROW_V) * table_cols + col]);
      pp = (gu32x2_ptr)(table[size_t(ROW_P16) * table_cols + col]);
    }
    const uint64_t u0 = uint64_t(tile) * TILE_UNITS + threadIdx.x;
    float dtile = k.decay;            // decay factor of the whole tile, when it has one
    bool cut = false;                 // a range edge falls inside this tile
    uint32_t r0 = 0, r1 = 0;          // ranges of this chunk from the first one that ends after the tile start
    if (MASKED) {
      const uint32_t c = mask_chunk0 + ci;
      r1 = nd_begin[c + 1];
      uint32_t lo = nd_begin[c], hi = r1;
      const uint64_t e0 = uint64_t(tile) * TILE_UNITS * 4, e1 = e0 + uint64_t(TILE_UNITS) * 4;
      while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (nd_ranges[2 * size_t(mid) + 1] <= e0) lo = mid + 1; else hi = mid;
      }
      r0 = lo;
      if (r0 < r1 && nd_ranges[2 * size_t(r0)] < e1) {
        if (nd_ranges[2 * size_t(r0)] <= e0 && nd_ranges[2 * size_t(r0) + 1] >= e1) dtile = 1.0f;
        else cut = true;
      }
    }
    if (MASKED && cut) {
      // element-wise decay factors; also covers a ragged last tile
      const uint64_t u_end = min(units, (uint64_t(tile) + 1) * TILE_UNITS);
      for (uint64_t u = u0; u < u_end; u += AW_THREADS) {
        float dk[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint64_t e = 4 * u + j;
          float d = k.decay;
          for (uint32_t r = r0; r < r1 && nd_ranges[2 * size_t(r)] <= e; ++r)
            if (e < nd_ranges[2 * size_t(r) + 1]) d = 1.0f;
          dk[j] = d;
        }
        gvec g = gp[u]; f32x4 w = wp[u], m = mp[u], v = vp[u]; u32x2 p;
        update_unit<DT, GF32>(k, dk, g, w, m, v, p);
        wp[u] = w; mp[u] = m; vp[u] = v; pp[u] = p;
        if (zero_grads) gp[u] = gzero;
      }
      continue;
    }
    const float dk[4] = {dtile, dtile, dtile, dtile};
    if ((uint64_t(tile) + 1) * TILE_UNITS <= units) {
      gvec g[UNROLL]; f32x4 w[UNROLL], m[UNROLL], v[UNROLL];
#pragma unroll
      for (int r = 0; r < UNROLL; ++r) {
        const uint64_t u = u0 + uint64_t(r) * AW_THREADS;
        g[r] = ld_stream<NT>(gp + u);
        w[r] = ld_stream<NT>(wp + u);
        m[r] = ld_stream<NT>(mp + u);
        v[r] = ld_stream<NT>(vp + u);
      }
#pragma unroll
      for (int r = 0; r < UNROLL; ++r) {
        const uint64_t u = u0 + uint64_t(r) * AW_THREADS;
        u32x2 p;
        update_unit<DT, GF32>(k, dk, g[r], w[r], m[r], v[r], p);
        st_stream<NT>(w[r], wp + u);
        st_stream<NT>(m[r], mp + u);
        st_stream<NT>(v[r], vp + u);
        st_stream<NT>(p, pp + u);
        if (zero_grads) st_stream<NT>(gzero, gp + u);
      }
    } else {
      // ragged last tile of a chunk
      for (uint64_t u = u0; u < units; u += AW_THREADS) {
        gvec g = gp[u]; f32x4 w = wp[u], m = mp[u], v = vp[u]; u32x2 p;
        update_unit<DT, GF32>(k, dk, g, w, m, v, p);
        wp[u] = w; mp[u] = m; vp[u] = v; pp[u] = p;
        if (zero_grads) gp[u] = gzero;
      }
    }
  }
}

// Measurement aid: the update's memory access pattern with the arithmetic taken out.  Same tiles, same
// block-to-tile mapping, the same four loads and four stores per unit with the same hints; master,
// momentum and variance are stored back as loaded and param16 is re-derived from the master weight
// (which is what it holds already), so the state does not change.  What this kernel attains is what the
// memory system gives this mix of streams on this placement; the update itself cannot be faster.
template <int AW_THREADS, int DT, int UNROLL, bool NT>
__global__ void __launch_bounds__(AW_THREADS)
k_adamw_pattern(const uint64_t* __restrict__ table, uint32_t table_cols, uint32_t first_col, uint32_t n_cols,
                uint64_t S, uint32_t tiles_per_chunk, uint32_t* __restrict__ sink) {
  constexpr uint32_t TILE_UNITS = AW_THREADS * UNROLL;
  const uint64_t units = S / 4;
  const uint32_t total_tiles = tiles_per_chunk * n_cols;
  uint32_t keep = 0;
  for (uint32_t T = blockIdx.x; T < total_tiles; T += gridDim.x) {
    const uint32_t ci = T / tiles_per_chunk, tile = T - ci * tiles_per_chunk;
    const uint32_t col = first_col + ci;
    cgu32x2_ptr gp = (cgu32x2_ptr)(table[size_t(ROW_GRAD) * table_cols + col]);
    gf32x4_ptr wp = (gf32x4_ptr)(table[size_t(ROW_MASTER) * table_cols + col]);
    gf32x4_ptr mp = (gf32x4_ptr)(table[size_t(ROW_M) * table_cols + col]);
    gf32x4_ptr vp = (gf32x4_ptr)(table[size_t(ROW_V) * table_cols + col]);
    gu32x2_ptr pp = (gu32x2_ptr)(table[size_t(ROW_P16) * table_cols + col]);
    const uint64_t u0 = uint64_t(tile) * TILE_UNITS + threadIdx.x;
    if ((uint64_t(tile) + 1) * TILE_UNITS > units) continue;      // ragged last tiles are left out (a few KiB per chunk)
    u32x2 g[UNROLL]; f32x4 w[UNROLL], m[UNROLL], v[UNROLL];
#pragma unroll
    for (int r = 0; r < UNROLL; ++r) {
      const uint64_t u = u0 + uint64_t(r) * AW_THREADS;
      g[r] = ld_stream<NT>(gp + u);
      w[r] = ld_stream<NT>(wp + u);
      m[r] = ld_stream<NT>(mp + u);
      v[r] = ld_stream<NT>(vp + u);
    }
#pragma unroll
    for (int r = 0; r < UNROLL; ++r) {
      const uint64_t u = u0 + uint64_t(r) * AW_THREADS;
      // opaque to the optimiser, so that the stores of unchanged values are not dropped
      asm volatile("" : "+v"(w[r]), "+v"(m[r]), "+v"(v[r]));
      u32x2 p;
      p.x = encode16<DT>(w[r][0]) | (encode16<DT>(w[r][1]) << 16);
      p.y = encode16<DT>(w[r][2]) | (encode16<DT>(w[r][3]) << 16);
      keep ^= g[r].x ^ g[r].y;
      st_stream<NT>(w[r], wp + u);
      st_stream<NT>(m[r], mp + u);
      st_stream<NT>(v[r], vp + u);
      st_stream<NT>(p, pp + u);
    }
  }
  if (keep == 0x9e3779b9u && sink) *sink = keep;      // keeps the gradient loads alive; practically never taken
}

typedef void (*adamw_kernel_t)(const uint64_t*, uint32_t, uint32_t, uint32_t, uint64_t, uint32_t,
                               const PtDevState*, int, const uint32_t*, const uint64_t*, uint32_t, int);

template <int TH, int DT, bool MASKED, bool GF32>
adamw_kernel_t pick_unroll(uint32_t unroll, bool nt) {
  switch (unroll) {
    case 1: return nt ? k_adamw<TH, DT, 1, true, MASKED, GF32> : k_adamw<TH, DT, 1, false, MASKED, GF32>;
    case 2: return nt ? k_adamw<TH, DT, 2, true, MASKED, GF32> : k_adamw<TH, DT, 2, false, MASKED, GF32>;
    case 8: return nt ? k_adamw<TH, DT, 8, true, MASKED, GF32> : k_adamw<TH, DT, 8, false, MASKED, GF32>;
    default: return nt ? k_adamw<TH, DT, 4, true, MASKED, GF32> : k_adamw<TH, DT, 4, false, MASKED, GF32>;
  }
}

template <int TH, int DT>
adamw_kernel_t pick_flags(uint32_t unroll, bool nt, bool masked, bool gf32) {
  if (masked) return gf32 ? pick_unroll<TH, DT, true, true>(unroll, nt) : pick_unroll<TH, DT, true, false>(unroll, nt);
  return gf32 ? pick_unroll<TH, DT, false, true>(unroll, nt) : pick_unroll<TH, DT, false, false>(unroll, nt);
}

template <int DT>
adamw_kernel_t pick_kernel(uint32_t threads, uint32_t unroll, bool nt, bool masked, bool gf32) {
  return threads == 256 ? pick_flags<256, DT>(unroll, nt, masked, gf32) : pick_flags<512, DT>(unroll, nt, masked, gf32);
}

typedef void (*pattern_kernel_t)(const uint64_t*, uint32_t, uint32_t, uint32_t, uint64_t, uint32_t, uint32_t*);

template <int TH, int DT>
pattern_kernel_t pick_pattern_unroll(uint32_t unroll, bool nt) {
  switch (unroll) {
    case 1: return nt ? k_adamw_pattern<TH, DT, 1, true> : k_adamw_pattern<TH, DT, 1, false>;
    case 2: return nt ? k_adamw_pattern<TH, DT, 2, true> : k_adamw_pattern<TH, DT, 2, false>;
    case 8: return nt ? k_adamw_pattern<TH, DT, 8, true> : k_adamw_pattern<TH, DT, 8, false>;
    default: return nt ? k_adamw_pattern<TH, DT, 4, true> : k_adamw_pattern<TH, DT, 4, false>;
  }
}

template <int DT>
pattern_kernel_t pick_pattern(uint32_t threads, uint32_t unroll, bool nt) {
  return threads == 256 ? pick_pattern_unroll<256, DT>(unroll, nt) : pick_pattern_unroll<512, DT>(unroll, nt);
}

}  // namespace

int pt_launch_adamw(pt_ctx* ctx, uint32_t first_col, uint32_t n_cols, hipStream_t stream, bool recast_on_skip,
                    uint32_t mask_chunk0, bool zero_grads) {
  if (n_cols == 0) return PT_OK;
  const uint32_t unroll = ctx->opt_adamw_unroll;
  const uint64_t units = ctx->S / 4;
  const uint32_t threads = pt_adamw_threads(ctx, n_cols);
  const uint64_t tile_units = uint64_t(threads) * unroll;
  const uint64_t tpc = (units + tile_units - 1) / tile_units;
  if (tpc * n_cols > 0x7fffffffull)
    return pt_fail(ctx, PT_ERR_UNSUPPORTED, "update launch of %u chunks exceeds 2^31 tiles", n_cols);
  const uint32_t total = uint32_t(tpc) * n_cols;
  // Grid: measured on MI355X, many short-lived workgroups (about three tiles each) keep the
  // memory system a few percent busier than a grid sized to what stays resident.
  uint32_t want = ctx->opt_adamw_grid > 0 ? ctx->opt_adamw_grid : (total + 2) / 3;
  if (ctx->opt_adamw_grid == 0 && want < PT_ADAMW_MIN_GRID) want = PT_ADAMW_MIN_GRID;
  dim3 grid(want < total ? want : total);
  const bool nt = pt_adamw_nt(ctx, n_cols), masked = ctx->d_nd_begin != nullptr;
  adamw_kernel_t kern = ctx->dtype == PT_BF16 ? pick_kernel<PT_BF16>(threads, unroll, nt, masked, ctx->grad_f32)
                                              : pick_kernel<PT_FP16>(threads, unroll, nt, masked, ctx->grad_f32);
  hipLaunchKernelGGL(kern, grid, dim3(threads), 0, stream, ctx->d_table, ctx->table_cols, first_col, n_cols,
                     ctx->S, uint32_t(tpc), ctx->d_state, recast_on_skip ? 1 : 0, ctx->d_nd_begin, ctx->d_nd_ranges,
                     mask_chunk0, zero_grads ? 1 : 0);
  PT_LAUNCH_CHECK(ctx, "k_adamw");
  return PT_OK;
}

extern "C" int pt_chunk_adamw_step(pt_ctx* ctx, const pt_hparams* hp, uint32_t first_chunk, uint32_t n_chunks,
                                   const void* const* grad, float* const* master, float* const* m,
                                   float* const* v, void* const* param16, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (!hp) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_adamw_step: hp is NULL");
  if (uint64_t(first_chunk) + n_chunks > ctx->C)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_adamw_step: chunks [%u, %u) outside the context's %u chunks",
                   first_chunk, first_chunk + n_chunks, ctx->C);
  if (n_chunks && (!grad || !master || !m || !v || !param16))
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_adamw_step: NULL pointer array");
  if (!ctx->norm_finalized)
    return pt_fail(ctx, PT_ERR_STATE, "pt_chunk_adamw_step: no finalized gradient norm in this step");
  if (n_chunks == 0) return PT_OK;
  int rc;
  if ((rc = pt_table_bind(ctx, ROW_GRAD, first_chunk, n_chunks, grad, false, st, nullptr)) != PT_OK) return rc;
  if ((rc = pt_table_bind(ctx, ROW_MASTER, first_chunk, n_chunks, (const void* const*)master, false, st, nullptr)) != PT_OK) return rc;
  if ((rc = pt_table_bind(ctx, ROW_M, first_chunk, n_chunks, (const void* const*)m, false, st, nullptr)) != PT_OK) return rc;
  if ((rc = pt_table_bind(ctx, ROW_V, first_chunk, n_chunks, (const void* const*)v, false, st, nullptr)) != PT_OK) return rc;
  if ((rc = pt_table_bind(ctx, ROW_P16, first_chunk, n_chunks, (const void* const*)param16, false, st, nullptr)) != PT_OK) return rc;
  if ((rc = pt_prepare_consts(ctx, hp, st)) != PT_OK) return rc;
  return pt_launch_adamw(ctx, first_chunk, n_chunks, st, false, first_chunk, ctx->opt_zero_grads != 0);
}

extern "C" int pt_calib_adamw_pattern(pt_ctx* ctx, uint32_t first_chunk, uint32_t n_chunks, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  if (uint64_t(first_chunk) + n_chunks > ctx->C)
    return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_calib_adamw_pattern: chunks [%u, %u) outside the context's %u chunks",
                   first_chunk, first_chunk + n_chunks, ctx->C);
  if (ctx->grad_f32 || ctx->d_nd_begin)
    return pt_fail(ctx, PT_ERR_UNSUPPORTED, "pt_calib_adamw_pattern: 16-bit gradient chunks without no-decay runs only");
  const uint64_t* h = ctx->h_table.data();
  for (uint32_t c = first_chunk; c < first_chunk + n_chunks; ++c)
    for (int row : {ROW_GRAD, ROW_MASTER, ROW_M, ROW_V, ROW_P16})
      if (!h[size_t(row) * ctx->table_cols + c])
        return pt_fail(ctx, PT_ERR_STATE, "pt_calib_adamw_pattern: chunk %u has not been through pt_chunk_adamw_step yet "
                       "(its pointers are not in the context's table)", c);
  if (n_chunks == 0) return PT_OK;
  const uint32_t unroll = ctx->opt_adamw_unroll;
  const uint32_t threads = pt_adamw_threads(ctx, n_chunks);
  const uint64_t units = ctx->S / 4, tile_units = uint64_t(threads) * unroll;
  const uint64_t tpc = (units + tile_units - 1) / tile_units;
  if (tpc * n_chunks > 0x7fffffffull) return pt_fail(ctx, PT_ERR_UNSUPPORTED, "pt_calib_adamw_pattern: more than 2^31 tiles");
  const uint32_t total = uint32_t(tpc) * n_chunks;
  uint32_t want = ctx->opt_adamw_grid > 0 ? ctx->opt_adamw_grid : (total + 2) / 3;      // as pt_launch_adamw
  if (ctx->opt_adamw_grid == 0 && want < PT_ADAMW_MIN_GRID) want = PT_ADAMW_MIN_GRID;
  dim3 grid(want < total ? want : total);
  const bool nt = pt_adamw_nt(ctx, n_chunks);
  pattern_kernel_t kern = ctx->dtype == PT_BF16 ? pick_pattern<PT_BF16>(threads, unroll, nt)
                                                : pick_pattern<PT_FP16>(threads, unroll, nt);
  hipLaunchKernelGGL(kern, grid, dim3(threads), 0, (hipStream_t)stream, ctx->d_table, ctx->table_cols, first_chunk,
                     n_chunks, ctx->S, uint32_t(tpc), (uint32_t*)nullptr);
  PT_LAUNCH_CHECK(ctx, "k_adamw_pattern");
  return PT_OK;
}
