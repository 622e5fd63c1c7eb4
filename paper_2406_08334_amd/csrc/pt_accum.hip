// Gradient accumulation over micro-batches: the 16-bit gradient tensors of one
// micro-batch are added into fp32 gradient chunks (or overwrite them, for the first
// micro-batch), over the same tile list as pack; on the last micro-batch the per-tile
// sum of squares and the non-finite scan of the ACCUMULATED values are taken on the way.
//
// HBM-bound: per element 2 bytes read + 4 written when overwriting, 6 read + 4 written
// when adding.  Work unit = 4 consecutive elements per lane: one 8-byte load on the tensor
// side, one 16-byte load and store on the chunk side, so that every wave instruction covers
// one contiguous span (512 B / 1 KiB); the body is aligned on the chunk side (16 bytes); a
// tensor side that is not congruent (8 bytes) falls back to 16-bit loads.
// Each element is one binary32 addition of the stored sum and the exactly decoded word.
#include "pt_common.h"

#include <hip/hip_fp16.h>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int AC_THREADS = PT_REDUCE_THREADS;

template <int DT>
__device__ __forceinline__ float word_to_f32(uint32_t w16) {
  if (DT == PT_BF16) {
    return __uint_as_float(w16 << 16);
  } else {
    __half_raw r; r.x = (unsigned short)w16;
    return __half2float(__half(r));
  }
}

__device__ __forceinline__ void take(float a, double inv_scale, double& sum, uint32_t& flag) {
  const double x = (double)a * inv_scale;
  sum = fma(x, x, sum);
  flag |= (__float_as_uint(a) & 0x7f800000u) == 0x7f800000u;
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// q: four 16-bit words; acc: the four sums they are added to (or that they replace)
template <int DT, bool OVERWRITE, bool NORM>
__device__ __forceinline__ void add4(const u32x2& q, f32x4& acc, double inv_scale, double& a0, double& a1,
                                     uint32_t& flag) {
  const float x[4] = {word_to_f32<DT>(q.x & 0xffffu), word_to_f32<DT>(q.x >> 16),
                      word_to_f32<DT>(q.y & 0xffffu), word_to_f32<DT>(q.y >> 16)};
#pragma unroll
  for (int k = 0; k < 4; ++k) acc[k] = OVERWRITE ? x[k] : acc[k] + x[k];
  if (NORM) {
    take(acc[0], inv_scale, a0, flag); take(acc[1], inv_scale, a1, flag);
    take(acc[2], inv_scale, a0, flag); take(acc[3], inv_scale, a1, flag);
  }
}

__device__ __forceinline__ u32x2 load4_unaligned(const PT_GLOBAL uint16_t* s) {
  u32x2 q;
  q.x = uint32_t(s[0]) | (uint32_t(s[1]) << 16);
  q.y = uint32_t(s[2]) | (uint32_t(s[3]) << 16);
  return q;
}

template <int DT, bool OVERWRITE, bool NORM>
__global__ void __launch_bounds__(AC_THREADS)
k_accum(const PtTile* __restrict__ tiles, const uint64_t* __restrict__ chunk_row,
        const PtDevState* __restrict__ st, double* __restrict__ tile_sq, uint32_t* __restrict__ tile_flag) {
  // Even workgroups walk the first half of the tile list (sorted by chunk), odd ones the second half:
  // the read-modify-write traffic of a moment then falls on two distant parts of the chunks.  Measured
  // on MI355X: 9 % faster when the two halves of the gradient chunks lie in different 96 GiB regions of
  // the memory, no slower when they do not.
  const uint32_t half = (gridDim.x + 1) >> 1;
  const uint32_t tidx = (blockIdx.x & 1u) ? half + (blockIdx.x >> 1) : (blockIdx.x >> 1);
  const PtTile t = tiles[tidx];
  PT_GLOBAL float* dst = (PT_GLOBAL float*)(chunk_row[t.chunk]) + t.chunk_off;
  const PT_GLOBAL uint16_t* src = (const PT_GLOBAL uint16_t*)(t.tensor_addr);
  const uint32_t len = t.len;

  // elements before the chunk side reaches a 16-byte boundary
  uint32_t head = uint32_t(((16u - (uint32_t((uintptr_t)dst) & 15u)) & 15u) >> 2);
  if (head > len) head = len;
  const uint32_t nvec = (len - head) / 4;
  const uint32_t tail0 = head + nvec * 4;

  const double inv_scale = NORM ? 1.0 / st->loss_scale : 1.0;
  double a0 = 0.0, a1 = 0.0;
  uint32_t flag = 0;

  // head and tail: at most 3 elements each, one lane per element
  if (threadIdx.x < head) {
    const float x = word_to_f32<DT>(src[threadIdx.x]);
    const float a = OVERWRITE ? x : dst[threadIdx.x] + x;
    dst[threadIdx.x] = a;
    if (NORM) take(a, inv_scale, a0, flag);
  }
  if (threadIdx.x >= 64 && threadIdx.x - 64 < len - tail0) {
    const uint32_t e = tail0 + (threadIdx.x - 64);
    const float x = word_to_f32<DT>(src[e]);
    const float a = OVERWRITE ? x : dst[e] + x;
    dst[e] = a;
    if (NORM) take(a, inv_scale, a1, flag);
  }

  const PT_GLOBAL uint16_t* sb = src + head;
  PT_GLOBAL f32x4* db = (PT_GLOBAL f32x4*)(dst + head);
  const bool src_aligned = ((uintptr_t)sb & 7u) == 0;
  const PT_GLOBAL u32x2* sv = (const PT_GLOBAL u32x2*)sb;
  uint32_t i = threadIdx.x;
  if (src_aligned) {
    constexpr int D = 4;               // units per lane in flight
    for (; i + (D - 1) * AC_THREADS < nvec; i += D * AC_THREADS) {
      u32x2 q[D];
      f32x4 a[D];
#pragma unroll
      for (int r = 0; r < D; ++r) {
        q[r] = __builtin_nontemporal_load(sv + i + r * AC_THREADS);
        if (OVERWRITE) a[r] = f32x4{};
        else a[r] = __builtin_nontemporal_load(db + i + r * AC_THREADS);
      }
#pragma unroll
      for (int r = 0; r < D; ++r) {
        add4<DT, OVERWRITE, NORM>(q[r], a[r], inv_scale, a0, a1, flag);
        __builtin_nontemporal_store(a[r], db + i + r * AC_THREADS);
      }
    }
  }
  for (; i < nvec; i += AC_THREADS) {
    u32x2 q = src_aligned ? sv[i] : load4_unaligned(sb + size_t(i) * 4);
    f32x4 a = {};
    if (!OVERWRITE) a = db[i];
    add4<DT, OVERWRITE, NORM>(q, a, inv_scale, a0, a1, flag);
    db[i] = a;
  }

  if (NORM) {
    double acc = a0 + a1;
    pt_block_sum(acc, flag);
    if (threadIdx.x == 0) {
      tile_sq[tidx] = acc;
      tile_flag[tidx] = flag;
    }
  }
}

typedef void (*accum_kernel_t)(const PtTile*, const uint64_t*, const PtDevState*, double*, uint32_t*);

template <int DT>
accum_kernel_t pick(bool overwrite, bool norm) {
  if (overwrite) return norm ? k_accum<DT, true, true> : k_accum<DT, true, false>;
  return norm ? k_accum<DT, false, true> : k_accum<DT, false, false>;
}

}  // namespace

extern "C" int pt_chunk_accum_grads(pt_ctx* ctx, const pt_pack_plan* plan, float* const* acc_chunks, int overwrite,
                                    int take_norm, void* stream) {
  if (!ctx) return PT_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (!plan || !acc_chunks) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_accum_grads: NULL argument");
  if (plan->ctx != ctx) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_accum_grads: plan belongs to another context");
  if (!ctx->grad_f32)
    return pt_fail(ctx, PT_ERR_STATE, "pt_chunk_accum_grads: the context holds 16-bit gradient chunks (set option grad_fp32)");
  int rc = pt_table_bind(ctx, ROW_PACK, 0, ctx->C, (const void* const*)acc_chunks, true, st, nullptr);
  if (rc != PT_OK) return rc;
  if (plan->n_tiles == 0) return PT_OK;
  const uint64_t* h = ctx->h_table.data() + size_t(ROW_PACK) * ctx->table_cols;
  for (uint32_t c : plan->touched)
    if (!h[c]) return pt_fail(ctx, PT_ERR_INVALID_ARG, "pt_chunk_accum_grads: chunk %u is used by the plan but its pointer is NULL", c);
  accum_kernel_t kern = ctx->dtype == PT_BF16 ? pick<PT_BF16>(overwrite != 0, take_norm != 0)
                                              : pick<PT_FP16>(overwrite != 0, take_norm != 0);
  hipLaunchKernelGGL(kern, dim3(plan->n_tiles), dim3(AC_THREADS), 0, st, plan->d_tiles, pt_row(ctx, ROW_PACK),
                     ctx->d_state, plan->d_tile_sq, plan->d_tile_flag);
  PT_LAUNCH_CHECK(ctx, "k_accum");
  if (take_norm) {
    rc = pt_launch_chunk_reduce(ctx, plan->d_tile_sq, plan->d_tile_flag, plan->d_chunk_tile_begin, 0, ctx->C, 0, st, plan,
                                plan->n_tiles, uint32_t(plan->touched.size()));
    if (rc != PT_OK) return rc;
    for (uint32_t c : plan->touched) ctx->chunk_fresh[c] = 1;
  }
  return PT_OK;
}
