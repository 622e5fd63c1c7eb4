// Host-side update of host-resident chunks: the paper's own placement of the update of
// non-persistent chunks ("CPU Adam" running concurrently with GPU work; Hierarchical Chunk
// Management for Model States; Appendix A.1, T_CPU_OPTIM).  Host threads walk the pinned
// master / momentum / variance arrays in place, so nothing but the 16-bit gradients and
// parameters ever needs to cross the CPU-GPU link.
//
// Same fp32 operation sequence as the device kernel, driven by the same nine fp32
// constants (read back from the device once per step), so host-updated and
// device-updated chunks are bit-identical.  The loop is plain scalar code that the
// compiler vectorises per x86 target (AVX-512 / AVX2 clones picked at load time).
#include "pt_common.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <thread>

#pragma clang fp contract(off)

namespace {

struct HostConsts { float b1, b2, omb1, omb2, decay, step_size, rsb2, eps, gm; };

inline float bf16_to_f32(uint16_t w) {
  uint32_t u = uint32_t(w) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

inline uint16_t f32_to_bf16(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x0040u);
  return uint16_t((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

inline float fp16_to_f32(uint16_t w) {
  _Float16 h;
  std::memcpy(&h, &w, 2);
  return float(h);
}

inline uint16_t f32_to_fp16(float x) {
  _Float16 h = _Float16(x);           // round to nearest even (the default rounding mode)
  uint16_t w;
  std::memcpy(&w, &h, 2);
  return w;
}

#define PT_HOST_UPDATE_BODY(DECODE, ENCODE)                                         \
  for (uint64_t i = 0; i < n; ++i) {                                               \
    float gg = DECODE(g[i]) * k.gm;                                                \
    float t1 = k.omb1 * gg;                                                        \
    float mn = std::fmaf(k.b1, m[i], t1);                                          \
    float t2 = k.omb2 * gg;                                                        \
    t2 = t2 * gg;                                                                  \
    float vn = std::fmaf(k.b2, v[i], t2);                                          \
    float d = std::fmaf(std::sqrt(vn), k.rsb2, k.eps);                             \
    float u = mn / d;                                                              \
    float t3 = w[i] * k.decay;                                                     \
    float wn = std::fmaf(-k.step_size, u, t3);                                     \
    m[i] = mn; v[i] = vn; w[i] = wn;                                               \
    p[i] = ENCODE(wn);                                                             \
  }

// x86 clones picked at load time; the device pass of the compiler only parses this host code
// and does not know function multiversioning, so it sees the plain declaration.
#if defined(__HIP_DEVICE_COMPILE__)
#define PT_HOST_CLONES
#else
#define PT_HOST_CLONES __attribute__((target_clones("arch=x86-64-v4", "arch=x86-64-v3", "default")))
#endif

PT_HOST_CLONES
void host_update_bf16(const HostConsts k, const uint16_t* __restrict__ g, float* __restrict__ w,
                      float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ p, uint64_t n) {
  PT_HOST_UPDATE_BODY(bf16_to_f32, f32_to_bf16)
}

inline float f32_identity(float x) { return x; }

// fp32 gradient chunks (accumulated micro-batches): the gradient is read as it is
PT_HOST_CLONES
void host_update_bf16_g32(const HostConsts k, const float* __restrict__ g, float* __restrict__ w,
                          float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ p, uint64_t n) {
  PT_HOST_UPDATE_BODY(f32_identity, f32_to_bf16)
}

PT_HOST_CLONES
void host_update_fp16_g32(const HostConsts k, const float* __restrict__ g, float* __restrict__ w,
                          float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ p, uint64_t n) {
  PT_HOST_UPDATE_BODY(f32_identity, f32_to_fp16)
}

PT_HOST_CLONES
void host_update_fp16(const HostConsts k, const uint16_t* __restrict__ g, float* __restrict__ w,
                      float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ p, uint64_t n) {
  PT_HOST_UPDATE_BODY(fp16_to_f32, f32_to_fp16)
}

constexpr uint64_t HOST_GRAIN = 1u << 18;   // elements one thread takes at a time

}  // namespace

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
  // ev_scalar was recorded right behind the scalar kernel of this step (pt_prepare_consts)
  PT_HIP(ctx, hipStreamWaitEvent(ctx->s_scalar, ctx->ev_scalar, 0));
  PT_HIP(ctx, hipMemcpyAsync(ctx->h_state, ctx->d_state, sizeof(PtDevState), hipMemcpyDeviceToHost, ctx->s_scalar));
  PT_HIP(ctx, hipStreamSynchronize(ctx->s_scalar));
  const PtDevState& hs = *ctx->h_state;
  if (hs.skip) return PT_OK;                     // skipped step: the host arrays stay as they are
  HostConsts k{hs.c[0], hs.c[1], hs.c[2], hs.c[3], hs.c[4], hs.c[5], hs.c[6], hs.c[7], hs.c[8]};

  const uint64_t S = ctx->S;
  const uint64_t grains_per_chunk = (S + HOST_GRAIN - 1) / HOST_GRAIN;
  const uint64_t total_grains = grains_per_chunk * n_chunks;
  std::atomic<uint64_t> next{0};
  const int dtype = ctx->dtype;
  const bool masked = !ctx->h_nd_begin.empty(), gf32 = ctx->grad_f32;
  const uint32_t* nd_begin = ctx->h_nd_begin.data();
  const uint64_t* nd_ranges = ctx->h_nd_ranges.data();
  auto worker = [&]() {
    for (;;) {
      const uint64_t gidx = next.fetch_add(1, std::memory_order_relaxed);
      if (gidx >= total_grains) return;
      const uint64_t c = gidx / grains_per_chunk, lo = (gidx % grains_per_chunk) * HOST_GRAIN;
      const uint64_t n = (lo + HOST_GRAIN <= S) ? HOST_GRAIN : S - lo;
      const uint16_t* g = static_cast<const uint16_t*>(h_grad[c]) + lo;       // 16-bit gradient chunks
      const float* g32 = static_cast<const float*>(h_grad[c]) + lo;          // fp32 gradient chunks
      uint16_t* p = static_cast<uint16_t*>(h_param16[c]) + lo;
      // runs of one decay factor: between and inside the chunk's no-decay ranges
      uint64_t pos = lo;
      const uint64_t end = lo + n;
      uint32_t r = masked ? nd_begin[first_chunk + c] : 0;
      const uint32_t r_end = masked ? nd_begin[first_chunk + c + 1] : 0;
      while (r < r_end && nd_ranges[2 * size_t(r) + 1] <= pos) ++r;
      while (pos < end) {
        uint64_t stop = end;
        HostConsts kk = k;
        if (r < r_end && nd_ranges[2 * size_t(r)] < end) {
          if (nd_ranges[2 * size_t(r)] > pos) stop = nd_ranges[2 * size_t(r)];          // decayed run up to the range
          else { kk.decay = 1.0f; stop = std::min<uint64_t>(end, nd_ranges[2 * size_t(r) + 1]); ++r; }
        }
        const uint64_t off = pos - lo, cnt = stop - pos;
        float* w_ = h_master[c] + pos; float* m_ = h_m[c] + pos; float* v_ = h_v[c] + pos;
        if (gf32) {
          if (dtype == PT_BF16) host_update_bf16_g32(kk, g32 + off, w_, m_, v_, p + off, cnt);
          else host_update_fp16_g32(kk, g32 + off, w_, m_, v_, p + off, cnt);
        } else {
          if (dtype == PT_BF16) host_update_bf16(kk, g + off, w_, m_, v_, p + off, cnt);
          else host_update_fp16(kk, g + off, w_, m_, v_, p + off, cnt);
        }
        pos = stop;
      }
    }
  };
  std::vector<std::thread> pool;
  const uint32_t extra = n_threads - 1;
  try {
    pool.reserve(extra);
    for (uint32_t t = 0; t < extra; ++t) pool.emplace_back(worker);
  } catch (...) {
    // could not start every thread: the shared work queue is drained by those that did start
  }
  worker();
  for (auto& th : pool) th.join();
  return PT_OK;
}
