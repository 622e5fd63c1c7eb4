// Host-side AdamW over chunks that live in host memory: the update loops, the grain queue and
// the persistent thread pool.  Pure host C++ (no HIP): pt_host.hip drives it with the constants
// read back from the device, and the CPU-only sanitizer harness (tests/pins) drives it on plain
// arrays.
//
// The paper updates non-persistent chunks with a CPU Adam that runs concurrently with GPU work
// ("Hierarchical Chunk Management for Model States"; Appendix A.1, T_CPU_OPTIM).  Same fp32
// operation sequence as the device kernel, written as plain scalar loops that the compiler
// vectorises per x86 target (AVX-512 / AVX2 clones picked at load time).
#pragma once

#include <algorithm>
#include <atomic>
#include <cmath>
#include <condition_variable>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <thread>
#include <vector>

#if defined(__clang__)
#pragma clang fp contract(off)
#endif

namespace pt_host {

struct Consts { float b1, b2, omb1, omb2, decay, step_size, rsb2, eps, gm; };

static inline float bf16_to_f32(uint16_t w) {
  uint32_t u = uint32_t(w) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

static inline uint16_t f32_to_bf16(float x) {
  uint32_t u;
  std::memcpy(&u, &x, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return uint16_t((u >> 16) | 0x0040u);
  return uint16_t((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

static inline float fp16_to_f32(uint16_t w) {
  _Float16 h;
  std::memcpy(&h, &w, 2);
  return float(h);
}

static inline uint16_t f32_to_fp16(float x) {
  _Float16 h = _Float16(x);           // round to nearest even (the default rounding mode)
  uint16_t w;
  std::memcpy(&w, &h, 2);
  return w;
}

static inline float f32_identity(float x) { return x; }

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

// x86 clones picked at load time; a device pass of a HIP compiler only parses this host code
// and does not know function multiversioning, so it sees the plain declaration.
#if defined(__HIP_DEVICE_COMPILE__) || defined(PT_HOST_NO_CLONES)
#define PT_HOST_CLONES
#else
#define PT_HOST_CLONES __attribute__((target_clones("arch=x86-64-v4", "arch=x86-64-v3", "default")))
#endif

PT_HOST_CLONES
static void update_bf16(const Consts k, const uint16_t* __restrict__ g, float* __restrict__ w,
                        float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ p, uint64_t n) {
  PT_HOST_UPDATE_BODY(bf16_to_f32, f32_to_bf16)
}

PT_HOST_CLONES
static void update_fp16(const Consts k, const uint16_t* __restrict__ g, float* __restrict__ w,
                        float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ p, uint64_t n) {
  PT_HOST_UPDATE_BODY(fp16_to_f32, f32_to_fp16)
}

// fp32 gradient chunks (accumulated micro-batches): the gradient is read as it is
PT_HOST_CLONES
static void update_bf16_g32(const Consts k, const float* __restrict__ g, float* __restrict__ w,
                            float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ p, uint64_t n) {
  PT_HOST_UPDATE_BODY(f32_identity, f32_to_bf16)
}

PT_HOST_CLONES
static void update_fp16_g32(const Consts k, const float* __restrict__ g, float* __restrict__ w,
                            float* __restrict__ m, float* __restrict__ v, uint16_t* __restrict__ p, uint64_t n) {
  PT_HOST_UPDATE_BODY(f32_identity, f32_to_fp16)
}

#undef PT_HOST_UPDATE_BODY

constexpr uint64_t GRAIN = 1u << 18;   // elements one thread takes at a time

// One call's work.  The chunks are cut into grains; threads take grains from a shared counter.
struct Job {
  Consts k{};
  int dtype_fp16 = 0;                   // 0: bf16 parameters / gradients, 1: fp16
  bool grad_f32 = false;                // gradient chunks hold fp32
  uint64_t S = 0;                       // elements per chunk
  uint32_t first_chunk = 0, n_chunks = 0;
  const void* const* h_grad = nullptr;  // n_chunks pointers each
  float* const* h_master = nullptr;
  float* const* h_m = nullptr;
  float* const* h_v = nullptr;
  void* const* h_param16 = nullptr;
  // element runs kept out of the weight decay: per chunk (absolute index) sorted disjoint
  // (lo, hi) pairs, nd_begin[c] .. nd_begin[c + 1]; nd_begin == NULL: none
  const uint32_t* nd_begin = nullptr;
  const uint64_t* nd_ranges = nullptr;
  std::atomic<uint64_t> next{0};
  uint64_t grains_per_chunk = 0, total_grains = 0;

  void prepare() {
    grains_per_chunk = (S + GRAIN - 1) / GRAIN;
    total_grains = grains_per_chunk * n_chunks;
    next.store(0, std::memory_order_relaxed);
  }
};

// Takes grains until none is left.  Every element belongs to exactly one grain, so no two threads
// ever touch the same element.
static inline void run_grains(Job& job) {
  const uint64_t S = job.S;
  for (;;) {
    const uint64_t gidx = job.next.fetch_add(1, std::memory_order_relaxed);
    if (gidx >= job.total_grains) return;
    const uint64_t c = gidx / job.grains_per_chunk, lo = (gidx % job.grains_per_chunk) * GRAIN;
    const uint64_t n = (lo + GRAIN <= S) ? GRAIN : S - lo;
    const uint16_t* g = static_cast<const uint16_t*>(job.h_grad[c]) + lo;       // 16-bit gradient chunks
    const float* g32 = static_cast<const float*>(job.h_grad[c]) + lo;          // fp32 gradient chunks
    uint16_t* p = static_cast<uint16_t*>(job.h_param16[c]) + lo;
    // runs of one decay factor: between and inside the chunk's no-decay ranges
    uint64_t pos = lo;
    const uint64_t end = lo + n;
    const bool masked = job.nd_begin != nullptr;
    uint32_t r = masked ? job.nd_begin[job.first_chunk + c] : 0;
    const uint32_t r_end = masked ? job.nd_begin[job.first_chunk + c + 1] : 0;
    const uint64_t* ranges = job.nd_ranges;
    while (r < r_end && ranges[2 * size_t(r) + 1] <= pos) ++r;
    while (pos < end) {
      uint64_t stop = end;
      Consts kk = job.k;
      if (r < r_end && ranges[2 * size_t(r)] < end) {
        if (ranges[2 * size_t(r)] > pos) stop = ranges[2 * size_t(r)];          // decayed run up to the range
        else { kk.decay = 1.0f; stop = std::min<uint64_t>(end, ranges[2 * size_t(r) + 1]); ++r; }
      }
      const uint64_t off = pos - lo, cnt = stop - pos;
      float* w_ = job.h_master[c] + pos; float* m_ = job.h_m[c] + pos; float* v_ = job.h_v[c] + pos;
      if (job.grad_f32) {
        if (!job.dtype_fp16) update_bf16_g32(kk, g32 + off, w_, m_, v_, p + off, cnt);
        else update_fp16_g32(kk, g32 + off, w_, m_, v_, p + off, cnt);
      } else {
        if (!job.dtype_fp16) update_bf16(kk, g + off, w_, m_, v_, p + off, cnt);
        else update_fp16(kk, g + off, w_, m_, v_, p + off, cnt);
      }
      pos = stop;
    }
  }
}

// Worker threads that outlive a call: they sleep on a condition variable between calls, so a step
// pays a wake-up instead of thread creation.  run() hands one Job to all workers, the caller works
// along, and run() returns when every worker has left the job.  One run() at a time.
class Pool {
 public:
  explicit Pool(uint32_t n_workers) {
    try {
      threads_.reserve(n_workers);
      for (uint32_t i = 0; i < n_workers; ++i) threads_.emplace_back([this] { worker(); });
    } catch (...) {
      // fewer threads than asked for: the grain queue is drained by those that did start
    }
  }
  Pool(const Pool&) = delete;
  Pool& operator=(const Pool&) = delete;
  ~Pool() {
    {
      std::lock_guard<std::mutex> lk(mu_);
      stop_ = true;
    }
    cv_work_.notify_all();
    for (auto& t : threads_) t.join();
  }
  uint32_t workers() const { return uint32_t(threads_.size()); }

  void run(Job& job) {
    job.prepare();
    {
      std::lock_guard<std::mutex> lk(mu_);
      job_ = &job;
      active_ = uint32_t(threads_.size());
      ++generation_;
    }
    cv_work_.notify_all();
    run_grains(job);
    std::unique_lock<std::mutex> lk(mu_);
    cv_done_.wait(lk, [this] { return active_ == 0; });
    job_ = nullptr;
  }

 private:
  void worker() {
    uint64_t seen = 0;
    for (;;) {
      Job* j;
      {
        std::unique_lock<std::mutex> lk(mu_);
        cv_work_.wait(lk, [&] { return stop_ || generation_ != seen; });
        if (stop_) return;
        seen = generation_;
        j = job_;
      }
      run_grains(*j);
      {
        std::lock_guard<std::mutex> lk(mu_);
        if (--active_ == 0) cv_done_.notify_one();
      }
    }
  }

  std::mutex mu_;
  std::condition_variable cv_work_, cv_done_;
  Job* job_ = nullptr;
  uint64_t generation_ = 0;
  uint32_t active_ = 0;
  bool stop_ = false;
  std::vector<std::thread> threads_;
};

}  // namespace pt_host
