// ptchunk_probe: a plain C++ driver of the C-ABI library, without Python or PyTorch.
//
// Runs `steps` optimizer steps (pack -> norm -> AdamW -> step end) over a synthetic state
// of n_chunks x chunk_elems elements, then `copies` launches of the calibration copy over
// one fp32 chunk, and prints hipEvent timings.  It exists so that hardware counters can be
// collected with `rocprofv3 --pmc ... -- ./ptchunk_probe ...` on a process that holds
// nothing but this library, and doubles as a usage example of the boundary.
//
//   ptchunk_probe [chunk_elems=67108864] [n_chunks=101] [steps=3] [copies=4]
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ptchunk.h"

#define CHECK_HIP(x)                                                                        \
  do {                                                                                      \
    hipError_t err_ = (x);                                                                  \
    if (err_ != hipSuccess) {                                                               \
      fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(err_));                      \
      return 1;                                                                             \
    }                                                                                       \
  } while (0)
#define CHECK_PT(ctx, x)                                                                    \
  do {                                                                                      \
    int rc = (x);                                                                           \
    if (rc != PT_OK) {                                                                      \
      fprintf(stderr, "%s -> %s: %s\n", #x, pt_status_string(rc), pt_last_error(ctx));      \
      return 1;                                                                             \
    }                                                                                       \
  } while (0)

static uint16_t bf16_of(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  return uint16_t((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

int main(int argc, char** argv) {
  const uint64_t S = argc > 1 ? strtoull(argv[1], nullptr, 10) : (1ull << 26);
  const uint32_t C = argc > 2 ? (uint32_t)atoi(argv[2]) : 101;
  const int steps = argc > 3 ? atoi(argv[3]) : 3;
  const int copies = argc > 4 ? atoi(argv[4]) : 4;
  printf("probe: %u chunks of %llu elements, %d steps, %d copies\n", C, (unsigned long long)S, steps, copies);

  const uint32_t n_host = getenv("PROBE_STREAM_CHUNKS") ? (uint32_t)atoi(getenv("PROBE_STREAM_CHUNKS")) : 0;
  pt_ctx* ctx = nullptr;
  CHECK_PT(nullptr, pt_ctx_create(&ctx, PT_BF16, S, C + n_host, nullptr));

  // one chunk of pseudo-random host data (LCG -> roughly uniform in +-1e-3 / +-0.03), replicated
  std::vector<uint16_t> hg(S), hp(S);
  std::vector<float> hw(S);
  uint32_t r = 12345u;
  for (uint64_t i = 0; i < S; ++i) {
    r = r * 1664525u + 1013904223u;
    float u1 = (float)((r >> 8) & 0xffff) / 32768.0f - 1.0f;
    r = r * 1664525u + 1013904223u;
    float u2 = (float)((r >> 8) & 0xffff) / 32768.0f - 1.0f;
    hg[i] = bf16_of(1.7e-3f * u1);
    hp[i] = bf16_of(0.035f * u2);
    uint32_t b = uint32_t(hp[i]) << 16;
    memcpy(&hw[i], &b, 4);
  }

  std::vector<void*> src(C), g(C), p(C);
  std::vector<float*> w(C), m(C), v(C);
  for (uint32_t c = 0; c < C; ++c) {
    char* q;
    CHECK_HIP(hipMalloc((void**)&q, 2 * S)); src[c] = q;
    CHECK_HIP(hipMalloc((void**)&q, 2 * S)); g[c] = q;
    CHECK_HIP(hipMalloc((void**)&q, 2 * S)); p[c] = q;
    CHECK_HIP(hipMalloc((void**)&q, 4 * S)); w[c] = (float*)q;
    CHECK_HIP(hipMalloc((void**)&q, 4 * S)); m[c] = (float*)q;
    CHECK_HIP(hipMalloc((void**)&q, 4 * S)); v[c] = (float*)q;
    CHECK_HIP(hipMemcpy(src[c], hg.data(), 2 * S, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(p[c], hp.data(), 2 * S, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(w[c], hw.data(), 4 * S, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(m[c], 0, 4 * S));
    CHECK_HIP(hipMemset(v[c], 0, 4 * S));
    CHECK_HIP(hipMemset(g[c], 0, 2 * S));
  }
  g.resize(C + n_host, nullptr);   // pack takes one entry per chunk of the context; host chunks have none
  // one "tensor" per chunk, filling it completely
  std::vector<pt_segment> segs(C);
  for (uint32_t c = 0; c < C; ++c) segs[c] = pt_segment{src[c], 0, S, 0, c, c};
  pt_pack_plan* plan = nullptr;
  CHECK_PT(ctx, pt_pack_plan_create(ctx, segs.data(), C, &plan));

  hipStream_t st;
  CHECK_HIP(hipStreamCreate(&st));
  hipEvent_t e[4];
  for (auto& x : e) CHECK_HIP(hipEventCreate(&x));
  const pt_hparams hpar{1e-4, 0.9, 0.95, 1e-8, 0.1, 1.0};

  for (int s = 0; s < steps; ++s) {
    CHECK_HIP(hipEventRecord(e[0], st));
    CHECK_PT(ctx, pt_chunk_pack_grads(ctx, plan, g.data(), st));
    CHECK_HIP(hipEventRecord(e[1], st));
    // host chunks (if any) were never reduced in this driver: their sums stay at their initial zero
    CHECK_PT(ctx, pt_chunk_grad_sqnorm(ctx, nullptr, 0, C, n_host ? PT_FINALIZE_CARRY : PT_FINALIZE_STRICT, st));
    CHECK_HIP(hipEventRecord(e[2], st));
    CHECK_PT(ctx, pt_chunk_adamw_step(ctx, &hpar, 0, C, g.data(), w.data(), m.data(), v.data(), p.data(), st));
    CHECK_HIP(hipEventRecord(e[3], st));
    CHECK_PT(ctx, pt_step_end(ctx, st));
    CHECK_HIP(hipStreamSynchronize(st));
    float t_pack, t_norm, t_adamw;
    CHECK_HIP(hipEventElapsedTime(&t_pack, e[0], e[1]));
    CHECK_HIP(hipEventElapsedTime(&t_norm, e[1], e[2]));
    CHECK_HIP(hipEventElapsedTime(&t_adamw, e[2], e[3]));
    pt_step_report rep;
    CHECK_PT(ctx, pt_step_report_read(ctx, &rep, st));
    const double n = double(S) * C;
    printf("step %d: pack %.3f ms (%.0f GB/s)  finalize %.3f ms  adamw %.3f ms (%.0f GB/s)  norm %.6f step %d\n", s,
           t_pack, 4.0 * n / t_pack / 1e6, t_norm, t_adamw, 28.0 * n / t_adamw / 1e6, rep.norm, rep.step);
  }
  // PROBE_STREAM_CHUNKS=<n> [PROBE_SLOTS=3]: n more chunks live in pinned host memory and go through
  // pt_chunk_stream_step while the resident chunks update (needs a context of C + n chunks: see main's top)
  if (n_host > 0) {
    std::vector<void*> hgp(n_host), hpp(n_host);
    std::vector<float*> hwp(n_host), hmp(n_host), hvp(n_host);
    for (uint32_t i = 0; i < n_host; ++i) {
      CHECK_HIP(hipHostMalloc(&hgp[i], 2 * S, hipHostMallocDefault));
      CHECK_HIP(hipHostMalloc(&hpp[i], 2 * S, hipHostMallocDefault));
      CHECK_HIP(hipHostMalloc((void**)&hwp[i], 4 * S, hipHostMallocDefault));
      CHECK_HIP(hipHostMalloc((void**)&hmp[i], 4 * S, hipHostMallocDefault));
      CHECK_HIP(hipHostMalloc((void**)&hvp[i], 4 * S, hipHostMallocDefault));
      memcpy(hgp[i], hg.data(), 2 * S); memcpy(hpp[i], hp.data(), 2 * S); memcpy(hwp[i], hw.data(), 4 * S);
      memset(hmp[i], 0, 4 * S); memset(hvp[i], 0, 4 * S);
    }
    // what the link gives bare copies of the same pinned arrays (one 4*S-byte array per copy, no kernels): one
    // direction at a time, then both at once on two streams - the rates the streamed step is measured against
    {
      void *d_up = nullptr, *d_dn = nullptr;
      hipStream_t sa, sb;
      CHECK_HIP(hipMalloc(&d_up, 4 * S)); CHECK_HIP(hipMalloc(&d_dn, 4 * S));
      CHECK_HIP(hipMemset(d_dn, 0, 4 * S));                 // what comes down is what the host arrays hold anyway
      CHECK_HIP(hipStreamCreateWithFlags(&sa, hipStreamNonBlocking)); CHECK_HIP(hipStreamCreateWithFlags(&sb, hipStreamNonBlocking));
      CHECK_HIP(hipDeviceSynchronize());
      auto run = [&](bool up, bool down, double* gbps) -> int {
        CHECK_HIP(hipDeviceSynchronize());
        const auto t0 = std::chrono::steady_clock::now();
        for (uint32_t i = 0; i < n_host; ++i) {
          if (up) CHECK_HIP(hipMemcpyAsync(d_up, hwp[i], 4 * S, hipMemcpyHostToDevice, sa));
          if (down) CHECK_HIP(hipMemcpyAsync(hvp[i], d_dn, 4 * S, hipMemcpyDeviceToHost, sb));
        }
        CHECK_HIP(hipDeviceSynchronize());
        const double sec = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
        *gbps = 4.0 * double(S) * n_host / sec / 1e9;
        return 0;
      };
      double warm, h2d, d2h, both;
      if (run(true, true, &warm) || run(true, false, &h2d) || run(false, true, &d2h) || run(true, true, &both)) return 1;
      printf("bare pinned copies, %u x %llu bytes: H2D alone %.2f GB/s, D2H alone %.2f GB/s, both at once %.2f GB/s per direction\n",
             n_host, (unsigned long long)(4 * S), h2d, d2h, both);
      CHECK_HIP(hipStreamDestroy(sa)); CHECK_HIP(hipStreamDestroy(sb));
      CHECK_HIP(hipFree(d_up)); CHECK_HIP(hipFree(d_dn));
    }
    const uint32_t slots = getenv("PROBE_SLOTS") ? (uint32_t)atoi(getenv("PROBE_SLOTS")) : 3;
    CHECK_PT(ctx, pt_stream_reserve(ctx, slots));
    {
      int32_t tested = 0, ok = 0, attempts = 0;
      CHECK_PT(ctx, pt_stream_status(ctx, &tested, &ok, &attempts, nullptr));
      printf("copy streams: duplex test %s, %s, %d stream pair(s) tried\n", tested ? "run" : "not run",
             ok ? "upload and offload overlap" : "no overlap seen", attempts);
    }
    for (int s = 0; s < steps; ++s) {
      CHECK_HIP(hipEventRecord(e[0], st));
      CHECK_PT(ctx, pt_chunk_pack_grads(ctx, plan, g.data(), st));
      CHECK_PT(ctx, pt_chunk_grad_sqnorm(ctx, nullptr, 0, C, PT_FINALIZE_CARRY, st));
      CHECK_PT(ctx, pt_chunk_stream_step(ctx, &hpar, C, n_host, hgp.data(), hwp.data(), hmp.data(), hvp.data(), hpp.data(), st));
      CHECK_PT(ctx, pt_chunk_adamw_step(ctx, &hpar, 0, C, g.data(), w.data(), m.data(), v.data(), p.data(), st));
      CHECK_PT(ctx, pt_step_end(ctx, st));
      CHECK_HIP(hipEventRecord(e[1], st));
      CHECK_HIP(hipStreamSynchronize(st));
      float t;
      CHECK_HIP(hipEventElapsedTime(&t, e[0], e[1]));
      int32_t rebuilds = 0;
      CHECK_PT(ctx, pt_stream_status(ctx, nullptr, nullptr, nullptr, &rebuilds));
      printf("streamed step %d: %u resident + %u host chunks, %u slots: %.2f ms, %.2f GB/s per direction (side streams replaced %d time(s) so far)\n",
             s, C, n_host, slots, t, 14.0 * double(S) * n_host / t / 1e6, rebuilds);
    }
  }
  // PROBE_ACCUM=<k> [PROBE_ZERO=1]: the gradient-accumulation variant on the same state: a second context
  // with fp32 gradient chunks, k micro-batches accumulated per step, then norm and update
  if (const char* ka = getenv("PROBE_ACCUM")) {
    const int K = atoi(ka) > 0 ? atoi(ka) : 1;
    pt_ctx* cx = nullptr;
    CHECK_PT(nullptr, pt_ctx_create(&cx, PT_BF16, S, C, nullptr));
    CHECK_PT(cx, pt_ctx_set_option(cx, "grad_fp32", 1));
    if (getenv("PROBE_ZERO")) CHECK_PT(cx, pt_ctx_set_option(cx, "adamw_zero_grads", 1));
    std::vector<float*> g32(C);
    for (uint32_t c = 0; c < C; ++c) {
      CHECK_HIP(hipMalloc((void**)&g32[c], 4 * S));
      CHECK_HIP(hipMemset(g32[c], 0, 4 * S));
    }
    pt_pack_plan* pl = nullptr;
    CHECK_PT(cx, pt_pack_plan_create(cx, segs.data(), C, &pl));
    for (int s = 0; s < steps; ++s) {
      CHECK_HIP(hipEventRecord(e[0], st));
      for (int k = 0; k < K; ++k) CHECK_PT(cx, pt_chunk_accum_grads(cx, pl, g32.data(), k == 0, k == K - 1, st));
      CHECK_HIP(hipEventRecord(e[1], st));
      CHECK_PT(cx, pt_chunk_grad_sqnorm(cx, nullptr, 0, C, 1, st));
      CHECK_HIP(hipEventRecord(e[2], st));
      CHECK_PT(cx, pt_chunk_adamw_step(cx, &hpar, 0, C, (const void* const*)g32.data(), w.data(), m.data(), v.data(), p.data(), st));
      CHECK_HIP(hipEventRecord(e[3], st));
      CHECK_PT(cx, pt_step_end(cx, st));
      CHECK_HIP(hipStreamSynchronize(st));
      float ta, tu;
      CHECK_HIP(hipEventElapsedTime(&ta, e[0], e[1]));
      CHECK_HIP(hipEventElapsedTime(&tu, e[2], e[3]));
      const double n = double(S) * C;
      printf("accumulate step %d: %d micro-batches %.3f ms (%.0f GB/s)  adamw on fp32 gradients %.3f ms (%.0f GB/s)\n", s, K, ta,
             (6.0 + 10.0 * (K - 1)) * n / ta / 1e6, tu, (getenv("PROBE_ZERO") ? 34.0 : 30.0) * n / tu / 1e6);
    }
    CHECK_PT(cx, pt_pack_plan_destroy(pl));
    CHECK_PT(cx, pt_ctx_destroy(cx));
    for (uint32_t c = 0; c < C; ++c) CHECK_HIP(hipFree(g32[c]));
  }
  // standalone norm over all chunks (reads 2 bytes per element)
  {
    CHECK_HIP(hipEventRecord(e[0], st));
    CHECK_PT(ctx, pt_chunk_grad_sqnorm(ctx, g.data(), 0, C, n_host ? PT_FINALIZE_CARRY : PT_FINALIZE_STRICT, st));
    CHECK_HIP(hipEventRecord(e[1], st));
    CHECK_HIP(hipStreamSynchronize(st));
    float t;
    CHECK_HIP(hipEventElapsedTime(&t, e[0], e[1]));
    printf("sqnorm standalone: %.3f ms (%.0f GB/s)\n", t, 2.0 * double(S) * C / t / 1e6);
    CHECK_PT(ctx, pt_step_end(ctx, st));
  }
  for (int k = 0; k < copies; ++k) {
    // 16 back-to-back copies between different arrays (4 GiB read + 4 GiB written): far beyond any cache
    const int reps = C >= 17 ? 16 : 1;
    CHECK_HIP(hipEventRecord(e[0], st));
    for (int r = 0; r < reps; ++r) CHECK_PT(nullptr, pt_calib_copy(m[(k + r + 1) % C], v[(k + r) % C], 4 * S, st));
    CHECK_HIP(hipEventRecord(e[1], st));
    CHECK_HIP(hipStreamSynchronize(st));
    float t;
    CHECK_HIP(hipEventElapsedTime(&t, e[0], e[1]));
    printf("calib copy %d: %d x %llu bytes read + written in %.3f ms (%.0f GB/s)\n", k, reps,
           (unsigned long long)(4 * S), t, reps * 8.0 * double(S) / t / 1e6);
  }
  CHECK_PT(ctx, pt_pack_plan_destroy(plan));
  CHECK_PT(ctx, pt_ctx_destroy(ctx));
  printf("probe done\n");
  return 0;
}
