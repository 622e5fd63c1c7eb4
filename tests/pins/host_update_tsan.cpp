// CPU-only harness for the host-side update's thread pool and grain queue (built with
// -fsanitize=thread by tests/test_sanitizers.py; no GPU, no HIP).  Runs several steps over plain
// host arrays with a pool of threads, with and without no-decay runs, bf16 and fp16, 16-bit and
// fp32 gradients, re-using one pool across calls and rebuilding it, and compares every result with
// a single-threaded pass over the same data.  A data race is reported by the sanitizer (exit code
// 66); a wrong result by exit code 1.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "pt_host_update.h"

namespace {

struct State {
  std::vector<std::vector<uint16_t>> g16, p;
  std::vector<std::vector<float>> g32, w, m, v;
};

uint32_t lcg(uint32_t& r) { r = r * 1664525u + 1013904223u; return r >> 8; }

State make(uint32_t C, uint64_t S, uint32_t seed) {
  State st;
  st.g16.assign(C, std::vector<uint16_t>(S)); st.p.assign(C, std::vector<uint16_t>(S));
  st.g32.assign(C, std::vector<float>(S)); st.w.assign(C, std::vector<float>(S));
  st.m.assign(C, std::vector<float>(S, 0.0f)); st.v.assign(C, std::vector<float>(S, 0.0f));
  uint32_t r = seed;
  for (uint32_t c = 0; c < C; ++c)
    for (uint64_t i = 0; i < S; ++i) {
      float a = float(int(lcg(r) & 0xffff) - 32768) / 32768.0f;
      float b = float(int(lcg(r) & 0xffff) - 32768) / 32768.0f;
      st.g32[c][i] = 1.5e-3f * a;
      st.g16[c][i] = pt_host::f32_to_bf16(1.5e-3f * a);     // a valid bf16 word; also a finite fp16 word pattern or not: masked below
      st.g16[c][i] &= 0xbbffu;                              // keeps the word finite in both 16-bit formats
      st.w[c][i] = 0.03f * b;
    }
  return st;
}

void fill_job(pt_host::Job& job, State& st, std::vector<const void*>& gp, std::vector<float*>& wp, std::vector<float*>& mp,
              std::vector<float*>& vp, std::vector<void*>& pp, bool fp16, bool g32, uint64_t S, uint32_t first, uint32_t n,
              const std::vector<uint32_t>* nd_begin, const std::vector<uint64_t>* nd_ranges, int step) {
  gp.clear(); wp.clear(); mp.clear(); vp.clear(); pp.clear();
  for (uint32_t c = first; c < first + n; ++c) {
    gp.push_back(g32 ? (const void*)st.g32[c].data() : (const void*)st.g16[c].data());
    wp.push_back(st.w[c].data()); mp.push_back(st.m[c].data()); vp.push_back(st.v[c].data()); pp.push_back(st.p[c].data());
  }
  job.k = pt_host::Consts{0.9f, 0.95f, 0.1f, 0.05f, 0.99999f, 1e-4f / (1.0f - std::pow(0.9f, float(step))),
                          1.0f / std::sqrt(1.0f - std::pow(0.95f, float(step))), 1e-8f, 0.0123f};
  job.dtype_fp16 = fp16; job.grad_f32 = g32; job.S = S; job.first_chunk = first; job.n_chunks = n;
  job.h_grad = gp.data(); job.h_master = wp.data(); job.h_m = mp.data(); job.h_v = vp.data(); job.h_param16 = pp.data();
  job.nd_begin = nd_begin ? nd_begin->data() : nullptr;
  job.nd_ranges = nd_ranges ? nd_ranges->data() : nullptr;
}

bool same(const State& a, const State& b) {
  return a.w == b.w && a.m == b.m && a.v == b.v && a.p == b.p;
}

}  // namespace

int main() {
  const uint64_t S = 2 * pt_host::GRAIN + 4104;      // several grains and a ragged last one
  const uint32_t C = 5;   // keep in step with nd_begin below
  // no-decay runs: chunk 0 head, chunk 1 across a grain boundary, chunk 3 whole, chunk 4 tail
  std::vector<uint32_t> nd_begin = {0, 1, 2, 2, 3, 4};
  std::vector<uint64_t> nd_ranges = {0, 100, pt_host::GRAIN - 7, pt_host::GRAIN + 9, 0, S, S - 50, S};
  int cases = 0;
  for (int fp16 = 0; fp16 < 2; ++fp16)
    for (int g32 = 0; g32 < 2; ++g32)
      for (int masked = 0; masked < 2; ++masked) {
        State par = make(C, S, 77u + fp16 * 3 + g32), ser = par;
        std::vector<const void*> gp; std::vector<float*> wp, mp, vp; std::vector<void*> pp;
        pt_host::Pool pool(7);
        pt_host::Pool none(0);
        for (int step = 1; step <= 2; ++step) {
          // chunks [1, 5) by the pool, chunk 0 by a pool rebuilt for the call; serial reference does all at once
          pt_host::Job job;
          fill_job(job, par, gp, wp, mp, vp, pp, fp16, g32, S, 1, 4, masked ? &nd_begin : nullptr, masked ? &nd_ranges : nullptr, step);
          pool.run(job);
          {
            pt_host::Pool fresh(3);
            pt_host::Job j0;
            fill_job(j0, par, gp, wp, mp, vp, pp, fp16, g32, S, 0, 1, masked ? &nd_begin : nullptr, masked ? &nd_ranges : nullptr, step);
            fresh.run(j0);
          }
          pt_host::Job js;
          fill_job(js, ser, gp, wp, mp, vp, pp, fp16, g32, S, 0, C, masked ? &nd_begin : nullptr, masked ? &nd_ranges : nullptr, step);
          none.run(js);
          if (!same(par, ser)) {
            fprintf(stderr, "threaded and serial results differ: fp16 %d g32 %d masked %d step %d\n", fp16, g32, masked, step);
            return 1;
          }
        }
        ++cases;
      }
  printf("host update under the thread pool: %d cases equal the serial pass\n", cases);
  return 0;
}
