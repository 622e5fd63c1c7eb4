// CPU-only harness that runs the oracle's C++ under AddressSanitizer + UndefinedBehaviorSanitizer
// (built by tests/test_sanitizers.py): ragged pack / unpack round trips, the general segment copy,
// norms over odd block sizes and thread counts, both evaluations of the update with a no-decay
// mask and several threads, a skipped step, fp32 accumulation.  It checks a few identities on the
// way; its main purpose is that every index the oracle forms stays inside its arrays.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../oracle/oracle.cpp"

#define EXPECT(cond)                                                                   \
  do {                                                                                 \
    if (!(cond)) { fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); return 1; } \
  } while (0)

int main() {
  uint32_t r = 2024u;
  auto next = [&]() { r = r * 1664525u + 1013904223u; return r >> 8; };
  // conversions on edge words
  for (int dt = 0; dt < 2; ++dt)
    for (uint32_t w = 0; w < 65536; w += 1) {
      float x = orc_decode16(uint16_t(w), dt);
      if (x == x) EXPECT(orc_encode16_rne(x, dt) == uint16_t(w));       // every non-NaN word survives the round trip
    }
  // pack / unpack, ragged
  for (uint64_t S : {8ull, 16ull, 24ull}) {
    const uint64_t sizes[] = {1, 3, 7, 8, 0, 9, 17};
    std::vector<std::vector<uint16_t>> src(7), back(7);
    std::vector<const uint16_t*> sp(7);
    std::vector<uint16_t*> bp(7);
    uint64_t total = 0;
    for (int t = 0; t < 7; ++t) {
      src[t].resize(sizes[t]); back[t].assign(sizes[t], 0xffff);
      for (auto& x : src[t]) x = uint16_t(next());
      sp[t] = src[t].data(); bp[t] = back[t].data();
      total += sizes[t];
    }
    const uint64_t C = (total + S - 1) / S;
    std::vector<uint16_t> chunks(C * S, 0xdead);
    EXPECT(orc_pack_dense(sp.data(), sizes, 7, S, chunks.data(), C) == int64_t(C));
    EXPECT(orc_pack_dense(sp.data(), sizes, 7, S, chunks.data(), C - 1) == -1);
    for (uint64_t k = total; k < C * S; ++k) EXPECT(chunks[k] == 0);
    EXPECT(orc_unpack_dense(chunks.data(), S, C, bp.data(), sizes, 7) == int64_t(C));
    for (int t = 0; t < 7; ++t) EXPECT(src[t] == back[t]);
    // the same layout through the general segment copy
    std::vector<uint16_t> chunks2(C * S, 0);
    std::vector<const uint16_t*> ssrc; std::vector<uint64_t> soff, slen, coff; std::vector<uint32_t> sch;
    uint64_t e = 0;
    for (int t = 0; t < 7; ++t) {
      uint64_t done = 0;
      while (done < sizes[t]) {
        uint64_t c = e / S, in = e % S, run = std::min(S - in, sizes[t] - done);
        ssrc.push_back(sp[t]); soff.push_back(done); slen.push_back(run); sch.push_back(uint32_t(c)); coff.push_back(in);
        done += run; e += run;
      }
    }
    orc_pack_segments(ssrc.data(), soff.data(), slen.data(), sch.data(), coff.data(), uint32_t(ssrc.size()), S, chunks2.data());
    EXPECT(chunks == chunks2);
  }
  // norm, update, step
  const uint64_t n = 10007, S = 1000;
  std::vector<uint16_t> g(n), p(n), p2(n);
  std::vector<float> w(n), m(n, 0.f), v(n, 0.f), w2, m2, v2;
  std::vector<uint8_t> mask(n);
  for (uint64_t i = 0; i < n; ++i) {
    g[i] = orc_encode16_rne(1e-3f * (float(int(next() & 0xffff) - 32768) / 32768.f), 0);
    w[i] = 0.02f * (float(int(next() & 0xffff) - 32768) / 32768.f);
    p[i] = orc_encode16_rne(w[i], 0);
    mask[i] = (i % 7) == 0;
  }
  double s1 = orc_sqnorm(g.data(), n, 0, 1.0, S, 1), s4 = orc_sqnorm(g.data(), n, 0, 1.0, S, 4);
  EXPECT(s1 == s4 && s1 > 0);
  EXPECT(orc_sqnorm(g.data(), 0, 0, 1.0, S, 3) == 0.0);
  EXPECT(orc_sqnorm(g.data(), n, 0, 4.0, 0, 5) > 0);
  orc_hparams hp{1e-4, 0.9, 0.95, 1e-8, 0.1, 1.0};
  w2 = w; m2 = m; v2 = v; p2 = p;
  orc_adamw_f64(&hp, 1, 0.0123, g.data(), w.data(), m.data(), v.data(), p.data(), n, 0, 3, mask.data());
  float c[9];
  orc_consts_f32(&hp, 1, 0.0123, c);
  orc_adamw_f32seq(c, g.data(), w2.data(), m2.data(), v2.data(), p2.data(), n, 0, 5, mask.data());
  for (uint64_t i = 0; i < n; ++i) EXPECT(std::fabs(double(w[i]) - double(w2[i])) <= 1e-6 * (std::fabs(w[i]) + 1e-4));
  orc_scaler_cfg sc{65536.0, 2.0, 0.5, 2, 1};
  orc_state st{0, 0, 65536.0};
  orc_report rep;
  std::vector<uint16_t> g16(n);
  for (uint64_t i = 0; i < n; ++i) g16[i] = orc_encode16_rne(orc_decode16(g[i], 0) * 65536.f, 1);
  for (uint64_t i = 0; i < n; ++i) p[i] = orc_encode16_rne(w[i], 1);
  orc_step(&hp, &sc, &st, g16.data(), w.data(), m.data(), v.data(), p.data(), n, S, 1, 1, 4, &rep, nullptr);
  EXPECT(rep.found_inf == 0 && st.t == 1);
  g16[n - 1] = 0x7c00;
  w2 = w;
  orc_step(&hp, &sc, &st, g16.data(), w.data(), m.data(), v.data(), p.data(), n, S, 1, 0, 4, &rep, mask.data());
  EXPECT(rep.found_inf == 1 && st.t == 1 && st.loss_scale == 32768.0 && w == w2);
  // fp32 accumulation
  std::vector<float> acc(n, 0.f);
  orc_accum_f32(g.data(), n, 0, 1, acc.data());
  orc_accum_f32(g.data(), n, 0, 0, acc.data());
  EXPECT(orc_found_nonfinite_f32(acc.data(), n) == 0);
  EXPECT(orc_sqnorm_f32(acc.data(), n, 1.0, S, 3) == 4.0 * s1);            // every sum is an exact doubling
  st = orc_state{0, 0, 1.0};
  orc_step_g32(&hp, nullptr, &st, acc.data(), w.data(), m.data(), v.data(), p.data(), n, S, 0, 1, 2, &rep, mask.data());
  EXPECT(st.t == 1);
  printf("oracle under the sanitizers: all checks held\n");
  return 0;
}
