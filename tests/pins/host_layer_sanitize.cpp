// CPU-only harness for the host-only layer of the library: layout builders, chunk-size search, cost
// model, chooser and the argument validation that returns before any HIP call.  Built together with
// the library's sources in a host-only compile under AddressSanitizer + UndefinedBehaviorSanitizer
// by tests/test_sanitizers.py; nothing here launches a kernel or needs a GPU.  Exit code 0 = every
// check held and no sanitizer report.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ptchunk.h"

#define EXPECT(cond)                                                                   \
  do {                                                                                 \
    if (!(cond)) { fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); return 1; } \
  } while (0)

int main() {
  // ---- dense layout: tiny ragged tensors, exact capacity, one slot too few
  {
    const uint64_t sizes[] = {1, 3, 7, 8, 0, 9, 17};
    uint32_t nseg = 0, nch = 0;
    EXPECT(pt_layout_dense(sizes, 7, 8, nullptr, 0, &nseg, &nch) == PT_OK);
    EXPECT(nch == 6 && nseg >= 6);                          // 45 elements in chunks of 8
    std::vector<pt_segment> segs(nseg);
    EXPECT(pt_layout_dense(sizes, 7, 8, segs.data(), nseg, &nseg, &nch) == PT_OK);
    uint64_t covered = 0;
    for (const pt_segment& s : segs) {
      EXPECT(s.len > 0 && s.chunk < nch && s.chunk_off + s.len <= 8);
      EXPECT(uint64_t(s.chunk) * 8 + s.chunk_off == covered);   // back to back in global order
      covered += s.len;
    }
    EXPECT(covered == 45);
    std::vector<pt_segment> fewer(nseg - 1);
    EXPECT(pt_layout_dense(sizes, 7, 8, fewer.data(), nseg - 1, &nseg, &nch) == PT_ERR_INVALID_ARG);
    EXPECT(pt_layout_dense(sizes, 7, 12, nullptr, 0, &nseg, &nch) == PT_ERR_ALIGNMENT);
    EXPECT(pt_layout_dense(sizes, 7, 0, nullptr, 0, &nseg, &nch) == PT_ERR_INVALID_ARG);
    EXPECT(pt_layout_dense(nullptr, 7, 8, nullptr, 0, &nseg, &nch) == PT_ERR_INVALID_ARG);
    EXPECT(pt_layout_dense(sizes, 0, 8, nullptr, 0, &nseg, &nch) == PT_OK && nseg == 0 && nch == 0);
    EXPECT(strlen(pt_last_error(nullptr)) > 0);
  }
  // ---- grouped layout and the chunk-size search
  {
    const uint64_t sizes[] = {10, 8, 8, 20, 4, 3};
    const uint32_t gids[] = {PT_NO_GROUP, 0, 0, 1, 1, PT_NO_GROUP};
    uint32_t nseg = 0, nch = 0;
    uint64_t waste = 0;
    {
      const uint32_t uses[] = {2, 0, 2, 5, 0};
      uint32_t order[6] = {9, 9, 9, 9, 9, 9};
      EXPECT(pt_layout_execution_order(uses, 5, 6, order) == PT_OK);
      EXPECT(order[0] == 2 && order[1] == 0 && order[2] == 5 && order[3] == 1 && order[4] == 3 && order[5] == 4);
      EXPECT(pt_layout_execution_order(uses, 5, 5, order) == PT_ERR_INVALID_ARG);    // tensor 5 of 5
      EXPECT(pt_layout_execution_order(nullptr, 0, 0, nullptr) == PT_OK);
      EXPECT(pt_layout_execution_order(nullptr, 0, 2, order) == PT_OK && order[0] == 0 && order[1] == 1);
      EXPECT(pt_layout_execution_order(nullptr, 1, 2, order) == PT_ERR_INVALID_ARG);
    }
    EXPECT(pt_layout_grouped(sizes, gids, 6, 32, nullptr, 0, &nseg, &nch, &waste) == PT_OK);
    EXPECT(nseg == 6 && nch == 3 && waste == 3 * 32 - 53);
    std::vector<pt_segment> segs(nseg);
    EXPECT(pt_layout_grouped(sizes, gids, 6, 32, segs.data(), nseg, &nseg, &nch, &waste) == PT_OK);
    EXPECT(segs[1].chunk == 0 && segs[1].chunk_off == 16 && segs[3].chunk == 1 && segs[3].chunk_off == 0);
    EXPECT(pt_layout_grouped(sizes, gids, 6, 32, segs.data(), 2, &nseg, &nch, &waste) == PT_ERR_INVALID_ARG);
    EXPECT(pt_layout_grouped(sizes, gids, 6, 16, nullptr, 0, &nseg, &nch, &waste) == PT_ERR_INVALID_ARG);   // 20 > 16
    EXPECT(pt_layout_grouped(sizes, nullptr, 6, 32, nullptr, 0, &nseg, &nch, nullptr) == PT_OK);
    uint64_t best = 0;
    EXPECT(pt_chunk_size_search(sizes, gids, 6, 0, 64, 8, &best, &nch, &waste) == PT_OK);
    EXPECT(best >= 24 && best <= 88 && best % 8 == 0 && waste == uint64_t(nch) * best - 53);
    EXPECT(pt_chunk_size_search(sizes, gids, 6, 0, 64, 12, &best, &nch, &waste) == PT_ERR_ALIGNMENT);
    EXPECT(pt_chunk_size_search(sizes, gids, 6, 0, 64, 8, nullptr, &nch, &waste) == PT_ERR_INVALID_ARG);
    EXPECT(pt_chunk_size_search(sizes, gids, 0, 0, 0, 8, &best, &nch, &waste) == PT_OK && nch == 0);
  }
  // ---- cost model and chooser
  {
    pt_optim_rates r{1e-3, 5e-12, 2e-3, 3e-10, 1e-4, 7e-11, 0.3, 0.125};
    double tg = 0, to = 0, ts = 0;
    EXPECT(pt_optim_predict(&r, 1 << 20, 10, 10, PT_OPTIM_STREAM, &tg, &to, &ts) == PT_OK && to == 0 && ts == tg);
    EXPECT(pt_optim_predict(&r, 1 << 20, 10, 0, PT_OPTIM_HOST, &tg, &to, &ts) == PT_OK && tg == 0 && ts == to);
    EXPECT(pt_optim_predict(&r, 1 << 20, 10, 4, PT_OPTIM_STREAM, nullptr, nullptr, &ts) == PT_OK && ts > 0);
    EXPECT(pt_optim_predict(&r, 1 << 20, 10, 11, PT_OPTIM_HOST, &tg, &to, &ts) == PT_ERR_INVALID_ARG);
    EXPECT(pt_optim_predict(nullptr, 1 << 20, 10, 1, PT_OPTIM_HOST, &tg, &to, &ts) == PT_ERR_INVALID_ARG);
    EXPECT(pt_optim_predict(&r, 1 << 20, 10, 1, 7, &tg, &to, &ts) == PT_ERR_INVALID_ARG);
    pt_optim_choice ch;
    const uint64_t per_chunk = 16ull << 20;
    EXPECT(pt_optim_choose(&r, 1 << 20, 10, 6 * per_chunk, PT_OPTIM_STREAM, 3, &ch) == PT_OK);
    EXPECT(ch.n_persist + ch.n_slots <= 6 && ch.hbm_bytes <= 6 * per_chunk);
    EXPECT(pt_optim_choose(&r, 1 << 20, 10, 2 * per_chunk, PT_OPTIM_STREAM, 3, &ch) == PT_ERR_INVALID_ARG);
    EXPECT(pt_optim_choose(&r, 1 << 20, 10, 100 * per_chunk, PT_OPTIM_HOST, 0, &ch) == PT_OK && ch.n_persist <= 10);
    EXPECT(pt_optim_choose(&r, 1 << 20, 10, per_chunk, PT_OPTIM_STREAM, 1, &ch) == PT_ERR_INVALID_ARG);
  }
  // ---- validation that answers before any HIP call
  {
    pt_ctx* ctx = nullptr;
    EXPECT(pt_ctx_create(nullptr, PT_BF16, 8, 1, nullptr) == PT_ERR_INVALID_ARG);
    EXPECT(pt_ctx_create(&ctx, 5, 8, 1, nullptr) == PT_ERR_INVALID_ARG && ctx == nullptr);
    EXPECT(pt_ctx_create(&ctx, PT_BF16, 0, 1, nullptr) == PT_ERR_INVALID_ARG);
    EXPECT(pt_ctx_create(&ctx, PT_BF16, 12, 1, nullptr) == PT_ERR_ALIGNMENT);
    EXPECT(pt_ctx_create(&ctx, PT_BF16, 8, 70000, nullptr) == PT_ERR_UNSUPPORTED);
    pt_scaler_cfg bad{0.5, 2.0, 0.5, 2000, 0};
    EXPECT(pt_ctx_create(&ctx, PT_FP16, 8, 1, &bad) == PT_ERR_INVALID_ARG);
    EXPECT(pt_ctx_destroy(nullptr) == PT_OK);
    EXPECT(pt_pack_plan_destroy(nullptr) == PT_OK);
    EXPECT(pt_chunk_adamw_step(nullptr, nullptr, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == PT_ERR_INVALID_ARG);
    EXPECT(pt_calib_copy(nullptr, nullptr, 16, nullptr) == PT_ERR_INVALID_ARG);
    double out[2]; int32_t flag;
    EXPECT(pt_chunk_grad_sqnorm_noalloc(nullptr, PT_BF16, 8, 1, 1.0, out, &flag, nullptr) == PT_ERR_INVALID_ARG);
    EXPECT(pt_chunk_grad_sqnorm_noalloc(out, PT_BF16, 1ull << 26, 512, 1.0, out, &flag, nullptr) == PT_ERR_UNSUPPORTED);
    EXPECT(strcmp(pt_status_string(PT_ERR_STATE), "PT_ERR_STATE") == 0 && strcmp(pt_status_string(99), "PT_ERR_UNKNOWN") == 0);
  }
  printf("host-only layer: all checks held\n");
  return 0;
}
