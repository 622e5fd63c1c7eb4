// OPTIM-phase cost model and n_persist chooser (host, no GPU work).
//
// The paper models an iteration as T_FWD + max{T_BWD + T_GPU_OPTIM, T_CPU_OPTIM}, with both
// update times "modeled based on parameter size", and the memory of model states as
// M_persist * n_persist + M_buffer * n_buffer (Appendix A, Eq. 2 and the last equation of
// A.2); it then searches the configurations exhaustively under the memory capacity
// (Automatic Memory Management).  This file is that structure restricted to the optimizer
// phase of this library: linear-in-elements times fitted from measurements, the max of the
// two concurrent parts, 16 bytes per element of HBM per resident chunk or chunk buffer, and
// an exhaustive scan over n_persist.
#include "pt_common.h"

namespace {

// a fitted intercept may be slightly negative: a time never is
inline double lin(double fixed, double per_elem, double elems) {
  if (!(elems > 0)) return 0.0;
  const double t = fixed + per_elem * elems;
  return t > 0.0 ? t : 0.0;
}

int predict(const pt_optim_rates* r, uint64_t S, uint32_t C, uint32_t n_persist, int mode, double* t_gpu,
            double* t_other, double* t_step) {
  const double res = double(S) * n_persist, rest = double(S) * (C - n_persist);
  const double tg = lin(r->gpu_s_fixed, r->gpu_s_per_elem, res);
  double to = 0.0;
  if (mode == PT_OPTIM_STREAM) to = lin(r->link_s_fixed, r->link_s_per_elem, rest);
  else to = lin(r->host_s_fixed, r->host_s_per_elem, rest);
  // The resident work that precedes the norm comes first; the rest of it and the other part run side by
  // side; a streamed part also shares the GPU with the resident one.
  double ts = tg;
  if (rest > 0) {
    const double first = r->gpu_serial_share * tg, beside = tg - first;
    ts = first + (beside > to ? beside : to);
    if (mode == PT_OPTIM_STREAM && res > 0) ts += r->stream_contention * (beside < to ? beside : to);
  }
  if (t_gpu) *t_gpu = tg;
  if (t_other) *t_other = to;
  if (t_step) *t_step = ts;
  return PT_OK;
}

}  // namespace

extern "C" int pt_optim_predict(const pt_optim_rates* rates, uint64_t chunk_elems, uint32_t n_chunks,
                                uint32_t n_persist, int mode, double* t_gpu, double* t_other, double* t_step) {
  if (!rates) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_predict: rates is NULL");
  if (chunk_elems == 0 || n_persist > n_chunks)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_predict: chunk_elems > 0 and n_persist <= n_chunks required");
  if (mode != PT_OPTIM_STREAM && mode != PT_OPTIM_HOST)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_predict: mode must be PT_OPTIM_STREAM or PT_OPTIM_HOST");
  if (!(rates->gpu_serial_share >= 0.0) || !(rates->gpu_serial_share <= 1.0))
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_predict: gpu_serial_share must be in [0, 1]");
  return predict(rates, chunk_elems, n_chunks, n_persist, mode, t_gpu, t_other, t_step);
}

extern "C" int pt_optim_choose(const pt_optim_rates* rates, uint64_t chunk_elems, uint32_t n_chunks,
                               uint64_t hbm_budget_bytes, int mode, uint32_t n_slots, pt_optim_choice* out) {
  if (!rates || !out) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_choose: NULL argument");
  if (chunk_elems == 0 || n_chunks == 0)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_choose: chunk_elems and n_chunks must be > 0");
  if (mode != PT_OPTIM_STREAM && mode != PT_OPTIM_HOST)
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_choose: mode must be PT_OPTIM_STREAM or PT_OPTIM_HOST");
  if (!(rates->gpu_serial_share >= 0.0) || !(rates->gpu_serial_share <= 1.0))
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_choose: gpu_serial_share must be in [0, 1]");
  if (mode == PT_OPTIM_STREAM && (n_slots < 2 || n_slots > PT_MAX_SLOTS))
    return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_choose: n_slots must be in [2, %u] for the streamed mode", PT_MAX_SLOTS);
  const uint64_t per_chunk = 16 * chunk_elems;
  bool found = false;
  pt_optim_choice best{};
  for (uint32_t n = 0; n <= n_chunks; ++n) {
    // chunk buffers are only needed while some chunk is not resident
    const uint64_t buffers = (mode == PT_OPTIM_STREAM && n < n_chunks) ? n_slots : 0;
    const uint64_t need = per_chunk * (uint64_t(n) + buffers);
    if (need > hbm_budget_bytes) continue;
    double tg, to, ts;
    predict(rates, chunk_elems, n_chunks, n, mode, &tg, &to, &ts);
    // least predicted time; at equal time the smaller footprint
    if (!found || ts < best.t_step) {
      found = true;
      best.n_persist = n; best.n_slots = uint32_t(buffers); best.mode = mode;
      best.t_step = ts; best.t_gpu = tg; best.t_other = to; best.hbm_bytes = need;
    }
  }
  if (!found) return pt_fail(nullptr, PT_ERR_INVALID_ARG, "pt_optim_choose: the budget does not even hold the chunk buffers");
  *out = best;
  return PT_OK;
}
