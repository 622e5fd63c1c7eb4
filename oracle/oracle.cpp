// CPU oracle for the chunked model-state path (pack -> global grad norm -> clip ->
// mixed-precision AdamW -> 16-bit recast, with dynamic loss scaling).
//
// TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct C++; fp64 arithmetic
// for everything that is floating point.  It shares no code, header, table or
// helper with the HIP library and must never be imported by the product path.
// Only tests, the smoke check and the bench's cpu_baseline leg may load it.
//
// What is followed:
//  * The five arrays of a model state (16-bit param, fp32 master, 16-bit grad,
//    fp32 momentum, fp32 variance = 16 bytes per parameter): paper, Introduction.
//  * Model states live in fixed-size flat chunks; a prefix of chunks is
//    persistent on the GPU: paper, "Hierarchical Chunk Management for Model
//    States".
//  * Reduced-precision forward/backward with an fp32 update: paper, Background.
//  * The optimizer itself is Adam ("FusedAdam"/"CPU Adam", Appendix A.1) and the
//    paper says nothing more about it.  The arithmetic below is the textbook
//    definition: Adam with bias correction (Kingma & Ba, Algorithm 1), decoupled
//    weight decay (Loshchilov & Hutter), global-L2-norm clipping with
//    clip = min(1, c / (norm + 1e-6)), dynamic loss scaling with skip on
//    non-finite gradients (Micikevicius et al.).
//
// The oracle works on UNCHUNKED flat arrays; chunking only appears as the index
// map e -> (e div S, e mod S) in orc_pack_dense / orc_unpack_dense and as the
// partial-sum block of orc_sqnorm, so a chunk-indexing bug on the GPU side cannot
// cancel against the same bug here.
//
// Parity pins (tests/, -m "not gpu"): 16-bit conversions vs a nearest-value brute
// force over all 2^32 inputs and vs numpy/torch conversions; norm vs math.fsum,
// closed forms and power-of-two scaling; AdamW vs closed forms, a 60-digit
// decimal evaluation and torch.optim.AdamW in fp64; pack vs per-element brute
// force and the round-trip invariant; the loss-scale machine vs a replay without
// the skipped step.  orc_adamw_f32seq (the fp32 operation sequence) is pinned bit for bit, in
// the general case where operations round, against the same sequence carried out in exact
// rational arithmetic with one value-domain nearest/ties-to-even rounding per operation
// (Python integers and fractions; square roots proven by exact squares), on 16-bit and on
// fp32 gradients, subnormal intermediates included; it also stays within tolerance of
// orc_adamw_f64.  The fp32 gradient-accumulation variant
// (orc_accum_f32, orc_sqnorm_f32, orc_*_g32): numpy float32 addition and exact rationals,
// math.fsum, bit-identity with the 16-bit-gradient functions on decoded words, a closed form
// on gradients no 16-bit word holds, torch.optim.AdamW in fp64 on accumulated gradients.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

inline uint32_t f32_bits(float x) { uint32_t u; std::memcpy(&u, &x, 4); return u; }
inline float bits_f32(uint32_t u) { float x; std::memcpy(&x, &u, 4); return x; }

// ---- 16-bit formats, integer arithmetic on the bit patterns -----------------

// bfloat16: the upper half of a binary32.
inline float bf16_decode(uint16_t w) { return bits_f32(uint32_t(w) << 16); }

inline uint16_t bf16_encode_rne(float x) {
  uint32_t u = f32_bits(x);
  if ((u & 0x7fffffffu) > 0x7f800000u)            // NaN: keep sign, force quiet
    return uint16_t((u >> 16) | 0x0040u);
  uint32_t keep_lsb = (u >> 16) & 1u;             // ties go to the even pattern
  u += 0x7fffu + keep_lsb;                        // carry may roll into exponent / inf
  return uint16_t(u >> 16);
}

// IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.
inline float fp16_decode(uint16_t w) {
  uint32_t sign = uint32_t(w & 0x8000u) << 16;
  uint32_t exp = (w >> 10) & 0x1fu;
  uint32_t frac = w & 0x3ffu;
  if (exp == 0x1fu) return bits_f32(sign | 0x7f800000u | (frac << 13));
  if (exp == 0) {
    // subnormal: frac * 2^-24, exact in binary32
    float mag = float(frac) * 5.9604644775390625e-08f;
    return sign ? -mag : mag;
  }
  return bits_f32(sign | ((exp + 112u) << 23) | (frac << 13));
}

inline uint16_t fp16_encode_rne(float x) {
  uint32_t u = f32_bits(x);
  uint16_t sign = uint16_t((u >> 16) & 0x8000u);
  uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return uint16_t(sign | 0x7e00u | ((a >> 13) & 0x3ffu));  // quiet NaN
  if (a == 0x7f800000u) return uint16_t(sign | 0x7c00u);
  int e = int(a >> 23) - 127;
  uint32_t h, rem, half;
  if (e >= -14) {
    if (e > 15) return uint16_t(sign | 0x7c00u);
    uint32_t frac = a & 0x7fffffu;
    h = (uint32_t(e + 15) << 10) | (frac >> 13);
    rem = frac & 0x1fffu;
    half = 0x1000u;
  } else {
    if (e < -25) return sign;                      // below half of the smallest subnormal
    uint32_t sig = (a & 0x7fffffu) | 0x800000u;    // 1.frac as a 24-bit integer
    int shift = -1 - e;                            // 14 .. 24
    h = sig >> shift;
    rem = sig & ((1u << shift) - 1u);
    half = 1u << (shift - 1);
  }
  if (rem > half || (rem == half && (h & 1u))) ++h;  // may carry up to 0x7c00 = inf
  return uint16_t(sign | h);
}

inline float decode16(uint16_t w, int dtype) { return dtype == 0 ? bf16_decode(w) : fp16_decode(w); }
inline uint16_t encode16(float x, int dtype) { return dtype == 0 ? bf16_encode_rne(x) : fp16_encode_rne(x); }
inline bool nonfinite16(uint16_t w, int dtype) {
  return dtype == 0 ? ((w & 0x7f80u) == 0x7f80u) : ((w & 0x7c00u) == 0x7c00u);
}

// ---- a plain parallel-for over [0, n) in contiguous ranges ------------------

template <class F>
void parallel_ranges(uint64_t n, int threads, F&& body) {
  if (threads <= 1 || n < 4096) { body(uint64_t(0), n); return; }
  uint64_t per = (n + uint64_t(threads) - 1) / uint64_t(threads);
  std::vector<std::thread> pool;
  for (int t = 0; t < threads; ++t) {
    uint64_t lo = uint64_t(t) * per, hi = std::min(n, lo + per);
    if (lo >= hi) break;
    pool.emplace_back([=, &body] { body(lo, hi); });
  }
  for (auto& th : pool) th.join();
}

}  // namespace

extern "C" {

typedef struct {
  double lr, beta1, beta2, eps, weight_decay, max_norm;   // max_norm <= 0: no clipping
} orc_hparams;

typedef struct {
  double init_scale, growth, backoff;                     // 65536, 2, 0.5
  int32_t growth_interval;                                // 2000
  int32_t enabled;                                        // 0: loss scale fixed at 1
} orc_scaler_cfg;

typedef struct {
  int32_t t;            // number of APPLIED updates so far
  int32_t good_steps;   // consecutive finite steps since the last scale change
  double loss_scale;
} orc_state;

typedef struct {
  double sqnorm, norm, clip_coef, grad_mult, loss_scale_used;
  int32_t found_inf, t_after;
} orc_report;

}  // extern "C"

namespace {

// The gradient of element i comes from `grad_at(i)` (its exact value as a double): 16-bit
// gradient chunks decode their word, fp32 accumulation chunks hand over the stored float.
template <class G>
void adamw_f64_any(const orc_hparams* hp, int32_t t, double grad_mult, G grad_at,
                   float* w, float* m, float* v, uint16_t* p16, uint64_t n, int dtype,
                   int threads, const uint8_t* no_decay) {
  const double b1 = hp->beta1, b2 = hp->beta2;
  const double bc1 = 1.0 - std::pow(b1, double(t));
  const double bc2 = 1.0 - std::pow(b2, double(t));
  const double step_size = hp->lr / bc1;
  const double decay = 1.0 - hp->lr * hp->weight_decay;
  const double sqrt_bc2 = std::sqrt(bc2);
  const double eps = hp->eps;
  parallel_ranges(n, threads, [&](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) {
      double g = grad_at(i) * grad_mult;
      double mn = b1 * double(m[i]) + (1.0 - b1) * g;
      double vn = b2 * double(v[i]) + (1.0 - b2) * g * g;
      double denom = std::sqrt(vn) / sqrt_bc2 + eps;
      double wn = double(w[i]) * ((no_decay && no_decay[i]) ? 1.0 : decay) - step_size * (mn / denom);
      m[i] = float(mn);
      v[i] = float(vn);
      w[i] = float(wn);
      p16[i] = encode16(w[i], dtype);
    }
  });
}

// The fp32 operation sequence of the update; `grad_at(i)` is the gradient as a binary32 value.
template <class G>
void adamw_f32seq_any(const float* c, G grad_at, float* w, float* m, float* v,
                      uint16_t* p16, uint64_t n, int dtype, int threads, const uint8_t* no_decay) {
  const float b1 = c[0], b2 = c[1], omb1 = c[2], omb2 = c[3], decay = c[4], step_size = c[5],
              rsb2 = c[6], eps = c[7], gm = c[8];
  parallel_ranges(n, threads, [&](uint64_t lo, uint64_t hi) {
    for (uint64_t i = lo; i < hi; ++i) {
      float g = grad_at(i) * gm;
      float t1 = omb1 * g;
      float mn = std::fmaf(b1, m[i], t1);
      float t2 = omb2 * g;
      t2 = t2 * g;
      float vn = std::fmaf(b2, v[i], t2);
      float d = std::fmaf(std::sqrt(vn), rsb2, eps);
      float u = mn / d;
      float t3 = w[i] * ((no_decay && no_decay[i]) ? 1.0f : decay);
      float wn = std::fmaf(-step_size, u, t3);
      m[i] = mn;
      v[i] = vn;
      w[i] = wn;
      p16[i] = encode16(wn, dtype);
    }
  });
}

}  // namespace

extern "C" {

// ---- conversions -------------------------------------------------------------

float orc_decode16(uint16_t w, int dtype) { return decode16(w, dtype); }
uint16_t orc_encode16_rne(float x, int dtype) { return encode16(x, dtype); }

void orc_decode16_array(const uint16_t* in, float* out, uint64_t n, int dtype) {
  for (uint64_t i = 0; i < n; ++i) out[i] = decode16(in[i], dtype);
}
void orc_encode16_array(const float* in, uint16_t* out, uint64_t n, int dtype) {
  for (uint64_t i = 0; i < n; ++i) out[i] = encode16(in[i], dtype);
}

// ---- pack / unpack -------------------------------------------------------------
// Dense layout: the tensors are concatenated in the order given; global element e
// lands in chunk e div S at position e mod S.  Only the tail of the last chunk is
// padding and it is zero.  Words are moved as 16-bit integers.
// Returns the number of chunks needed, or -1 if n_chunks is too small.
int64_t orc_pack_dense(const uint16_t* const* tensors, const uint64_t* elems, uint32_t n_tensors,
                       uint64_t S, uint16_t* chunks, uint64_t n_chunks) {
  uint64_t total = 0;
  for (uint32_t i = 0; i < n_tensors; ++i) total += elems[i];
  uint64_t need = (total + S - 1) / S;
  if (need > n_chunks) return -1;
  for (uint64_t k = total; k < n_chunks * S; ++k) chunks[k] = 0;
  uint64_t e = 0;
  for (uint32_t i = 0; i < n_tensors; ++i)
    for (uint64_t j = 0; j < elems[i]; ++j, ++e) {
      uint64_t c = e / S, pos = e % S;
      chunks[c * S + pos] = tensors[i][j];
    }
  return int64_t(need);
}

// General form of the copy: segment i puts words [src_off, src_off + len) of its tensor into
// chunk `chunk` at position chunk_off (the dense layout above is one such table; the paper's own
// layout, which never splits a tensor, another).  Words no segment covers are left as they are.
void orc_pack_segments(const uint16_t* const* src, const uint64_t* src_off, const uint64_t* len,
                       const uint32_t* chunk, const uint64_t* chunk_off, uint32_t n_segs, uint64_t S,
                       uint16_t* chunks) {
  for (uint32_t i = 0; i < n_segs; ++i)
    for (uint64_t j = 0; j < len[i]; ++j)
      chunks[uint64_t(chunk[i]) * S + chunk_off[i] + j] = src[i][src_off[i] + j];
}

int64_t orc_unpack_dense(const uint16_t* chunks, uint64_t S, uint64_t n_chunks,
                         uint16_t* const* tensors, const uint64_t* elems, uint32_t n_tensors) {
  uint64_t e = 0;
  for (uint32_t i = 0; i < n_tensors; ++i)
    for (uint64_t j = 0; j < elems[i]; ++j, ++e) {
      uint64_t c = e / S, pos = e % S;
      if (c >= n_chunks) return -1;
      tensors[i][j] = chunks[c * S + pos];
    }
  return int64_t((e + S - 1) / S);
}

// ---- non-finite scan -------------------------------------------------------------
int32_t orc_found_nonfinite(const uint16_t* g, uint64_t n, int dtype) {
  for (uint64_t i = 0; i < n; ++i)
    if (nonfinite16(g[i], dtype)) return 1;
  return 0;
}

// ---- global squared L2 norm of the unscaled gradients ----------------------------
// sum_e (double(g_e) / loss_scale)^2, accumulated in fp64 in index order inside
// each block of `block` elements (one chunk), the block sums then added in block
// order.  block == 0 means one single run.  The thread count never changes the
// result: threads only decide who computes which block.
double orc_sqnorm(const uint16_t* g, uint64_t n, int dtype, double loss_scale, uint64_t block,
                  int threads) {
  if (n == 0) return 0.0;
  if (block == 0) block = n;
  uint64_t nb = (n + block - 1) / block;
  std::vector<double> part(nb, 0.0);
  parallel_ranges(nb, threads, [&](uint64_t b0, uint64_t b1) {
    for (uint64_t b = b0; b < b1; ++b) {
      uint64_t lo = b * block, hi = std::min(n, lo + block);
      double s = 0.0;
      for (uint64_t i = lo; i < hi; ++i) {
        double x = double(decode16(g[i], dtype)) / loss_scale;
        s += x * x;
      }
      part[b] = s;
    }
  });
  double total = 0.0;
  for (uint64_t b = 0; b < nb; ++b) total += part[b];
  return total;
}

// clip = min(1, c / (norm + 1e-6)); c <= 0 switches clipping off.
double orc_clip_coef(double norm, double max_norm) {
  if (!(max_norm > 0.0)) return 1.0;
  double c = max_norm / (norm + 1e-6);
  return c < 1.0 ? c : 1.0;
}

// ---- AdamW, fp64 evaluation ---------------------------------------------------
// t is the index of this update (the first applied update has t = 1).
// Every element (padding included):
//   g  = decode(g16) * grad_mult
//   m' = beta1 m + (1 - beta1) g
//   v' = beta2 v + (1 - beta2) g^2
//   w' = w (1 - lr wd) - lr/(1 - beta1^t) * m' / ( sqrt(v') / sqrt(1 - beta2^t) + eps )
// evaluated in fp64 from the fp32 state, each result rounded once to fp32 (the
// state arrays ARE fp32: that rounding is part of the method, not of the oracle),
// and p16 = RNE16(w').
// no_decay (may be NULL): one byte per element; a non-zero byte switches the decay factor of
// that element to 1 (weight-decay groups: biases and normalisation gains are commonly kept out
// of the decay; the paper does not speak of weight decay at all).
void orc_adamw_f64(const orc_hparams* hp, int32_t t, double grad_mult, const uint16_t* g16,
                   float* w, float* m, float* v, uint16_t* p16, uint64_t n, int dtype,
                   int threads, const uint8_t* no_decay) {
  adamw_f64_any(hp, t, grad_mult, [=](uint64_t i) { return double(decode16(g16[i], dtype)); }, w, m, v, p16, n,
                dtype, threads, no_decay);
}

// ---- AdamW, the fp32 operation sequence ---------------------------------------
// Nine binary32 constants, each computed in fp64 and rounded once:
//   c[0]=beta1  c[1]=beta2  c[2]=1-beta1  c[3]=1-beta2  c[4]=1-lr*wd
//   c[5]=lr/(1-beta1^t)  c[6]=1/sqrt(1-beta2^t)  c[7]=eps  c[8]=grad_mult
void orc_consts_f32(const orc_hparams* hp, int32_t t, double grad_mult, float* c) {
  c[0] = float(hp->beta1);
  c[1] = float(hp->beta2);
  c[2] = float(1.0 - hp->beta1);
  c[3] = float(1.0 - hp->beta2);
  c[4] = float(1.0 - hp->lr * hp->weight_decay);
  c[5] = float(hp->lr / (1.0 - std::pow(hp->beta1, double(t))));
  c[6] = float(1.0 / std::sqrt(1.0 - std::pow(hp->beta2, double(t))));
  c[7] = float(hp->eps);
  c[8] = float(grad_mult);
}

// One IEEE binary32 operation per line (this file is built with -ffp-contract=off;
// fmaf is a single rounding).  A device kernel that performs the same correctly
// rounded operations in the same order gives the same bits.
void orc_adamw_f32seq(const float* c, const uint16_t* g16, float* w, float* m, float* v,
                      uint16_t* p16, uint64_t n, int dtype, int threads, const uint8_t* no_decay) {
  adamw_f32seq_any(c, [=](uint64_t i) { return decode16(g16[i], dtype); }, w, m, v, p16, n, dtype, threads, no_decay);
}

// Scalars of a step from its squared norm and non-finite flag (rep->sqnorm, rep->found_inf set by
// the caller).  Returns false for a skipped step: state untouched, the update counter does not
// advance, the loss scale backs off.  Otherwise the counter advances and the update may run.
static bool step_scalars(const orc_hparams* hp, const orc_scaler_cfg* sc, orc_state* st, orc_report* rep) {
  const double sigma = st->loss_scale;
  rep->norm = std::sqrt(rep->sqnorm);
  rep->clip_coef = orc_clip_coef(rep->norm, hp->max_norm);
  rep->grad_mult = rep->clip_coef / sigma;
  if (rep->found_inf) {
    if (sc && sc->enabled) {
      st->loss_scale = std::max(sigma * sc->backoff, 1.0);
      st->good_steps = 0;
    }
    rep->t_after = st->t;
    return false;
  }
  st->t += 1;
  return true;
}

// After an applied update: the loss scale grows every growth_interval good steps in a row.
static void step_grow(const orc_scaler_cfg* sc, orc_state* st, orc_report* rep) {
  if (sc && sc->enabled) {
    st->good_steps += 1;
    if (st->good_steps >= sc->growth_interval) {
      st->loss_scale = st->loss_scale * sc->growth;
      st->good_steps = 0;
    }
  }
  rep->t_after = st->t;
}

// ---- one whole optimizer step on flat arrays --------------------------------------
// g16 holds the (loss-scaled) 16-bit gradients of all n elements, padding
// included (padding words are zero).  S is the chunk size: it only fixes the
// order of the fp64 partial sums of the norm.  use_f32seq selects the fp32
// sequence for the update instead of the fp64 evaluation; the scalars (norm,
// clip, grad_mult) are always fp64.
void orc_step(const orc_hparams* hp, const orc_scaler_cfg* sc, orc_state* st, const uint16_t* g16,
              float* w, float* m, float* v, uint16_t* p16, uint64_t n, uint64_t S, int dtype,
              int use_f32seq, int threads, orc_report* rep, const uint8_t* no_decay) {
  const double sigma = st->loss_scale;
  rep->loss_scale_used = sigma;
  rep->found_inf = orc_found_nonfinite(g16, n, dtype);
  rep->sqnorm = orc_sqnorm(g16, n, dtype, sigma, S, threads);
  if (!step_scalars(hp, sc, st, rep)) return;
  if (use_f32seq) {
    float c[9];
    orc_consts_f32(hp, st->t, rep->grad_mult, c);
    orc_adamw_f32seq(c, g16, w, m, v, p16, n, dtype, threads, no_decay);
  } else {
    orc_adamw_f64(hp, st->t, rep->grad_mult, g16, w, m, v, p16, n, dtype, threads, no_decay);
  }
  step_grow(sc, st, rep);
}

// ---- gradient accumulation in fp32 (micro-batches) ----------------------------------
// Not in the paper, whose gradients are the 16-bit array of the model state; a variant of the
// same path: the 16-bit gradients of several micro-batches are summed into an fp32 array of
// the same layout, and norm, clipping and update read that array.
//   overwrite: acc[i] = decode(src[i])           (first micro-batch)
//   else:      acc[i] = acc[i] + decode(src[i])  (one binary32 addition)
void orc_accum_f32(const uint16_t* src, uint64_t n, int dtype, int overwrite, float* acc) {
  for (uint64_t i = 0; i < n; ++i) {
    float x = decode16(src[i], dtype);
    acc[i] = overwrite ? x : acc[i] + x;
  }
}

int32_t orc_found_nonfinite_f32(const float* g, uint64_t n) {
  for (uint64_t i = 0; i < n; ++i)
    if (!std::isfinite(g[i])) return 1;
  return 0;
}

// As orc_sqnorm, over binary32 gradients.
double orc_sqnorm_f32(const float* g, uint64_t n, double loss_scale, uint64_t block, int threads) {
  if (n == 0) return 0.0;
  if (block == 0) block = n;
  uint64_t nb = (n + block - 1) / block;
  std::vector<double> part(nb, 0.0);
  parallel_ranges(nb, threads, [&](uint64_t b0, uint64_t b1) {
    for (uint64_t b = b0; b < b1; ++b) {
      uint64_t lo = b * block, hi = std::min(n, lo + block);
      double s = 0.0;
      for (uint64_t i = lo; i < hi; ++i) {
        double x = double(g[i]) / loss_scale;
        s += x * x;
      }
      part[b] = s;
    }
  });
  double total = 0.0;
  for (uint64_t b = 0; b < nb; ++b) total += part[b];
  return total;
}

void orc_adamw_f64_g32(const orc_hparams* hp, int32_t t, double grad_mult, const float* g32,
                       float* w, float* m, float* v, uint16_t* p16, uint64_t n, int dtype,
                       int threads, const uint8_t* no_decay) {
  adamw_f64_any(hp, t, grad_mult, [=](uint64_t i) { return double(g32[i]); }, w, m, v, p16, n, dtype, threads,
                no_decay);
}

void orc_adamw_f32seq_g32(const float* c, const float* g32, float* w, float* m, float* v,
                          uint16_t* p16, uint64_t n, int dtype, int threads, const uint8_t* no_decay) {
  adamw_f32seq_any(c, [=](uint64_t i) { return g32[i]; }, w, m, v, p16, n, dtype, threads, no_decay);
}

// orc_step over accumulated binary32 gradients (dtype is that of the 16-bit parameters).
void orc_step_g32(const orc_hparams* hp, const orc_scaler_cfg* sc, orc_state* st, const float* g32,
                  float* w, float* m, float* v, uint16_t* p16, uint64_t n, uint64_t S, int dtype,
                  int use_f32seq, int threads, orc_report* rep, const uint8_t* no_decay) {
  const double sigma = st->loss_scale;
  rep->loss_scale_used = sigma;
  rep->found_inf = orc_found_nonfinite_f32(g32, n);
  rep->sqnorm = orc_sqnorm_f32(g32, n, sigma, S, threads);
  if (!step_scalars(hp, sc, st, rep)) return;
  if (use_f32seq) {
    float c[9];
    orc_consts_f32(hp, st->t, rep->grad_mult, c);
    orc_adamw_f32seq_g32(c, g32, w, m, v, p16, n, dtype, threads, no_decay);
  } else {
    orc_adamw_f64_g32(hp, st->t, rep->grad_mult, g32, w, m, v, p16, n, dtype, threads, no_decay);
  }
  step_grow(sc, st, rep);
}

int orc_hardware_threads(void) {
  unsigned h = std::thread::hardware_concurrency();
  return h ? int(h) : 1;
}

}  // extern "C"
