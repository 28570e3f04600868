// CPU oracle for the FP8 gradient cast + FP8 Adam step of FP8-LM (arXiv 2310.18313).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, scalar, obviously-correct statement of what
// the GPU path must compute.  Only the test-suite, the smoke check and the benchmark's
// cpu_baseline leg may load it.  It shares no code, header, table or constant generator with the
// HIP library: every struct below is declared here on its own, and the layout merely has to agree
// with the library's because both describe the same device-resident metadata.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fPIC -shared   (no -ffast-math; one rounding per
// written operation; std::fmaf only where a fused multiply-add is written).
//
// What the paper fixes and where:
//   * the two FP8 encodings, their largest values 448 / 57344 and which of them has inf
//     (Appendix A.1 and its range table);
//   * "scaling tensor" semantics: stored payload = value * scale, value = payload / scale
//     (Sec. 2.1, the paragraph before Eq. 4; Appendix A.2);
//   * just-in-time scaling = scale from the amax of the tensor being cast (Appendix A.2);
//   * the auto-scaling factor mu with its 0.001 % saturation threshold, the drop to 1/2 and the
//     ramp to 2 over 1000 steps (Sec. 2.1, Eq. 3 and the paragraph after it);
//   * the optimizer's storage types: FP8 gradient, FP8 first moment, FP16 second moment, FP16
//     master weight with tensor scaling (Sec. 2.2, Eq. 8), AdamW with beta1 .9, beta2 .95,
//     weight decay .1 (Sec. 3.1.2).
// What the paper leaves open (rounding mode, scale formula, eps placement, how each scale is
// refreshed) follows the readings stated at each function below; each says
// which reading it takes.
//
// Parity pins (tests marked "not gpu"): decode tables against the paper's printed range table and
// numpy's IEEE half; encoders against a brute-force nearest-value search and a library FP8 cast;
// FP16 conversion against numpy; amax against a float loop; the Adam recurrences against float64
// closed forms.  PARITY UNPINNED: the mu state machine and the v / master-weight / weight-copy
// scale refresh rules have no printed example or closed form; they are held only by invariants.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>

namespace {

inline uint32_t f32_bits(float x) { uint32_t u; std::memcpy(&u, &x, 4); return u; }
inline float bits_f32(uint32_t u) { float x; std::memcpy(&x, &u, 4); return x; }

// Description of a small binary floating-point format with IEEE-style subnormals.
struct SmallFmt {
  int mbits;        // explicit mantissa bits
  int bias;         // exponent bias
  uint32_t maxcode; // magnitude code of the largest finite value
  float fmax;       // that value
  uint32_t nancode; // canonical NaN magnitude code
};

// Appendix A.1: E4M3 = 1/4/3 bits, largest value 448, NaN but no infinity.
constexpr SmallFmt kE4M3{3, 7, 0x7E, 448.0f, 0x7F};
// Appendix A.1: E5M2 = 1/5/2 bits, largest value 57344, has +-inf and NaN.
constexpr SmallFmt kE5M2{2, 15, 0x7B, 57344.0f, 0x7F};
// IEEE half: 1/5/10, largest finite 65504 (range table, FP16 row).
constexpr SmallFmt kF16{10, 15, 0x7BFF, 65504.0f, 0x7E00};

// Round a non-negative finite fp32 below fmt.fmax (given by its bit pattern) to the nearest
// magnitude code of `fmt`, ties to the even code.
uint32_t round_mag_rne(uint32_t abits, const SmallFmt& fmt) {
  const int e32 = int(abits >> 23);
  if (e32 == 0) return 0;                       // fp32 zero/subnormal: far below every format's half-ulp
  const int E = e32 - 127;                      // value = sig * 2^(E-23), sig in [2^23, 2^24)
  const uint32_t sig = (abits & 0x7FFFFFu) | 0x800000u;
  const int emin = 1 - fmt.bias;                // exponent of the smallest normal
  int shift = 23 - fmt.mbits;                   // bits dropped for a normal result
  if (E < emin) shift += emin - E;              // subnormal result: drop more
  if (shift > 25) return 0;                     // below half of the smallest subnormal
  uint32_t q = sig >> shift;
  const uint32_t rem = sig & ((1u << shift) - 1u);
  const uint32_t half = 1u << (shift - 1);
  if (rem > half || (rem == half && (q & 1u))) q += 1;
  if (E < emin) return q;                       // q == 2^mbits lands exactly on the smallest normal
  // normal: q in [2^mbits, 2^(mbits+1)]; a mantissa carry walks into the exponent field
  return (uint32_t(E + fmt.bias) << fmt.mbits) + (q - (1u << fmt.mbits));
}

// Saturating round-to-nearest-even encoder: NaN -> canonical NaN code (sign dropped),
// |x| >= fmax (incl. inf) -> sign | maxcode, else nearest code, -0 keeps its sign.
uint32_t encode_sat(float x, const SmallFmt& fmt, int total_bits) {
  const uint32_t b = f32_bits(x);
  const uint32_t abits = b & 0x7FFFFFFFu;
  if (abits > 0x7F800000u) return fmt.nancode;
  const uint32_t sign = (b >> 31) << (total_bits - 1);
  if (bits_f32(abits) >= fmt.fmax) return sign | fmt.maxcode;
  return sign | round_mag_rne(abits, fmt);       // a < fmax never rounds past the top code
}

float decode_small(uint32_t code, int ebits, int mbits, int bias, bool has_inf, int total_bits) {
  const uint32_t s = (code >> (total_bits - 1)) & 1u;
  const uint32_t e = (code >> mbits) & ((1u << ebits) - 1u);
  const uint32_t f = code & ((1u << mbits) - 1u);
  const uint32_t emax = (1u << ebits) - 1u;
  float mag;
  if (has_inf && e == emax) {
    mag = f == 0 ? std::numeric_limits<float>::infinity() : std::numeric_limits<float>::quiet_NaN();
  } else if (!has_inf && e == emax && f == (1u << mbits) - 1u) {
    mag = std::numeric_limits<float>::quiet_NaN();
  } else if (e == 0) {
    mag = std::ldexp(float(f), 1 - bias - mbits);
  } else {
    mag = std::ldexp(float((1u << mbits) + f), int(e) - bias - mbits);
  }
  return s ? -mag : mag;
}

inline float dec_e4m3(uint8_t c) { return decode_small(c, 4, 3, 7, false, 8); }
inline float dec_e5m2(uint8_t c) { return decode_small(c, 5, 2, 15, true, 8); }
inline float dec_f16(uint16_t c) { return decode_small(c, 5, 10, 15, true, 16); }
inline float dec_bf16(uint16_t c) { return bits_f32(uint32_t(c) << 16); }
inline uint8_t enc_e4m3(float x) { return uint8_t(encode_sat(x, kE4M3, 8)); }
inline uint8_t enc_e5m2(float x) { return uint8_t(encode_sat(x, kE5M2, 8)); }
inline uint16_t enc_f16_sat(float x) { return uint16_t(encode_sat(x, kF16, 16)); }

// fp32 -> bf16, round to nearest even, IEEE overflow to inf, NaN -> 0x7FC0.
uint16_t enc_bf16(float x) {
  const uint32_t b = f32_bits(x);
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
  return uint16_t((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

inline float dec_fp8(int fmt, uint8_t c) { return fmt == 0 ? dec_e4m3(c) : dec_e5m2(c); }
inline uint8_t enc_fp8(int fmt, float x) { return fmt == 0 ? enc_e4m3(x) : enc_e5m2(x); }
inline uint32_t maxcode_fp8(int fmt) { return fmt == 0 ? kE4M3.maxcode : kE5M2.maxcode; }
inline float fmax_fp8(int fmt) { return fmt == 0 ? kE4M3.fmax : kE5M2.fmax; }

// The power-of-two scale rule: for A > 0 finite, the unique integer k with
//   2^k * A <= fmax < 2^(k+1) * A.
// Written with frexp in double so that fp32 subnormal A needs no special case.
int pow2_exp(float fmax, float A) {
  int ea, ef;
  const double ma = std::frexp(double(A), &ea);     // A    = ma * 2^ea, ma in [0.5, 1)
  const double mf = std::frexp(double(fmax), &ef);  // fmax = mf * 2^ef
  return ma <= mf ? ef - ea : ef - ea - 1;
}

inline int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

}  // namespace

extern "C" {

// ---- metadata, declared independently of the library's header (same byte layout) -------------
enum { ORACLE_HIST = 16 };
enum { ORACLE_FLAG_NONFINITE = 1u, ORACLE_FLAG_AMAX_ZERO = 2u, ORACLE_FLAG_SCALE_CLAMPED = 4u,
       ORACLE_FLAG_SATURATED = 8u };

typedef struct { int64_t offset; int64_t numel; } oracle_tensor;

typedef struct {
  float scale;       // power of two; stored payload = value * scale
  float inv_scale;   // exact reciprocal
  float amax;        // max |value| before quantisation (+inf when a non-finite value was seen)
  float amax_deq;    // max |stored payload| / scale over the non-NaN stored codes
  float amax_hist[ORACLE_HIST];
  int32_t hist_pos;
  int32_t mu_exp;      // log2 of the auto-scaling factor: -1, 0, +1
  int32_t clean_steps; // consecutive steps without overflow, capped at ramp_steps
  uint32_t flags;
  uint64_t n_sat;
  uint64_t n_underflow;
} oracle_meta;

typedef struct {
  int32_t sat_num, sat_den, ramp_steps, hist_window, margin;
  int32_t mu_rule;     // 0: the reading taken (set to 1/2, ramp back to 2); 1: the alternative (halve / double)
  int32_t mu_min_exp;  // rule 1: lowest log2(mu)
} oracle_autoscale_cfg;

typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  int64_t step;        // >= 1
  int32_t v_scaled;    // 1: second moment stored as scaled FP16; 0: plain FP16 (scale 1)
  int32_t wcopy;       // 0: E4M3 weight copy with its own scale; 1: bf16 weight copy
  int32_t m_predict;   // 0: first-moment scale from the exact amax of the new moment (just-in-time);
                       // 1: from the bound fma(beta1, amax_deq(m), (1-beta1) * amax_deq(g)), no extra pass
  // Storage formats of the precision-decoupling study (Sec. 3.3, the table of optimizer settings):
  int32_t master_fmt;  // 0 FP16 with tensor scaling (setting 2a, the default), 1 BF16 (2b), 2 E4M3 with
                       // tensor scaling (3), 3 FP32 (the alternative named in Sec. 2.2)
  int32_t v_fmt;       // 0 FP16 (scaled or plain as v_scaled says), 2 E4M3 with tensor scaling (setting 4)
} oracle_adam_hparams;

// ---- scalar format functions exported for the pins -------------------------------------------
float oracle_decode_e4m3(uint8_t c) { return dec_e4m3(c); }
float oracle_decode_e5m2(uint8_t c) { return dec_e5m2(c); }
float oracle_decode_f16(uint16_t c) { return dec_f16(c); }
float oracle_decode_bf16(uint16_t c) { return dec_bf16(c); }
uint8_t oracle_encode_e4m3(float x) { return enc_e4m3(x); }
uint8_t oracle_encode_e5m2(float x) { return enc_e5m2(x); }
uint16_t oracle_encode_f16_sat(float x) { return enc_f16_sat(x); }
uint16_t oracle_encode_bf16(float x) { return enc_bf16(x); }
int oracle_pow2_exp(float fmax, float A) { return pow2_exp(fmax, A); }

// Second, independent FP8 encoder: nearest of the finite non-negative code values by exhaustive
// search in double precision, ties to the even code.  Used only to pin the bit-level encoder.
uint8_t oracle_encode_fp8_nearest(int fmt, float x) {
  if (x != x) return 0x7F;
  const uint32_t sign = f32_bits(x) >> 31 << 7;
  const double a = std::fabs(double(x));
  const uint32_t top = maxcode_fp8(fmt);
  if (a >= double(fmax_fp8(fmt))) return uint8_t(sign | top);
  uint32_t best = 0;
  double best_d = a;  // distance to code 0 (value 0)
  for (uint32_t c = 1; c <= top; ++c) {
    const double d = std::fabs(a - double(dec_fp8(fmt, uint8_t(c))));
    if (d < best_d || (d == best_d && (c & 1u) == 0)) { best = c; best_d = d; }
  }
  return uint8_t(sign | best);
}

void oracle_encode_fp8_array(int fmt, const float* x, uint8_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = enc_fp8(fmt, x[i]);
}
void oracle_encode_fp8_nearest_array(int fmt, const float* x, uint8_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = oracle_encode_fp8_nearest(fmt, x[i]);
}
void oracle_encode_f16_sat_array(const float* x, uint16_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = enc_f16_sat(x[i]);
}
void oracle_encode_bf16_array(const float* x, uint16_t* out, int64_t n) {
  for (int64_t i = 0; i < n; ++i) out[i] = enc_bf16(x[i]);
}

// ---- metadata initial state ---------------------------------------------------------------------
// scale 1, empty history, mu = 1: the clean-step counter starts halfway up the ramp.
void oracle_meta_init(oracle_meta* meta, int32_t n, const oracle_autoscale_cfg* cfg) {
  for (int32_t t = 0; t < n; ++t) {
    oracle_meta& M = meta[t];
    std::memset(&M, 0, sizeof(M));
    M.scale = 1.0f;
    M.inv_scale = 1.0f;
    M.clean_steps = cfg->mu_rule == 1 ? 0 : cfg->ramp_steps / 2;
    M.mu_exp = 0;
  }
}

// ---- the auto-scaling state machine (Sec. 2.1, the paragraph after Eq. 3) ------------------------
// The statistic is the share of stored payloads on the largest finite code; "overflow" means it is above
// sat_num / sat_den (0.001 %).  The sentence that says what happens then is garbled; two readings:
//   rule 0 (taken by default): on overflow mu is SET to 1/2 and the count of clean steps restarts; mu is a
//     function of that count alone: 1/2 for the first ramp_steps/2 clean steps, 1 for the next
//     ramp_steps/2, 2 from ramp_steps on (the paper has mu grow exponentially back to 2 within a thousand steps).
//   rule 1 (alternative): every overflowing step HALVES mu, down to 2^mu_min_exp; every ramp_steps/2
//     clean steps in a row double it, up to 2.  Unlike rule 0 it can follow a sum that grows by more than 2.
// Takes effect in the next scale computation.
static void autoscale_step(oracle_meta& M, uint64_t n_sat, int64_t n, const oracle_autoscale_cfg* cfg) {
  const int R = cfg->ramp_steps < 2 ? 2 : cfg->ramp_steps;
  const bool overflow = int64_t(n_sat) * int64_t(cfg->sat_den) > n * int64_t(cfg->sat_num);
  if (cfg->mu_rule == 1) {
    if (overflow) {
      M.mu_exp = M.mu_exp - 1 < cfg->mu_min_exp ? cfg->mu_min_exp : M.mu_exp - 1;
      M.clean_steps = 0;
    } else if (++M.clean_steps >= R / 2) {
      M.mu_exp = M.mu_exp + 1 > 1 ? 1 : M.mu_exp + 1;
      M.clean_steps = 0;
    }
    return;
  }
  if (overflow) M.clean_steps = 0;
  else M.clean_steps = M.clean_steps + 1 > R ? R : M.clean_steps + 1;
  const int ramp = (2 * M.clean_steps) / R;
  M.mu_exp = -1 + (ramp > 2 ? 2 : ramp);
}

// ---- the high-precision source of a cast ------------------------------------------------------
// Gradients reach the cast as bf16, IEEE half or fp32 (Sec. 2.1 casts "high-precision" gradients;
// the mixed-precision baselines of Sec. 3.1 keep them in 16 or 32 bits).  Every one of them is
// widened to fp32 exactly before anything else happens.
enum { ORACLE_SRC_BF16 = 0, ORACLE_SRC_F16 = 1, ORACLE_SRC_F32 = 2 };
static float src_value(const void* src, int src_type, int64_t i) {
  if (src_type == ORACLE_SRC_F32) return static_cast<const float*>(src)[i];
  const uint16_t b = static_cast<const uint16_t*>(src)[i];
  return src_type == ORACLE_SRC_F16 ? dec_f16(b) : dec_bf16(b);
}

// ---- step a1 + a2: per-tensor amax of the gradient and the scale update -----------------------
// amax is just-in-time (Appendix A.2): it is taken over the tensor that is about to be cast.
// The scale is the largest power of two that keeps scale * amax_eff inside the target format,
// times the auto-scaling factor mu = 2^mu_exp (Sec. 2.1, Eq. 3: g' = mu * g), divided by
// 2^margin.  amax_eff is the largest of the hist_window most recent amax values (Appendix A.2,
// delayed scaling keeps such a history; a window of 1 is pure just-in-time scaling).
void oracle_amax_scale_src(const void* src, int src_type, const oracle_tensor* tensors, int32_t n_tensors,
                           int target_fmt, oracle_meta* meta, const oracle_autoscale_cfg* cfg) {
  for (int32_t t = 0; t < n_tensors; ++t) {
    const int64_t n = tensors[t].numel;
    if (n == 0) continue;
    const int64_t off = tensors[t].offset;
    oracle_meta& M = meta[t];
    bool nonfinite = false;
    float A = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
      const float a = std::fabs(src_value(src, src_type, off + i));
      if (!(a <= std::numeric_limits<float>::max())) nonfinite = true;  // inf or NaN
      else if (a > A) A = a;
    }
    uint32_t flags = 0;
    if (nonfinite) {
      M.amax = std::numeric_limits<float>::infinity();
      M.flags = ORACLE_FLAG_NONFINITE;  // scale and history left as they were
      continue;
    }
    M.amax = A;
    const int H = clampi(cfg->hist_window, 1, ORACLE_HIST);
    const int slot = M.hist_pos % H;
    M.amax_hist[slot] = A;
    M.hist_pos = (slot + 1) % H;
    float Aeff = 0.0f;
    for (int h = 0; h < H; ++h) Aeff = M.amax_hist[h] > Aeff ? M.amax_hist[h] : Aeff;
    if (Aeff == 0.0f) {
      flags |= ORACLE_FLAG_AMAX_ZERO;  // nothing to scale by: keep the previous scale
    } else {
      const int k = pow2_exp(fmax_fp8(target_fmt), Aeff) + M.mu_exp - cfg->margin;
      const int e = clampi(k, -126, 126);
      if (e != k) flags |= ORACLE_FLAG_SCALE_CLAMPED;
      M.scale = std::ldexp(1.0f, e);
      M.inv_scale = std::ldexp(1.0f, -e);
    }
    M.flags = flags;
  }
}
void oracle_amax_scale(const uint16_t* src_bf16, const oracle_tensor* tensors, int32_t n_tensors,
                       int target_fmt, oracle_meta* meta, const oracle_autoscale_cfg* cfg) {
  oracle_amax_scale_src(src_bf16, ORACLE_SRC_BF16, tensors, n_tensors, target_fmt, meta, cfg);
}

// ---- step a3 + a4: the scaled saturating cast and the auto-scaling state machine --------------
// payload = FP8(scale * g), round to nearest even, saturating (Sec. 2.1: the value is
// payload / scale).  The statistic of Sec. 2.1 is the share of payloads whose magnitude is the
// largest finite code; above sat_num/sat_den (0.001 %) the next step uses mu = 1/2, and after
// that mu climbs back one doubling per ramp_steps/2 clean steps until it reaches 2.
void oracle_cast_fp8_src(const void* src, int src_type, const oracle_tensor* tensors, int32_t n_tensors,
                         uint8_t* dst, int fmt, oracle_meta* meta, const oracle_autoscale_cfg* cfg) {
  const uint32_t top = maxcode_fp8(fmt);
  for (int32_t t = 0; t < n_tensors; ++t) {
    const int64_t n = tensors[t].numel;
    if (n == 0) continue;
    const int64_t off = tensors[t].offset;
    uint8_t* q = dst + tensors[t].offset;
    oracle_meta& M = meta[t];
    uint64_t n_sat = 0, n_under = 0;
    float stored_max = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
      const float x = src_value(src, src_type, off + i);
      const float y = x * M.scale;
      const uint8_t c = enc_fp8(fmt, y);
      q[i] = c;
      const uint32_t mag = c & 0x7Fu;
      if (mag == top) ++n_sat;
      if (x != 0.0f && mag == 0) ++n_under;   // a non-zero input (NaN included) stored as +-0
      const float d = std::fabs(dec_fp8(fmt, c));
      if (d == d && d > stored_max) stored_max = d;   // NaN codes carry no magnitude
    }
    M.n_sat = n_sat;
    M.n_underflow = n_under;
    M.amax_deq = stored_max * M.inv_scale;
    if (n_sat > 0) M.flags |= ORACLE_FLAG_SATURATED; else M.flags &= ~uint32_t(ORACLE_FLAG_SATURATED);
    autoscale_step(M, n_sat, n, cfg);
  }
}
void oracle_cast_fp8(const uint16_t* src_bf16, const oracle_tensor* tensors, int32_t n_tensors,
                     uint8_t* dst, int fmt, oracle_meta* meta, const oracle_autoscale_cfg* cfg) {
  oracle_cast_fp8_src(src_bf16, ORACLE_SRC_BF16, tensors, n_tensors, dst, fmt, meta, cfg);
}

// ---- delayed scaling for the gradient cast (Appendix A.2) --------------------------------------
// The scale comes from the amax values of preceding steps only (the history ring as it stands
// before this call), so amax and cast need a single pass over the data: the tensor is cast with
// that scale (saturating: a gradient that grew past the history clips and is counted in n_sat),
// and this step's amax is pushed into the ring for the steps to come.  An all-zero history (first
// step) keeps the scale that is already in the metadata.
void oracle_cast_fp8_delayed_src(const void* src, int src_type, const oracle_tensor* tensors, int32_t n_tensors,
                                 uint8_t* dst, int fmt, oracle_meta* meta, const oracle_autoscale_cfg* cfg) {
  const int H = clampi(cfg->hist_window, 1, ORACLE_HIST);
  for (int32_t t = 0; t < n_tensors; ++t) {
    const int64_t n = tensors[t].numel;
    if (n == 0) continue;
    oracle_meta& M = meta[t];
    // 1. scale from the history before this step
    uint32_t flags = 0;
    float Aeff = 0.0f;
    for (int h = 0; h < H; ++h) Aeff = M.amax_hist[h] > Aeff ? M.amax_hist[h] : Aeff;
    if (Aeff == 0.0f) {
      flags |= ORACLE_FLAG_AMAX_ZERO;
    } else {
      const int k = pow2_exp(fmax_fp8(fmt), Aeff) + M.mu_exp - cfg->margin;
      const int e = clampi(k, -126, 126);
      if (e != k) flags |= ORACLE_FLAG_SCALE_CLAMPED;
      M.scale = std::ldexp(1.0f, e);
      M.inv_scale = std::ldexp(1.0f, -e);
    }
    // 2. this step's amax, for the history
    const int64_t off = tensors[t].offset;
    bool nonfinite = false;
    float A = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
      const float a = std::fabs(src_value(src, src_type, off + i));
      if (!(a <= std::numeric_limits<float>::max())) nonfinite = true;
      else if (a > A) A = a;
    }
    if (nonfinite) {
      M.amax = std::numeric_limits<float>::infinity();
      flags |= ORACLE_FLAG_NONFINITE;
    } else {
      M.amax = A;
      const int slot = M.hist_pos % H;
      M.amax_hist[slot] = A;
      M.hist_pos = (slot + 1) % H;
    }
    M.flags = flags;
  }
  // 3. the cast itself, counters and the auto-scaling state: identical to the two-pass path
  oracle_cast_fp8_src(src, src_type, tensors, n_tensors, dst, fmt, meta, cfg);
}
void oracle_cast_fp8_delayed(const uint16_t* src_bf16, const oracle_tensor* tensors, int32_t n_tensors,
                             uint8_t* dst, int fmt, oracle_meta* meta, const oracle_autoscale_cfg* cfg) {
  oracle_cast_fp8_delayed_src(src_bf16, ORACLE_SRC_BF16, tensors, n_tensors, dst, fmt, meta, cfg);
}

// ---- shared-scale re-quantisation and the FP8 gradient sum (Sec. 2.1, Eq. 4-6) -------------------
// Eq. 4: the shared scale of a tensor is the smallest of the ranks' scales.
void oracle_shared_scale(const oracle_meta* const* metas, int32_t n_ranks, int32_t n_tensors, float* shared) {
  for (int32_t t = 0; t < n_tensors; ++t) {
    float s = metas[0][t].scale;
    for (int32_t r = 1; r < n_ranks; ++r) s = metas[r][t].scale < s ? metas[r][t].scale : s;
    shared[t] = s;
  }
}

// Eq. 5: g'' = FP8(s_g * (g' / s')).  Scales are powers of two and s_g <= s', so the value only moves
// down in exponent: nothing can saturate, small values may fall into the subnormals or to zero.
void oracle_requantize_fp8(const uint8_t* src, int fmt, const oracle_meta* src_meta, const float* shared,
                           const oracle_tensor* tensors, int32_t n_tensors, uint8_t* dst, oracle_meta* dst_meta) {
  const uint32_t top = maxcode_fp8(fmt);
  for (int32_t t = 0; t < n_tensors; ++t) {
    const int64_t n = tensors[t].numel;
    if (n == 0) continue;
    const int64_t off = tensors[t].offset;
    const float sg = shared[t];
    oracle_meta& M = dst_meta[t];
    uint64_t n_sat = 0, n_under = 0;
    float stored = 0.0f;
    bool nonfinite = false;
    for (int64_t i = 0; i < n; ++i) {
      const float value = dec_fp8(fmt, src[off + i]) * src_meta[t].inv_scale;   // g' / s'
      const uint8_t c = enc_fp8(fmt, value * sg);
      dst[off + i] = c;
      const float d = std::fabs(dec_fp8(fmt, c));
      if (d == d && d > stored) stored = d;
      if (!(std::fabs(value) <= std::numeric_limits<float>::max())) nonfinite = true;
      if ((c & 0x7Fu) == top) ++n_sat;
      if (value != 0.0f && (c & 0x7Fu) == 0) ++n_under;
    }
    const float inv = 1.0f / sg;           // exact: sg is a power of two
    M.scale = sg;
    M.inv_scale = inv;
    M.amax = nonfinite ? std::numeric_limits<float>::infinity() : src_meta[t].amax;
    M.amax_deq = stored * inv;
    M.n_sat = n_sat;
    M.n_underflow = n_under;
    M.flags = (nonfinite ? uint32_t(ORACLE_FLAG_NONFINITE) : 0u) | (n_sat ? uint32_t(ORACLE_FLAG_SATURATED) : 0u);
  }
}

// Eq. 6: g = g''_1 + ... + g''_N with scale N * s_g.  The payloads are added in rank order in an fp32
// accumulator and rounded once to FP8 (nearest even, saturating): sums that leave the FP8 range clip,
// which is what the auto-scaling statistic of Sec. 2.1 watches.
void oracle_sum_fp8(const uint8_t* const* payloads, int32_t n_ranks, int fmt, const float* shared,
                    const oracle_tensor* tensors, int32_t n_tensors, uint8_t* dst, oracle_meta* dst_meta,
                    const oracle_autoscale_cfg* cfg) {
  const uint32_t top = maxcode_fp8(fmt);
  for (int32_t t = 0; t < n_tensors; ++t) {
    const int64_t n = tensors[t].numel;
    if (n == 0) continue;
    const int64_t off = tensors[t].offset;
    oracle_meta& M = dst_meta[t];
    uint64_t n_sat = 0, n_under = 0;
    float stored = 0.0f, amax = 0.0f;
    bool nonfinite = false;
    for (int64_t i = 0; i < n; ++i) {
      float acc = 0.0f;
      for (int32_t r = 0; r < n_ranks; ++r) acc = acc + dec_fp8(fmt, payloads[r][off + i]);
      const uint8_t c = enc_fp8(fmt, acc);
      dst[off + i] = c;
      const float d = std::fabs(dec_fp8(fmt, c));
      if (d == d && d > stored) stored = d;
      const float a = std::fabs(acc);
      if (!(a <= std::numeric_limits<float>::max())) nonfinite = true; else if (a > amax) amax = a;
      if ((c & 0x7Fu) == top) ++n_sat;
      if (acc != 0.0f && (c & 0x7Fu) == 0) ++n_under;
    }
    const float s = float(n_ranks) * shared[t];
    M.scale = s;
    M.inv_scale = 1.0f / s;
    M.amax = nonfinite ? std::numeric_limits<float>::infinity() : amax * M.inv_scale;
    M.amax_deq = stored * M.inv_scale;
    M.n_sat = n_sat;
    M.n_underflow = n_under;
    M.flags = (nonfinite ? uint32_t(ORACLE_FLAG_NONFINITE) : 0u) | (n_sat ? uint32_t(ORACLE_FLAG_SATURATED) : 0u);
    autoscale_step(M, n_sat, n, cfg);
  }
}

// ---- storage formats of the optimizer state (precision decoupling, Sec. 2.2 and 3.3) ------------
enum { ST_F16 = 0, ST_BF16 = 1, ST_E4M3 = 2, ST_F32 = 3 };
static float st_decode(int kind, uint32_t code) {
  switch (kind) {
    case ST_F16: return dec_f16(uint16_t(code));
    case ST_BF16: return dec_bf16(uint16_t(code));
    case ST_E4M3: return dec_e4m3(uint8_t(code));
    default: return bits_f32(code);
  }
}
static uint32_t st_load(int kind, const void* buf, int64_t i) {
  switch (kind) {
    case ST_F16: case ST_BF16: return static_cast<const uint16_t*>(buf)[i];
    case ST_E4M3: return static_cast<const uint8_t*>(buf)[i];
    default: return static_cast<const uint32_t*>(buf)[i];
  }
}
static void st_store(int kind, void* buf, int64_t i, uint32_t code) {
  switch (kind) {
    case ST_F16: case ST_BF16: static_cast<uint16_t*>(buf)[i] = uint16_t(code); break;
    case ST_E4M3: static_cast<uint8_t*>(buf)[i] = uint8_t(code); break;
    default: static_cast<uint32_t*>(buf)[i] = code;
  }
}
// FP16 and E4M3 saturate; BF16 and FP32 follow IEEE (overflow to infinity), NaN is canonical
static uint32_t st_encode(int kind, float x) {
  switch (kind) {
    case ST_F16: return enc_f16_sat(x);
    case ST_BF16: return enc_bf16(x);
    case ST_E4M3: return enc_e4m3(x);
    default: return x != x ? 0x7FC00000u : f32_bits(x);
  }
}
static uint32_t st_mag(int kind, uint32_t code) {
  switch (kind) {
    case ST_F16: case ST_BF16: return code & 0x7FFFu;
    case ST_E4M3: return code & 0x7Fu;
    default: return code & 0x7FFFFFFFu;
  }
}
// the code counted by n_sat: the largest finite code of a saturating format, infinity otherwise
static uint32_t st_topcode(int kind) {
  switch (kind) {
    case ST_F16: return 0x7BFFu;
    case ST_BF16: return 0x7F80u;
    case ST_E4M3: return 0x7Eu;
    default: return 0x7F800000u;
  }
}
static bool st_scaled(int kind) { return kind == ST_F16 || kind == ST_E4M3; }
static float st_fmax(int kind) { return kind == ST_E4M3 ? kE4M3.fmax : kF16.fmax; }

// ---- master-weight initialisation ----------------------------------------------------------------
// Sec. 2.2: master weights are FP16 with tensor scaling.  The scale leaves one binade of
// headroom above the initial amax so that weights can grow between scale refreshes.
void oracle_init_master_as(const uint16_t* w_bf16, const oracle_tensor* tensors, int32_t n_tensors,
                           void* w_out, oracle_meta* w_meta, int master_fmt) {
  const int wk = master_fmt;
  for (int32_t t = 0; t < n_tensors; ++t) {
    const int64_t n = tensors[t].numel;
    if (n == 0) continue;
    const int64_t off = tensors[t].offset;
    const uint16_t* src = w_bf16 + off;
    oracle_meta& M = w_meta[t];
    bool nonfinite = false;
    float A = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
      const float a = std::fabs(dec_bf16(src[i]));
      if (!(a <= std::numeric_limits<float>::max())) nonfinite = true;
      else if (a > A) A = a;
    }
    uint32_t flags = 0;
    M.amax = nonfinite ? std::numeric_limits<float>::infinity() : A;
    // an initialisation has no earlier scale to keep: a tensor of zeros (biases), a non-finite one and the
    // formats without tensor scaling all get scale 1, whatever the caller's buffer held
    M.scale = 1.0f;
    M.inv_scale = 1.0f;
    if (nonfinite) flags |= ORACLE_FLAG_NONFINITE;
    else if (A == 0.0f) flags |= ORACLE_FLAG_AMAX_ZERO;
    else if (st_scaled(wk)) {
      const int k = pow2_exp(st_fmax(wk), A) - 1;
      const int e = clampi(k, -126, 126);
      if (e != k) flags |= ORACLE_FLAG_SCALE_CLAMPED;
      M.scale = std::ldexp(1.0f, e);
      M.inv_scale = std::ldexp(1.0f, -e);
    }
    float stored_max = 0.0f;
    uint64_t n_sat = 0, n_under = 0;
    for (int64_t i = 0; i < n; ++i) {
      const float x = dec_bf16(src[i]);
      const uint32_t c = st_encode(wk, x * M.scale);
      st_store(wk, w_out, off + i, c);
      const float d = std::fabs(st_decode(wk, c));
      if (d <= std::numeric_limits<float>::max() && d > stored_max) stored_max = d;
      if (st_mag(wk, c) == st_topcode(wk)) ++n_sat;
      if ((src[i] & 0x7FFFu) != 0 && st_mag(wk, c) == 0) ++n_under;
    }
    M.amax_deq = stored_max * M.inv_scale;
    M.n_sat = n_sat;
    M.n_underflow = n_under;
    if (n_sat > 0) flags |= ORACLE_FLAG_SATURATED;
    M.flags = flags;
  }
}

void oracle_init_master(const uint16_t* w_bf16, const oracle_tensor* tensors, int32_t n_tensors,
                        uint16_t* w_f16, oracle_meta* w_meta) {
  oracle_init_master_as(w_bf16, tensors, n_tensors, w_f16, w_meta, ST_F16);
}

// ---- step a5 + a6: the FP8 Adam step ---------------------------------------------------------
// Sec. 2.2 / Eq. 8: gradient FP8, first moment FP8 (E4M3 with a per-tensor scale), second moment
// FP16, master weight FP16 with tensor scaling; AdamW (Sec. 3.1.2) with bias correction and the
// usual sqrt(v_hat) + eps denominator.  All arithmetic in fp32; the update uses the fp32 moments
// before they are quantised for storage.
//
// Scales of the values written back:
//   first moment : just-in-time, from the exact amax of the new moment (Appendix A.2);
//   second moment: from the bound B_v = fma(beta2, amax_deq(v), (1-beta2) * amax_deq(g)^2), which
//                  by monotonicity of rounding is >= every new v, so the FP16 store never clips;
//   master weight: from the amax of the stored weights before the step, minus one binade;
//   weight copy  : E4M3 from the same amax without headroom (saturating), or plain bf16.
static void derive_hparams(const oracle_adam_hparams* hp, float& b1, float& omb1, float& rbc1,
                           float& b2, float& omb2, float& rbc2, float& decay) {
  b1 = hp->beta1;
  b2 = hp->beta2;
  omb1 = float(1.0 - double(b1));
  omb2 = float(1.0 - double(b2));
  rbc1 = float(1.0 / (1.0 - std::pow(double(b1), double(hp->step))));
  rbc2 = float(1.0 / (1.0 - std::pow(double(b2), double(hp->step))));
  decay = float(1.0 - double(hp->lr) * double(hp->weight_decay));
}

// Picks the stored scale of one output buffer from a magnitude bound.  Keeps the old scale when the
// bound is zero or not finite and reports why.
static void refresh_scale(float fmax, float bound, int headroom, float old_scale, float old_inv,
                          float& scale, float& inv, uint32_t& flags) {
  scale = old_scale;
  inv = old_inv;
  if (!(bound <= std::numeric_limits<float>::max())) { flags |= ORACLE_FLAG_NONFINITE; return; }
  if (bound == 0.0f) { flags |= ORACLE_FLAG_AMAX_ZERO; return; }
  const int k = pow2_exp(fmax, bound) - headroom;
  const int e = clampi(k, -126, 126);
  if (e != k) flags |= ORACLE_FLAG_SCALE_CLAMPED;
  scale = std::ldexp(1.0f, e);
  inv = std::ldexp(1.0f, -e);
}

void oracle_adam_step_fp8(const oracle_tensor* tensors, int32_t n_tensors,
                          const uint8_t* grad, int grad_fmt, const oracle_meta* grad_meta,
                          uint8_t* m, oracle_meta* m_meta,
                          void* v, oracle_meta* v_meta,
                          void* w, oracle_meta* w_meta,
                          void* wcopy, oracle_meta* wcopy_meta,
                          const oracle_adam_hparams* hp) {
  float b1, omb1, rbc1, b2, omb2, rbc2, decay;
  derive_hparams(hp, b1, omb1, rbc1, b2, omb2, rbc2, decay);
  const float lr = hp->lr, eps = hp->eps;
  const float INF = std::numeric_limits<float>::infinity();
  const int wk = hp->master_fmt, vk = hp->v_fmt;

  for (int32_t t = 0; t < n_tensors; ++t) {
    const int64_t n = tensors[t].numel;
    if (n == 0) continue;
    const int64_t off = tensors[t].offset;
    const uint8_t* qg = grad + off;
    uint8_t* qm = m + off;
    const float inv_sg = grad_meta[t].inv_scale;
    const float inv_sm = m_meta[t].inv_scale;
    const float inv_sv = v_meta[t].inv_scale;
    const float inv_sw = w_meta[t].inv_scale;

    // phase A: exact amax of the new first moment
    bool m_nonfinite = false;
    float A_m = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
      const float g = dec_fp8(grad_fmt, qg[i]) * inv_sg;
      const float m0 = dec_e4m3(qm[i]) * inv_sm;
      const float m1 = std::fmaf(b1, m0, omb1 * g);
      const float a = std::fabs(m1);
      if (!(a <= std::numeric_limits<float>::max())) m_nonfinite = true;
      else if (a > A_m) A_m = a;
    }

    // scales for the four writes
    uint32_t fm = 0, fv = 0, fw = 0, fq = 0;
    float sm, ism, sv, isv, sw, isw, sq, isq;
    if (hp->m_predict) {
      // Single-pass variant (Appendix A.2 names the extra passes as the cost of just-in-time scaling):
      // |m'| <= beta1 * max|m| + (1-beta1) * max|g|, and with monotone rounding the fp32 value of
      // that bound is >= every fp32 m', so the E4M3 store cannot clip.
      const float Bm = std::fmaf(b1, m_meta[t].amax_deq, omb1 * grad_meta[t].amax_deq);
      refresh_scale(kE4M3.fmax, Bm, 0, m_meta[t].scale, m_meta[t].inv_scale, sm, ism, fm);
    } else {
      refresh_scale(kE4M3.fmax, m_nonfinite ? INF : A_m, 0, m_meta[t].scale, m_meta[t].inv_scale, sm, ism, fm);
    }
    if (hp->v_scaled || vk == ST_E4M3) {
      const float Ag = grad_meta[t].amax_deq;
      const float Bv = std::fmaf(b2, v_meta[t].amax_deq, omb2 * (Ag * Ag));
      refresh_scale(st_fmax(vk), Bv, 0, v_meta[t].scale, v_meta[t].inv_scale, sv, isv, fv);
    } else {
      sv = 1.0f; isv = 1.0f;
    }
    if (st_scaled(wk)) {
      refresh_scale(st_fmax(wk), w_meta[t].amax_deq, 1, w_meta[t].scale, w_meta[t].inv_scale, sw, isw, fw);
    } else {
      sw = 1.0f; isw = 1.0f;       // BF16 and FP32 master weights carry no scale
    }
    if (hp->wcopy == 0) {
      refresh_scale(kE4M3.fmax, w_meta[t].amax_deq, 0, wcopy_meta[t].scale, wcopy_meta[t].inv_scale, sq, isq, fq);
    } else {
      sq = 1.0f; isq = 1.0f;
    }

    // phase B: the update
    bool v_nonfinite = false, w_nonfinite = false;
    float A_v = 0.0f, A_w = 0.0f;
    float st_m = 0.0f, st_v = 0.0f, st_w = 0.0f, st_q = 0.0f;       // max |stored payload|
    uint64_t sat_m = 0, sat_v = 0, sat_w = 0, sat_q = 0;
    uint64_t und_m = 0, und_v = 0, und_w = 0, und_q = 0;
    for (int64_t i = 0; i < n; ++i) {
      const float g = dec_fp8(grad_fmt, qg[i]) * inv_sg;
      const float m0 = dec_e4m3(qm[i]) * inv_sm;
      const float v0 = st_decode(vk, st_load(vk, v, off + i)) * inv_sv;
      const float w0 = st_decode(wk, st_load(wk, w, off + i)) * inv_sw;
      const float m1 = std::fmaf(b1, m0, omb1 * g);
      const float v1 = std::fmaf(b2, v0, omb2 * (g * g));
      const float den = std::sqrt(v1 * rbc2) + eps;
      const float upd = (m1 * rbc1) / den;
      const float w1 = std::fmaf(-lr, upd, w0 * decay);

      const uint8_t cm = enc_e4m3(m1 * sm);
      const uint32_t cv = st_encode(vk, v1 * sv);
      const uint32_t cw = st_encode(wk, w1 * sw);
      qm[i] = cm;
      st_store(vk, v, off + i, cv);
      st_store(wk, w, off + i, cw);

      float d;
      d = std::fabs(dec_e4m3(cm)); if (d == d && d > st_m) st_m = d;
      d = std::fabs(st_decode(vk, cv)); if (d <= std::numeric_limits<float>::max() && d > st_v) st_v = d;
      d = std::fabs(st_decode(wk, cw)); if (d <= std::numeric_limits<float>::max() && d > st_w) st_w = d;
      if ((cm & 0x7Fu) == kE4M3.maxcode) ++sat_m;
      if (st_mag(vk, cv) == st_topcode(vk)) ++sat_v;
      if (st_mag(wk, cw) == st_topcode(wk)) ++sat_w;
      if (m1 != 0.0f && (cm & 0x7Fu) == 0) ++und_m;
      if (v1 != 0.0f && st_mag(vk, cv) == 0) ++und_v;
      if (w1 != 0.0f && st_mag(wk, cw) == 0) ++und_w;

      float a = std::fabs(v1);
      if (!(a <= std::numeric_limits<float>::max())) v_nonfinite = true; else if (a > A_v) A_v = a;
      a = std::fabs(w1);
      if (!(a <= std::numeric_limits<float>::max())) w_nonfinite = true; else if (a > A_w) A_w = a;

      if (hp->wcopy == 0) {
        const uint8_t cq = enc_e4m3(w1 * sq);
        static_cast<uint8_t*>(wcopy)[off + i] = cq;
        d = std::fabs(dec_e4m3(cq)); if (d == d && d > st_q) st_q = d;
        if ((cq & 0x7Fu) == kE4M3.maxcode) ++sat_q;
        if (w1 != 0.0f && (cq & 0x7Fu) == 0) ++und_q;
      } else {
        const uint16_t cq = enc_bf16(w1);
        static_cast<uint16_t*>(wcopy)[off + i] = cq;
        d = std::fabs(dec_bf16(cq));
        if (d <= std::numeric_limits<float>::max() && d > st_q) st_q = d;
        if ((cq & 0x7FFFu) == 0x7F80u) ++sat_q;                 // rounded to infinity
        if (w1 != 0.0f && (cq & 0x7FFFu) == 0) ++und_q;
      }
    }

    auto finish = [&](oracle_meta& M, float scale, float inv, float amax, bool nonfinite,
                      float stored, uint64_t n_sat, uint64_t n_und, uint32_t flags) {
      M.scale = scale;
      M.inv_scale = inv;
      M.amax = nonfinite ? INF : amax;
      M.amax_deq = stored * inv;
      M.n_sat = n_sat;
      M.n_underflow = n_und;
      if (nonfinite) flags |= ORACLE_FLAG_NONFINITE;
      if (n_sat > 0) flags |= ORACLE_FLAG_SATURATED;
      M.flags = flags;
    };
    finish(m_meta[t], sm, ism, A_m, m_nonfinite, st_m, sat_m, und_m, fm);
    finish(v_meta[t], sv, isv, A_v, v_nonfinite, st_v, sat_v, und_v, fv);
    finish(w_meta[t], sw, isw, A_w, w_nonfinite, st_w, sat_w, und_w, fw);
    finish(wcopy_meta[t], sq, isq, A_w, w_nonfinite, st_q, sat_q, und_q, fq);
  }
}

// ---- quantisation error of an FP8 gradient against a high-precision reference -----------------------
// The quantities of the communication ablation (Sec. 3.3, the figure comparing pre-scaling,
// post-scaling and auto-scaling): per tensor, the signal-to-noise ratio of the FP8 gradient, the share
// of its entries that underflowed and the share that sits on the largest finite code.  The paper does
// not define them; the reading taken is the textbook one.  With r_i the reference and
// x_i = payload_i / scale the value the scaling tensor stands for (Sec. 2.1):
//   signal = sum r_i^2,  noise = sum (r_i - x_i)^2   (SNR = 10 log10(signal / noise), left to the caller),
//   n_nonzero = #{r_i != 0},  n_underflow = #{r_i != 0 and payload_i = +-0},
//   n_overflow = #{|payload_i| is the largest finite code}.
// Entries whose reference is inf/NaN or whose payload is a NaN/inf code are counted in n_nonfinite
// and take part in nothing else.  Sums are float64; x_i = double(payload_i) * (1.0 / double(scale)).
typedef struct {
  double signal, noise;
  uint64_t n_nonzero, n_underflow, n_overflow, n_nonfinite;
} oracle_quant_stats;

void oracle_quant_error_stats(const void* ref, int ref_type, const uint8_t* q, int fmt, const oracle_meta* meta,
                              const oracle_tensor* tensors, int32_t n_tensors, oracle_quant_stats* out) {
  const uint32_t top = maxcode_fp8(fmt);
  for (int32_t t = 0; t < n_tensors; ++t) {
    oracle_quant_stats S{};
    const int64_t off = tensors[t].offset;
    const double rs = 1.0 / double(meta[t].scale);
    for (int64_t i = 0; i < tensors[t].numel; ++i) {
      const float r = src_value(ref, ref_type, off + i);
      const uint8_t c = q[off + i];
      const float p = dec_fp8(fmt, c);
      if (!(std::fabs(r) <= std::numeric_limits<float>::max()) || !(std::fabs(p) <= std::numeric_limits<float>::max())) {
        ++S.n_nonfinite;
        continue;
      }
      const double x = double(p) * rs;
      const double e = double(r) - x;
      S.signal += double(r) * double(r);
      S.noise += e * e;
      const uint32_t mag = c & 0x7Fu;
      if (r != 0.0f) {
        ++S.n_nonzero;
        if (mag == 0) ++S.n_underflow;
      }
      if (mag == top) ++S.n_overflow;
    }
    out[t] = S;
  }
}

// ---- whole-tensor greedy distribution (Sec. 2.3, Alg. 1) -----------------------------------------
// Tensors are visited in descending order of size (equal sizes in their original order); each goes
// to the GPU with the least memory in use so far (the lowest-numbered one among equals).
void oracle_greedy_partition(const int64_t* sizes, int32_t n, int32_t n_gpus, int32_t* owner, int64_t* usage) {
  for (int32_t j = 0; j < n_gpus; ++j) usage[j] = 0;
  for (int32_t i = 0; i < n; ++i) owner[i] = -1;
  for (int32_t round = 0; round < n; ++round) {
    int32_t pick = -1;                       // the largest tensor not yet placed
    for (int32_t i = 0; i < n; ++i)
      if (owner[i] < 0 && (pick < 0 || sizes[i] > sizes[pick])) pick = i;
    int32_t j = 0;
    for (int32_t k = 1; k < n_gpus; ++k)
      if (usage[k] < usage[j]) j = k;
    owner[pick] = j;
    usage[j] += sizes[pick];
  }
}

// Derived host scalars, exported so a test can check them against float64 arithmetic.
void oracle_derive_hparams(const oracle_adam_hparams* hp, float* out7) {
  derive_hparams(hp, out7[0], out7[1], out7[2], out7[3], out7[4], out7[5], out7[6]);
}

uint32_t oracle_sizeof_meta(void) { return uint32_t(sizeof(oracle_meta)); }

}  // extern "C"
