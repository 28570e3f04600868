// Gradient quantisation (Sec. 2.1, Appendix A): amax + scale update, scaled saturating FP8 cast with the
// auto-scaling state, delayed scaling, and the shared-scale re-quantisation and FP8 sum of Eq. 4-6.
#ifndef FP8LM_QUANTIZE_HPP
#define FP8LM_QUANTIZE_HPP

#include "walk.hpp"

namespace fp8lm {

// ================================================================================================
// Kernel 1: per-tensor amax of a bf16 buffer, then the scale update (Appendix A.2; Sec. 2.1 Eq. 3)
// ================================================================================================
// |x| of a bf16 is monotone in (bits & 0x7FFF), so the maximum is taken on packed 16-bit integers:
// exact, order independent, and inf/NaN show up as a result >= 0x7F80.
enum : int { kAmaxForGradient = 0, kAmaxForMaster = 1 };

// The high-precision source of a cast: bf16, IEEE half or fp32 (Sec. 2.1 casts "high-precision"
// gradients).  |x| is monotone in the magnitude bits of all three, so the amax is an integer maximum;
// for the 16-bit types two maxima are kept packed in one register.
enum : int { kSrcBF16 = 0, kSrcF16 = 1, kSrcF32 = 2 };
template <int SRC> struct SrcTraits;
template <> struct SrcTraits<kSrcBF16> {
  using elem_t = uint16_t;
  static constexpr uint32_t kNonfinite = 0x7F80u;
  static __device__ __forceinline__ float dec(uint32_t bits) { return u2f(bits << 16); }
};
template <> struct SrcTraits<kSrcF16> {
  using elem_t = uint16_t;
  static constexpr uint32_t kNonfinite = 0x7C00u;
  static __device__ __forceinline__ float dec(uint32_t bits) { return f16_to_f32(bits); }
};
template <> struct SrcTraits<kSrcF32> {
  using elem_t = uint32_t;
  static constexpr uint32_t kNonfinite = 0x7F800000u;
  static __device__ __forceinline__ float dec(uint32_t bits) { return u2f(bits); }
};
template <int SRC> constexpr bool kSrc16 = sizeof(typename SrcTraits<SRC>::elem_t) == 2;
template <int SRC> constexpr int kSrcWords = kSrc16<SRC> ? 8 : 16;     // 32-bit words of a 16-element group
// folds one 32-bit word of the source (two 16-bit elements or one fp32) into a running maximum
template <int SRC> __device__ __forceinline__ void src_fold(uint32_t& acc, uint32_t word) {
  if constexpr (kSrc16<SRC>)
    acc = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, acc),
                                                                 __builtin_bit_cast(ushort2_t, word & 0x7FFF7FFFu)));
  else
    acc = max(acc, word & 0x7FFFFFFFu);
}
// the same for a single element given by its bit pattern
template <int SRC> __device__ __forceinline__ void src_fold1(uint32_t& acc, uint32_t bits) {
  if constexpr (kSrc16<SRC>) acc = (acc & 0xFFFF0000u) | max(acc & 0xFFFFu, bits & 0x7FFFu);
  else acc = max(acc, bits & 0x7FFFFFFFu);
}
template <int SRC> __device__ __forceinline__ uint32_t src_final(uint32_t acc) {
  if constexpr (kSrc16<SRC>) return max(acc & 0xFFFFu, acc >> 16);
  else return acc;
}

struct AmaxParams {
  const void* src;
  fp8lm_meta* meta;
  uint32_t fmax_bits;     // gradient mode: largest finite value of the target format
  int32_t hist_window;
  int32_t margin;
};

// Scale of a gradient tensor from the amax history as it stands: the largest of the last H entries,
// times 2^(mu_exp - margin).  Returns the flags (amax zero / clamped) and leaves the scale alone
// when the history is all zero.
__device__ __forceinline__ uint32_t scale_from_history(fp8lm_meta& M, uint32_t fmax_bits, int hist_window, int margin) {
  const int H = hist_window < 1 ? 1 : (hist_window > FP8LM_HIST ? FP8LM_HIST : hist_window);
  float Aeff = 0.0f;
  for (int h = 0; h < H; ++h) Aeff = M.amax_hist[h] > Aeff ? M.amax_hist[h] : Aeff;
  if (Aeff == 0.0f) return FP8LM_FLAG_AMAX_ZERO;
  uint32_t flags = 0;
  const int k = pow2_exp(fmax_bits, Aeff) + M.mu_exp - margin;
  const int e = k < -126 ? -126 : (k > 126 ? 126 : k);
  if (e != k) flags |= FP8LM_FLAG_SCALE_CLAMPED;
  M.scale = pow2f(e);
  M.inv_scale = pow2f(-e);
  return flags;
}
__device__ __forceinline__ void push_history(fp8lm_meta& M, float A, int hist_window) {
  const int H = hist_window < 1 ? 1 : (hist_window > FP8LM_HIST ? FP8LM_HIST : hist_window);
  const int slot = M.hist_pos % H;
  M.amax_hist[slot] = A;
  M.hist_pos = (slot + 1) % H;
}

template <int MODE, int SRC>
struct AmaxOp {
  using elem_t = typename SrcTraits<SRC>::elem_t;
  static constexpr int kPer = 16 / (int)sizeof(elem_t);   // elements per 128-bit load
  static constexpr int kLoads = kGroup / kPer;            // loads per thread and tile
  const AmaxParams& p;
  const Tables& tb;
  uint32_t acc;   // running maximum of the magnitude bits (two packed maxima for 16-bit sources)
  __device__ AmaxOp(const AmaxParams& p_, const Tables& tb_) : p(p_), tb(tb_), acc(0) {}
  __device__ __forceinline__ void begin(int, const TensorDesc&) { acc = 0; }
  __device__ __forceinline__ bool fast() const { return true; }
  template <int UN> __device__ __forceinline__ void tiles(long long pos) {
    // a pure reduction: each load instruction of a wavefront covers 1 KiB contiguous
    uint4 r[UN][kLoads];
    const elem_t* q = static_cast<const elem_t*>(p.src) + pos + threadIdx.x * kPer;
#pragma unroll
    for (int u = 0; u < UN; ++u)
#pragma unroll
      for (int k = 0; k < kLoads; ++k) r[u][k] = ld16<kNtLoadRO>(q + u * kTile + k * (kThreads * kPer));
#pragma unroll
    for (int u = 0; u < UN; ++u)
#pragma unroll
      for (int k = 0; k < kLoads; ++k) {
        src_fold<SRC>(acc, r[u][k].x);
        src_fold<SRC>(acc, r[u][k].y);
        src_fold<SRC>(acc, r[u][k].z);
        src_fold<SRC>(acc, r[u][k].w);
      }
  }
  // 16 consecutive elements at `pos`, by this thread alone
  __device__ __forceinline__ void full_group(long long pos) {
    const elem_t* q = static_cast<const elem_t*>(p.src) + pos;
    uint4 r[kLoads];
#pragma unroll
    for (int k = 0; k < kLoads; ++k) r[k] = ld16<kNtLoadRO>(q + k * kPer);
#pragma unroll
    for (int k = 0; k < kLoads; ++k) {
      src_fold<SRC>(acc, r[k].x);
      src_fold<SRC>(acc, r[k].y);
      src_fold<SRC>(acc, r[k].z);
      src_fold<SRC>(acc, r[k].w);
    }
  }
  __device__ __forceinline__ void group(long long pos, int valid) {
    const elem_t* q = static_cast<const elem_t*>(p.src) + pos;
    for (int j = 0; j < valid; ++j) src_fold1<SRC>(acc, q[j]);
  }
  using Stats = BlockStats<1, 0>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.mx[0] = src_final<SRC>(acc);
    s.orv = 0;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  // scalar epilogue, one thread per tensor
  __device__ void finalize(int t, const TensorDesc&, const Stats& s) {
    const uint32_t abits = s.mx[0];
    fp8lm_meta& M = p.meta[t];
    if constexpr (MODE == kAmaxForMaster) {
      // an initialisation has no earlier scale to keep: zero tensors, non-finite ones and unscaled formats get 1
      M.scale = 1.0f;
      M.inv_scale = 1.0f;
    }
    if (abits >= SrcTraits<SRC>::kNonfinite) {
      M.amax = __builtin_inff();
      M.flags = FP8LM_FLAG_NONFINITE;
      return;
    }
    const float A = SrcTraits<SRC>::dec(abits);
    M.amax = A;
    uint32_t flags = 0;
    if constexpr (MODE == kAmaxForGradient) {
      push_history(M, A, p.hist_window);
      M.flags = scale_from_history(M, p.fmax_bits, p.hist_window, p.margin);
    } else {
      // master weights: one binade of headroom; flags and the rest are completed by the cast pass
      if (A == 0.0f) {
        flags |= FP8LM_FLAG_AMAX_ZERO;
      } else if (p.fmax_bits != 0u) {      // 0: BF16 / FP32 master weights carry no scale
        const int k = pow2_exp(p.fmax_bits, A) - 1;
        const int e = k < -126 ? -126 : (k > 126 ? 126 : k);
        if (e != k) flags |= FP8LM_FLAG_SCALE_CLAMPED;
        M.scale = pow2f(e);
        M.inv_scale = pow2f(-e);
      }
      M.flags = flags;
    }
  }
};

template <int MODE, int SRC>
__global__ __launch_bounds__(kThreads) void amax_kernel(Tables tb, AmaxParams p) {
  AmaxOp<MODE, SRC> op(p, tb);
  walk_chunks<FP8LM_UN_READ>(tb, op);
}

// ================================================================================================
// Kernel 2: scaled saturating FP8 cast + auto-scaling state (Sec. 2.1; Appendix A.1)
// ================================================================================================
// The auto-scaling state machine of Sec. 2.1 (text after Eq. 3), shared by the cast and the sum.
// mu_rule 0: an overflow sets mu to 1/2; mu then follows the count of clean steps (1/2, 1, 2 as it passes
// 0, ramp_steps/2, ramp_steps).  mu_rule 1, the other reading of the same sentence: every overflowing step
// halves mu down to 2^mu_min_exp, every ramp_steps/2 clean steps in a row double it up to 2.
struct AutoscaleRule {
  int32_t sat_num, sat_den, ramp_steps, mu_rule, mu_min_exp;
};
__device__ __forceinline__ void autoscale_update(fp8lm_meta& M, unsigned long long n_sat, long long numel,
                                                 const AutoscaleRule& a) {
  const int R = a.ramp_steps < 2 ? 2 : a.ramp_steps;
  const bool overflow = (long long)n_sat * (long long)a.sat_den > numel * (long long)a.sat_num;
  if (a.mu_rule == 1) {
    if (overflow) {
      M.mu_exp = M.mu_exp - 1 < a.mu_min_exp ? a.mu_min_exp : M.mu_exp - 1;
      M.clean_steps = 0;
    } else if (M.clean_steps + 1 >= R / 2) {
      M.mu_exp = M.mu_exp + 1 > 1 ? 1 : M.mu_exp + 1;
      M.clean_steps = 0;
    } else {
      M.clean_steps = M.clean_steps + 1;
    }
    return;
  }
  const int clean = overflow ? 0 : (M.clean_steps + 1 > R ? R : M.clean_steps + 1);
  M.clean_steps = clean;
  const int ramp = (2 * clean) / R;
  M.mu_exp = -1 + (ramp > 2 ? 2 : ramp);
}

struct CastParams {
  const void* src;
  uint8_t* dst;
  fp8lm_meta* meta;
  AutoscaleRule rule;
  int32_t hist_window;   // delayed scaling and speculation
  int32_t speculative;   // DELAYED pass of the speculative just-in-time quantisation (see CastOp::speculation_verdict)
  uint32_t fmax_bits;    // speculation: largest finite value of the target format
  int32_t margin;
  // fused first pass of the Adam step (FUSE): the first moment as it stands and beta1
  const uint8_t* m;
  const fp8lm_meta* m_meta;
  float b1, omb1;
};

// number of non-zero bytes among the four 7-bit fields of x (each byte of x must be <= 0x7F)
__device__ __forceinline__ uint32_t nonzero_bytes7(uint32_t x) { return __popc((x + 0x7F7F7F7Fu) & 0x80808080u); }

// DELAYED: the scale was fixed from the amax history before the launch (Appendix A.2, delayed
// scaling); this pass also measures the amax of the source for the history, and since no amax pass
// has looked for inf/NaN it checks every 16-element group itself.
// FUSE: on one GPU the Adam step follows the cast directly, so this pass also measures what the Adam
// step's first pass would: max |fma(beta1, m, (1-beta1) * g)| with g the value just stored in FP8.
template <int FMT, bool DELAYED, bool FUSE, int SRC>
struct CastOp {
  using elem_t = typename SrcTraits<SRC>::elem_t;
  static constexpr int kPer = 16 / (int)sizeof(elem_t);   // elements per 128-bit load
  static constexpr int kLoads = kGroup / kPer;            // loads per 16-element group
  static constexpr int kW = kSrcWords<SRC>;
  const CastParams& p;
  const Tables& tb;
  float scale;
  bool careful;
  float inv_sg, inv_sm;   // FUSE
  uint32_t macc;          // FUSE: running max of the |m'| bit patterns
  uint32_t amax16;        // DELAYED: running maximum of the source's magnitude bits (packed pair for 16-bit types)
  float vmax;             // max |clamped scaled value|
  uint32_t n_elems;       // elements seen (full groups * 16 + tails) since the last flush
  uint32_t nz_top;        // codes whose magnitude differs from the top code
  uint32_t nz_code;       // codes with non-zero magnitude
  uint32_t z_in;          // inputs that are +-0
  __device__ CastOp(const CastParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void reset() { vmax = 0.0f; n_elems = nz_top = nz_code = z_in = 0; amax16 = 0; macc = 0; }
  __device__ __forceinline__ void begin(int t, const TensorDesc&) {
    scale = p.meta[t].scale;
    careful = !DELAYED && (p.meta[t].flags & FP8LM_FLAG_NONFINITE) != 0;
    if constexpr (FUSE) {
      inv_sg = p.meta[t].inv_scale;
      inv_sm = p.m_meta[t].inv_scale;
    }
    reset();
  }
  // FUSE: the new first moment of one element, from the decoded FP8 gradient and moment codes
  __device__ __forceinline__ void moment(float dg, float dm) {
    const float g = dg * inv_sg, m0 = dm * inv_sm;
    const float m1 = __builtin_fmaf(p.b1, m0, p.omb1 * g);
    macc = max(macc, f2u(m1) & 0x7FFFFFFFu);
  }
  __device__ __forceinline__ void moment_word(uint32_t gw, uint32_t mw) {
    const float2_t g01 = fp8x2_to_f32<FMT, false>(gw), g23 = fp8x2_to_f32<FMT, true>(gw);
    const float2_t m01 = fp8x2_to_f32<kE4M3, false>(mw), m23 = fp8x2_to_f32<kE4M3, true>(mw);
    moment(g01.x, m01.x);
    moment(g01.y, m01.y);
    moment(g23.x, m23.x);
    moment(g23.y, m23.y);
  }
  // DELAYED: folds one group's source bits into the running amax; true if the group holds inf or NaN
  __device__ __forceinline__ bool note_source(const uint32_t (&w)[kW]) {
    uint32_t gm = 0;
#pragma unroll
    for (int j = 0; j < kW; ++j) src_fold<SRC>(gm, w[j]);
    if constexpr (kSrc16<SRC>)
      amax16 = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, amax16),
                                                                      __builtin_bit_cast(ushort2_t, gm)));
    else
      amax16 = max(amax16, gm);
    return src_final<SRC>(gm) >= SrcTraits<SRC>::kNonfinite;
  }
  // four consecutive elements of a group (quad q = 0..3) widened to fp32
  __device__ __forceinline__ uint32_t quad(const uint32_t (&w)[kW], int q) {
    float f0, f1, f2, f3;
    if constexpr (SRC == kSrcBF16) {
      f0 = bf16lo_to_f32(w[2 * q]); f1 = bf16hi_to_f32(w[2 * q]);
      f2 = bf16lo_to_f32(w[2 * q + 1]); f3 = bf16hi_to_f32(w[2 * q + 1]);
    } else if constexpr (SRC == kSrcF16) {
      const float2_t lo = f16x2_to_f32(w[2 * q]), hi = f16x2_to_f32(w[2 * q + 1]);
      f0 = lo.x; f1 = lo.y; f2 = hi.x; f3 = hi.y;
    } else {
      f0 = u2f(w[4 * q]); f1 = u2f(w[4 * q + 1]); f2 = u2f(w[4 * q + 2]); f3 = u2f(w[4 * q + 3]);
    }
    const float y0 = clamp_fp8<FMT>(f0 * scale), y1 = clamp_fp8<FMT>(f1 * scale);
    const float y2 = clamp_fp8<FMT>(f2 * scale), y3 = clamp_fp8<FMT>(f3 * scale);
    vmax = fmaxf(fmaxf(vmax, fmaxf(fabsf(y0), fabsf(y1))), fmaxf(fabsf(y2), fabsf(y3)));
    z_in += (f0 == 0.0f) + (f1 == 0.0f) + (f2 == 0.0f) + (f3 == 0.0f);
    uint32_t c = f32x2_to_fp8<FMT, false>(y0, y1, 0u);
    c = f32x2_to_fp8<FMT, true>(y2, y3, c);
    const uint32_t mag = c & 0x7F7F7F7Fu;
    nz_code += nonzero_bytes7(mag);
    nz_top += nonzero_bytes7(mag ^ Fp8Traits<FMT>::kTopX4);
    return c;
  }
  __device__ __forceinline__ uint32_t one(uint32_t bits, uint32_t mcode) {
    const float f = SrcTraits<SRC>::dec(bits);
    const float y = f * scale;
    uint32_t c;
    if (y != y) {
      c = 0x7Fu;
    } else {
      const float yc = clamp_fp8<FMT>(y);
      vmax = fmaxf(vmax, fabsf(yc));
      c = f32x2_to_fp8<FMT, false>(yc, 0.0f, 0u) & 0xFFu;
    }
    z_in += (f == 0.0f);
    nz_code += (c & 0x7Fu) != 0;
    nz_top += (c & 0x7Fu) != Fp8Traits<FMT>::kTop;
    if constexpr (DELAYED) src_fold1<SRC>(amax16, bits);
    if constexpr (FUSE) moment(fp8_to_f32<FMT>(c), fp8_to_f32<kE4M3>(mcode));
    return c;
  }
  __device__ __forceinline__ bool fast() const { return !careful; }
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) { tiles_as<UN, FP8LM_CAST_SPLIT && kSrc16<SRC>>(pos0); }
  // kSplit: the thread's 16 elements are [8L, 8L+8) of each half of the tile (every 128-bit load contiguous
  // over the workgroup, 64-bit stores); otherwise 16 consecutive elements.
  template <int UN, bool kSplit> __device__ __forceinline__ void tiles_as(long long pos0) {
    uint4 r[UN][kLoads], mm[UN];
    const long long pos = pos0 + threadIdx.x * (kSplit ? 8 : kGroup);
    const elem_t* q = static_cast<const elem_t*>(p.src) + pos;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int k = 0; k < kLoads; ++k) r[u][k] = ld16<kNtLoadRO>(q + u * kTile + k * (kSplit ? kTile / 2 : kPer));
      if constexpr (FUSE) {
        if constexpr (kSplit) {
          const uint2 lo = ld8<kNtLoadRO>(p.m + pos + u * kTile), hi = ld8<kNtLoadRO>(p.m + pos + u * kTile + kTile / 2);
          mm[u] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        } else {
          mm[u] = ld16<kNtLoadRO>(p.m + pos + u * kTile);
        }
      }
    }
    // called by all lanes of a wavefront together (the 128-bit form exchanges halves between neighbouring lanes)
    auto store = [&](int u, const uint4& o) {
      if constexpr (kSplit && FP8LM_CAST_STORE16) {
        // lanes 2k and 2k+1 hold 8 codes each of both halves of the tile: the even lane takes the pair's 16 codes
        // of the first half, the odd lane those of the second half, and each stores once with 128 bits
        const bool odd = (threadIdx.x & 1) != 0;
        const uint32_t g0 = (uint32_t)__shfl_xor((int)(odd ? o.x : o.z), 1, 64);
        const uint32_t g1 = (uint32_t)__shfl_xor((int)(odd ? o.y : o.w), 1, 64);
        const long long at = pos0 + u * kTile + (threadIdx.x & ~1) * 8 + (odd ? kTile / 2 : 0);
        st16<kNtStoreWO>(p.dst + at, odd ? make_uint4(g0, g1, o.z, o.w) : make_uint4(o.x, o.y, g0, g1));
      } else if constexpr (kSplit) {
        st8<kNtStoreWO>(p.dst + pos + u * kTile, make_uint2(o.x, o.y));
        st8<kNtStoreWO>(p.dst + pos + u * kTile + kTile / 2, make_uint2(o.z, o.w));
      } else {
        st16<kNtStoreWO>(p.dst + pos + u * kTile, o);
      }
    };
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      uint32_t w[kW];
#pragma unroll
      for (int k = 0; k < kLoads; ++k) {
        w[4 * k] = r[u][k].x; w[4 * k + 1] = r[u][k].y; w[4 * k + 2] = r[u][k].z; w[4 * k + 3] = r[u][k].w;
      }
      uint4 o = make_uint4(0, 0, 0, 0);
      bool slow = false;
      if constexpr (DELAYED) slow = note_source(w);
      if (slow) {             // rare: this group holds inf/NaN, encode it element by element
        const uint32_t mw[4] = {mm[u].x, mm[u].y, mm[u].z, mm[u].w};
        const uint32_t keep = amax16;
        uint32_t* ow = &o.x;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const uint32_t bits = kSrc16<SRC> ? (w[(j >> 1) % kW] >> ((j & 1) * 16)) & 0xFFFFu : w[j % kW];
          ow[j >> 2] |= one(bits, FUSE ? (mw[j >> 2] >> ((j & 3) * 8)) & 0xFFu : 0u) << ((j & 3) * 8);
        }
        amax16 = keep;
      } else {
        o.x = quad(w, 0);
        o.y = quad(w, 1);
        o.z = quad(w, 2);
        o.w = quad(w, 3);
        if constexpr (FUSE) {
          moment_word(o.x, mm[u].x);
          moment_word(o.y, mm[u].y);
          moment_word(o.z, mm[u].z);
          moment_word(o.w, mm[u].w);
        }
      }
      store(u, o);            // all lanes again: the store may exchange data between lanes
    }
    n_elems += UN * kGroup;
  }
  // 16 consecutive elements at `pos`, by this thread alone (the layout without the split)
  __device__ __forceinline__ void full_group(long long pos) { tiles_as<1, false>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    const elem_t* q = static_cast<const elem_t*>(p.src) + pos;
    for (int j = 0; j < valid; ++j) p.dst[pos + j] = (uint8_t)one(q[j], FUSE ? p.m[pos + j] : 0u);
    n_elems += valid;
  }
  using Stats = BlockStats<3, 2>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.mx[0] = f2u(vmax);
    s.mx[1] = src_final<SRC>(amax16);
    s.mx[2] = macc;
    s.ct[0] = n_elems - nz_top;                 // codes on the top magnitude
    s.ct[1] = (n_elems - nz_code) - z_in;       // zero codes that did not come from zero inputs
    s.orv = 0;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  __device__ void finalize(int t, const TensorDesc& d, const Stats& s) {
    const float vm = u2f(s.mx[0]);
    const uint32_t abits = s.mx[1];
    if constexpr (FUSE) tb.scratch[t].pend.amax_m_bits = s.mx[2];
    const unsigned long long n_sat = s.ct[0], n_und = s.ct[1];
    if constexpr (DELAYED) {
      if (p.speculative) {
        if (speculation_verdict(t, abits)) finish(t, d, vm, n_sat, n_und);
        return;
      }
      fp8lm_meta& M = p.meta[t];
      if (abits >= SrcTraits<SRC>::kNonfinite) {
        M.amax = __builtin_inff();
        M.flags |= FP8LM_FLAG_NONFINITE;
      } else {
        M.amax = SrcTraits<SRC>::dec(abits);
        push_history(M, M.amax, p.hist_window);
      }
    }
    finish(t, d, vm, n_sat, n_und);
  }
  // Speculative just-in-time quantisation (Appendix A.2): this pass has cast the tensor with the scale its amax
  // history predicted and measured the true amax on the way.  Now the metadata is brought to exactly what the amax
  // pass of the two-pass form would have left (scale from the true amax, history pushed, flags); if that scale is
  // the one the cast used, the codes already written are the just-in-time result and the caller finishes the cast's
  // bookkeeping; otherwise the tensor is marked to be cast again.  Returns true if the speculation held.
  __device__ bool speculation_verdict(int t, uint32_t abits) {
    fp8lm_meta& M = p.meta[t];
    Scratch& S = tb.scratch[t];
    const float used = M.scale;
    M.scale = S.old_scale;
    M.inv_scale = S.old_inv;
    bool held;
    if (abits >= SrcTraits<SRC>::kNonfinite) {
      M.amax = __builtin_inff();
      M.flags = FP8LM_FLAG_NONFINITE;       // the second cast takes the path that knows NaN
      held = false;
    } else {
      const float A = SrcTraits<SRC>::dec(abits);
      M.amax = A;
      push_history(M, A, p.hist_window);
      M.flags = scale_from_history(M, p.fmax_bits, p.hist_window, p.margin);
      held = M.scale == used;
    }
    S.redo = held ? 0u : 1u;
    return held;
  }
  __device__ void finish(int t, const TensorDesc& d, float vm, unsigned long long n_sat, unsigned long long n_und) {
    fp8lm_meta& M = p.meta[t];
    M.n_sat = n_sat;
    M.n_underflow = n_und;
    M.amax_deq = fp8_to_f32<FMT>(encode1_fp8<FMT>(vm)) * M.inv_scale;
    M.flags = n_sat ? (M.flags | FP8LM_FLAG_SATURATED) : (M.flags & ~FP8LM_FLAG_SATURATED);
    autoscale_update(M, n_sat, d.numel, p.rule);
  }
};

template <int FMT, bool DELAYED, bool FUSE, int SRC>
__global__ __launch_bounds__(kThreads) void cast_kernel(Tables tb, CastParams p) {
  CastOp<FMT, DELAYED, FUSE, SRC> op(p, tb);
  walk_chunks<FP8LM_UN_CAST>(tb, op);
}

// Speculative just-in-time quantisation, step 1: one thread per tensor keeps the scale the meta holds and sets the
// scale its amax history predicts (the rule of delayed scaling; with an all-zero history the scale stays).
__global__ void speculate_scale_kernel(const TensorDesc* desc, fp8lm_meta* meta, Scratch* scratch, int n, uint32_t fmax_bits,
                                       int hist_window, int margin) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n || desc[t].numel == 0) return;
  scratch[t].old_scale = meta[t].scale;
  scratch[t].old_inv = meta[t].inv_scale;
  scratch[t].redo = 0;
  meta[t].flags = scale_from_history(meta[t], fmax_bits, hist_window, margin);
}

// Step 3: the chunk list of the tensors whose speculation failed.  One workgroup scans the tensors in order and
// gives each marked tensor its run of chunks (first_chunk = chunks of the marked tensors before it); the others
// get none.  Also adds to the running totals that fp8lm_get_speculation_stats reports.
constexpr int kScanThreads = 1024;
__global__ __launch_bounds__(kScanThreads) void redo_scan_kernel(const TensorDesc* desc, const Scratch* scratch, TensorDesc* redo_desc,
                                                                 int n, int32_t* n_chunks_out, unsigned long long* totals) {
  __shared__ int l_scan[kScanThreads];
  __shared__ int l_base;
  if (threadIdx.x == 0) l_base = 0;
  __syncthreads();
  unsigned long long redone_elems = 0, redone_tensors = 0;
  for (int t0 = 0; t0 < n; t0 += kScanThreads) {
    const int t = t0 + threadIdx.x;
    TensorDesc d{};
    int c = 0;
    if (t < n) {
      d = desc[t];
      if (d.numel > 0 && scratch[t].redo) { c = d.n_chunks; redone_elems += (unsigned long long)d.numel; redone_tensors += 1; }
    }
    l_scan[threadIdx.x] = c;
    __syncthreads();
    for (int o = 1; o < kScanThreads; o <<= 1) {             // inclusive scan over the block
      const int add = threadIdx.x >= o ? l_scan[threadIdx.x - o] : 0;
      __syncthreads();
      l_scan[threadIdx.x] += add;
      __syncthreads();
    }
    const int base = l_base;
    if (t < n) {
      d.first_chunk = base + l_scan[threadIdx.x] - c;
      d.n_chunks = c;
      redo_desc[t] = d;
    }
    __syncthreads();
    if (threadIdx.x == kScanThreads - 1) l_base = base + l_scan[threadIdx.x];
    __syncthreads();
  }
  // totals: calls, tensors cast twice, elements cast twice (exact sums, one workgroup)
  __shared__ unsigned long long l_e[kScanThreads / 64], l_t[kScanThreads / 64];
  redone_elems = wave_sum_u64(redone_elems);
  redone_tensors = wave_sum_u64(redone_tensors);
  if ((threadIdx.x & 63) == 0) { l_e[threadIdx.x >> 6] = redone_elems; l_t[threadIdx.x >> 6] = redone_tensors; }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long e = 0, k = 0;
    for (int w = 0; w < kScanThreads / 64; ++w) { e += l_e[w]; k += l_t[w]; }
    *n_chunks_out = l_base;
    totals[0] += 1;
    totals[1] += k;
    totals[2] += e;
  }
}
// ... and its chunk table: workgroup t (and t + grid, ...) writes tensor t's id into its run of chunks.
__global__ void redo_fill_kernel(const TensorDesc* redo_desc, int32_t* chunk_tensor, int n) {
  for (int t = blockIdx.x; t < n; t += gridDim.x) {
    const TensorDesc d = redo_desc[t];
    for (int i = threadIdx.x; i < d.n_chunks; i += blockDim.x) chunk_tensor[d.first_chunk + i] = t;
  }
}

// Delayed scaling, step 1: one thread per tensor fixes the scale from the history before the cast.
__global__ void delayed_scale_kernel(const TensorDesc* desc, fp8lm_meta* meta, int n, uint32_t fmax_bits,
                                     int hist_window, int margin) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n || desc[t].numel == 0) return;
  meta[t].flags = scale_from_history(meta[t], fmax_bits, hist_window, margin);
}

// ================================================================================================
// Shared-scale re-quantisation and the FP8 gradient sum (Sec. 2.1, Eq. 4-6)
// ================================================================================================
constexpr int kMaxRanks = 128;      // rank pointers travel as kernel arguments (1 KiB)
constexpr int kUnrolledRanks = 8;   // rank counts up to this have a kernel of their own
struct RankMetas { const fp8lm_meta* m[kMaxRanks]; int32_t n_ranks; };
struct RankPayloads { const uint8_t* p[kMaxRanks]; int32_t n_ranks; };

// Eq. 4: one thread per tensor takes the smallest scale among the ranks.
__global__ void shared_scale_kernel(RankMetas rm, int n, float* shared) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  float s = rm.m[0][t].scale;
  for (int r = 1; r < rm.n_ranks; ++r) s = rm.m[r][t].scale < s ? rm.m[r][t].scale : s;
  shared[t] = s;
}

// Sec. 2.1, text after Eq. 3: the factor mu chosen from the summed gradient's statistic is what every rank
// applies to its next gradient.  One thread per tensor copies the auto-scaling state into the ranks' metas.
struct RankMetasOut { fp8lm_meta* m[kMaxRanks]; int32_t n_ranks; };
__global__ void autoscale_broadcast_kernel(const fp8lm_meta* from, RankMetasOut rm, int n) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  const int32_t mu_exp = from[t].mu_exp, clean = from[t].clean_steps;
  for (int r = 0; r < rm.n_ranks; ++r) {
    rm.m[r][t].mu_exp = mu_exp;
    rm.m[r][t].clean_steps = clean;
  }
}
// Sec. 2.1, Eq. 1-2: a fixed factor mu = 2^mu_exp (pre-scaling 1/N, post-scaling 1) for every tensor.
__global__ void set_mu_kernel(fp8lm_meta* meta, int n, int32_t mu_exp) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) meta[t].mu_exp = mu_exp;
}

struct RequantParams {
  const uint8_t* src;
  const fp8lm_meta* src_meta;
  const float* shared;
  uint8_t* dst;
  fp8lm_meta* dst_meta;
};

// Eq. 5: dst = FP8(s_g * (src / s')).  Both scales are powers of two with s_g <= s': an exponent shift
// that can only lose bits at the bottom of the range.
template <int FMT>
struct RequantOp {
  const RequantParams& p;
  const Tables& tb;
  float inv_src, sg;
  bool careful;
  float vmax;
  uint32_t n_elems, nz_top, nz_code, nz_in, nonfinite;
  __device__ RequantOp(const RequantParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc&) {
    inv_src = p.src_meta[t].inv_scale;
    sg = p.shared[t];
    careful = (p.src_meta[t].flags & FP8LM_FLAG_NONFINITE) != 0;
    vmax = 0.0f;
    n_elems = nz_top = nz_code = nz_in = nonfinite = 0;
  }
  __device__ __forceinline__ bool fast() const { return !careful; }
  __device__ __forceinline__ uint32_t word(uint32_t w) {
    const float2_t a = fp8x2_to_f32<FMT, false>(w), b = fp8x2_to_f32<FMT, true>(w);
    const float y0 = (a.x * inv_src) * sg, y1 = (a.y * inv_src) * sg, y2 = (b.x * inv_src) * sg, y3 = (b.y * inv_src) * sg;
    vmax = fmaxf(fmaxf(vmax, fmaxf(fabsf(y0), fabsf(y1))), fmaxf(fabsf(y2), fabsf(y3)));
    const uint32_t c = encode4_fp8<FMT>(y0, y1, y2, y3);
    const uint32_t mag = c & 0x7F7F7F7Fu;
    nz_in += nonzero_bytes7(w & 0x7F7F7F7Fu);
    nz_code += nonzero_bytes7(mag);
    nz_top += nonzero_bytes7(mag ^ Fp8Traits<FMT>::kTopX4);
    return c;
  }
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) {
    uint4 a[UN];
    const long long pos = pos0 + threadIdx.x * kGroup;
#pragma unroll
    for (int u = 0; u < UN; ++u) a[u] = ld16<false>(p.src + pos + u * kTile);   // may be in place: cached loads
#pragma unroll
    for (int u = 0; u < UN; ++u) st16<false>(p.dst + pos + u * kTile, make_uint4(word(a[u].x), word(a[u].y), word(a[u].z), word(a[u].w)));
    n_elems += UN * kGroup;
  }
  // 16 consecutive elements at `pos`, by this thread alone: the tile body with the thread's own offset taken out
  __device__ __forceinline__ void full_group(long long pos) { tiles<1>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    for (int j = 0; j < valid; ++j) {
      const uint32_t in = p.src[pos + j];
      const float y = (fp8_to_f32<FMT>(in) * inv_src) * sg;
      const uint32_t c = encode1_fp8_careful<FMT>(y);
      if (y == y) vmax = fmaxf(vmax, fabsf(clamp_fp8<FMT>(y)));
      nonfinite |= !(fabsf(y) <= 3.4028234663852886e38f);
      nz_in += (in & 0x7Fu) != 0;
      nz_code += (c & 0x7Fu) != 0;
      nz_top += (c & 0x7Fu) != Fp8Traits<FMT>::kTop;
      p.dst[pos + j] = (uint8_t)c;
    }
    n_elems += valid;
  }
  using Stats = BlockStats<1, 2>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.mx[0] = f2u(vmax);
    s.ct[0] = n_elems - nz_top;
    s.ct[1] = nz_in - nz_code;                 // non-zero codes in, zero codes out (a NaN code is non-zero on both sides)
    s.orv = nonfinite;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  __device__ void finalize(int t, const TensorDesc&, const Stats& s) {
    const float vm = u2f(s.mx[0]);
    const unsigned long long n_sat = s.ct[0], n_und = s.ct[1];
    const uint32_t nf = s.orv;
    fp8lm_meta& M = p.dst_meta[t];
    const float src_amax = p.src_meta[t].amax;
    const float inv = 1.0f / sg;
    M.scale = sg;
    M.inv_scale = inv;
    M.amax = nf ? __builtin_inff() : src_amax;
    M.amax_deq = fp8_to_f32<FMT>(encode1_fp8<FMT>(vm)) * inv;
    M.n_sat = n_sat;
    M.n_underflow = n_und;
    M.flags = (nf ? FP8LM_FLAG_NONFINITE : 0u) | (n_sat ? FP8LM_FLAG_SATURATED : 0u);
  }
};

template <int FMT>
__global__ __launch_bounds__(kThreads) void requantize_kernel(Tables tb, RequantParams p) {
  RequantOp<FMT> op(p, tb);
  walk_chunks<2>(tb, op);
}

struct SumParams {
  RankPayloads in;
  const float* shared;
  uint8_t* dst;
  fp8lm_meta* dst_meta;
  AutoscaleRule rule;
};

// Eq. 6 on one GPU: the payloads of all ranks (same shared scale) are added in rank order in fp32 and
// rounded once to FP8, saturating; the result carries the scale N * s_g.
template <int FMT, int NR>
struct SumOp {
  const SumParams& p;
  const Tables& tb;
  float vmax;
  uint32_t amax_bits, n_elems, n_top, n_und;   // n_top / n_und: counted element by element (tails, NaN groups)
  uint32_t n_fast, nz_top, nz_code, z_acc;     // whole groups: counted on the packed codes, as in the cast
  __device__ SumOp(const SumParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int, const TensorDesc&) {
    vmax = 0.0f;
    amax_bits = n_elems = n_top = n_und = n_fast = nz_top = nz_code = z_acc = 0;
  }
  __device__ __forceinline__ bool fast() const { return true; }
  __device__ __forceinline__ uint32_t finish_one(float acc) {
    const uint32_t c = encode1_fp8_careful<FMT>(acc);
    amax_bits = max(amax_bits, f2u(acc) & 0x7FFFFFFFu);
    if (acc == acc) vmax = fmaxf(vmax, fabsf(clamp_fp8<FMT>(acc)));
    n_top += (c & 0x7Fu) == Fp8Traits<FMT>::kTop;
    n_und += (acc != 0.0f) && ((c & 0x7Fu) == 0);
    return c;
  }
  // four sums without a NaN among them: clamp, convert in pairs, count on the packed codes
  __device__ __forceinline__ uint32_t finish_quad(const float* acc) {
    const float y0 = clamp_fp8<FMT>(acc[0]), y1 = clamp_fp8<FMT>(acc[1]);
    const float y2 = clamp_fp8<FMT>(acc[2]), y3 = clamp_fp8<FMT>(acc[3]);
    vmax = fmaxf(fmaxf(vmax, fmaxf(fabsf(y0), fabsf(y1))), fmaxf(fabsf(y2), fabsf(y3)));
    amax_bits = max(max(amax_bits, max(f2u(acc[0]) & 0x7FFFFFFFu, f2u(acc[1]) & 0x7FFFFFFFu)),
                    max(f2u(acc[2]) & 0x7FFFFFFFu, f2u(acc[3]) & 0x7FFFFFFFu));
    z_acc += (acc[0] == 0.0f) + (acc[1] == 0.0f) + (acc[2] == 0.0f) + (acc[3] == 0.0f);
    uint32_t c = f32x2_to_fp8<FMT, false>(y0, y1, 0u);
    c = f32x2_to_fp8<FMT, true>(y2, y3, c);
    const uint32_t mag = c & 0x7F7F7F7Fu;
    nz_code += nonzero_bytes7(mag);
    nz_top += nonzero_bytes7(mag ^ Fp8Traits<FMT>::kTopX4);
    return c;
  }
  // one rank's 16 payloads added to the running sums: rank order, one fp32 addition per rank
  __device__ __forceinline__ void add_rank(float* acc, const uint4& a) {
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float2_t lo = fp8x2_to_f32<FMT, false>(w[k]), hi = fp8x2_to_f32<FMT, true>(w[k]);
      acc[4 * k + 0] = acc[4 * k + 0] + lo.x;
      acc[4 * k + 1] = acc[4 * k + 1] + lo.y;
      acc[4 * k + 2] = acc[4 * k + 2] + hi.x;
      acc[4 * k + 3] = acc[4 * k + 3] + hi.y;
    }
  }
  // rounds 16 sums to FP8 and stores them
  __device__ __forceinline__ void finish_group(const float* acc, long long pos) {
    bool any_nan = false;
#pragma unroll
    for (int j = 0; j < kGroup; ++j) any_nan |= acc[j] != acc[j];
    uint32_t o[4] = {0, 0, 0, 0};
    if (!any_nan) {
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = finish_quad(acc + 4 * k);
      n_fast += kGroup;
    } else {
#pragma unroll
      for (int j = 0; j < kGroup; ++j) o[j >> 2] |= finish_one(acc[j]) << ((j & 3) * 8);
    }
    st16<kNtStoreWO>(p.dst + pos, make_uint4(o[0], o[1], o[2], o[3]));
  }
  // NR > 0: that many ranks, all loads of UN tiles issued up front.  NR == 0: any number of ranks
  // (p.in.n_ranks), loaded eight at a time.
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) {
    const long long pos = pos0 + threadIdx.x * kGroup;
    if constexpr (NR == 0) {
      const int n = p.in.n_ranks;
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        float acc[kGroup];
#pragma unroll
        for (int j = 0; j < kGroup; ++j) acc[j] = 0.0f;
        for (int r0 = 0; r0 < n; r0 += kUnrolledRanks) {
          uint4 a[kUnrolledRanks];
#pragma unroll
          for (int k = 0; k < kUnrolledRanks; ++k)
            if (r0 + k < n) a[k] = ld16<kNtLoadRO>(p.in.p[r0 + k] + pos + u * kTile);
#pragma unroll
          for (int k = 0; k < kUnrolledRanks; ++k)
            if (r0 + k < n) add_rank(acc, a[k]);
        }
        finish_group(acc, pos + u * kTile);
      }
    } else {
      uint4 a[UN][NR > 0 ? NR : 1];
#pragma unroll
      for (int u = 0; u < UN; ++u)
#pragma unroll
        for (int r = 0; r < NR; ++r) a[u][r] = ld16<kNtLoadRO>(p.in.p[r] + pos + u * kTile);
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        float acc[kGroup];
#pragma unroll
        for (int j = 0; j < kGroup; ++j) acc[j] = 0.0f;
#pragma unroll
        for (int r = 0; r < NR; ++r) add_rank(acc, a[u][r]);
        finish_group(acc, pos + u * kTile);
      }
    }
    n_elems += UN * kGroup;
  }
  // 16 consecutive elements at `pos`, by this thread alone: the tile body with the thread's own offset taken out
  __device__ __forceinline__ void full_group(long long pos) { tiles<1>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    for (int j = 0; j < valid; ++j) {
      float acc = 0.0f;
      const int n = NR > 0 ? NR : p.in.n_ranks;
      for (int r = 0; r < n; ++r) acc = acc + fp8_to_f32<FMT>(p.in.p[r][pos + j]);
      p.dst[pos + j] = (uint8_t)finish_one(acc);
    }
    n_elems += valid;
  }
  using Stats = BlockStats<2, 2>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.mx[0] = f2u(vmax);
    s.mx[1] = amax_bits;
    s.ct[0] = n_top + (n_fast - nz_top);              // codes on the top magnitude
    s.ct[1] = n_und + ((n_fast - nz_code) - z_acc);   // zero codes that did not come from zero sums
    s.orv = 0;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  __device__ void finalize(int t, const TensorDesc& d, const Stats& s) {
    const float vm = u2f(s.mx[0]);
    const uint32_t ab = s.mx[1];
    const unsigned long long n_sat = s.ct[0], n_under = s.ct[1];
    fp8lm_meta& M = p.dst_meta[t];
    const float sc_out = (float)p.in.n_ranks * p.shared[t];
    const bool nf = ab >= 0x7F800000u;
    M.scale = sc_out;
    M.inv_scale = 1.0f / sc_out;
    M.amax = nf ? __builtin_inff() : u2f(ab) * M.inv_scale;
    M.amax_deq = fp8_to_f32<FMT>(encode1_fp8<FMT>(vm)) * M.inv_scale;
    M.n_sat = n_sat;
    M.n_underflow = n_under;
    M.flags = (nf ? FP8LM_FLAG_NONFINITE : 0u) | (n_sat ? FP8LM_FLAG_SATURATED : 0u);
    autoscale_update(M, n_sat, d.numel, p.rule);
  }
};

template <int FMT, int NR>
__global__ __launch_bounds__(kThreads) void sum_fp8_kernel(Tables tb, SumParams p) {
  SumOp<FMT, NR> op(p, tb);
  walk_chunks<(NR == 0 ? 1 : NR <= 2 ? 4 : NR <= 4 ? 2 : 1)>(tb, op);   // about eight 128-bit loads in flight per thread
}

}  // namespace fp8lm

#endif
