// The FP8 Adam step (Sec. 2.2, Eq. 8; Sec. 3.1.2) and the master-weight initialisation: scale selection,
// the read-only first pass, the update pass, and the update pass for the other storage formats (Sec. 3.3).
#ifndef FP8LM_ADAM_HPP
#define FP8LM_ADAM_HPP

#include "walk.hpp"
#include "quantize.hpp"

namespace fp8lm {

// ================================================================================================
// Master-weight initialisation: bf16 -> scaled FP16 (Sec. 2.2)
// ================================================================================================
struct InitParams {
  const uint16_t* src;
  void* dst;
  fp8lm_meta* meta;
};

template <int MASTER>
struct InitCastOp {
  typedef StTraits<MASTER> WT;
  const InitParams& p;
  const Tables& tb;
  float scale;
  float vmax;
  uint32_t n_sat, n_und;
  bool careful;
  __device__ InitCastOp(const InitParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc&) {
    scale = p.meta[t].scale;
    careful = (p.meta[t].flags & FP8LM_FLAG_NONFINITE) != 0;   // set by the amax pass just before
    vmax = 0.0f;
    n_sat = n_und = 0;
  }
  __device__ __forceinline__ bool fast() const { return !careful; }
  // what the stored code of a (NaN-free) scaled value will be, for the counters
  __device__ __forceinline__ void note(float y, bool nonzero_in) {
    const uint32_t c = WT::enc(y);
    if constexpr (WT::kSaturating) vmax = fmaxf(vmax, fabsf(WT::dec(c)));
    else if (fabsf(WT::dec(c)) <= 3.4028234663852886e38f) vmax = fmaxf(vmax, fabsf(WT::dec(c)));
    n_sat += (c & WT::kMagMask) == WT::kTopCode;
    n_und += nonzero_in && ((c & WT::kMagMask) == 0);
  }
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) {
    static_assert(UN == 1, "one group at a time");
    const long long pos = pos0 + threadIdx.x * kGroup;
    const uint4 a = ld16<kNtLoadRO>(p.src + pos), b = ld16<kNtLoadRO>(p.src + pos + 8);
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    float y[kGroup];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      y[2 * k] = bf16lo_to_f32(w[k]) * scale;
      y[2 * k + 1] = bf16hi_to_f32(w[k]) * scale;
      note(y[2 * k], (w[k] & 0x7FFFu) != 0);
      note(y[2 * k + 1], (w[k] & 0x7FFF0000u) != 0);
    }
    st_store16<MASTER>(p.dst, pos, y);
  }
  // 16 consecutive elements at `pos`, by this thread alone: the tile body with the thread's own offset taken out
  __device__ __forceinline__ void full_group(long long pos) { tiles<1>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    for (int j = 0; j < valid; ++j) {
      const uint32_t bits = p.src[pos + j];
      const float y = u2f(bits << 16) * scale;
      const uint32_t h = WT::enc_careful(y);
      const float d = fabsf(WT::dec(h));
      if (d <= 3.4028234663852886e38f) vmax = fmaxf(vmax, d);
      n_sat += (h & WT::kMagMask) == WT::kTopCode;
      n_und += ((bits & 0x7FFFu) != 0) && ((h & WT::kMagMask) == 0);
      st_store1<MASTER>(p.dst, pos + j, h);
    }
  }
  using Stats = BlockStats<1, 2>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.mx[0] = f2u(vmax);
    s.ct[0] = n_sat;
    s.ct[1] = n_und;
    s.orv = 0;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  __device__ void finalize(int t, const TensorDesc&, const Stats& s) {
    const float vm = u2f(s.mx[0]);
    fp8lm_meta& M = p.meta[t];
    M.n_sat = s.ct[0];
    M.n_underflow = s.ct[1];
    M.amax_deq = vm * M.inv_scale;        // vm is already a stored value
    if (M.n_sat) M.flags |= FP8LM_FLAG_SATURATED;
  }
};

template <int MASTER>
__global__ __launch_bounds__(kThreads) void init_master_cast_kernel(Tables tb, InitParams p) {
  InitCastOp<MASTER> op(p, tb);
  walk_chunks<1>(tb, op);
}

// ================================================================================================
// Kernels 3 + 4: the FP8 Adam step (Sec. 2.2, Eq. 8; Sec. 3.1.2)
// ================================================================================================
struct AdamParams {
  const uint8_t* grad;
  const fp8lm_meta* grad_meta;
  uint8_t* m;              // first moment, written (and read, unless m_in points elsewhere)
  fp8lm_meta* m_meta;
  void* v;                 // FP16 (default) or E4M3
  fp8lm_meta* v_meta;
  void* w;                 // FP16 (default), BF16, E4M3 or FP32
  fp8lm_meta* w_meta;
  void* wcopy;
  fp8lm_meta* wcopy_meta;
  float b1, omb1, rbc1, b2, omb2, rbc2, lr, eps, decay;
  int32_t v_scaled;
  uint32_t v_fmax_bits;    // largest finite value of the second moment's storage format
  uint32_t w_fmax_bits;    // ... of the master weight's, 0 if that format carries no scale (BF16, FP32)
  const uint8_t* m_in;     // where the first moment is read: m itself (in place), or the other buffer of a pair
  int32_t speculative_m;   // the first-moment scale was predicted; the update pass's epilogue verifies it (see
                           // AdamUpdateOp::finish)
};

// Chooses a stored scale from a magnitude bound; keeps the old one when the bound is 0 or not finite.
__device__ __forceinline__ void refresh_scale(uint32_t fmax_bits, float bound, int headroom, float old_scale,
                                              float old_inv, float& scale, float& inv, uint32_t& flags) {
  scale = old_scale;
  inv = old_inv;
  if (!(bound <= 3.4028234663852886e38f)) { flags |= FP8LM_FLAG_NONFINITE; return; }
  if (bound == 0.0f) { flags |= FP8LM_FLAG_AMAX_ZERO; return; }
  const int k = pow2_exp(fmax_bits, bound) - headroom;
  const int e = k < -126 ? -126 : (k > 126 ? 126 : k);
  if (e != k) flags |= FP8LM_FLAG_SCALE_CLAMPED;
  scale = pow2f(e);
  inv = pow2f(-e);
}

// Chooses the scales of the four buffers the update pass writes, from a bound on the new first moment
// (its exact amax, or the predicted bound) and the metadata of the inputs; decides whether the tensor
// may take the fast update path.
template <int WCOPY>
__device__ void adam_choose_scales(const AdamParams& p, Scratch::Pending& P, int t, float bound_m) {
  const fp8lm_meta& G = p.grad_meta[t];
  const fp8lm_meta& Mm = p.m_meta[t];
  const fp8lm_meta& Mv = p.v_meta[t];
  const fp8lm_meta& Mw = p.w_meta[t];
  const fp8lm_meta& Mq = p.wcopy_meta[t];
  uint32_t fm = 0, fv = 0, fw = 0, fq = 0;
  refresh_scale(kBitsE4M3Max, bound_m, 0, Mm.scale, Mm.inv_scale, P.sm, P.ism, fm);
  if (p.v_scaled) {
    const float Ag = G.amax_deq;
    const float Bv = __builtin_fmaf(p.b2, Mv.amax_deq, p.omb2 * (Ag * Ag));
    refresh_scale(p.v_fmax_bits, Bv, 0, Mv.scale, Mv.inv_scale, P.sv, P.isv, fv);
  } else {
    P.sv = 1.0f;
    P.isv = 1.0f;
  }
  if (p.w_fmax_bits) {
    refresh_scale(p.w_fmax_bits, Mw.amax_deq, 1, Mw.scale, Mw.inv_scale, P.sw, P.isw, fw);
  } else {
    P.sw = 1.0f;
    P.isw = 1.0f;
  }
  if constexpr (WCOPY == FP8LM_WCOPY_E4M3) {
    refresh_scale(kBitsE4M3Max, Mw.amax_deq, 0, Mq.scale, Mq.inv_scale, P.sq, P.isq, fq);
  } else {
    P.sq = 1.0f;
    P.isq = 1.0f;
  }
  P.fm = fm; P.fv = fv; P.fw = fw; P.fq = fq;
  // The fast update path assumes that no NaN and no fp32 overflow can occur.  That holds when every
  // input magnitude is moderate; anything else takes the careful path, which checks every element.
  const float kBig = 1.0995116e12f;     // 2^40
  const float kHuge = 1.2089258e24f;    // 2^80
  const uint32_t anyflag = (G.flags | Mm.flags | Mv.flags | Mw.flags) & FP8LM_FLAG_NONFINITE;
  const bool calm = !anyflag && (bound_m < kBig) && (G.amax_deq < kBig) && (Mm.amax_deq < kBig) &&
                    (Mv.amax_deq < kHuge) && (Mw.amax_deq < kHuge);
  P.careful = calm ? 0u : 1u;
}

// Single-pass variant: the first-moment scale comes from the bound
// fma(beta1, amax_deq(m), (1-beta1) * amax_deq(g)) >= every new |m| (monotone rounding), so no pass
// over the data is needed before the update.  One thread per tensor.
template <int WCOPY>
__global__ void adam_predict_scales_kernel(Tables tb, AdamParams p, int n) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n || tb.desc[t].numel == 0) return;
  const float Bm = __builtin_fmaf(p.b1, p.m_meta[t].amax_deq, p.omb1 * p.grad_meta[t].amax_deq);
  adam_choose_scales<WCOPY>(p, tb.scratch[t].pend, t, Bm);
}

// The first pass was done by a fused cast: its result sits in the scratch.  One thread per tensor.
template <int WCOPY>
__global__ void adam_scales_from_cast_kernel(Tables tb, AdamParams p, int n) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n || tb.desc[t].numel == 0) return;
  const uint32_t bits = tb.scratch[t].pend.amax_m_bits;
  adam_choose_scales<WCOPY>(p, tb.scratch[t].pend, t, bits >= 0x7F800000u ? __builtin_inff() : u2f(bits));
}

// Speculative first-moment scale (the update pass verifies it): the scale that the previous step's exact amax gives,
// which is the one in the metadata unless that amax was zero or not finite.  The decision for the careful path cannot
// wait for the exact amax either: it is taken from the bound fma(beta1, amax_deq(m), (1-beta1) * amax_deq(g)), which
// no new |m| exceeds.  Keeps the scale the moment is stored with for the pass that repairs a failed speculation.
template <int WCOPY>
__global__ void adam_speculate_scales_kernel(Tables tb, AdamParams p, int n) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n || tb.desc[t].numel == 0) return;
  Scratch& S = tb.scratch[t];
  S.redo = 0;
  S.old_scale = p.m_meta[t].scale;
  S.old_inv = p.m_meta[t].inv_scale;
  adam_choose_scales<WCOPY>(p, S.pend, t, p.m_meta[t].amax);
  const float Bm = __builtin_fmaf(p.b1, p.m_meta[t].amax_deq, p.omb1 * p.grad_meta[t].amax_deq);
  if (!(Bm < 1.0995116e12f)) S.pend.careful = 1u;      // 2^40, as in adam_choose_scales
}

// ---- pass A: exact amax of the new first moment, then all four scales ---------------------------
template <int GFMT, int WCOPY>
struct AdamAmaxOp {
  const AdamParams& p;
  const Tables& tb;
  float inv_sg, inv_sm;
  uint32_t acc;
  __device__ AdamAmaxOp(const AdamParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc&) {
    inv_sg = p.grad_meta[t].inv_scale;
    inv_sm = p.m_meta[t].inv_scale;
    acc = 0;
  }
  __device__ __forceinline__ void elem(float dg, float dm) {
    const float g = dg * inv_sg, m0 = dm * inv_sm;
    const float m1 = __builtin_fmaf(p.b1, m0, p.omb1 * g);
    acc = max(acc, f2u(m1) & 0x7FFFFFFFu);
  }
  __device__ __forceinline__ void word(uint32_t gw, uint32_t mw) {
    const float2_t g01 = fp8x2_to_f32<GFMT, false>(gw), g23 = fp8x2_to_f32<GFMT, true>(gw);
    const float2_t m01 = fp8x2_to_f32<kE4M3, false>(mw), m23 = fp8x2_to_f32<kE4M3, true>(mw);
    elem(g01.x, m01.x);
    elem(g01.y, m01.y);
    elem(g23.x, m23.x);
    elem(g23.y, m23.y);
  }
  __device__ __forceinline__ bool fast() const { return true; }
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) {
    uint4 g[UN], m[UN];
    const long long pos = pos0 + threadIdx.x * kGroup;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      g[u] = ld16<kNtLoadRO>(p.grad + pos + u * kTile);
      m[u] = ld16<kNtLoadRO>(p.m + pos + u * kTile);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      word(g[u].x, m[u].x);
      word(g[u].y, m[u].y);
      word(g[u].z, m[u].z);
      word(g[u].w, m[u].w);
    }
  }
  // 16 consecutive elements at `pos`, by this thread alone: the tile body with the thread's own offset taken out
  __device__ __forceinline__ void full_group(long long pos) { tiles<1>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    for (int j = 0; j < valid; ++j) elem(fp8_to_f32<GFMT>(p.grad[pos + j]), fp8_to_f32<kE4M3>(p.m[pos + j]));
  }
  using Stats = BlockStats<1, 0>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.mx[0] = acc;
    s.orv = 0;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  __device__ void finalize(int t, const TensorDesc&, const Stats& s) {
    const uint32_t abits = s.mx[0];
    const bool m_nonfinite = abits >= 0x7F800000u;
    adam_choose_scales<WCOPY>(p, tb.scratch[t].pend, t, m_nonfinite ? __builtin_inff() : u2f(abits));
  }
};

template <int GFMT, int WCOPY>
__global__ __launch_bounds__(kThreads) void adam_amax_kernel(Tables tb, AdamParams p) {
  AdamAmaxOp<GFMT, WCOPY> op(p, tb);
  walk_chunks<FP8LM_UN_READ>(tb, op);
}

// ---- pass B: the update ----------------------------------------------------------------------------
// FAST: v_sqrt_f32 / v_rcp_f32 (1 ulp each) instead of correctly rounded sqrt and divide in the weight
// update; m and v are unaffected (multiply/fma only).  STATS: count n_sat / n_underflow per output.
template <bool FAST> __device__ __forceinline__ float adam_update(float m1, float v1, float w0, float decay, const AdamParams& p) {
  if constexpr (FAST) {
    const float den = __builtin_amdgcn_sqrtf(v1 * p.rbc2) + p.eps;
    const float upd = (m1 * p.rbc1) * __builtin_amdgcn_rcpf(den);
    return __builtin_fmaf(-p.lr, upd, w0 * decay);
  } else {
    const float den = __builtin_sqrtf(v1 * p.rbc2) + p.eps;
    const float upd = ((m1 * p.rbc1) / den);
    return __builtin_fmaf(-p.lr, upd, w0 * decay);
  }
}

template <int GFMT, int WCOPY, bool FAST, bool STATS>
struct AdamUpdateOp {
  const AdamParams& p;
  const Tables& tb;
  float inv_sg, inv_sm, inv_sv, inv_sw;   // scales of the inputs
  float sm, sv, sw, sq;                   // scales of the outputs
  float decay;                            // 1 - lr * weight_decay, or 1 for a tensor that is exempt
  bool careful;
  float vmax, wmax, mmax;                 // running maxima of v', |w'| (and |m'| on the careful path)
  uint32_t nf;
  uint32_t cnt[8];                        // sat m,v,w,q ; underflow m,v,w,q: per lane (tails, careful path)
  uint32_t wcnt[8];                       // the same for whole tiles: wave totals, identical in every lane
  __device__ AdamUpdateOp(const AdamParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc& d) {
    const Scratch::Pending& P = tb.scratch[t].pend;
    decay = (d.flags & FP8LM_TENSOR_NO_WEIGHT_DECAY) ? 1.0f : p.decay;
    inv_sg = p.grad_meta[t].inv_scale;
    inv_sm = p.m_meta[t].inv_scale;
    inv_sv = p.v_meta[t].inv_scale;
    inv_sw = p.w_meta[t].inv_scale;
    sm = P.sm; sv = P.sv; sw = P.sw; sq = P.sq;
    careful = P.careful != 0;
    vmax = wmax = mmax = 0.0f;
    nf = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) cnt[i] = wcnt[i] = 0;
  }

  // Exact counters, from the scaled values before clamping.  WAVE: called by all 64 lanes together (whole
  // tiles); a condition then costs one compare, the count of lanes that meet it is taken from the lane mask
  // with scalar instructions and kept once per wavefront instead of once per lane.
  template <bool WAVE> __device__ __forceinline__ void count(int i, bool cond) {
    if constexpr (WAVE) wcnt[i] += (uint32_t)__popcll(__ballot(cond));
    else cnt[i] += cond;
  }
  // both conditions hold; WAVE: the two lane masks are combined with one scalar instruction
  template <bool WAVE> __device__ __forceinline__ void count2(int i, bool a, bool b) {
    if constexpr (WAVE) wcnt[i] += (uint32_t)__popcll(__ballot(a) & __ballot(b));
    else cnt[i] += a && b;
  }
  template <bool WAVE>
  __device__ __forceinline__ void stats(float m1, float v1, float w1, float tm, float tv, float tw, float tq) {
    if constexpr (STATS) {
      count<WAVE>(0, fabsf(tm) >= 432.0f);                       // rounds to (or beyond) the top E4M3 code
      count<WAVE>(1, fabsf(tv) > 65488.0f);                      // rounds to the top FP16 code
      count<WAVE>(2, fabsf(tw) > 65488.0f);
      count2<WAVE>(4, fabsf(tm) <= 0x1p-10f, m1 != 0.0f);        // rounds to zero
      count2<WAVE>(5, fabsf(tv) <= 0x1p-25f, v1 != 0.0f);
      count2<WAVE>(6, fabsf(tw) <= 0x1p-25f, w1 != 0.0f);
      if constexpr (WCOPY == FP8LM_WCOPY_E4M3) {
        count<WAVE>(3, fabsf(tq) >= 432.0f);
        count2<WAVE>(7, fabsf(tq) <= 0x1p-10f, w1 != 0.0f);
      } else {
        const uint32_t ab = f2u(w1) & 0x7FFFFFFFu;
        count<WAVE>(3, (ab - 0x7F7F8000u) <= 0x8000u);          // 0x7F7F8000 .. 0x7F800000: rounds to infinity
        count<WAVE>(7, (ab - 1u) < 0x8000u);                    // 1 .. 0x8000: rounds to zero
      }
    }
  }

  struct Quad { uint32_t m, v01, v23, w01, w23, q, q2; };

  // four elements: one word of gradient codes, one of moment codes, two words each of v and w
  template <bool WAVE>
  __device__ __forceinline__ Quad quad(uint32_t gw, uint32_t mw, uint32_t v01, uint32_t v23, uint32_t w01, uint32_t w23) {
    const float2_t dg01 = fp8x2_to_f32<GFMT, false>(gw), dg23 = fp8x2_to_f32<GFMT, true>(gw);
    const float2_t dm01 = fp8x2_to_f32<kE4M3, false>(mw), dm23 = fp8x2_to_f32<kE4M3, true>(mw);
    const float2_t dv01 = f16x2_to_f32(v01), dv23 = f16x2_to_f32(v23);
    const float2_t dw01 = f16x2_to_f32(w01), dw23 = f16x2_to_f32(w23);
    const float dg[4] = {dg01.x, dg01.y, dg23.x, dg23.y};
    const float dm[4] = {dm01.x, dm01.y, dm23.x, dm23.y};
    const float dv[4] = {dv01.x, dv01.y, dv23.x, dv23.y};
    const float dw[4] = {dw01.x, dw01.y, dw23.x, dw23.y};
    float tm[4], tv[4], tw[4], tq[4], w1s[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float g = dg[j] * inv_sg, m0 = dm[j] * inv_sm, v0 = dv[j] * inv_sv, w0 = dw[j] * inv_sw;
      const float m1 = __builtin_fmaf(p.b1, m0, p.omb1 * g);
      const float v1 = __builtin_fmaf(p.b2, v0, p.omb2 * (g * g));
      const float w1 = adam_update<FAST>(m1, v1, w0, decay, p);
      vmax = fmaxf(vmax, v1);
      wmax = fmaxf(wmax, fabsf(w1));
      mmax = fmaxf(mmax, fabsf(m1));
      tm[j] = m1 * sm;
      tv[j] = v1 * sv;
      tw[j] = w1 * sw;
      tq[j] = w1 * sq;
      w1s[j] = w1;
      stats<WAVE>(m1, v1, w1, tm[j], tv[j], tw[j], tq[j]);
    }
    Quad o;
    o.m = encode4_fp8<kE4M3>(tm[0], tm[1], tm[2], tm[3]);
    o.v01 = encode2_f16(tv[0], tv[1]);
    o.v23 = encode2_f16(tv[2], tv[3]);
    o.w01 = encode2_f16(tw[0], tw[1]);
    o.w23 = encode2_f16(tw[2], tw[3]);
    if constexpr (WCOPY == FP8LM_WCOPY_E4M3) {
      o.q = encode4_fp8<kE4M3>(tq[0], tq[1], tq[2], tq[3]);
      o.q2 = 0;
    } else {
      o.q = encode1_bf16(w1s[0]) | (encode1_bf16(w1s[1]) << 16);
      o.q2 = encode1_bf16(w1s[2]) | (encode1_bf16(w1s[3]) << 16);
    }
    return o;
  }

  // one element with every special case handled (NaN codes, infinities, fp32 overflow)
  __device__ __forceinline__ void one_careful(long long i) {
    const float g = fp8_to_f32<GFMT>(p.grad[i]) * inv_sg;
    const float m0 = fp8_to_f32<kE4M3>(p.m_in[i]) * inv_sm;
    uint16_t* pv = static_cast<uint16_t*>(p.v);
    uint16_t* pw = static_cast<uint16_t*>(p.w);
    const float v0 = f16_to_f32(pv[i]) * inv_sv;
    const float w0 = f16_to_f32(pw[i]) * inv_sw;
    const float m1 = __builtin_fmaf(p.b1, m0, p.omb1 * g);
    const float v1 = __builtin_fmaf(p.b2, v0, p.omb2 * (g * g));
    const float den = __builtin_sqrtf(v1 * p.rbc2) + p.eps;
    const float upd = ((m1 * p.rbc1) / den);
    const float w1 = __builtin_fmaf(-p.lr, upd, w0 * decay);
    const float tm = m1 * sm, tv = v1 * sv, tw = w1 * sw, tq = w1 * sq;
    p.m[i] = (uint8_t)encode1_fp8_careful<kE4M3>(tm);
    pv[i] = (uint16_t)encode1_f16_careful(tv);
    pw[i] = (uint16_t)encode1_f16_careful(tw);
    if constexpr (WCOPY == FP8LM_WCOPY_E4M3) static_cast<uint8_t*>(p.wcopy)[i] = (uint8_t)encode1_fp8_careful<kE4M3>(tq);
    else static_cast<uint16_t*>(p.wcopy)[i] = (uint16_t)encode1_bf16(w1);
    const float kMaxF = 3.4028234663852886e38f;
    const float am = fabsf(m1), av = fabsf(v1), aw = fabsf(w1);
    if (am <= kMaxF) mmax = fmaxf(mmax, am); else nf |= (m1 != m1) ? 1u : 2u;
    if (av <= kMaxF) vmax = fmaxf(vmax, av); else nf |= (v1 != v1) ? 4u : 8u;
    if (aw <= kMaxF) wmax = fmaxf(wmax, aw); else nf |= (w1 != w1) ? 16u : 32u;
    stats<false>(m1, v1, w1, tm, tv, tw, tq);
  }

  __device__ __forceinline__ bool fast() const { return !careful; }
  // Split layout: the 16-bit streams are walked with 128-bit accesses that are contiguous over the whole
  // workgroup (4 KiB per instruction) instead of pairs of adjacent ones; the 8-bit streams then take
  // 64-bit accesses.  Measured 1.6 % faster in a memory-only skeleton of this kernel.
  template <int UN> __device__ __forceinline__ void tiles_split(long long tile0) {
    uint2 ga[UN], gb[UN], ma[UN], mb[UN];
    uint4 va[UN], vb[UN], wa[UN], wb[UN];
    const long long pos0 = tile0 + threadIdx.x * 8;
    uint16_t* pv = static_cast<uint16_t*>(p.v);
    uint16_t* pw = static_cast<uint16_t*>(p.w);
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const long long a = pos0 + u * kTile, b = a + kTile / 2;
      ga[u] = ld8<kNtLoadRO>(p.grad + a);
      gb[u] = ld8<kNtLoadRO>(p.grad + b);
      ma[u] = ld8<kNtLoadRW>(p.m_in + a);
      mb[u] = ld8<kNtLoadRW>(p.m_in + b);
      va[u] = ld16<kNtLoadRW>(pv + a);
      vb[u] = ld16<kNtLoadRW>(pv + b);
      wa[u] = ld16<kNtLoadRW>(pw + a);
      wb[u] = ld16<kNtLoadRW>(pw + b);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const long long a = pos0 + u * kTile, b = a + kTile / 2;
      const Quad q0 = quad<true>(ga[u].x, ma[u].x, va[u].x, va[u].y, wa[u].x, wa[u].y);
      const Quad q1 = quad<true>(ga[u].y, ma[u].y, va[u].z, va[u].w, wa[u].z, wa[u].w);
      const Quad q2 = quad<true>(gb[u].x, mb[u].x, vb[u].x, vb[u].y, wb[u].x, wb[u].y);
      const Quad q3 = quad<true>(gb[u].y, mb[u].y, vb[u].z, vb[u].w, wb[u].z, wb[u].w);
      st8<kNtStoreRW>(p.m + a, make_uint2(q0.m, q1.m));
      st8<kNtStoreRW>(p.m + b, make_uint2(q2.m, q3.m));
      st16<kNtStoreRW>(pv + a, make_uint4(q0.v01, q0.v23, q1.v01, q1.v23));
      st16<kNtStoreRW>(pv + b, make_uint4(q2.v01, q2.v23, q3.v01, q3.v23));
      st16<kNtStoreRW>(pw + a, make_uint4(q0.w01, q0.w23, q1.w01, q1.w23));
      st16<kNtStoreRW>(pw + b, make_uint4(q2.w01, q2.w23, q3.w01, q3.w23));
      if constexpr (WCOPY == FP8LM_WCOPY_E4M3) {
        uint8_t* q = static_cast<uint8_t*>(p.wcopy);
        st8<kNtStoreWO>(q + a, make_uint2(q0.q, q1.q));
        st8<kNtStoreWO>(q + b, make_uint2(q2.q, q3.q));
      } else {
        uint16_t* q = static_cast<uint16_t*>(p.wcopy);
        st16<kNtStoreWO>(q + a, make_uint4(q0.q, q0.q2, q1.q, q1.q2));
        st16<kNtStoreWO>(q + b, make_uint4(q2.q, q2.q2, q3.q, q3.q2));
      }
    }
  }
  template <int UN> __device__ __forceinline__ void tiles(long long tile0) {
    if constexpr (FP8LM_UPDATE_SPLIT) tiles_split<UN>(tile0);
    else tiles_plain<UN>(tile0);
  }
  // a thread takes 16 consecutive elements of the tile
  template <int UN> __device__ __forceinline__ void tiles_plain(long long tile0) {
    uint4 g[UN], m[UN], va[UN], vb[UN], wa[UN], wb[UN];
    const long long pos0 = tile0 + threadIdx.x * kGroup;
    uint16_t* pv = static_cast<uint16_t*>(p.v);
    uint16_t* pw = static_cast<uint16_t*>(p.w);
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const long long pos = pos0 + u * kTile;
      g[u] = ld16<kNtLoadRO>(p.grad + pos);
      m[u] = ld16<kNtLoadRW>(p.m_in + pos);
      va[u] = ld16<kNtLoadRW>(pv + pos);
      vb[u] = ld16<kNtLoadRW>(pv + pos + 8);
      wa[u] = ld16<kNtLoadRW>(pw + pos);
      wb[u] = ld16<kNtLoadRW>(pw + pos + 8);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const long long pos = pos0 + u * kTile;
      const Quad q0 = quad<true>(g[u].x, m[u].x, va[u].x, va[u].y, wa[u].x, wa[u].y);
      const Quad q1 = quad<true>(g[u].y, m[u].y, va[u].z, va[u].w, wa[u].z, wa[u].w);
      const Quad q2 = quad<true>(g[u].z, m[u].z, vb[u].x, vb[u].y, wb[u].x, wb[u].y);
      const Quad q3 = quad<true>(g[u].w, m[u].w, vb[u].z, vb[u].w, wb[u].z, wb[u].w);
      st16<kNtStoreRW>(p.m + pos, make_uint4(q0.m, q1.m, q2.m, q3.m));
      st16<kNtStoreRW>(pv + pos, make_uint4(q0.v01, q0.v23, q1.v01, q1.v23));
      st16<kNtStoreRW>(pv + pos + 8, make_uint4(q2.v01, q2.v23, q3.v01, q3.v23));
      st16<kNtStoreRW>(pw + pos, make_uint4(q0.w01, q0.w23, q1.w01, q1.w23));
      st16<kNtStoreRW>(pw + pos + 8, make_uint4(q2.w01, q2.w23, q3.w01, q3.w23));
      if constexpr (WCOPY == FP8LM_WCOPY_E4M3) {
        st16<kNtStoreWO>(static_cast<uint8_t*>(p.wcopy) + pos, make_uint4(q0.q, q1.q, q2.q, q3.q));
      } else {
        uint16_t* q = static_cast<uint16_t*>(p.wcopy);
        st16<kNtStoreWO>(q + pos, make_uint4(q0.q, q0.q2, q1.q, q1.q2));
        st16<kNtStoreWO>(q + pos + 8, make_uint4(q2.q, q2.q2, q3.q, q3.q2));
      }
    }
  }
  // 16 consecutive elements at `pos`, by this thread alone (the layout without the split)
  __device__ __forceinline__ void full_group(long long pos) { tiles_plain<1>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    if (!careful) {
      // ragged tail of a tensor: same arithmetic, element by element
      uint16_t* pv = static_cast<uint16_t*>(p.v);
      uint16_t* pw = static_cast<uint16_t*>(p.w);
      for (int j = 0; j < valid; ++j) {
        const long long i = pos + j;
        const Quad o = quad<false>(p.grad[i], p.m_in[i], pv[i], 0u, pw[i], 0u);
        p.m[i] = (uint8_t)o.m;
        pv[i] = (uint16_t)o.v01;
        pw[i] = (uint16_t)o.w01;
        if constexpr (WCOPY == FP8LM_WCOPY_E4M3) static_cast<uint8_t*>(p.wcopy)[i] = (uint8_t)o.q;
        else static_cast<uint16_t*>(p.wcopy)[i] = (uint16_t)o.q;
      }
    } else {
      for (int j = 0; j < valid; ++j) one_careful(pos + j);
    }
  }

  using Stats = BlockStats<3, STATS ? 8 : 0>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.mx[0] = f2u(vmax);
    s.mx[1] = f2u(wmax);
    s.mx[2] = f2u(mmax);
    if constexpr (STATS) {
      const bool first_lane = (threadIdx.x & 63) == 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) s.ct[i] = cnt[i] + (first_lane ? wcnt[i] : 0u);
    }
    s.orv = nf;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  __device__ void finalize(int t, const TensorDesc&, const Stats& s) {
    unsigned long long c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (STATS) {
#pragma unroll
      for (int i = 0; i < 8; ++i) c[i] = s.ct[i];
    }
    finish(t, u2f(s.mx[0]), u2f(s.mx[1]), u2f(s.mx[2]), s.orv, c);
  }

  // Fills one output meta.  amax_deq is the stored value of the largest element: rounding is monotone,
  // so quantising the maximum gives the maximum of the quantised values.  An infinity is stored as the
  // top code of a saturating format, so it pins amax_deq to fmax / scale.
  template <class Enc, class Dec>
  __device__ __forceinline__ void fill(fp8lm_meta& M, float scale, float inv, float amax, uint32_t nan_inf_bits,
                                       uint32_t flags, float fmax, bool saturating, unsigned long long n_sat,
                                       unsigned long long n_und, Enc enc, Dec dec, uint32_t magmask, uint32_t topcode) {
    const bool nonfinite = nan_inf_bits != 0;
    const bool inf_stored = (nan_inf_bits & 2u) != 0;          // as the top code, or as infinity in bf16
    const bool inf_seen = saturating && inf_stored;
    M.scale = scale;
    M.inv_scale = inv;
    M.amax = nonfinite ? __builtin_inff() : amax;
    const uint32_t code = enc(amax * scale);
    const float stored = inf_seen ? fmax : dec(code);
    M.amax_deq = stored * inv;
    if (nonfinite) flags |= FP8LM_FLAG_NONFINITE;
    bool sat = inf_stored || (code & magmask) == topcode;
    if constexpr (STATS) sat = n_sat != 0;
    if (sat) flags |= FP8LM_FLAG_SATURATED;
    M.flags = flags;
    M.n_sat = STATS ? n_sat : 0;
    M.n_underflow = STATS ? n_und : 0;
  }

  __device__ void finish(int t, float A_v, float A_w, float A_mc, uint32_t nfb, const unsigned long long* c) {
    Scratch::Pending& P = tb.scratch[t].pend;
    const float A_m = A_mc;    // measured by this pass on both paths (equals what pass A saw)
    uint32_t m_nf = nfb & 3u;
    if (p.speculative_m) {
      // The moment was stored with a predicted scale.  The scale its exact amax demands, by the rule pass A applies:
      // equal -> what was stored is the just-in-time result; different -> the tensor's moment is computed again with
      // the right scale from the untouched inputs (grad and the other buffer of the pair); v, w and the copy never
      // depend on it.  Either way the metadata gets the exact scale and the flags that go with it.
      float sm = 0.0f, ism = 0.0f;
      uint32_t fm = 0;
      refresh_scale(kBitsE4M3Max, m_nf ? __builtin_inff() : A_m, 0, tb.scratch[t].old_scale, tb.scratch[t].old_inv, sm, ism, fm);
      tb.scratch[t].redo = sm != P.sm ? 1u : 0u;
      P.sm = sm;
      P.ism = ism;
      P.fm = fm;
    }
    auto enc8 = [](float x) { return encode1_fp8<kE4M3>(x); };
    auto dec8 = [](uint32_t cc) { return fp8_to_f32<kE4M3>(cc); };
    auto enc16 = [](float x) { return encode1_f16(x); };
    auto dec16 = [](uint32_t cc) { return f16_to_f32(cc); };
    fill(p.m_meta[t], P.sm, P.ism, A_m, m_nf, P.fm, 448.0f, true, c[0], c[4], enc8, dec8, 0x7Fu, 0x7Eu);
    fill(p.v_meta[t], P.sv, P.isv, A_v, (nfb >> 2) & 3u, P.fv, 65504.0f, true, c[1], c[5], enc16, dec16, 0x7FFFu, 0x7BFFu);
    fill(p.w_meta[t], P.sw, P.isw, A_w, (nfb >> 4) & 3u, P.fw, 65504.0f, true, c[2], c[6], enc16, dec16, 0x7FFFu, 0x7BFFu);
    if constexpr (WCOPY == FP8LM_WCOPY_E4M3) {
      fill(p.wcopy_meta[t], P.sq, P.isq, A_w, (nfb >> 4) & 3u, P.fq, 448.0f, true, c[3], c[7], enc8, dec8, 0x7Fu, 0x7Eu);
    } else {
      // bf16 is not saturating: an overflow is stored as infinity, which carries no magnitude
      auto encb = [](float x) { return encode1_bf16(x); };
      auto decb = [](uint32_t cc) { return u2f(cc << 16); };
      fill(p.wcopy_meta[t], 1.0f, 1.0f, A_w, (nfb >> 4) & 3u, 0u, 0.0f, false, c[3], c[7], encb, decb, 0x7FFFu, 0x7F80u);
    }
  }
};

template <int GFMT, int WCOPY, bool FAST, bool STATS>
__global__ __launch_bounds__(kThreads) void adam_update_kernel(Tables tb, AdamParams p) {
  AdamUpdateOp<GFMT, WCOPY, FAST, STATS> op(p, tb);
  walk_chunks<FP8LM_UN_UPDATE>(tb, op);
}

// ---- repair of a failed first-moment speculation ---------------------------------------------------
// Walks the chunk list of the marked tensors: m' = fma(beta1, m_in / s_m, (1-beta1) * g / s_g) once more, stored to
// m with the exact scale that the update pass's epilogue left in the scratch.
template <int GFMT>
struct AdamMomentRedoOp {
  const AdamParams& p;
  const Tables& tb;
  float inv_sg, inv_sm, sm;
  bool careful;
  __device__ AdamMomentRedoOp(const AdamParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc&) {
    inv_sg = p.grad_meta[t].inv_scale;
    inv_sm = tb.scratch[t].old_inv;                 // the scale m_in is stored with (m_meta already holds the new one)
    sm = tb.scratch[t].pend.sm;
    careful = tb.scratch[t].pend.careful != 0;
  }
  __device__ __forceinline__ float moment(float dg, float dm) const {
    return __builtin_fmaf(p.b1, dm * inv_sm, p.omb1 * (dg * inv_sg));
  }
  __device__ __forceinline__ uint32_t word(uint32_t gw, uint32_t mw) const {
    const float2_t g01 = fp8x2_to_f32<GFMT, false>(gw), g23 = fp8x2_to_f32<GFMT, true>(gw);
    const float2_t m01 = fp8x2_to_f32<kE4M3, false>(mw), m23 = fp8x2_to_f32<kE4M3, true>(mw);
    return encode4_fp8<kE4M3>(moment(g01.x, m01.x) * sm, moment(g01.y, m01.y) * sm, moment(g23.x, m23.x) * sm,
                              moment(g23.y, m23.y) * sm);
  }
  __device__ __forceinline__ bool fast() const { return !careful; }
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) {
    const long long pos = pos0 + threadIdx.x * kGroup;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const uint4 g = ld16<kNtLoadRO>(p.grad + pos + u * kTile), m = ld16<kNtLoadRO>(p.m_in + pos + u * kTile);
      st16<kNtStoreWO>(p.m + pos + u * kTile, make_uint4(word(g.x, m.x), word(g.y, m.y), word(g.z, m.z), word(g.w, m.w)));
    }
  }
  __device__ __forceinline__ void full_group(long long pos) { tiles<1>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    for (int j = 0; j < valid; ++j) {
      const long long i = pos + j;
      p.m[i] = (uint8_t)encode1_fp8_careful<kE4M3>(moment(fp8_to_f32<GFMT>(p.grad[i]), fp8_to_f32<kE4M3>(p.m_in[i])) * sm);
    }
  }
  using Stats = BlockStats<1, 0>;
  __device__ __forceinline__ void flush(int, const TensorDesc&, int) {}      // nothing to reduce: the metadata is complete
  __device__ void finalize(int, const TensorDesc&, const Stats&) {}
};

template <int GFMT>
__global__ __launch_bounds__(kThreads) void adam_moment_redo_kernel(Tables tb, AdamParams p) {
  AdamMomentRedoOp<GFMT> op(p, tb);
  walk_chunks<2>(tb, op);
}

// ---- pass B for the other storage formats of the precision-decoupling study ----------------------
// Master weight FP16-scaled / BF16 / E4M3-scaled / FP32 and second moment FP16 / E4M3-scaled (Sec. 2.2;
// Sec. 3.3, table of optimizer settings).  Same arithmetic as above, correctly rounded sqrt and divide,
// E4M3 weight copy, no counters; one 16-element group per thread and iteration.
template <int GFMT, int MASTER, int VFMT>
struct AdamUpdateVarOp {
  typedef StTraits<MASTER> WT;
  typedef StTraits<VFMT> VT;
  const AdamParams& p;
  const Tables& tb;
  float inv_sg, inv_sm, inv_sv, inv_sw, sm, sv, sw, sq, decay;
  bool careful;
  float vmax, wmax, mmax;
  uint32_t nf;
  __device__ AdamUpdateVarOp(const AdamParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc& d) {
    const Scratch::Pending& P = tb.scratch[t].pend;
    decay = (d.flags & FP8LM_TENSOR_NO_WEIGHT_DECAY) ? 1.0f : p.decay;
    inv_sg = p.grad_meta[t].inv_scale;
    inv_sm = p.m_meta[t].inv_scale;
    inv_sv = p.v_meta[t].inv_scale;
    inv_sw = p.w_meta[t].inv_scale;
    sm = P.sm; sv = P.sv; sw = P.sw; sq = P.sq;
    careful = P.careful != 0;
    vmax = wmax = mmax = 0.0f;
    nf = 0;
  }
  __device__ __forceinline__ bool fast() const { return !careful; }
  __device__ __forceinline__ void update(float dg, float dm, float dv, float dw, float& m1, float& v1, float& w1) {
    const float g = dg * inv_sg, m0 = dm * inv_sm, v0 = dv * inv_sv, w0 = dw * inv_sw;
    m1 = __builtin_fmaf(p.b1, m0, p.omb1 * g);
    v1 = __builtin_fmaf(p.b2, v0, p.omb2 * (g * g));
    const float den = __builtin_sqrtf(v1 * p.rbc2) + p.eps;
    const float upd = (m1 * p.rbc1) / den;
    w1 = __builtin_fmaf(-p.lr, upd, w0 * decay);
  }
  template <int UN> __device__ __forceinline__ void tiles(long long tile0) {
    static_assert(UN == 1, "one group at a time");
    const long long pos = tile0 + threadIdx.x * kGroup;
    const uint4 gq = ld16<kNtLoadRO>(p.grad + pos), mq = ld16<false>(p.m + pos);
    float dv[kGroup], dw[kGroup], dg[kGroup], dm[kGroup];
    st_load16<VFMT>(p.v, pos, dv);
    st_load16<MASTER>(p.w, pos, dw);
    const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w}, mw[4] = {mq.x, mq.y, mq.z, mq.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float2_t g01 = fp8x2_to_f32<GFMT, false>(gw[k]), g23 = fp8x2_to_f32<GFMT, true>(gw[k]);
      const float2_t m01 = fp8x2_to_f32<kE4M3, false>(mw[k]), m23 = fp8x2_to_f32<kE4M3, true>(mw[k]);
      dg[4 * k] = g01.x; dg[4 * k + 1] = g01.y; dg[4 * k + 2] = g23.x; dg[4 * k + 3] = g23.y;
      dm[4 * k] = m01.x; dm[4 * k + 1] = m01.y; dm[4 * k + 2] = m23.x; dm[4 * k + 3] = m23.y;
    }
    float tm[kGroup], tq[kGroup];
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
      float m1, v1, w1;
      update(dg[j], dm[j], dv[j], dw[j], m1, v1, w1);
      vmax = fmaxf(vmax, v1);
      wmax = fmaxf(wmax, fabsf(w1));
      mmax = fmaxf(mmax, fabsf(m1));
      tm[j] = m1 * sm;
      dv[j] = v1 * sv;
      dw[j] = w1 * sw;
      tq[j] = w1 * sq;
    }
    st_store16<kStE4M3>(p.m, pos, tm);
    st_store16<VFMT>(p.v, pos, dv);
    st_store16<MASTER>(p.w, pos, dw);
    st_store16<kStE4M3>(p.wcopy, pos, tq);
  }
  // 16 consecutive elements at `pos`, by this thread alone: the tile body with the thread's own offset taken out
  __device__ __forceinline__ void full_group(long long pos) { tiles<1>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    for (int j = 0; j < valid; ++j) {
      const long long i = pos + j;
      float m1, v1, w1;
      update(fp8_to_f32<GFMT>(p.grad[i]), fp8_to_f32<kE4M3>(p.m[i]), st_load1<VFMT>(p.v, i), st_load1<MASTER>(p.w, i), m1, v1, w1);
      p.m[i] = (uint8_t)encode1_fp8_careful<kE4M3>(m1 * sm);
      st_store1<VFMT>(p.v, i, VT::enc_careful(v1 * sv));
      st_store1<MASTER>(p.w, i, WT::enc_careful(w1 * sw));
      static_cast<uint8_t*>(p.wcopy)[i] = (uint8_t)encode1_fp8_careful<kE4M3>(w1 * sq);
      const float kMaxF = 3.4028234663852886e38f;
      const float am = fabsf(m1), av = fabsf(v1), aw = fabsf(w1);
      if (am <= kMaxF) mmax = fmaxf(mmax, am); else nf |= (m1 != m1) ? 1u : 2u;
      if (av <= kMaxF) vmax = fmaxf(vmax, av); else nf |= (v1 != v1) ? 4u : 8u;
      if (aw <= kMaxF) wmax = fmaxf(wmax, aw); else nf |= (w1 != w1) ? 16u : 32u;
    }
  }
  template <class T>
  __device__ __forceinline__ void fill(fp8lm_meta& M, float scale, float inv, float amax, uint32_t nan_inf_bits, uint32_t flags) {
    const bool nonfinite = nan_inf_bits != 0;
    const bool inf_stored = (nan_inf_bits & 2u) != 0;          // as the top code, or as infinity where the format has one
    M.scale = scale;
    M.inv_scale = inv;
    M.amax = nonfinite ? __builtin_inff() : amax;
    const uint32_t code = T::enc(amax * scale);
    M.amax_deq = ((T::kSaturating && inf_stored) ? T::kMax : T::dec(code)) * inv;
    if (nonfinite) flags |= FP8LM_FLAG_NONFINITE;
    if (inf_stored || (code & T::kMagMask) == T::kTopCode) flags |= FP8LM_FLAG_SATURATED;
    M.flags = flags;
    M.n_sat = 0;
    M.n_underflow = 0;
  }
  using Stats = BlockStats<3, 0>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.mx[0] = f2u(vmax);
    s.mx[1] = f2u(wmax);
    s.mx[2] = f2u(mmax);
    s.orv = nf;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  __device__ void finalize(int t, const TensorDesc&, const Stats& s) {
    const float A_v = u2f(s.mx[0]), A_w = u2f(s.mx[1]), A_m = u2f(s.mx[2]);
    const uint32_t nfb = s.orv;
    const Scratch::Pending& P = tb.scratch[t].pend;
    fill<StTraits<kStE4M3>>(p.m_meta[t], P.sm, P.ism, A_m, nfb & 3u, P.fm);
    fill<VT>(p.v_meta[t], P.sv, P.isv, A_v, (nfb >> 2) & 3u, P.fv);
    fill<WT>(p.w_meta[t], P.sw, P.isw, A_w, (nfb >> 4) & 3u, P.fw);
    fill<StTraits<kStE4M3>>(p.wcopy_meta[t], P.sq, P.isq, A_w, (nfb >> 4) & 3u, P.fq);
  }
};

template <int GFMT, int MASTER, int VFMT>
__global__ __launch_bounds__(kThreads) void adam_update_var_kernel(Tables tb, AdamParams p) {
  AdamUpdateVarOp<GFMT, MASTER, VFMT> op(p, tb);
  walk_chunks<1>(tb, op);
}

}  // namespace fp8lm

#endif
