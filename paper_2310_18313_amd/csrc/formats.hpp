// Device-side number-format helpers for gfx950 (CDNA4): OCP FP8 via the native convert
// instructions, IEEE half via v_cvt_f16_f32 / v_cvt_f32_f16, bf16 by bit manipulation.
//
// Encoders here are "saturating round-to-nearest-even": the input is clamped to the largest finite
// value of the target with v_med3_f32 and then handed to the hardware converter, which rounds to
// nearest even and keeps subnormals (FP8 formats: Appendix A.1 of the FP8-LM paper).  v_med3_f32
// does not propagate NaN, so callers that may see NaN use the *_careful variants, which select the
// canonical NaN code explicitly.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp8lm {

enum : int { kE4M3 = 0, kE5M2 = 1 };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t f2u(float x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ float u2f(uint32_t x) { return __builtin_bit_cast(float, x); }

template <int FMT> struct Fp8Traits;
template <> struct Fp8Traits<kE4M3> {
  static constexpr float kMax = 448.0f;          // largest finite value
  static constexpr uint32_t kTop = 0x7E;         // its code
  static constexpr uint32_t kTopX4 = 0x7E7E7E7Eu;
};
template <> struct Fp8Traits<kE5M2> {
  static constexpr float kMax = 57344.0f;
  static constexpr uint32_t kTop = 0x7B;
  static constexpr uint32_t kTopX4 = 0x7B7B7B7Bu;
};

// ---- FP8 decode: two codes of a 32-bit word -> two floats ---------------------------------------
template <int FMT, bool HI> __device__ __forceinline__ float2_t fp8x2_to_f32(uint32_t w) {
  if constexpr (FMT == kE4M3) return __builtin_amdgcn_cvt_pk_f32_fp8((int)w, HI);
  else return __builtin_amdgcn_cvt_pk_f32_bf8((int)w, HI);
}
template <int FMT> __device__ __forceinline__ float fp8_to_f32(uint32_t code) {
  return fp8x2_to_f32<FMT, false>(code & 0xFFu).x;
}

// ---- FP8 encode: inputs must already be inside [-max, max] (or NaN-free by construction) ---------
template <int FMT, bool HI> __device__ __forceinline__ uint32_t f32x2_to_fp8(float a, float b, uint32_t old) {
  if constexpr (FMT == kE4M3) return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, HI);
  else return (uint32_t)__builtin_amdgcn_cvt_pk_bf8_f32(a, b, (int)old, HI);
}
template <int FMT> __device__ __forceinline__ float clamp_fp8(float x) {
  return __builtin_amdgcn_fmed3f(x, -Fp8Traits<FMT>::kMax, Fp8Traits<FMT>::kMax);
}
// four floats -> four codes in one word (element 0 in the low byte)
template <int FMT> __device__ __forceinline__ uint32_t encode4_fp8(float a, float b, float c, float d) {
  uint32_t w = f32x2_to_fp8<FMT, false>(clamp_fp8<FMT>(a), clamp_fp8<FMT>(b), 0u);
  return f32x2_to_fp8<FMT, true>(clamp_fp8<FMT>(c), clamp_fp8<FMT>(d), w);
}
// single value, NaN -> 0x7F
template <int FMT> __device__ __forceinline__ uint32_t encode1_fp8_careful(float x) {
  const uint32_t c = f32x2_to_fp8<FMT, false>(clamp_fp8<FMT>(x), 0.0f, 0u) & 0xFFu;
  return (x != x) ? 0x7Fu : c;
}
template <int FMT> __device__ __forceinline__ uint32_t encode1_fp8(float x) {
  return f32x2_to_fp8<FMT, false>(clamp_fp8<FMT>(x), 0.0f, 0u) & 0xFFu;
}

// ---- IEEE half ---------------------------------------------------------------------------------
__device__ __forceinline__ float clamp_f16(float x) { return __builtin_amdgcn_fmed3f(x, -65504.0f, 65504.0f); }
__device__ __forceinline__ uint32_t encode2_f16(float a, float b) {
  half2_t h;
  h.x = (_Float16)clamp_f16(a);
  h.y = (_Float16)clamp_f16(b);
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ uint32_t encode1_f16(float a) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)clamp_f16(a));
}
__device__ __forceinline__ uint32_t encode1_f16_careful(float a) {
  return (a != a) ? 0x7E00u : encode1_f16(a);
}
__device__ __forceinline__ float2_t f16x2_to_f32(uint32_t w) {
  const half2_t h = __builtin_bit_cast(half2_t, w);
  float2_t r;
  r.x = (float)h.x;
  r.y = (float)h.y;
  return r;
}
__device__ __forceinline__ float f16_to_f32(uint32_t code) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)code);
}

// ---- bf16 --------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return u2f(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return u2f(w & 0xFFFF0000u); }
// round to nearest even; overflow goes to infinity as in IEEE; NaN -> 0x7FC0
__device__ __forceinline__ uint32_t encode1_bf16(float x) {
  const uint32_t b = f2u(x);
  const uint32_t r = (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
  return ((b & 0x7FFFFFFFu) > 0x7F800000u) ? 0x7FC0u : r;
}

// ---- storage formats of the optimizer state (precision-decoupling settings of the paper, Sec. 3.3) ----
enum : int { kStF16 = 0, kStBF16 = 1, kStE4M3 = 2, kStF32 = 3 };

template <int K> struct StTraits;
template <> struct StTraits<kStF16> {
  typedef uint16_t elem_t;
  static constexpr bool kScaled = true, kSaturating = true;
  static constexpr float kMax = 65504.0f;
  static constexpr uint32_t kMaxBits = 0x477FE000u, kMagMask = 0x7FFFu, kTopCode = 0x7BFFu;
  static __device__ __forceinline__ float dec(uint32_t c) { return f16_to_f32(c); }
  static __device__ __forceinline__ uint32_t enc(float x) { return encode1_f16(x); }
  static __device__ __forceinline__ uint32_t enc_careful(float x) { return encode1_f16_careful(x); }
};
template <> struct StTraits<kStBF16> {
  typedef uint16_t elem_t;
  static constexpr bool kScaled = false, kSaturating = false;
  static constexpr float kMax = 0.0f;
  static constexpr uint32_t kMaxBits = 0u, kMagMask = 0x7FFFu, kTopCode = 0x7F80u;   // "top" = rounded to infinity
  static __device__ __forceinline__ float dec(uint32_t c) { return u2f(c << 16); }
  static __device__ __forceinline__ uint32_t enc(float x) { return encode1_bf16(x); }
  static __device__ __forceinline__ uint32_t enc_careful(float x) { return encode1_bf16(x); }
};
template <> struct StTraits<kStE4M3> {
  typedef uint8_t elem_t;
  static constexpr bool kScaled = true, kSaturating = true;
  static constexpr float kMax = 448.0f;
  static constexpr uint32_t kMaxBits = 0x43E00000u, kMagMask = 0x7Fu, kTopCode = 0x7Eu;
  static __device__ __forceinline__ float dec(uint32_t c) { return fp8_to_f32<kE4M3>(c); }
  static __device__ __forceinline__ uint32_t enc(float x) { return encode1_fp8<kE4M3>(x); }
  static __device__ __forceinline__ uint32_t enc_careful(float x) { return encode1_fp8_careful<kE4M3>(x); }
};
template <> struct StTraits<kStF32> {
  typedef uint32_t elem_t;
  static constexpr bool kScaled = false, kSaturating = false;
  static constexpr float kMax = 0.0f;
  static constexpr uint32_t kMaxBits = 0u, kMagMask = 0x7FFFFFFFu, kTopCode = 0x7F800000u;
  static __device__ __forceinline__ float dec(uint32_t c) { return u2f(c); }
  static __device__ __forceinline__ uint32_t enc(float x) { return f2u(x); }
  static __device__ __forceinline__ uint32_t enc_careful(float x) { return x != x ? 0x7FC00000u : f2u(x); }
};

// 16 consecutive elements: 128-bit accesses, decoded to / encoded from fp32 payloads
template <int K> __device__ __forceinline__ void st_load16(const void* buf, long long pos, float* out) {
  const typename StTraits<K>::elem_t* q = static_cast<const typename StTraits<K>::elem_t*>(buf) + pos;
  if constexpr (K == kStE4M3) {
    const uint4 a = *reinterpret_cast<const uint4*>(q);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float2_t lo = fp8x2_to_f32<kE4M3, false>(w[k]), hi = fp8x2_to_f32<kE4M3, true>(w[k]);
      out[4 * k] = lo.x; out[4 * k + 1] = lo.y; out[4 * k + 2] = hi.x; out[4 * k + 3] = hi.y;
    }
  } else if constexpr (K == kStF32) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint4 a = *reinterpret_cast<const uint4*>(q + 4 * k);
      out[4 * k] = u2f(a.x); out[4 * k + 1] = u2f(a.y); out[4 * k + 2] = u2f(a.z); out[4 * k + 3] = u2f(a.w);
    }
  } else {
    const uint4 a = *reinterpret_cast<const uint4*>(q), b = *reinterpret_cast<const uint4*>(q + 8);
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if constexpr (K == kStF16) {
        const float2_t f = f16x2_to_f32(w[k]);
        out[2 * k] = f.x; out[2 * k + 1] = f.y;
      } else {
        out[2 * k] = bf16lo_to_f32(w[k]); out[2 * k + 1] = bf16hi_to_f32(w[k]);
      }
    }
  }
}
template <int K> __device__ __forceinline__ void st_store16(void* buf, long long pos, const float* x) {
  typename StTraits<K>::elem_t* q = static_cast<typename StTraits<K>::elem_t*>(buf) + pos;
  if constexpr (K == kStE4M3) {
    *reinterpret_cast<uint4*>(q) = make_uint4(encode4_fp8<kE4M3>(x[0], x[1], x[2], x[3]), encode4_fp8<kE4M3>(x[4], x[5], x[6], x[7]),
                                              encode4_fp8<kE4M3>(x[8], x[9], x[10], x[11]), encode4_fp8<kE4M3>(x[12], x[13], x[14], x[15]));
  } else if constexpr (K == kStF32) {
#pragma unroll
    for (int k = 0; k < 4; ++k)
      *reinterpret_cast<uint4*>(q + 4 * k) = make_uint4(f2u(x[4 * k]), f2u(x[4 * k + 1]), f2u(x[4 * k + 2]), f2u(x[4 * k + 3]));
  } else {
    uint32_t w[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if constexpr (K == kStF16) w[k] = encode2_f16(x[2 * k], x[2 * k + 1]);
      else w[k] = encode1_bf16(x[2 * k]) | (encode1_bf16(x[2 * k + 1]) << 16);
    }
    *reinterpret_cast<uint4*>(q) = make_uint4(w[0], w[1], w[2], w[3]);
    *reinterpret_cast<uint4*>(q + 8) = make_uint4(w[4], w[5], w[6], w[7]);
  }
}
template <int K> __device__ __forceinline__ float st_load1(const void* buf, long long i) {
  return StTraits<K>::dec(static_cast<const typename StTraits<K>::elem_t*>(buf)[i]);
}
template <int K> __device__ __forceinline__ void st_store1(void* buf, long long i, uint32_t code) {
  static_cast<typename StTraits<K>::elem_t*>(buf)[i] = (typename StTraits<K>::elem_t)code;
}

// ---- the power-of-two scale rule ------------------------------------------------------------------
// For A > 0 finite returns the integer k with 2^k * A <= fmax < 2^(k+1) * A, using only integer
// compares on the bit patterns.  fmax_bits is the fp32 pattern of a normal number.
__device__ __forceinline__ int pow2_exp(uint32_t fmax_bits, float A) {
  const uint32_t ab = f2u(A) & 0x7FFFFFFFu;
  int ea = (int)(ab >> 23) - 127;
  uint32_t ma = ab & 0x7FFFFFu;
  if ((ab >> 23) == 0) {                    // fp32 subnormal: normalise
    const int sh = __clz(ma) - 8;
    ma = (ma << sh) & 0x7FFFFFu;
    ea = -126 - sh;
  }
  const int ef = (int)(fmax_bits >> 23) - 127;
  const uint32_t mf = fmax_bits & 0x7FFFFFu;
  return ma <= mf ? ef - ea : ef - ea - 1;
}
__device__ __forceinline__ float pow2f(int e) { return u2f((uint32_t)(e + 127) << 23); }  // e in [-126, 127]

constexpr uint32_t kBitsE4M3Max = 0x43E00000u;  // 448
constexpr uint32_t kBitsE5M2Max = 0x47600000u;  // 57344
constexpr uint32_t kBitsF16Max = 0x477FE000u;   // 65504

}  // namespace fp8lm
