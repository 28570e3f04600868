// Quantisation-error statistics of an FP8 gradient (Sec. 3.3, communication ablation) and the small
// utility kernels (metadata initialisation, streaming copy).
#ifndef FP8LM_STATS_HPP
#define FP8LM_STATS_HPP

#include <type_traits>

#include "walk.hpp"

namespace fp8lm {

// ================================================================================================
// Quantisation error of an FP8 gradient against a high-precision reference (Sec. 3.3, the figure
// of the communication ablation: SNR, underflow rate, overflow rate)
// ================================================================================================
struct StatsParams {
  const void* ref;
  const uint8_t* q;
  const fp8lm_meta* meta;
  fp8lm_quant_stats* out;
};

template <int FMT, int SRC>
struct QuantStatsOp {
  using elem_t = typename SrcTraits<SRC>::elem_t;
  static constexpr int kPer = 16 / (int)sizeof(elem_t);
  static constexpr int kLoads = kGroup / kPer;
  static constexpr int kW = kSrcWords<SRC>;
  const StatsParams& p;
  const Tables& tb;
  double rs, signal, noise;
  uint32_t n_nonzero, n_under, n_over, n_nonfinite;
  __device__ QuantStatsOp(const StatsParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc&) {
    rs = 1.0 / (double)p.meta[t].scale;
    signal = noise = 0.0;
    n_nonzero = n_under = n_over = n_nonfinite = 0;
  }
  __device__ __forceinline__ bool fast() const { return true; }
  __device__ __forceinline__ void one(uint32_t rbits, uint32_t code) {
    const float r = SrcTraits<SRC>::dec(rbits);
    const float pv = fp8_to_f32<FMT>(code);
    if (!(fabsf(r) <= 3.4028234664e38f) || !(fabsf(pv) <= 3.4028234664e38f)) {
      ++n_nonfinite;
      return;
    }
    const double rd = (double)r;
    const double e = rd - (double)pv * rs;
    signal += rd * rd;
    noise += e * e;
    const uint32_t mag = code & 0x7Fu;
    n_nonzero += (r != 0.0f);
    n_under += (r != 0.0f) && mag == 0u;
    n_over += mag == Fp8Traits<FMT>::kTop;
  }
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) {
    const long long pos = pos0 + threadIdx.x * kGroup;
    const elem_t* rp = static_cast<const elem_t*>(p.ref) + pos;
    uint4 r[UN][kLoads], qq[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int k = 0; k < kLoads; ++k) r[u][k] = ld16<kNtLoadRO>(rp + u * kTile + k * kPer);
      qq[u] = ld16<kNtLoadRO>(p.q + pos + u * kTile);
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      uint32_t w[kW];
#pragma unroll
      for (int k = 0; k < kLoads; ++k) {
        w[4 * k] = r[u][k].x; w[4 * k + 1] = r[u][k].y; w[4 * k + 2] = r[u][k].z; w[4 * k + 3] = r[u][k].w;
      }
      const uint32_t qw[4] = {qq[u].x, qq[u].y, qq[u].z, qq[u].w};
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const uint32_t bits = kSrc16<SRC> ? (w[(j >> 1) % kW] >> ((j & 1) * 16)) & 0xFFFFu : w[j % kW];
        one(bits, (qw[j >> 2] >> ((j & 3) * 8)) & 0xFFu);
      }
    }
  }
  // 16 consecutive elements at `pos`, by this thread alone: the tile body with the thread's own offset taken out
  __device__ __forceinline__ void full_group(long long pos) { tiles<1>(pos - (long long)threadIdx.x * kGroup); }
  __device__ __forceinline__ void group(long long pos, int valid) {
    const elem_t* rp = static_cast<const elem_t*>(p.ref) + pos;
    for (int j = 0; j < valid; ++j) one(rp[j], p.q[pos + j]);
  }
  using Stats = BlockStats<0, 4, 2>;
  __device__ __forceinline__ void flush(int t, const TensorDesc& d, int done) {
    Stats s;
    s.ct[0] = n_nonzero; s.ct[1] = n_under; s.ct[2] = n_over; s.ct[3] = n_nonfinite;
    s.fs[0] = signal; s.fs[1] = noise;
    s.orv = 0;
    block_combine(s);
    if (collect(tb, t, d, done, s) && threadIdx.x == 0) finalize(t, d, s);
  }
  __device__ void finalize(int t, const TensorDesc&, const Stats& s) {
    p.out[t] = fp8lm_quant_stats{s.fs[0], s.fs[1], s.ct[0], s.ct[1], s.ct[2], s.ct[3]};
  }
};

template <int FMT, int SRC>
__global__ __launch_bounds__(kThreads) void quant_stats_kernel(Tables tb, StatsParams p) {
  QuantStatsOp<FMT, SRC> op(p, tb);
  walk_chunks<1>(tb, op);
}

__global__ void quant_stats_zero_kernel(fp8lm_quant_stats* out, int n) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) out[t] = fp8lm_quant_stats{0.0, 0.0, 0, 0, 0, 0};
}

__global__ void meta_init_kernel(fp8lm_meta* meta, int n, int clean0) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  fp8lm_meta M;
  M.scale = 1.0f; M.inv_scale = 1.0f; M.amax = 0.0f; M.amax_deq = 0.0f;
  for (int h = 0; h < FP8LM_HIST; ++h) M.amax_hist[h] = 0.0f;
  M.hist_pos = 0; M.mu_exp = 0; M.clean_steps = clean0; M.flags = 0; M.n_sat = 0; M.n_underflow = 0;
  meta[t] = M;
}

// Plain streaming copy: every workgroup owns one contiguous range, four 128-bit loads in flight per
// thread, non-temporal on both sides.
__global__ __launch_bounds__(kThreads) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, long long n16) {
  const long long b0 = n16 * blockIdx.x / gridDim.x, b1 = n16 * (blockIdx.x + 1) / gridDim.x;
  long long i = b0 + threadIdx.x;
  for (; i + 3 * kThreads < b1; i += 4 * kThreads) {
    const uint4 a = ld16<true>(src + i), b = ld16<true>(src + i + kThreads), c = ld16<true>(src + i + 2 * kThreads),
                d = ld16<true>(src + i + 3 * kThreads);
    st16<true>(dst + i, a);
    st16<true>(dst + i + kThreads, b);
    st16<true>(dst + i + 2 * kThreads, c);
    st16<true>(dst + i + 3 * kThreads, d);
  }
  for (; i < b1; i += kThreads) st16<true>(dst + i, ld16<true>(src + i));
}

// Memory-only skeletons of the hot kernels: the same persistent grid, tile walk, access widths, access layout and
// cache policies as the kernels they stand for, with the arithmetic replaced by XORs.  What they reach is the
// bandwidth ceiling of that access pattern on this machine; the real kernels are measured against it.
//   NS1 / NS2 : number of 8-bit / 16-bit streams read;  ND1 / ND2 : number of 8-bit / 16-bit streams written.
// A thread takes elements [8L, 8L+8) of both halves of a 4096-element tile (L = thread index), like the update and
// cast kernels: 64-bit accesses on 8-bit streams, 128-bit accesses on 16-bit streams, contiguous over the workgroup.
struct SkeletonParams {
  const uint8_t* s1[2];
  const uint16_t* s2[2];
  uint8_t* d1[2];
  uint16_t* d2[2];
  long long n_tiles;
  uint32_t* sink;        // one word per workgroup, so that pure reads cannot be optimised away
};
template <int NS1, int NS2, int ND1, int ND2, int UN>
__global__ __launch_bounds__(kThreads) void skeleton_kernel(SkeletonParams p) {
  const long long t0 = p.n_tiles * blockIdx.x / gridDim.x, t1 = p.n_tiles * (blockIdx.x + 1) / gridDim.x;
  uint32_t acc = 0;
  auto body = [&](long long tile, auto un_tag) {
    constexpr int U = decltype(un_tag)::value;
    uint2 a1[U][NS1 > 0 ? NS1 : 1][2];
    uint4 a2[U][NS2 > 0 ? NS2 : 1][2];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long a = (tile + u) * kTile + threadIdx.x * 8, b = a + kTile / 2;
#pragma unroll
      for (int i = 0; i < NS1; ++i) { a1[u][i][0] = ld8<true>(p.s1[i] + a); a1[u][i][1] = ld8<true>(p.s1[i] + b); }
#pragma unroll
      for (int i = 0; i < NS2; ++i) { a2[u][i][0] = ld16<true>(p.s2[i] + a); a2[u][i][1] = ld16<true>(p.s2[i] + b); }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long a = (tile + u) * kTile + threadIdx.x * 8, b = a + kTile / 2;
      uint32_t x = acc, y = ~acc;
#pragma unroll
      for (int i = 0; i < NS1; ++i) { x ^= a1[u][i][0].x ^ a1[u][i][1].y; y ^= a1[u][i][0].y ^ a1[u][i][1].x; }
#pragma unroll
      for (int i = 0; i < NS2; ++i) {
        x ^= a2[u][i][0].x ^ a2[u][i][0].z ^ a2[u][i][1].y ^ a2[u][i][1].w;
        y ^= a2[u][i][0].y ^ a2[u][i][0].w ^ a2[u][i][1].x ^ a2[u][i][1].z;
      }
      acc = x + y;
#pragma unroll
      for (int i = 0; i < ND1; ++i) { st8<true>(p.d1[i] + a, make_uint2(x, y)); st8<true>(p.d1[i] + b, make_uint2(y, x)); }
#pragma unroll
      for (int i = 0; i < ND2; ++i) { st16<true>(p.d2[i] + a, make_uint4(x, y, y, x)); st16<true>(p.d2[i] + b, make_uint4(y, x, x, y)); }
    }
  };
  long long tile = t0;
  for (; tile + UN <= t1; tile += UN) body(tile, std::integral_constant<int, UN>{});
  for (; tile < t1; ++tile) body(tile, std::integral_constant<int, 1>{});
  if constexpr (ND1 + ND2 == 0) {
    acc = wave_or_u32(acc);
    if ((threadIdx.x & 63) == 0) p.sink[blockIdx.x * kWaves + (threadIdx.x >> 6)] = acc;
  }
}

}  // namespace fp8lm

#endif
