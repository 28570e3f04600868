// libfp8lm: FP8 gradient quantisation and FP8 Adam step of FP8-LM (arXiv 2310.18313, Sec. 2.1, 2.2,
// Appendix A) for MI355X / gfx950.  See include/fp8lm.h for the boundary.
//
// Shape of every hot kernel
//   * The tensor list is cut into chunks of `chunk_elems` elements that never straddle a tensor.  A
//     persistent grid of 256-thread workgroups (a few per compute unit) walks the chunk table, so a
//     5 K-element bias and a 250 M-element matrix are served by the same launch.
//   * A thread handles 16 consecutive elements per iteration: one 128-bit access for 8-bit buffers,
//     two adjacent 128-bit accesses for 16-bit buffers; a wavefront covers 1 KiB / 2 KiB contiguous.
//   * Per-tensor statistics (amax, counters) are kept in registers while a workgroup stays inside one
//     tensor, then reduced wavefront -> LDS -> one atomic per workgroup into a per-tensor scratch slot.
//     A ticket counter of finished chunks tells the last workgroup of a tensor to run the scalar
//     epilogue (scale update, auto-scaling state, metadata) and to clear the scratch: a single pass,
//     no second launch.
//   * These kernels are HBM-bandwidth bound (2..12 bytes per element against ~40 ALU operations); no
//     matrix cores are involved.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <numeric>
#include <queue>
#include <string>
#include <vector>

#include "fp8lm.h"
#include "formats.hpp"

namespace fp8lm {

constexpr int kThreads = 256;
constexpr int kGroup = 16;                 // elements per thread per iteration
constexpr int kTile = kThreads * kGroup;   // elements per workgroup per iteration
constexpr int kWaves = kThreads / 64;
constexpr int kMaxBlocksPerCu = 16;        // upper limit of the launch tuning; sizes the record array

struct TensorDesc {
  int64_t offset;
  int64_t numel;
  int32_t first_chunk;
  int32_t n_chunks;
};

// Per-tensor scratch.  The ticket is zero between launches; the `pend` block carries the scales chosen
// by the first Adam pass to the second.
struct Scratch {
  uint32_t ticket;                // chunks finished
  uint32_t pad[3];
  struct Pending {
    float sm, ism, sv, isv, sw, isw, sq, isq;
    uint32_t fm, fv, fw, fq;      // flags gathered while choosing the scales
    uint32_t careful;
    uint32_t amax_m_bits;   // written by a fused cast: bit pattern of max |m'|
  } pend;
};

// What one workgroup found in its part of one tensor: maxima (bit patterns of non-negative values),
// counters and an OR-mask.  One record per (workgroup, tensor) pair, each in a cache line of its own.
struct alignas(128) Partial {
  uint32_t mx[3];
  uint32_t orv;
  unsigned long long ct[8];
};

struct Tables {
  const TensorDesc* desc;
  const int32_t* chunk_tensor;
  Scratch* scratch;
  Partial* partials;              // [grid + n_tensors]
  int32_t n_chunks;
  int32_t chunk_elems;
  int32_t deferred;               // 1: workgroups only leave their records; an epilogue launch finishes the tensors
};

// ---- reductions ----------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, o, 64));
  return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ uint32_t wave_or_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v |= (uint32_t)__shfl_xor((int)v, o, 64);
  return v;
}

// Workgroup-wide combine of up to NV maxima, NC counters and one OR-mask; result valid in thread 0.
template <int NV, int NC>
struct BlockStats {
  uint32_t mx[NV > 0 ? NV : 1];
  unsigned long long ct[NC > 0 ? NC : 1];
  uint32_t orv;
};

template <int NV, int NC>
__device__ __forceinline__ void block_combine(BlockStats<NV, NC>& s) {
  __shared__ uint32_t l_mx[kWaves][NV > 0 ? NV : 1];
  __shared__ unsigned long long l_ct[kWaves][NC > 0 ? NC : 1];
  __shared__ uint32_t l_or[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < NV; ++i) s.mx[i] = wave_max_u32(s.mx[i]);
#pragma unroll
  for (int i = 0; i < NC; ++i) s.ct[i] = wave_sum_u64(s.ct[i]);
  s.orv = wave_or_u32(s.orv);
  __syncthreads();   // the previous use of the LDS arrays is over
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) l_mx[wave][i] = s.mx[i];
#pragma unroll
    for (int i = 0; i < NC; ++i) l_ct[wave][i] = s.ct[i];
    l_or[wave] = s.orv;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
#pragma unroll
      for (int i = 0; i < NV; ++i) s.mx[i] = max(s.mx[i], l_mx[w][i]);
#pragma unroll
      for (int i = 0; i < NC; ++i) s.ct[i] += l_ct[w][i];
      s.orv |= l_or[w];
    }
  }
}

// Cross-workgroup reduction of a tensor's statistics.
//
// Workgroup b walks the chunk range [b*C/G, (b+1)*C/G), so the workgroups that touch tensor t are
// consecutive and a workgroup touches consecutive tensors: record b + t is unique to the pair (b, t) and
// the records of one tensor are contiguous.  Every workgroup stores its partial result into its record
// (each record has a cache line of its own).  What happens next has two forms:
//
//  * single pass: the workgroup adds its finished chunks to the tensor's ticket with one atomic; the
//    workgroup whose addition completes the ticket reads the records of all the others, combines them
//    and runs the tensor's scalar epilogue.  Measured on MI355X, a ticket costs every workgroup about
//    20 ns that do not overlap with those of other workgroups (12 ns for an atomic on an address all
//    workgroups share, 8 ns for the release that makes the record visible): 80 us for a launch of 4096
//    workgroups, nothing beside the milliseconds of a 13B-parameter model, more than the data of a
//    100M-parameter one.
//  * deferred: no ticket; a second, tiny launch (one workgroup per tensor) combines the records after the
//    first has ended and runs the epilogues.  Costs one launch (about 3 us), independent of the grid.
//
// The host picks the form per launch from the chunks each workgroup has (fp8lm_set_tuning); the default is
// the deferred form at every size.
//
// Ordering in the single pass: records are written and read with agent-scope atomic accesses (they bypass
// the caches that are not coherent across the chip); the ticket is bumped with release/acquire semantics,
// so the completing workgroup observes every record written before the other workgroups' bumps.
template <int NV, int NC>
__device__ __forceinline__ void store_record(const Tables& tb, int t, const BlockStats<NV, NC>& s) {
  Partial* rec = tb.partials + ((long long)blockIdx.x + t);
#pragma unroll
  for (int i = 0; i < NV; ++i) __hip_atomic_store(&rec->mx[i], s.mx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
  for (int i = 0; i < NC; ++i) __hip_atomic_store(&rec->ct[i], s.ct[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(&rec->orv, s.orv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Combines the records of all workgroups of a launch with `grid` workgroups that touched tensor t.  Called
// by all threads; the totals end up in thread 0's `s`.
template <int NV, int NC>
__device__ __forceinline__ void gather_records(const Tables& tb, int t, const TensorDesc& d, long long grid, BlockStats<NV, NC>& s) {
  // owner(c) = the b with b*C/G <= c < (b+1)*C/G
  const long long C = tb.n_chunks;
  const long long c0 = d.first_chunk, c1 = c0 + d.n_chunks - 1;
  const long long b_lo = ((c0 + 1) * grid - 1) / C, b_hi = ((c1 + 1) * grid - 1) / C;
#pragma unroll
  for (int i = 0; i < NV; ++i) s.mx[i] = 0;
#pragma unroll
  for (int i = 0; i < NC; ++i) s.ct[i] = 0;
  s.orv = 0;
  for (long long b = b_lo + threadIdx.x; b <= b_hi; b += kThreads) {
    const Partial* rec = tb.partials + (b + t);
#pragma unroll
    for (int i = 0; i < NV; ++i) s.mx[i] = max(s.mx[i], __hip_atomic_load(&rec->mx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
#pragma unroll
    for (int i = 0; i < NC; ++i) s.ct[i] += __hip_atomic_load(&rec->ct[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s.orv |= __hip_atomic_load(&rec->orv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  block_combine(s);
}

// Called by all threads at the end of a workgroup's part of tensor t, after block_combine(s).  Returns
// true in every thread of the workgroup that has to run the tensor's epilogue, with the tensor's totals in
// thread 0's `s`; always false in the deferred form.
template <int NV, int NC>
__device__ __forceinline__ bool collect(const Tables& tb, int t, const TensorDesc& d, int done, BlockStats<NV, NC>& s) {
  if (tb.deferred) {
    if (threadIdx.x == 0) store_record(tb, t, s);
    return false;
  }
  __shared__ int l_last;
  if (threadIdx.x == 0) {
    store_record(tb, t, s);
    Scratch* sc = tb.scratch + t;
    const uint32_t old = __hip_atomic_fetch_add(&sc->ticket, (uint32_t)done, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = old + (uint32_t)done == (uint32_t)d.n_chunks;
    if (last) __hip_atomic_store(&sc->ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch
    l_last = last;
  }
  __syncthreads();
  const bool last = l_last != 0;
  __syncthreads();                 // l_last may be rewritten by the next flush
  if (!last) return false;
  gather_records(tb, t, d, gridDim.x, s);
  return true;
}

// The second launch of the deferred form: workgroup t finishes tensor t.
template <class Op, class Params>
__global__ __launch_bounds__(kThreads) void epilogue_kernel(Tables tb, Params p, int main_grid, int n_tensors) {
  Op op(p, tb);
  for (int t = blockIdx.x; t < n_tensors; t += gridDim.x) {
    const TensorDesc d = tb.desc[t];
    if (d.n_chunks == 0) continue;
    op.begin(t, d);
    typename Op::Stats s;
    gather_records(tb, t, d, main_grid, s);
    if (threadIdx.x == 0) op.finalize(t, d, s);
  }
}

__device__ __forceinline__ void atomic_add_u64(unsigned long long* p, unsigned long long v) {
  if (v) __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- the chunk walk shared by all kernels -------------------------------------------------------
// Op must provide: begin(t, desc); fast() (uniform: may the vector path be used for this tensor);
// tiles<UN>(pos): UN complete 4096-element tiles starting at element `pos` of the flat buffers, handled
// by the whole workgroup (all loads issued before the first use; the op chooses which 16 elements of
// a tile a thread takes); group(pos, valid) with 1 <= valid <= 16 for everything else, element by
// element; flush(t, desc, chunks_done) (called by all threads).
template <int UN, class Op>
__device__ __forceinline__ void walk_chunks(const Tables& tb, Op& op) {
  // workgroup b walks the contiguous chunk range [b*C/G, (b+1)*C/G): `collect` relies on this mapping
  const long long G = gridDim.x, b = blockIdx.x;
  long long c = b * tb.n_chunks / G;
  const long long c_end = (b + 1) * tb.n_chunks / G, step = 1;
  int cur = -1, done = 0;
  TensorDesc d{};
  // the tensor id of the next chunk is fetched one iteration ahead, so its latency hides behind the body
  int t_next = c < c_end ? tb.chunk_tensor[c] : -1;
  for (; c < c_end; c += step) {
    const int t = t_next;
    t_next = c + step < c_end ? tb.chunk_tensor[c + step] : -1;
    if (t != cur) {
      if (cur >= 0) op.flush(cur, d, done);
      cur = t;
      done = 0;
      d = tb.desc[t];
      op.begin(t, d);
    }
    const long long e0 = (long long)((int)c - d.first_chunk) * tb.chunk_elems;
    const long long rest = d.numel - e0;
    const int len = rest < tb.chunk_elems ? (int)rest : tb.chunk_elems;
    const long long base = d.offset + e0;
    const int ntiles = len / kTile;
    int tile = 0;
    if (op.fast()) {
      if constexpr (UN > 1)
        for (; tile + UN <= ntiles; tile += UN) op.template tiles<UN>(base + (long long)tile * kTile);
      for (; tile < ntiles; ++tile) op.template tiles<1>(base + (long long)tile * kTile);
    }
    for (int i = tile * kTile + threadIdx.x * kGroup; i < len; i += kTile) {
      const int valid = len - i < kGroup ? len - i : kGroup;
      op.group(base + i, valid);
    }
    ++done;
  }
  if (cur >= 0) op.flush(cur, d, done);
}

// Build-time tuning knobs (defaults are the measured best on MI355X).
#ifndef FP8LM_NT_MASK
#define FP8LM_NT_MASK 15  // bit0 non-temporal loads of read-only streams, bit1 non-temporal stores of write-only
                          // streams, bit2 / bit3 the same for the in-place (read-modify-write) streams.  All four
                          // measured best with the split access layout (bits 2+3 together: -1 % on the update
                          // kernel; bit 3 alone: +0.7 %)
#endif
#ifndef FP8LM_UN_READ
#define FP8LM_UN_READ 4   // 16-element groups a thread keeps in flight in the read-only kernels
#endif
#ifndef FP8LM_UN_CAST
#define FP8LM_UN_CAST 2
#endif
#ifndef FP8LM_UN_UPDATE
#define FP8LM_UN_UPDATE 1
#endif
#ifndef FP8LM_SINGLE_PASS_MIN_CHUNKS
#define FP8LM_SINGLE_PASS_MIN_CHUNKS (1 << 30)   // launches with fewer chunks per workgroup finish their tensors in
                                                 // a second launch instead of through tickets (see collect); the
                                                 // default never uses tickets: the second launch measured faster
                                                 // at every size, 2 % on the read-only kernels even at 13e9 parameters
#endif
#ifndef FP8LM_CAST_SPLIT
#define FP8LM_CAST_SPLIT 1     // cast kernel, 16-bit sources: the same split layout as the update kernel
#endif
#ifndef FP8LM_UPDATE_SPLIT
#define FP8LM_UPDATE_SPLIT 1   // update kernel: a thread takes elements [8L, 8L+8) of both halves of a tile, so
                               // that every access of the workgroup is contiguous (0: 16 consecutive elements)
#endif
constexpr bool kNtLoadRO = (FP8LM_NT_MASK & 1) != 0, kNtStoreWO = (FP8LM_NT_MASK & 2) != 0;
constexpr bool kNtLoadRW = (FP8LM_NT_MASK & 4) != 0, kNtStoreRW = (FP8LM_NT_MASK & 8) != 0;

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <bool NT = false> __device__ __forceinline__ uint4 ld16(const void* p) {
  if constexpr (NT) {
    const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
  } else {
    return *reinterpret_cast<const uint4*>(p);
  }
}
template <bool NT = false> __device__ __forceinline__ void st16(void* p, uint4 v) {
  if constexpr (NT) {
    const u32x4_t r = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(r, reinterpret_cast<u32x4_t*>(p));
  } else {
    *reinterpret_cast<uint4*>(p) = v;
  }
}

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <bool NT = false> __device__ __forceinline__ uint2 ld8(const void* p) {
  if constexpr (NT) {
    const u32x2_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
    return make_uint2(r.x, r.y);
  } else {
    return *reinterpret_cast<const uint2*>(p);
  }
}
template <bool NT = false> __device__ __forceinline__ void st8(void* p, uint2 v) {
  if constexpr (NT) {
    const u32x2_t r = {v.x, v.y};
    __builtin_nontemporal_store(r, reinterpret_cast<u32x2_t*>(p));
  } else {
    *reinterpret_cast<uint2*>(p) = v;
  }
}

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
      } else if (p.fmax_bits == 0u) {      // BF16 / FP32 master weights carry no scale
        M.scale = 1.0f;
        M.inv_scale = 1.0f;
      } else {
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
__device__ __forceinline__ void autoscale_update(fp8lm_meta& M, unsigned long long n_sat, long long numel, int sat_num,
                                                 int sat_den, int ramp_steps) {
  const int R = ramp_steps < 2 ? 2 : ramp_steps;
  const bool overflow = (long long)n_sat * (long long)sat_den > numel * (long long)sat_num;
  const int clean = overflow ? 0 : (M.clean_steps + 1 > R ? R : M.clean_steps + 1);
  M.clean_steps = clean;
  const int ramp = (2 * clean) / R;
  M.mu_exp = -1 + (ramp > 2 ? 2 : ramp);
}

struct CastParams {
  const void* src;
  uint8_t* dst;
  fp8lm_meta* meta;
  int32_t sat_num, sat_den, ramp_steps;
  int32_t hist_window;   // delayed scaling only
  // fused first pass of the Adam step (FUSE): the first moment as it stands and beta1
  const uint8_t* m;
  const fp8lm_meta* m_meta;
  float b1, omb1;
};

// number of zero bytes among the four 7-bit fields of x (each byte of x must be <= 0x7F)
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
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) {
    // kSplit: the thread's 16 elements are [8L, 8L+8) of each half of the tile (every 128-bit load contiguous
    // over the workgroup, 64-bit stores); otherwise 16 consecutive elements.
    constexpr bool kSplit = FP8LM_CAST_SPLIT && kSrc16<SRC>;
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
    auto store = [&](int u, const uint4& o) {
      if constexpr (kSplit) {
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
      if constexpr (DELAYED) {
        if (note_source(w)) {   // rare: this group holds inf/NaN, encode it element by element
          const uint32_t mw[4] = {mm[u].x, mm[u].y, mm[u].z, mm[u].w};
          const uint32_t keep = amax16;
          uint4 o = make_uint4(0, 0, 0, 0);
          uint32_t* ow = &o.x;
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const uint32_t bits = kSrc16<SRC> ? (w[(j >> 1) % kW] >> ((j & 1) * 16)) & 0xFFFFu : w[j % kW];
            ow[j >> 2] |= one(bits, FUSE ? (mw[j >> 2] >> ((j & 3) * 8)) & 0xFFu : 0u) << ((j & 3) * 8);
          }
          amax16 = keep;
          store(u, o);
          continue;
        }
      }
      uint4 o;
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
      store(u, o);
    }
    n_elems += UN * kGroup;
  }
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
    {
      {
        const float vm = u2f(s.mx[0]);
        const uint32_t abits = s.mx[1];
        if constexpr (FUSE) tb.scratch[t].pend.amax_m_bits = s.mx[2];
        const unsigned long long n_sat = s.ct[0], n_und = s.ct[1];
        if constexpr (DELAYED) {
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
    }
  }
  __device__ void finish(int t, const TensorDesc& d, float vm, unsigned long long n_sat, unsigned long long n_und) {
    fp8lm_meta& M = p.meta[t];
    M.n_sat = n_sat;
    M.n_underflow = n_und;
    M.amax_deq = fp8_to_f32<FMT>(encode1_fp8<FMT>(vm)) * M.inv_scale;
    M.flags = n_sat ? (M.flags | FP8LM_FLAG_SATURATED) : (M.flags & ~FP8LM_FLAG_SATURATED);
    autoscale_update(M, n_sat, d.numel, p.sat_num, p.sat_den, p.ramp_steps);
  }
};

template <int FMT, bool DELAYED, bool FUSE, int SRC>
__global__ __launch_bounds__(kThreads) void cast_kernel(Tables tb, CastParams p) {
  CastOp<FMT, DELAYED, FUSE, SRC> op(p, tb);
  walk_chunks<FP8LM_UN_CAST>(tb, op);
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
constexpr int kMaxRanks = 8;
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
    {
      {
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
    }
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
  int32_t sat_num, sat_den, ramp_steps;
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
  template <int UN> __device__ __forceinline__ void tiles(long long pos0) {
    const long long pos = pos0 + threadIdx.x * kGroup;
    uint4 a[UN][NR];
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
      for (int r = 0; r < NR; ++r) {            // rank order, one fp32 addition per rank
        const uint32_t w[4] = {a[u][r].x, a[u][r].y, a[u][r].z, a[u][r].w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float2_t lo = fp8x2_to_f32<FMT, false>(w[k]), hi = fp8x2_to_f32<FMT, true>(w[k]);
          acc[4 * k + 0] = acc[4 * k + 0] + lo.x;
          acc[4 * k + 1] = acc[4 * k + 1] + lo.y;
          acc[4 * k + 2] = acc[4 * k + 2] + hi.x;
          acc[4 * k + 3] = acc[4 * k + 3] + hi.y;
        }
      }
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
      st16<kNtStoreWO>(p.dst + pos + u * kTile, make_uint4(o[0], o[1], o[2], o[3]));
    }
    n_elems += UN * kGroup;
  }
  __device__ __forceinline__ void group(long long pos, int valid) {
    for (int j = 0; j < valid; ++j) {
      float acc = 0.0f;
#pragma unroll
      for (int r = 0; r < NR; ++r) acc = acc + fp8_to_f32<FMT>(p.in.p[r][pos + j]);
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
    {
      {
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
        autoscale_update(M, n_sat, d.numel, p.sat_num, p.sat_den, p.ramp_steps);
      }
    }
  }
};

template <int FMT, int NR>
__global__ __launch_bounds__(kThreads) void sum_fp8_kernel(Tables tb, SumParams p) {
  SumOp<FMT, NR> op(p, tb);
  walk_chunks<(NR <= 2 ? 4 : NR <= 4 ? 2 : 1)>(tb, op);   // about eight 128-bit loads in flight per thread
}

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
    {
      {
        const float vm = u2f(s.mx[0]);
        fp8lm_meta& M = p.meta[t];
        M.n_sat = s.ct[0];
        M.n_underflow = s.ct[1];
        M.amax_deq = vm * M.inv_scale;        // vm is already a stored value
        if (M.n_sat) M.flags |= FP8LM_FLAG_SATURATED;
      }
    }
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
  uint8_t* m;
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
template <bool FAST> __device__ __forceinline__ float adam_update(float m1, float v1, float w0, const AdamParams& p) {
  if constexpr (FAST) {
    const float den = __builtin_amdgcn_sqrtf(v1 * p.rbc2) + p.eps;
    const float upd = (m1 * p.rbc1) * __builtin_amdgcn_rcpf(den);
    return __builtin_fmaf(-p.lr, upd, w0 * p.decay);
  } else {
    const float den = __builtin_sqrtf(v1 * p.rbc2) + p.eps;
    const float upd = ((m1 * p.rbc1) / den);
    return __builtin_fmaf(-p.lr, upd, w0 * p.decay);
  }
}

template <int GFMT, int WCOPY, bool FAST, bool STATS>
struct AdamUpdateOp {
  const AdamParams& p;
  const Tables& tb;
  float inv_sg, inv_sm, inv_sv, inv_sw;   // scales of the inputs
  float sm, sv, sw, sq;                   // scales of the outputs
  bool careful;
  float vmax, wmax, mmax;                 // running maxima of v', |w'| (and |m'| on the careful path)
  uint32_t nf;
  uint32_t cnt[8];                        // sat m,v,w,q ; underflow m,v,w,q: per lane (tails, careful path)
  uint32_t wcnt[8];                       // the same for whole tiles: wave totals, identical in every lane
  __device__ AdamUpdateOp(const AdamParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc&) {
    const Scratch::Pending& P = tb.scratch[t].pend;
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
      const float w1 = adam_update<FAST>(m1, v1, w0, p);
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
    const float m0 = fp8_to_f32<kE4M3>(p.m[i]) * inv_sm;
    uint16_t* pv = static_cast<uint16_t*>(p.v);
    uint16_t* pw = static_cast<uint16_t*>(p.w);
    const float v0 = f16_to_f32(pv[i]) * inv_sv;
    const float w0 = f16_to_f32(pw[i]) * inv_sw;
    const float m1 = __builtin_fmaf(p.b1, m0, p.omb1 * g);
    const float v1 = __builtin_fmaf(p.b2, v0, p.omb2 * (g * g));
    const float den = __builtin_sqrtf(v1 * p.rbc2) + p.eps;
    const float upd = ((m1 * p.rbc1) / den);
    const float w1 = __builtin_fmaf(-p.lr, upd, w0 * p.decay);
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
      ma[u] = ld8<kNtLoadRW>(p.m + a);
      mb[u] = ld8<kNtLoadRW>(p.m + b);
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
    if constexpr (FP8LM_UPDATE_SPLIT) {
      tiles_split<UN>(tile0);
      return;
    }
    uint4 g[UN], m[UN], va[UN], vb[UN], wa[UN], wb[UN];
    const long long pos0 = tile0 + threadIdx.x * kGroup;
    uint16_t* pv = static_cast<uint16_t*>(p.v);
    uint16_t* pw = static_cast<uint16_t*>(p.w);
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const long long pos = pos0 + u * kTile;
      g[u] = ld16<kNtLoadRO>(p.grad + pos);
      m[u] = ld16<kNtLoadRW>(p.m + pos);
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
  __device__ __forceinline__ void group(long long pos, int valid) {
    if (!careful) {
      // ragged tail of a tensor: same arithmetic, element by element
      uint16_t* pv = static_cast<uint16_t*>(p.v);
      uint16_t* pw = static_cast<uint16_t*>(p.w);
      for (int j = 0; j < valid; ++j) {
        const long long i = pos + j;
        const Quad o = quad<false>(p.grad[i], p.m[i], pv[i], 0u, pw[i], 0u);
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
    {
      unsigned long long c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if constexpr (STATS) {
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = s.ct[i];
      }
      finish(t, u2f(s.mx[0]), u2f(s.mx[1]), u2f(s.mx[2]), s.orv, c);
    }
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
    const Scratch::Pending& P = tb.scratch[t].pend;
    const float A_m = A_mc;    // measured by this pass on both paths (equals what pass A saw)
    uint32_t m_nf = nfb & 3u;
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
  float inv_sg, inv_sm, inv_sv, inv_sw, sm, sv, sw, sq;
  bool careful;
  float vmax, wmax, mmax;
  uint32_t nf;
  __device__ AdamUpdateVarOp(const AdamParams& p_, const Tables& tb_) : p(p_), tb(tb_) {}
  __device__ __forceinline__ void begin(int t, const TensorDesc&) {
    const Scratch::Pending& P = tb.scratch[t].pend;
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
    w1 = __builtin_fmaf(-p.lr, upd, w0 * p.decay);
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
    {
      {
        const float A_v = u2f(s.mx[0]), A_w = u2f(s.mx[1]), A_m = u2f(s.mx[2]);
        const uint32_t nfb = s.orv;
        const Scratch::Pending& P = tb.scratch[t].pend;
        fill<StTraits<kStE4M3>>(p.m_meta[t], P.sm, P.ism, A_m, nfb & 3u, P.fm);
        fill<VT>(p.v_meta[t], P.sv, P.isv, A_v, (nfb >> 2) & 3u, P.fv);
        fill<WT>(p.w_meta[t], P.sw, P.isw, A_w, (nfb >> 4) & 3u, P.fw);
        fill<StTraits<kStE4M3>>(p.wcopy_meta[t], P.sq, P.isq, A_w, (nfb >> 4) & 3u, P.fq);
      }
    }
  }
};

template <int GFMT, int MASTER, int VFMT>
__global__ __launch_bounds__(kThreads) void adam_update_var_kernel(Tables tb, AdamParams p) {
  AdamUpdateVarOp<GFMT, MASTER, VFMT> op(p, tb);
  walk_chunks<1>(tb, op);
}

// ---- small kernels ---------------------------------------------------------------------------------
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

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// workgroup-wide sum of two doubles; result valid in thread 0
__device__ __forceinline__ void block_sum2_f64(double& a, double& b) {
  __shared__ double l[kWaves][2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  a = wave_sum_f64(a);
  b = wave_sum_f64(b);
  __syncthreads();
  if (lane == 0) { l[wave][0] = a; l[wave][1] = b; }
  __syncthreads();
  if (threadIdx.x == 0)
#pragma unroll
    for (int w = 1; w < kWaves; ++w) { a += l[w][0]; b += l[w][1]; }
}

template <int FMT, int SRC>
struct QuantStatsOp {
  using elem_t = typename SrcTraits<SRC>::elem_t;
  static constexpr int kPer = 16 / (int)sizeof(elem_t);
  static constexpr int kLoads = kGroup / kPer;
  static constexpr int kW = kSrcWords<SRC>;
  const StatsParams& p;
  double rs, signal, noise;
  uint32_t n_nonzero, n_under, n_over, n_nonfinite;
  __device__ QuantStatsOp(const StatsParams& p_) : p(p_) {}
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
  __device__ __forceinline__ void group(long long pos, int valid) {
    const elem_t* rp = static_cast<const elem_t*>(p.ref) + pos;
    for (int j = 0; j < valid; ++j) one(rp[j], p.q[pos + j]);
  }
  __device__ __forceinline__ void flush(int t, const TensorDesc&, int) {
    BlockStats<0, 4> s;
    s.ct[0] = n_nonzero; s.ct[1] = n_under; s.ct[2] = n_over; s.ct[3] = n_nonfinite;
    s.orv = 0;
    block_combine(s);
    block_sum2_f64(signal, noise);
    if (threadIdx.x == 0) {
      fp8lm_quant_stats* o = p.out + t;
      if (signal != 0.0) __hip_atomic_fetch_add(&o->signal, signal, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (noise != 0.0) __hip_atomic_fetch_add(&o->noise, noise, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      atomic_add_u64(reinterpret_cast<unsigned long long*>(&o->n_nonzero), s.ct[0]);
      atomic_add_u64(reinterpret_cast<unsigned long long*>(&o->n_underflow), s.ct[1]);
      atomic_add_u64(reinterpret_cast<unsigned long long*>(&o->n_overflow), s.ct[2]);
      atomic_add_u64(reinterpret_cast<unsigned long long*>(&o->n_nonfinite), s.ct[3]);
    }
  }
};

template <int FMT, int SRC>
__global__ __launch_bounds__(kThreads) void quant_stats_kernel(Tables tb, StatsParams p) {
  QuantStatsOp<FMT, SRC> op(p);
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

}  // namespace fp8lm

// ====================================================================================================
// Host side: context, validation, launches
// ====================================================================================================
using namespace fp8lm;

static thread_local std::string g_hip_error;

struct fp8lm_ctx {
  int device = 0;
  int n_tensors = 0;
  int num_cus = 0;
  std::vector<fp8lm_tensor> tensors;
  int32_t chunk_elems = 16384;
  int32_t blocks_per_cu = kMaxBlocksPerCu;
  int32_t single_pass_min_chunks = FP8LM_SINGLE_PASS_MIN_CHUNKS;
  int32_t n_chunks = 0;
  TensorDesc* d_desc = nullptr;
  int32_t* d_chunk_tensor = nullptr;
  Scratch* d_scratch = nullptr;
  Partial* d_partials = nullptr;    // [num_cus * kMaxBlocksPerCu + n_tensors]
  // what the last fused cast measured for (checked by the Adam step that wants to use it)
  struct Fused { bool valid; const uint8_t* grad; const uint8_t* m; const fp8lm_meta* m_meta; float b1; int fmt; };
  Fused fused{false, nullptr, nullptr, nullptr, 0.0f, 0};
  // timing
  bool timing = false;
  struct Stamp { int kernel; hipEvent_t a, b; };
  std::vector<Stamp> stamps;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> free_events;
};

#define HIP_TRY(expr)                                                      \
  do {                                                                     \
    hipError_t e_ = (expr);                                                \
    if (e_ != hipSuccess) {                                                \
      g_hip_error = std::string(#expr) + ": " + hipGetErrorString(e_);     \
      return FP8LM_ERR_HIP;                                                \
    }                                                                      \
  } while (0)

namespace {

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
    if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
    if (prev == dev) prev = -1;
  }
  ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

fp8lm_status build_tables(fp8lm_ctx* c) {
  std::vector<TensorDesc> desc(c->n_tensors);
  std::vector<int32_t> chunk_tensor;
  long long total_chunks = 0;
  for (int t = 0; t < c->n_tensors; ++t) {
    const long long n = c->tensors[t].numel;
    const long long nc = (n + c->chunk_elems - 1) / c->chunk_elems;
    if (total_chunks + nc > 0x7FFFFFF0LL) return FP8LM_ERR_TOO_LARGE;
    desc[t] = TensorDesc{c->tensors[t].offset, n, (int32_t)total_chunks, (int32_t)nc};
    total_chunks += nc;
  }
  chunk_tensor.resize((size_t)total_chunks);
  for (int t = 0; t < c->n_tensors; ++t)
    std::fill(chunk_tensor.begin() + desc[t].first_chunk, chunk_tensor.begin() + desc[t].first_chunk + desc[t].n_chunks, t);
  if (c->d_desc) HIP_TRY(hipFree(c->d_desc));
  if (c->d_chunk_tensor) HIP_TRY(hipFree(c->d_chunk_tensor));
  c->d_desc = nullptr;
  c->d_chunk_tensor = nullptr;
  c->n_chunks = (int32_t)total_chunks;
  HIP_TRY(hipMalloc((void**)&c->d_desc, std::max<size_t>(1, desc.size()) * sizeof(TensorDesc)));
  HIP_TRY(hipMalloc((void**)&c->d_chunk_tensor, std::max<size_t>(1, chunk_tensor.size()) * sizeof(int32_t)));
  if (!desc.empty()) HIP_TRY(hipMemcpy(c->d_desc, desc.data(), desc.size() * sizeof(TensorDesc), hipMemcpyHostToDevice));
  if (!chunk_tensor.empty())
    HIP_TRY(hipMemcpy(c->d_chunk_tensor, chunk_tensor.data(), chunk_tensor.size() * sizeof(int32_t), hipMemcpyHostToDevice));
  return FP8LM_OK;
}

// Workgroups per launch: blocks_per_cu per compute unit, but never more than there are chunks.
int grid_of(const fp8lm_ctx* c) {
  const long long full = (long long)c->num_cus * c->blocks_per_cu;
  return (int)std::max<long long>(1, std::min<long long>(full, c->n_chunks));
}

// The single-pass form of the cross-workgroup reduction costs every workgroup a ticket (about 20 ns that
// do not overlap between workgroups); with few chunks per workgroup that is more than the data.  The
// deferred form (a second, tiny launch) is used below single_pass_min_chunks chunks per workgroup.
bool deferred_of(const fp8lm_ctx* c) {
  return c->single_pass_min_chunks > 0 && c->n_chunks / grid_of(c) < c->single_pass_min_chunks;
}

Tables tables_of(const fp8lm_ctx* c) {
  return Tables{c->d_desc, c->d_chunk_tensor, c->d_scratch, c->d_partials, c->n_chunks, c->chunk_elems,
                deferred_of(c) ? 1 : 0};
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct Timed {
  fp8lm_ctx* c;
  hipStream_t s;
  int kernel;
  hipEvent_t a = nullptr, b = nullptr;
  Timed(fp8lm_ctx* c_, hipStream_t s_, int k) : c(c_), s(s_), kernel(k) {
    if (!c->timing || c->free_events.empty()) return;
    a = c->free_events.back().first;
    b = c->free_events.back().second;
    c->free_events.pop_back();
    (void)hipEventRecord(a, s);
  }
  ~Timed() {
    if (!a) return;
    (void)hipEventRecord(b, s);
    c->stamps.push_back({kernel, a, b});
  }
};

fp8lm_status after_launch() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    g_hip_error = std::string("kernel launch: ") + hipGetErrorString(e);
    return FP8LM_ERR_HIP;
  }
  return FP8LM_OK;
}

// Launches a chunk-walking kernel and, in the deferred form, the launch that finishes its tensors.
template <class Op, class Params, class Kernel>
void launch_walk(fp8lm_ctx* c, hipStream_t s, Kernel kernel, const Params& p) {
  const Tables tb = tables_of(c);
  const dim3 g(grid_of(c)), b(kThreads);
  hipLaunchKernelGGL(kernel, g, b, 0, s, tb, p);
  if (tb.deferred)
    hipLaunchKernelGGL((epilogue_kernel<Op, Params>), dim3(std::min<int>(c->n_tensors, 4 * c->num_cus)), b, 0, s, tb, p,
                       (int)g.x, (int)c->n_tensors);
}

// Selects the adam_update_kernel instantiation.
template <int GFMT, int WCOPY>
void launch_update(fp8lm_ctx* c, hipStream_t s, const AdamParams& p, bool fast, bool stats) {
  const dim3 g(grid_of(c)), b(kThreads);
  const Tables tb = tables_of(c);
  if (fast) {
    if (stats) launch_walk<AdamUpdateOp<GFMT, WCOPY, true, true>>(c, s, adam_update_kernel<GFMT, WCOPY, true, true>, p);
    else launch_walk<AdamUpdateOp<GFMT, WCOPY, true, false>>(c, s, adam_update_kernel<GFMT, WCOPY, true, false>, p);
  } else {
    if (stats) launch_walk<AdamUpdateOp<GFMT, WCOPY, false, true>>(c, s, adam_update_kernel<GFMT, WCOPY, false, true>, p);
    else launch_walk<AdamUpdateOp<GFMT, WCOPY, false, false>>(c, s, adam_update_kernel<GFMT, WCOPY, false, false>, p);
  }
}

// Selects the adam_update_var_kernel instantiation (every master / second-moment format pair except the default).
template <int GFMT>
void launch_update_variant_g(fp8lm_ctx* c, hipStream_t s, const AdamParams& p, int master, int vfmt) {
  const dim3 g(grid_of(c)), b(kThreads);
  const Tables tb = tables_of(c);
#define FP8LM_VAR(M, V) launch_walk<AdamUpdateVarOp<GFMT, M, V>>(c, s, adam_update_var_kernel<GFMT, M, V>, p)
  if (vfmt == kStF16) {
    if (master == kStBF16) FP8LM_VAR(kStBF16, kStF16);
    else if (master == kStE4M3) FP8LM_VAR(kStE4M3, kStF16);
    else FP8LM_VAR(kStF32, kStF16);
  } else {
    if (master == kStF16) FP8LM_VAR(kStF16, kStE4M3);
    else if (master == kStBF16) FP8LM_VAR(kStBF16, kStE4M3);
    else if (master == kStE4M3) FP8LM_VAR(kStE4M3, kStE4M3);
    else FP8LM_VAR(kStF32, kStE4M3);
  }
#undef FP8LM_VAR
}
void launch_update_variant(fp8lm_ctx* c, hipStream_t s, const AdamParams& p, bool e5, int master, int vfmt) {
  if (e5) launch_update_variant_g<kE5M2>(c, s, p, master, vfmt);
  else launch_update_variant_g<kE4M3>(c, s, p, master, vfmt);
}

bool src_ok(fp8lm_src t) { return t == FP8LM_SRC_BF16 || t == FP8LM_SRC_F16 || t == FP8LM_SRC_F32; }
bool cfg_ok(const fp8lm_autoscale_cfg* cfg) {
  return cfg && cfg->sat_num >= 0 && cfg->sat_den > 0 && cfg->ramp_steps >= 2 && cfg->hist_window >= 1 &&
         cfg->hist_window <= FP8LM_HIST && cfg->margin >= -64 && cfg->margin <= 64;
}

}  // namespace

extern "C" {

const char* fp8lm_status_string(fp8lm_status s) {
  switch (s) {
    case FP8LM_OK: return "ok";
    case FP8LM_ERR_INVALID_ARGUMENT: return "invalid argument";
    case FP8LM_ERR_MISALIGNED: return "misaligned offset or buffer";
    case FP8LM_ERR_OVERLAP: return "tensors overlap";
    case FP8LM_ERR_HIP: return "HIP runtime error";
    case FP8LM_ERR_TOO_LARGE: return "too many chunks or tensors";
  }
  return "unknown status";
}

const char* fp8lm_last_hip_error(void) { return g_hip_error.c_str(); }
uint32_t fp8lm_sizeof_meta(void) { return (uint32_t)sizeof(fp8lm_meta); }

fp8lm_status fp8lm_create(fp8lm_ctx** out, const fp8lm_tensor* tensors, int32_t n, int device) {
  if (!out || n < 0 || (n > 0 && !tensors)) return FP8LM_ERR_INVALID_ARGUMENT;
  *out = nullptr;
  for (int t = 0; t < n; ++t) {
    if (tensors[t].numel < 0 || tensors[t].offset < 0) return FP8LM_ERR_INVALID_ARGUMENT;
    if (tensors[t].offset % 16 != 0) return FP8LM_ERR_MISALIGNED;
  }
  {
    std::vector<std::pair<long long, long long>> spans;
    for (int t = 0; t < n; ++t)
      if (tensors[t].numel > 0) spans.emplace_back(tensors[t].offset, tensors[t].offset + tensors[t].numel);
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
      if (spans[i].first < spans[i - 1].second) return FP8LM_ERR_OVERLAP;
  }
  int count = 0;
  HIP_TRY(hipGetDeviceCount(&count));
  if (device < 0 || device >= count) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(device);
  if (!guard.ok) { g_hip_error = "hipSetDevice failed"; return FP8LM_ERR_HIP; }
  hipDeviceProp_t prop;
  HIP_TRY(hipGetDeviceProperties(&prop, device));
  fp8lm_ctx* c = new fp8lm_ctx();
  c->device = device;
  c->n_tensors = n;
  c->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  c->tensors.assign(tensors, tensors + n);
  fp8lm_status st = build_tables(c);
  if (st == FP8LM_OK) {
    const size_t bytes = std::max<size_t>(1, (size_t)n) * sizeof(Scratch);
    hipError_t e = hipMalloc((void**)&c->d_scratch, bytes);
    if (e == hipSuccess) e = hipMemset(c->d_scratch, 0, bytes);
    const size_t records = (size_t)c->num_cus * kMaxBlocksPerCu + (size_t)n + 1;
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_partials, records * sizeof(Partial));
    if (e == hipSuccess) e = hipMemset(c->d_partials, 0, records * sizeof(Partial));
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) { g_hip_error = hipGetErrorString(e); st = FP8LM_ERR_HIP; }
  }
  if (st != FP8LM_OK) { fp8lm_destroy(c); return st; }
  *out = c;
  return FP8LM_OK;
}

fp8lm_status fp8lm_destroy(fp8lm_ctx* c) {
  if (!c) return FP8LM_OK;
  DeviceGuard guard(c->device);
  if (c->d_desc) (void)hipFree(c->d_desc);
  if (c->d_chunk_tensor) (void)hipFree(c->d_chunk_tensor);
  if (c->d_scratch) (void)hipFree(c->d_scratch);
  if (c->d_partials) (void)hipFree(c->d_partials);
  for (auto& s : c->stamps) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
  for (auto& e : c->free_events) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
  delete c;
  return FP8LM_OK;
}

fp8lm_status fp8lm_set_tuning(fp8lm_ctx* c, int32_t chunk_elems, int32_t blocks_per_cu, int32_t single_pass_min_chunks) {
  if (!c || chunk_elems < kTile || chunk_elems > (1 << 20) || chunk_elems % kTile != 0 || blocks_per_cu < 1 ||
      blocks_per_cu > kMaxBlocksPerCu || single_pass_min_chunks < 0 || single_pass_min_chunks > (1 << 30))
    return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  HIP_TRY(hipDeviceSynchronize());
  c->chunk_elems = chunk_elems;
  c->blocks_per_cu = blocks_per_cu;
  c->single_pass_min_chunks = single_pass_min_chunks;
  return build_tables(c);
}

fp8lm_status fp8lm_meta_init(fp8lm_ctx* c, fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, void* stream) {
  if (!c || !cfg_ok(cfg) || (c->n_tensors > 0 && !meta)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_tensors == 0) return FP8LM_OK;
  DeviceGuard guard(c->device);
  const int blocks = (c->n_tensors + 255) / 256;
  hipLaunchKernelGGL(meta_init_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, meta, c->n_tensors,
                     cfg->ramp_steps / 2);
  return after_launch();
}

fp8lm_status fp8lm_amax_scale(fp8lm_ctx* c, const void* src, fp8lm_src src_type, fp8lm_fmt target, fp8lm_meta* meta,
                              const fp8lm_autoscale_cfg* cfg, void* stream) {
  if (!c || !cfg_ok(cfg) || !src_ok(src_type) || (target != FP8LM_E4M3 && target != FP8LM_E5M2))
    return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!src || !meta) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(src)) return FP8LM_ERR_MISALIGNED;
  DeviceGuard guard(c->device);
  AmaxParams p{src, meta, target == FP8LM_E4M3 ? kBitsE4M3Max : kBitsE5M2Max, cfg->hist_window, cfg->margin};
  const dim3 g(grid_of(c)), b(kThreads);
  hipStream_t s = (hipStream_t)stream;
  const Tables tb = tables_of(c);
  Timed tm(c, s, FP8LM_K_AMAX);
  if (src_type == FP8LM_SRC_F32) launch_walk<AmaxOp<kAmaxForGradient, kSrcF32>>(c, s, amax_kernel<kAmaxForGradient, kSrcF32>, p);
  else if (src_type == FP8LM_SRC_F16) launch_walk<AmaxOp<kAmaxForGradient, kSrcF16>>(c, s, amax_kernel<kAmaxForGradient, kSrcF16>, p);
  else launch_walk<AmaxOp<kAmaxForGradient, kSrcBF16>>(c, s, amax_kernel<kAmaxForGradient, kSrcBF16>, p);
  return after_launch();
}

// Common body of the three cast entry points.
static fp8lm_status cast_impl(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                              fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, bool delayed, bool fuse,
                              const uint8_t* m, const fp8lm_meta* m_meta, float beta1, void* stream) {
  if (!c || !cfg_ok(cfg) || !src_ok(src_type) || (fmt != FP8LM_E4M3 && fmt != FP8LM_E5M2))
    return FP8LM_ERR_INVALID_ARGUMENT;
  c->fused.valid = false;
  if (fuse && !(beta1 >= 0.0f && beta1 < 1.0f)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!src || !dst || !meta || (fuse && (!m || !m_meta))) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(src) || !aligned16(dst) || (fuse && !aligned16(m))) return FP8LM_ERR_MISALIGNED;
  DeviceGuard guard(c->device);
  hipStream_t s = (hipStream_t)stream;
  if (delayed) {
    Timed tm(c, s, FP8LM_K_SCALARS);
    hipLaunchKernelGGL(delayed_scale_kernel, dim3((c->n_tensors + 255) / 256), dim3(256), 0, s, c->d_desc, meta,
                       c->n_tensors, fmt == FP8LM_E4M3 ? kBitsE4M3Max : kBitsE5M2Max, cfg->hist_window, cfg->margin);
    fp8lm_status st = after_launch();
    if (st != FP8LM_OK) return st;
  }
  CastParams p{};
  p.src = src;
  p.dst = dst;
  p.meta = meta;
  p.sat_num = cfg->sat_num; p.sat_den = cfg->sat_den; p.ramp_steps = cfg->ramp_steps; p.hist_window = cfg->hist_window;
  p.m = m;
  p.m_meta = m_meta;
  p.b1 = beta1;
  p.omb1 = (float)(1.0 - (double)beta1);
  const dim3 g(grid_of(c)), b(kThreads);
  const Tables tb = tables_of(c);
  {
    Timed tm(c, s, FP8LM_K_CAST);
#define FP8LM_CAST_LAUNCH(F, S)                                                                           \
    do {                                                                                                    \
      if (delayed && fuse) launch_walk<CastOp<F, true, true, S>>(c, s, cast_kernel<F, true, true, S>, p);          \
      else if (delayed) launch_walk<CastOp<F, true, false, S>>(c, s, cast_kernel<F, true, false, S>, p);            \
      else if (fuse) launch_walk<CastOp<F, false, true, S>>(c, s, cast_kernel<F, false, true, S>, p);               \
      else launch_walk<CastOp<F, false, false, S>>(c, s, cast_kernel<F, false, false, S>, p);                        \
    } while (0)
#define FP8LM_CAST_SRC(S)                                                                                   \
    do {                                                                                                    \
      if (fmt == FP8LM_E4M3) FP8LM_CAST_LAUNCH(kE4M3, S);                                                   \
      else FP8LM_CAST_LAUNCH(kE5M2, S);                                                                     \
    } while (0)
    if (src_type == FP8LM_SRC_F32) FP8LM_CAST_SRC(kSrcF32);
    else if (src_type == FP8LM_SRC_F16) FP8LM_CAST_SRC(kSrcF16);
    else FP8LM_CAST_SRC(kSrcBF16);
#undef FP8LM_CAST_SRC
#undef FP8LM_CAST_LAUNCH
  }
  fp8lm_status st = after_launch();
  if (st == FP8LM_OK && fuse) c->fused = {true, dst, m, m_meta, p.b1, fmt};
  return st;
}

fp8lm_status fp8lm_cast_fp8(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                            fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, void* stream) {
  return cast_impl(c, src, src_type, dst, fmt, meta, cfg, false, false, nullptr, nullptr, 0.0f, stream);
}

fp8lm_status fp8lm_cast_fp8_delayed(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                                    fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, void* stream) {
  return cast_impl(c, src, src_type, dst, fmt, meta, cfg, true, false, nullptr, nullptr, 0.0f, stream);
}

fp8lm_status fp8lm_cast_fp8_for_adam(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                                     fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, int32_t delayed,
                                     const uint8_t* m, const fp8lm_meta* m_meta, float beta1, void* stream) {
  return cast_impl(c, src, src_type, dst, fmt, meta, cfg, delayed != 0, true, m, m_meta, beta1, stream);
}

fp8lm_status fp8lm_shared_scale(fp8lm_ctx* c, const fp8lm_meta* const* metas, int32_t n_ranks, float* shared,
                                void* stream) {
  if (!c || !metas || n_ranks < 1 || n_ranks > kMaxRanks) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_tensors == 0) return FP8LM_OK;
  if (!shared) return FP8LM_ERR_INVALID_ARGUMENT;
  RankMetas rm{};
  rm.n_ranks = n_ranks;
  for (int r = 0; r < n_ranks; ++r) {
    if (!metas[r]) return FP8LM_ERR_INVALID_ARGUMENT;
    rm.m[r] = metas[r];
  }
  DeviceGuard guard(c->device);
  Timed tm(c, (hipStream_t)stream, FP8LM_K_SCALARS);
  hipLaunchKernelGGL(shared_scale_kernel, dim3((c->n_tensors + 255) / 256), dim3(256), 0, (hipStream_t)stream, rm,
                     c->n_tensors, shared);
  return after_launch();
}

fp8lm_status fp8lm_requantize_fp8(fp8lm_ctx* c, const uint8_t* src, fp8lm_fmt fmt, const fp8lm_meta* src_meta,
                                  const float* shared, uint8_t* dst, fp8lm_meta* dst_meta, void* stream) {
  if (!c || (fmt != FP8LM_E4M3 && fmt != FP8LM_E5M2)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!src || !src_meta || !shared || !dst || !dst_meta || src_meta == dst_meta) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(src) || !aligned16(dst)) return FP8LM_ERR_MISALIGNED;
  DeviceGuard guard(c->device);
  RequantParams p{src, src_meta, shared, dst, dst_meta};
  Timed tm(c, (hipStream_t)stream, FP8LM_K_REQUANT);
  if (fmt == FP8LM_E4M3)
    launch_walk<RequantOp<kE4M3>>(c, (hipStream_t)stream, requantize_kernel<kE4M3>, p);
  else
    launch_walk<RequantOp<kE5M2>>(c, (hipStream_t)stream, requantize_kernel<kE5M2>, p);
  return after_launch();
}

fp8lm_status fp8lm_sum_fp8(fp8lm_ctx* c, const uint8_t* const* payloads, int32_t n_ranks, fp8lm_fmt fmt,
                           const float* shared, uint8_t* dst, fp8lm_meta* dst_meta, const fp8lm_autoscale_cfg* cfg,
                           void* stream) {
  if (!c || !cfg_ok(cfg) || !payloads || n_ranks < 1 || n_ranks > kMaxRanks || (fmt != FP8LM_E4M3 && fmt != FP8LM_E5M2))
    return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!shared || !dst || !dst_meta) return FP8LM_ERR_INVALID_ARGUMENT;
  SumParams p{};
  p.in.n_ranks = n_ranks;
  for (int r = 0; r < n_ranks; ++r) {
    if (!payloads[r]) return FP8LM_ERR_INVALID_ARGUMENT;
    if (!aligned16(payloads[r])) return FP8LM_ERR_MISALIGNED;
    p.in.p[r] = payloads[r];
  }
  if (!aligned16(dst)) return FP8LM_ERR_MISALIGNED;
  p.shared = shared; p.dst = dst; p.dst_meta = dst_meta;
  p.sat_num = cfg->sat_num; p.sat_den = cfg->sat_den; p.ramp_steps = cfg->ramp_steps;
  DeviceGuard guard(c->device);
  Timed tm(c, (hipStream_t)stream, FP8LM_K_SUM);
  const dim3 g(grid_of(c)), b(kThreads);
  hipStream_t s = (hipStream_t)stream;
  const Tables tb = tables_of(c);
#define FP8LM_SUM_N(N)                                                                          \
  case N:                                                                                       \
    if (fmt == FP8LM_E4M3) launch_walk<SumOp<kE4M3, N>>(c, s, sum_fp8_kernel<kE4M3, N>, p);   \
    else launch_walk<SumOp<kE5M2, N>>(c, s, sum_fp8_kernel<kE5M2, N>, p);                     \
    break
  static_assert(kMaxRanks == 8, "one case per rank count");
  switch (n_ranks) {
    FP8LM_SUM_N(1); FP8LM_SUM_N(2); FP8LM_SUM_N(3); FP8LM_SUM_N(4);
    FP8LM_SUM_N(5); FP8LM_SUM_N(6); FP8LM_SUM_N(7); FP8LM_SUM_N(8);
    default: return FP8LM_ERR_INVALID_ARGUMENT;
  }
#undef FP8LM_SUM_N
  return after_launch();
}

fp8lm_status fp8lm_init_master_as(fp8lm_ctx* c, const void* w_bf16, void* w_out, fp8lm_meta* w_meta,
                                  fp8lm_state_fmt master_fmt, void* stream) {
  if (!c || (int)master_fmt < 0 || (int)master_fmt > 3) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!w_bf16 || !w_out || !w_meta) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(w_bf16) || !aligned16(w_out)) return FP8LM_ERR_MISALIGNED;
  DeviceGuard guard(c->device);
  hipStream_t s = (hipStream_t)stream;
  Timed tm(c, s, FP8LM_K_INIT_MASTER);
  const uint32_t fmax_bits = master_fmt == FP8LM_STATE_F16 ? kBitsF16Max : (master_fmt == FP8LM_STATE_E4M3 ? kBitsE4M3Max : 0u);
  AmaxParams pa{static_cast<const uint16_t*>(w_bf16), w_meta, fmax_bits, 1, 0};
  launch_walk<AmaxOp<kAmaxForMaster, kSrcBF16>>(c, s, amax_kernel<kAmaxForMaster, kSrcBF16>, pa);
  fp8lm_status st = after_launch();
  if (st != FP8LM_OK) return st;
  InitParams pi{static_cast<const uint16_t*>(w_bf16), w_out, w_meta};
  const dim3 g(grid_of(c)), b(kThreads);
  switch (master_fmt) {
    case FP8LM_STATE_F16: launch_walk<InitCastOp<kStF16>>(c, s, init_master_cast_kernel<kStF16>, pi); break;
    case FP8LM_STATE_BF16: launch_walk<InitCastOp<kStBF16>>(c, s, init_master_cast_kernel<kStBF16>, pi); break;
    case FP8LM_STATE_E4M3: launch_walk<InitCastOp<kStE4M3>>(c, s, init_master_cast_kernel<kStE4M3>, pi); break;
    default: launch_walk<InitCastOp<kStF32>>(c, s, init_master_cast_kernel<kStF32>, pi); break;
  }
  return after_launch();
}

fp8lm_status fp8lm_init_master(fp8lm_ctx* c, const void* w_bf16, uint16_t* w_f16, fp8lm_meta* w_meta, void* stream) {
  return fp8lm_init_master_as(c, w_bf16, w_f16, w_meta, FP8LM_STATE_F16, stream);
}

fp8lm_status fp8lm_adam_step_fp8(fp8lm_ctx* c, const uint8_t* grad, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta,
                                 uint8_t* m, fp8lm_meta* m_meta, void* v, fp8lm_meta* v_meta, void* w,
                                 fp8lm_meta* w_meta, void* wcopy, fp8lm_meta* wcopy_meta, const fp8lm_adam_hparams* hp,
                                 void* stream) {
  if (!c || !hp || (grad_fmt != FP8LM_E4M3 && grad_fmt != FP8LM_E5M2)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (hp->wcopy != FP8LM_WCOPY_E4M3 && hp->wcopy != FP8LM_WCOPY_BF16) return FP8LM_ERR_INVALID_ARGUMENT;
  if (hp->m_scale_mode < 0 || hp->m_scale_mode > 2) return FP8LM_ERR_INVALID_ARGUMENT;
  if (hp->master_fmt < 0 || hp->master_fmt > 3 || (hp->v_fmt != FP8LM_STATE_F16 && hp->v_fmt != FP8LM_STATE_E4M3))
    return FP8LM_ERR_INVALID_ARGUMENT;
  const bool variant = hp->master_fmt != FP8LM_STATE_F16 || hp->v_fmt != FP8LM_STATE_F16;
  if (variant && (hp->wcopy != FP8LM_WCOPY_E4M3 || hp->stats)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!(hp->lr >= 0.0f && hp->lr <= 1024.0f) || !(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) ||
      !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f) || !(hp->eps >= 0x1p-36f && hp->eps < INFINITY) ||
      !(hp->weight_decay >= 0.0f && hp->weight_decay <= 1024.0f) || hp->step < 1)
    return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!grad || !grad_meta || !m || !m_meta || !v || !v_meta || !w || !w_meta || !wcopy || !wcopy_meta)
    return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(grad) || !aligned16(m) || !aligned16(v) || !aligned16(w) || !aligned16(wcopy)) return FP8LM_ERR_MISALIGNED;
  DeviceGuard guard(c->device);

  AdamParams p{};
  p.grad = grad; p.grad_meta = grad_meta; p.m = m; p.m_meta = m_meta; p.v = v; p.v_meta = v_meta;
  p.w = w; p.w_meta = w_meta; p.wcopy = wcopy; p.wcopy_meta = wcopy_meta;
  // scalars derived once on the host, in double, then rounded to fp32
  p.b1 = hp->beta1;
  p.b2 = hp->beta2;
  p.omb1 = (float)(1.0 - (double)p.b1);
  p.omb2 = (float)(1.0 - (double)p.b2);
  p.rbc1 = (float)(1.0 / (1.0 - std::pow((double)p.b1, (double)hp->step)));
  p.rbc2 = (float)(1.0 / (1.0 - std::pow((double)p.b2, (double)hp->step)));
  p.lr = hp->lr;
  p.eps = hp->eps;
  p.decay = (float)(1.0 - (double)hp->lr * (double)hp->weight_decay);
  p.v_scaled = (hp->v_scaled || hp->v_fmt == FP8LM_STATE_E4M3) ? 1 : 0;
  p.v_fmax_bits = hp->v_fmt == FP8LM_STATE_E4M3 ? kBitsE4M3Max : kBitsF16Max;
  p.w_fmax_bits = hp->master_fmt == FP8LM_STATE_F16 ? kBitsF16Max : (hp->master_fmt == FP8LM_STATE_E4M3 ? kBitsE4M3Max : 0u);

  const bool stats = hp->stats != 0, fast = hp->exact == 0;
  hipStream_t s = (hipStream_t)stream;
  const dim3 g(grid_of(c)), b(kThreads);
  const Tables tb = tables_of(c);
  const bool e5 = grad_fmt == FP8LM_E5M2, q8 = hp->wcopy == FP8LM_WCOPY_E4M3;
  if (hp->m_scale_mode == FP8LM_MSCALE_FROM_CAST) {
    const fp8lm_ctx::Fused f = c->fused;
    c->fused.valid = false;
    if (!f.valid || f.grad != grad || f.m != m || f.m_meta != m_meta || f.b1 != p.b1 || f.fmt != (int)grad_fmt)
      return FP8LM_ERR_INVALID_ARGUMENT;
    Timed tm(c, s, FP8LM_K_SCALARS);
    const dim3 gs((c->n_tensors + 255) / 256), bs(256);
    if (q8) hipLaunchKernelGGL((adam_scales_from_cast_kernel<FP8LM_WCOPY_E4M3>), gs, bs, 0, s, tb, p, c->n_tensors);
    else hipLaunchKernelGGL((adam_scales_from_cast_kernel<FP8LM_WCOPY_BF16>), gs, bs, 0, s, tb, p, c->n_tensors);
  } else if (hp->m_scale_mode == FP8LM_MSCALE_PREDICTED) {
    Timed tm(c, s, FP8LM_K_SCALARS);
    const dim3 gs((c->n_tensors + 255) / 256), bs(256);
    if (q8) hipLaunchKernelGGL((adam_predict_scales_kernel<FP8LM_WCOPY_E4M3>), gs, bs, 0, s, tb, p, c->n_tensors);
    else hipLaunchKernelGGL((adam_predict_scales_kernel<FP8LM_WCOPY_BF16>), gs, bs, 0, s, tb, p, c->n_tensors);
  } else {
    Timed tm(c, s, FP8LM_K_ADAM_AMAX);
    if (e5 && q8) launch_walk<AdamAmaxOp<kE5M2, FP8LM_WCOPY_E4M3>>(c, s, adam_amax_kernel<kE5M2, FP8LM_WCOPY_E4M3>, p);
    else if (e5) launch_walk<AdamAmaxOp<kE5M2, FP8LM_WCOPY_BF16>>(c, s, adam_amax_kernel<kE5M2, FP8LM_WCOPY_BF16>, p);
    else if (q8) launch_walk<AdamAmaxOp<kE4M3, FP8LM_WCOPY_E4M3>>(c, s, adam_amax_kernel<kE4M3, FP8LM_WCOPY_E4M3>, p);
    else launch_walk<AdamAmaxOp<kE4M3, FP8LM_WCOPY_BF16>>(c, s, adam_amax_kernel<kE4M3, FP8LM_WCOPY_BF16>, p);
  }
  fp8lm_status st = after_launch();
  if (st != FP8LM_OK) return st;
  if (variant) {
    Timed tm(c, s, FP8LM_K_ADAM_UPDATE);
    launch_update_variant(c, s, p, e5, hp->master_fmt, hp->v_fmt);
  } else {
    Timed tm(c, s, FP8LM_K_ADAM_UPDATE);
    if (e5 && q8) launch_update<kE5M2, FP8LM_WCOPY_E4M3>(c, s, p, fast, stats);
    else if (e5) launch_update<kE5M2, FP8LM_WCOPY_BF16>(c, s, p, fast, stats);
    else if (q8) launch_update<kE4M3, FP8LM_WCOPY_E4M3>(c, s, p, fast, stats);
    else launch_update<kE4M3, FP8LM_WCOPY_BF16>(c, s, p, fast, stats);
  }
  return after_launch();
}

// Host only.  Whole-tensor greedy distribution of Sec. 2.3, Alg. 1, with a heap over the GPUs.
fp8lm_status fp8lm_quant_error_stats(fp8lm_ctx* c, const void* ref, fp8lm_src ref_type, const uint8_t* q, fp8lm_fmt fmt,
                                     const fp8lm_meta* q_meta, fp8lm_quant_stats* out, void* stream) {
  if (!c || !src_ok(ref_type) || (fmt != FP8LM_E4M3 && fmt != FP8LM_E5M2)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_tensors == 0) return FP8LM_OK;
  if (!out) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  hipStream_t s = (hipStream_t)stream;
  {
    Timed tm(c, s, FP8LM_K_SCALARS);
    hipLaunchKernelGGL(quant_stats_zero_kernel, dim3((c->n_tensors + 255) / 256), dim3(256), 0, s, out, c->n_tensors);
    fp8lm_status st = after_launch();
    if (st != FP8LM_OK) return st;
  }
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!ref || !q || !q_meta) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(ref) || !aligned16(q)) return FP8LM_ERR_MISALIGNED;
  StatsParams p{ref, q, q_meta, out};
  const dim3 g(grid_of(c)), b(kThreads);
  const Tables tb = tables_of(c);
  Timed tm(c, s, FP8LM_K_STATS);
#define FP8LM_STATS_SRC(S)                                                                                   \
  do {                                                                                                       \
    if (fmt == FP8LM_E4M3) hipLaunchKernelGGL((quant_stats_kernel<kE4M3, S>), g, b, 0, s, tb, p);            \
    else hipLaunchKernelGGL((quant_stats_kernel<kE5M2, S>), g, b, 0, s, tb, p);                              \
  } while (0)
  if (ref_type == FP8LM_SRC_F32) FP8LM_STATS_SRC(kSrcF32);
  else if (ref_type == FP8LM_SRC_F16) FP8LM_STATS_SRC(kSrcF16);
  else FP8LM_STATS_SRC(kSrcBF16);
#undef FP8LM_STATS_SRC
  return after_launch();
}

fp8lm_status fp8lm_greedy_partition(const int64_t* sizes, int32_t n, int32_t n_gpus, int32_t* owner, int64_t* usage) {
  if (n < 0 || n_gpus < 1 || (n > 0 && (!sizes || !owner)) || !usage) return FP8LM_ERR_INVALID_ARGUMENT;
  for (int32_t i = 0; i < n; ++i)
    if (sizes[i] < 0) return FP8LM_ERR_INVALID_ARGUMENT;
  std::vector<int32_t> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return sizes[a] > sizes[b]; });
  typedef std::pair<int64_t, int32_t> Load;   // (memory in use, gpu): the smallest pair is the next receiver
  std::priority_queue<Load, std::vector<Load>, std::greater<Load>> heap;
  for (int32_t j = 0; j < n_gpus; ++j) heap.emplace(0, j);
  for (int32_t i : order) {
    Load top = heap.top();
    heap.pop();
    owner[i] = top.second;
    top.first += sizes[i];
    heap.push(top);
  }
  for (int32_t j = 0; j < n_gpus; ++j) usage[j] = 0;
  for (int32_t i = 0; i < n; ++i) usage[owner[i]] += sizes[i];
  return FP8LM_OK;
}

fp8lm_status fp8lm_copy_bytes(fp8lm_ctx* c, const void* src, void* dst, int64_t bytes, void* stream) {
  if (!c || !src || !dst || bytes < 0 || bytes % 16 != 0) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(src) || !aligned16(dst)) return FP8LM_ERR_MISALIGNED;
  if (bytes == 0) return FP8LM_OK;
  DeviceGuard guard(c->device);
  const long long n16 = bytes / 16;
  const long long want = (long long)c->num_cus * c->blocks_per_cu;
  const int grid = (int)std::max<long long>(1, std::min<long long>(want, (n16 + kThreads - 1) / kThreads));
  Timed tm(c, (hipStream_t)stream, FP8LM_K_COPY);
  hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), n16);
  return after_launch();
}

fp8lm_status fp8lm_set_timing(fp8lm_ctx* c, int32_t enable) {
  if (!c) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  if (enable && c->free_events.empty() && c->stamps.empty()) {
    for (int i = 0; i < 4096; ++i) {
      hipEvent_t a, b;
      HIP_TRY(hipEventCreate(&a));
      HIP_TRY(hipEventCreate(&b));
      c->free_events.emplace_back(a, b);
    }
  }
  c->timing = enable != 0;
  return FP8LM_OK;
}

fp8lm_status fp8lm_get_timing(fp8lm_ctx* c, int32_t* launches, double* total_ms) {
  if (!c || !launches || !total_ms) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  for (int k = 0; k < FP8LM_K_COUNT; ++k) { launches[k] = 0; total_ms[k] = 0.0; }
  for (auto& s : c->stamps) {
    HIP_TRY(hipEventSynchronize(s.b));
    float ms = 0.0f;
    HIP_TRY(hipEventElapsedTime(&ms, s.a, s.b));
    launches[s.kernel] += 1;
    total_ms[s.kernel] += ms;
    c->free_events.emplace_back(s.a, s.b);
  }
  c->stamps.clear();
  return FP8LM_OK;
}

}  // extern "C"
