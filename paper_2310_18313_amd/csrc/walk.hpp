// Shared by every kernel of libfp8lm: tensor and chunk tables, wavefront / workgroup / grid-wide
// reductions, the chunk walk, 128-bit and 64-bit access helpers and the build-time tuning knobs.
#ifndef FP8LM_WALK_HPP
#define FP8LM_WALK_HPP

#include "fp8lm.h"
#include "formats.hpp"

namespace fp8lm {

constexpr int kThreads = 256;
constexpr int kGroup = 16;                 // elements per thread per iteration
constexpr int kTile = kThreads * kGroup;   // elements per workgroup per iteration
constexpr int kWaves = kThreads / 64;
#ifndef FP8LM_MAX_BLOCKS_PER_CU
#define FP8LM_MAX_BLOCKS_PER_CU 16         // the step gains up to 16 workgroups per compute unit and is flat from 16 to 64
#endif
constexpr int kMaxBlocksPerCu = FP8LM_MAX_BLOCKS_PER_CU;   // upper limit (and default) of the launch tuning; sizes the record array

struct TensorDesc {
  int64_t offset;
  int64_t numel;
  int32_t first_chunk;
  int32_t n_chunks;
  uint32_t flags;       // FP8LM_TENSOR_* attributes of the tensor
  uint32_t pad;
};

// Per-tensor scratch.  The ticket is zero between launches; the `pend` block carries the scales chosen
// by the first Adam pass to the second.
struct Scratch {
  uint32_t ticket;                // chunks finished
  uint32_t redo;                  // speculative quantisation: 1 if the tensor has to be cast again with the scale now in its meta
  float old_scale, old_inv;       // ... and the scale the meta held before the speculation
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
  double fs[2];                   // float64 sums (error statistics)
};

struct Tables {
  const TensorDesc* desc;
  const int32_t* chunk_tensor;
  Scratch* scratch;
  Partial* partials;              // [grid + n_tensors]
  int32_t n_chunks;
  int32_t chunk_elems;
  int32_t deferred;               // 1: workgroups only leave their records; an epilogue launch finishes the tensors
  const int32_t* n_chunks_dev;    // if set: the number of chunks is read from here (a chunk list built on the device);
                                  // n_chunks is then only the host's upper bound
};
__device__ __forceinline__ long long chunk_count(const Tables& tb) { return tb.n_chunks_dev ? *tb.n_chunks_dev : tb.n_chunks; }

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
__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Workgroup-wide combine of up to NV maxima, NC counters, NF float64 sums and one OR-mask; result valid in
// thread 0.  Every step is done in a fixed order, so the float64 sums are reproducible from run to run.
template <int NV, int NC, int NF = 0>
struct BlockStats {
  uint32_t mx[NV > 0 ? NV : 1];
  unsigned long long ct[NC > 0 ? NC : 1];
  double fs[NF > 0 ? NF : 1];
  uint32_t orv;
};

template <int NV, int NC, int NF>
__device__ __forceinline__ void block_combine(BlockStats<NV, NC, NF>& s) {
  __shared__ uint32_t l_mx[kWaves][NV > 0 ? NV : 1];
  __shared__ unsigned long long l_ct[kWaves][NC > 0 ? NC : 1];
  __shared__ double l_fs[kWaves][NF > 0 ? NF : 1];
  __shared__ uint32_t l_or[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < NV; ++i) s.mx[i] = wave_max_u32(s.mx[i]);
#pragma unroll
  for (int i = 0; i < NC; ++i) s.ct[i] = wave_sum_u64(s.ct[i]);
#pragma unroll
  for (int i = 0; i < NF; ++i) s.fs[i] = wave_sum_f64(s.fs[i]);
  s.orv = wave_or_u32(s.orv);
  __syncthreads();   // the previous use of the LDS arrays is over
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) l_mx[wave][i] = s.mx[i];
#pragma unroll
    for (int i = 0; i < NC; ++i) l_ct[wave][i] = s.ct[i];
#pragma unroll
    for (int i = 0; i < NF; ++i) l_fs[wave][i] = s.fs[i];
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
#pragma unroll
      for (int i = 0; i < NF; ++i) s.fs[i] += l_fs[w][i];
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
template <int NV, int NC, int NF>
__device__ __forceinline__ void store_record(const Tables& tb, int t, const BlockStats<NV, NC, NF>& s) {
  Partial* rec = tb.partials + ((long long)blockIdx.x + t);
#pragma unroll
  for (int i = 0; i < NV; ++i) __hip_atomic_store(&rec->mx[i], s.mx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
  for (int i = 0; i < NC; ++i) __hip_atomic_store(&rec->ct[i], s.ct[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
  for (int i = 0; i < NF; ++i) __hip_atomic_store(&rec->fs[i], s.fs[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(&rec->orv, s.orv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Combines the records of all workgroups of a launch with `grid` workgroups that touched tensor t.  Called
// by all threads; the totals end up in thread 0's `s`.
template <int NV, int NC, int NF>
__device__ __forceinline__ void gather_records(const Tables& tb, int t, const TensorDesc& d, long long grid, BlockStats<NV, NC, NF>& s) {
  // owner(c) = the b with b*C/G <= c < (b+1)*C/G
  const long long C = chunk_count(tb);
  if (grid > C) grid = C;         // a launch with more workgroups than chunks uses only the first C (see walk_chunks)
  const long long c0 = d.first_chunk, c1 = c0 + d.n_chunks - 1;
  const long long b_lo = ((c0 + 1) * grid - 1) / C, b_hi = ((c1 + 1) * grid - 1) / C;
#pragma unroll
  for (int i = 0; i < NV; ++i) s.mx[i] = 0;
#pragma unroll
  for (int i = 0; i < NC; ++i) s.ct[i] = 0;
#pragma unroll
  for (int i = 0; i < NF; ++i) s.fs[i] = 0.0;
  s.orv = 0;
  for (long long b = b_lo + threadIdx.x; b <= b_hi; b += kThreads) {
    const Partial* rec = tb.partials + (b + t);
#pragma unroll
    for (int i = 0; i < NV; ++i) s.mx[i] = max(s.mx[i], __hip_atomic_load(&rec->mx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
#pragma unroll
    for (int i = 0; i < NC; ++i) s.ct[i] += __hip_atomic_load(&rec->ct[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int i = 0; i < NF; ++i) s.fs[i] += __hip_atomic_load(&rec->fs[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s.orv |= __hip_atomic_load(&rec->orv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  block_combine(s);
}

// Called by all threads at the end of a workgroup's part of tensor t, after block_combine(s).  Returns
// true in every thread of the workgroup that has to run the tensor's epilogue, with the tensor's totals in
// thread 0's `s`; always false in the deferred form.
template <int NV, int NC, int NF>
__device__ __forceinline__ bool collect(const Tables& tb, int t, const TensorDesc& d, int done, BlockStats<NV, NC, NF>& s) {
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

// ---- the chunk walk shared by all kernels -------------------------------------------------------
// Op must provide: begin(t, desc); fast() (uniform: may the vector path be used for this tensor);
// tiles<UN>(pos): UN complete 4096-element tiles starting at element `pos` of the flat buffers, handled
// by the whole workgroup (all loads issued before the first use; the op chooses which 16 elements of
// a tile a thread takes); full_group(pos): the 16 consecutive elements starting at `pos`, handled by the calling
// thread alone with vector accesses (any subset of the threads may call it); group(pos, valid) with
// 1 <= valid <= 16 for everything else, element by element; flush(t, desc, chunks_done) (called by all threads when the workgroup leaves tensor t: it fills
// a Stats = BlockStats<..>, combines it over the workgroup and hands it to `collect`); and for the tensor's
// scalar epilogue finalize(t, desc, stats), run by one thread once the totals of all workgroups are known.
template <int UN, class Op>
__device__ __forceinline__ void walk_chunks(const Tables& tb, Op& op) {
  // workgroup b walks the contiguous chunk range [b*C/G, (b+1)*C/G): `collect` relies on this mapping
  // With fewer chunks than workgroups (a chunk list built on the device) only the first C workgroups take part, so
  // that every one of them owns a chunk and leaves a record wherever `gather_records` expects one.
  const long long C = chunk_count(tb), b = blockIdx.x;
  const long long G = C < (long long)gridDim.x ? C : (long long)gridDim.x;
  if (b >= G) return;
  long long c = b * C / G;
  const long long c_end = (b + 1) * C / G;
  int cur = -1, done = 0;
  TensorDesc d{};
  // the tensor id of the next chunk is fetched one iteration ahead, so its latency hides behind the body
  int t_next = c < c_end ? tb.chunk_tensor[c] : -1;
  for (; c < c_end; ++c) {
    const int t = t_next;
    t_next = c + 1 < c_end ? tb.chunk_tensor[c + 1] : -1;
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
    // what is left of the chunk (less than a tile; a whole small tensor): complete 16-element groups still take
    // 128-bit accesses, only the last, incomplete group of a tensor goes element by element
    for (int i = tile * kTile + threadIdx.x * kGroup; i < len; i += kTile) {
      const int valid = len - i < kGroup ? len - i : kGroup;
      if (valid == kGroup && op.fast()) op.full_group(base + i);
      else op.group(base + i, valid);
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
#ifndef FP8LM_CAST_STORE16
#define FP8LM_CAST_STORE16 0   // cast kernel, split layout: neighbouring lanes swap halves so that each stores 128 bits once
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

}  // namespace fp8lm

#endif
