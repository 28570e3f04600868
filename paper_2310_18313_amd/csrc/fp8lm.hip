// libfp8lm: FP8 gradient quantisation and FP8 Adam step of FP8-LM (arXiv 2310.18313, Sec. 2.1, 2.2,
// Appendix A) for MI355X / gfx950.  See include/fp8lm.h for the boundary.  This file holds the host side
// (context, validation, launches); the kernels live in the headers it includes:
//   walk.hpp      tables, reductions, the chunk walk every kernel shares, access helpers, tuning knobs
//   quantize.hpp  amax + scale, FP8 cast + auto-scaling, delayed scaling, Eq. 4-6 (re-quantise, sum)
//   adam.hpp      master-weight initialisation and the two passes of the FP8 Adam step
//   stats.hpp     quantisation-error statistics, metadata initialisation, streaming copy
//   formats.hpp   FP8 / FP16 / bf16 conversions and the power-of-two scale rule
//
// Shape of every hot kernel
//   * The tensor list is cut into chunks of `chunk_elems` elements that never straddle a tensor.  A grid
//     of 256-thread workgroups (up to 16 per compute unit) walks contiguous ranges of the chunk table,
//     so a 5 K-element bias and a 250 M-element matrix are served by the same launch.
//   * A thread handles 16 elements of a 4096-element tile per iteration, with 128-bit (64-bit on 8-bit
//     streams of the update and cast kernels) accesses that are contiguous over the whole workgroup.
//   * Per-tensor statistics (amax, counters) stay in registers while a workgroup is inside one tensor,
//     then go wavefront -> LDS -> one record per (workgroup, tensor).  A second, tiny launch (one
//     workgroup per tensor) combines the records and runs the scalar epilogue (scale update,
//     auto-scaling state, metadata); a single-pass form with a per-tensor ticket is selectable.
//   * These kernels are HBM-bandwidth bound (2..12 bytes per element against ~10-60 ALU operations); no
//     matrix cores are involved.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <numeric>
#include <queue>
#include <string>
#include <vector>

#include "fp8lm.h"
#include "formats.hpp"

#include "walk.hpp"
#include "quantize.hpp"
#include "adam.hpp"
#include "stats.hpp"


// ====================================================================================================
// Fixed device array for fp8lm_adam_step_fp8_static (callers that cannot allocate)
// ====================================================================================================
namespace fp8lm {

// Everything a context keeps in hipMalloc'd memory, at fixed maximum sizes.
constexpr int kStaticMaxGrid = 4096;                      // workgroups of a launch: bounds the reduction records
constexpr int kStaticChunkElems = 16384;
struct StaticArena {
  TensorDesc desc[FP8LM_STATIC_MAX_TENSORS];              // 128 KiB
  Scratch scratch[FP8LM_STATIC_MAX_TENSORS];              // 288 KiB
  Partial partials[kStaticMaxGrid + FP8LM_STATIC_MAX_TENSORS + 1];   // 1 MiB
  int32_t chunk_tensor[FP8LM_STATIC_MAX_CHUNKS];          // 4 MiB
};

// A batch of tensor descriptors travels as kernel arguments: no copy from host memory is enqueued.
constexpr int kDescBatch = 96;                            // 3 KiB of arguments per launch
struct DescBatch {
  TensorDesc d[kDescBatch];
  int32_t first, count;
};
__global__ void static_desc_kernel(DescBatch b, TensorDesc* desc) {
  const int i = threadIdx.x;
  if (i < b.count) desc[b.first + i] = b.d[i];
}
// Workgroup t (and t + grid, ...) writes tensor t's id into its chunks; also returns the tickets to zero.
__global__ void static_chunks_kernel(const TensorDesc* desc, int32_t* chunk_tensor, Scratch* scratch, int n) {
  for (int t = blockIdx.x; t < n; t += gridDim.x) {
    const TensorDesc d = desc[t];
    for (int i = threadIdx.x; i < d.n_chunks; i += blockDim.x) chunk_tensor[d.first_chunk + i] = t;
    if (threadIdx.x == 0) scratch[t].ticket = 0;
  }
}

}  // namespace fp8lm

// The array itself.  In host code this name is only a handle for hipGetSymbolAddress: the device address is
// looked up once per GPU (static_arena_of) and that pointer is what kernels and launches are given.
static __device__ __align__(256) unsigned char scratch[sizeof(fp8lm::StaticArena)];

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
  std::vector<uint32_t> tensor_flags;   // FP8LM_TENSOR_* per tensor
  int32_t chunk_elems = 16384;
  int32_t blocks_per_cu = kMaxBlocksPerCu;
  int32_t single_pass_min_chunks = FP8LM_SINGLE_PASS_MIN_CHUNKS;
  int32_t n_chunks = 0;
  TensorDesc* d_desc = nullptr;
  int32_t* d_chunk_tensor = nullptr;
  Scratch* d_scratch = nullptr;
  Partial* d_partials = nullptr;    // [num_cus * kMaxBlocksPerCu + n_tensors]
  // speculative quantisation: tensor and chunk tables of the tensors that have to be cast again, their chunk
  // count, and running totals (calls, tensors cast twice, elements cast twice)
  TensorDesc* d_redo_desc = nullptr;
  int32_t* d_redo_chunk_tensor = nullptr;
  int32_t* d_redo_count = nullptr;
  unsigned long long* d_spec_totals = nullptr;
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

// Builds the tensor and chunk tables for chunks of chunk_elems elements and installs them.  On failure the
// context keeps the tables (and the chunk size) it had.
fp8lm_status build_tables(fp8lm_ctx* c, int32_t chunk_elems) {
  std::vector<TensorDesc> desc(c->n_tensors);
  std::vector<int32_t> chunk_tensor;
  long long total_chunks = 0;
  for (int t = 0; t < c->n_tensors; ++t) {
    const long long n = c->tensors[t].numel;
    const long long nc = (n + chunk_elems - 1) / chunk_elems;
    if (total_chunks + nc > 0x7FFFFFF0LL) return FP8LM_ERR_TOO_LARGE;
    desc[t] = TensorDesc{c->tensors[t].offset, n, (int32_t)total_chunks, (int32_t)nc, c->tensor_flags[t], 0u};
    total_chunks += nc;
  }
  chunk_tensor.resize((size_t)total_chunks);
  for (int t = 0; t < c->n_tensors; ++t)
    std::fill(chunk_tensor.begin() + desc[t].first_chunk, chunk_tensor.begin() + desc[t].first_chunk + desc[t].n_chunks, t);
  TensorDesc* d_desc = nullptr;
  TensorDesc* d_redo_desc = nullptr;
  int32_t* d_chunk_tensor = nullptr;
  int32_t* d_redo_chunk_tensor = nullptr;
  hipError_t e = hipMalloc((void**)&d_desc, std::max<size_t>(1, desc.size()) * sizeof(TensorDesc));
  if (e == hipSuccess) e = hipMalloc((void**)&d_chunk_tensor, std::max<size_t>(1, chunk_tensor.size()) * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&d_redo_desc, std::max<size_t>(1, desc.size()) * sizeof(TensorDesc));
  if (e == hipSuccess) e = hipMalloc((void**)&d_redo_chunk_tensor, std::max<size_t>(1, chunk_tensor.size()) * sizeof(int32_t));
  if (e == hipSuccess && !desc.empty())
    e = hipMemcpy(d_desc, desc.data(), desc.size() * sizeof(TensorDesc), hipMemcpyHostToDevice);
  if (e == hipSuccess && !chunk_tensor.empty())
    e = hipMemcpy(d_chunk_tensor, chunk_tensor.data(), chunk_tensor.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    g_hip_error = std::string("chunk tables: ") + hipGetErrorString(e);
    if (d_desc) (void)hipFree(d_desc);
    if (d_chunk_tensor) (void)hipFree(d_chunk_tensor);
    if (d_redo_desc) (void)hipFree(d_redo_desc);
    if (d_redo_chunk_tensor) (void)hipFree(d_redo_chunk_tensor);
    return FP8LM_ERR_HIP;
  }
  if (c->d_desc) (void)hipFree(c->d_desc);
  if (c->d_chunk_tensor) (void)hipFree(c->d_chunk_tensor);
  if (c->d_redo_desc) (void)hipFree(c->d_redo_desc);
  if (c->d_redo_chunk_tensor) (void)hipFree(c->d_redo_chunk_tensor);
  c->d_desc = d_desc;
  c->d_chunk_tensor = d_chunk_tensor;
  c->d_redo_desc = d_redo_desc;
  c->d_redo_chunk_tensor = d_redo_chunk_tensor;
  c->chunk_elems = chunk_elems;
  c->n_chunks = (int32_t)total_chunks;
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
                deferred_of(c) ? 1 : 0, nullptr};
}
// The tables of the tensors a speculative quantisation has to cast again: built on the device, so the number of
// chunks is only known there; tensors always finished by the second launch.
Tables redo_tables_of(const fp8lm_ctx* c) {
  return Tables{c->d_redo_desc, c->d_redo_chunk_tensor, c->d_scratch, c->d_partials, c->n_chunks, c->chunk_elems, 1,
                c->d_redo_count};
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
void launch_walk_on(fp8lm_ctx* c, hipStream_t s, Kernel kernel, const Params& p, const Tables& tb) {
  const dim3 g(grid_of(c)), b(kThreads);
  hipLaunchKernelGGL(kernel, g, b, 0, s, tb, p);
  if (tb.deferred)
    hipLaunchKernelGGL((epilogue_kernel<Op, Params>), dim3(std::min<int>(c->n_tensors, 8 * c->num_cus)), b, 0, s, tb, p,
                       (int)g.x, (int)c->n_tensors);
}
template <class Op, class Params, class Kernel>
void launch_walk(fp8lm_ctx* c, hipStream_t s, Kernel kernel, const Params& p) {
  const Tables tb = tables_of(c);
  const dim3 g(grid_of(c)), b(kThreads);
  hipLaunchKernelGGL(kernel, g, b, 0, s, tb, p);
  if (tb.deferred)
    hipLaunchKernelGGL((epilogue_kernel<Op, Params>), dim3(std::min<int>(c->n_tensors, 8 * c->num_cus)), b, 0, s, tb, p,
                       (int)g.x, (int)c->n_tensors);
}

// Selects the adam_update_kernel instantiation.
template <int GFMT, int WCOPY>
void launch_update(fp8lm_ctx* c, hipStream_t s, const AdamParams& p, bool fast, bool stats) {
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
AutoscaleRule rule_of(const fp8lm_autoscale_cfg* cfg) {
  return AutoscaleRule{cfg->sat_num, cfg->sat_den, cfg->ramp_steps, cfg->mu_rule, cfg->mu_min_exp};
}
bool cfg_ok(const fp8lm_autoscale_cfg* cfg) {
  if (cfg && cfg->mu_rule != FP8LM_MU_SET_HALF &&
      !(cfg->mu_rule == FP8LM_MU_HALVE && cfg->mu_min_exp >= -64 && cfg->mu_min_exp <= -1))
    return false;
  // sat_num, sat_den <= 2^24: the overflow test multiplies them with element counts in 64 bits
  return cfg && cfg->sat_num >= 0 && cfg->sat_num <= (1 << 24) && cfg->sat_den > 0 && cfg->sat_den <= (1 << 24) &&
         cfg->ramp_steps >= 2 && cfg->hist_window >= 1 &&
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
  c->tensor_flags.assign((size_t)n, 0u);
  fp8lm_status st = build_tables(c, c->chunk_elems);
  if (st == FP8LM_OK) {
    const size_t bytes = std::max<size_t>(1, (size_t)n) * sizeof(Scratch);
    hipError_t e = hipMalloc((void**)&c->d_scratch, bytes);
    if (e == hipSuccess) e = hipMemset(c->d_scratch, 0, bytes);
    const size_t records = (size_t)c->num_cus * kMaxBlocksPerCu + (size_t)n + 1;
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_partials, records * sizeof(Partial));
    if (e == hipSuccess) e = hipMemset(c->d_partials, 0, records * sizeof(Partial));
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_redo_count, sizeof(int32_t));
    if (e == hipSuccess) e = hipMemset(c->d_redo_count, 0, sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&c->d_spec_totals, 6 * sizeof(unsigned long long));     // gradient, first moment
    if (e == hipSuccess) e = hipMemset(c->d_spec_totals, 0, 6 * sizeof(unsigned long long));
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
  if (c->d_redo_desc) (void)hipFree(c->d_redo_desc);
  if (c->d_redo_chunk_tensor) (void)hipFree(c->d_redo_chunk_tensor);
  if (c->d_redo_count) (void)hipFree(c->d_redo_count);
  if (c->d_spec_totals) (void)hipFree(c->d_spec_totals);
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
  HIP_TRY(hipDeviceSynchronize());   // no launch may still be reading the tables that are about to go
  const fp8lm_status st = build_tables(c, chunk_elems);
  if (st != FP8LM_OK) return st;
  c->blocks_per_cu = blocks_per_cu;
  c->single_pass_min_chunks = single_pass_min_chunks;
  return FP8LM_OK;
}

fp8lm_status fp8lm_set_tensor_flags(fp8lm_ctx* c, const uint32_t* flags, int32_t n) {
  if (!c || n != c->n_tensors || (n > 0 && !flags)) return FP8LM_ERR_INVALID_ARGUMENT;
  for (int t = 0; t < n; ++t)
    if (flags[t] & ~(uint32_t)FP8LM_TENSOR_NO_WEIGHT_DECAY) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  HIP_TRY(hipDeviceSynchronize());   // no launch may still be reading the tables that are about to go
  const std::vector<uint32_t> before = c->tensor_flags;
  c->tensor_flags.assign(flags, flags + n);
  const fp8lm_status st = build_tables(c, c->chunk_elems);
  if (st != FP8LM_OK) c->tensor_flags = before;
  return st;
}

fp8lm_status fp8lm_meta_init(fp8lm_ctx* c, fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, void* stream) {
  if (!c || !cfg_ok(cfg) || (c->n_tensors > 0 && !meta)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_tensors == 0) return FP8LM_OK;
  DeviceGuard guard(c->device);
  const int blocks = (c->n_tensors + 255) / 256;
  hipLaunchKernelGGL(meta_init_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, meta, c->n_tensors,
                     cfg->mu_rule == FP8LM_MU_HALVE ? 0 : cfg->ramp_steps / 2);
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
  hipStream_t s = (hipStream_t)stream;
  Timed tm(c, s, FP8LM_K_AMAX);
  if (src_type == FP8LM_SRC_F32) launch_walk<AmaxOp<kAmaxForGradient, kSrcF32>>(c, s, amax_kernel<kAmaxForGradient, kSrcF32>, p);
  else if (src_type == FP8LM_SRC_F16) launch_walk<AmaxOp<kAmaxForGradient, kSrcF16>>(c, s, amax_kernel<kAmaxForGradient, kSrcF16>, p);
  else launch_walk<AmaxOp<kAmaxForGradient, kSrcBF16>>(c, s, amax_kernel<kAmaxForGradient, kSrcBF16>, p);
  return after_launch();
}

// Common body of the three cast entry points.
enum CastMode { kCastPlain = 0, kCastDelayed = 1, kCastSpeculative = 2 };
static fp8lm_status cast_impl(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                              fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, int mode, bool fuse,
                              const uint8_t* m, const fp8lm_meta* m_meta, float beta1, void* stream) {
  const bool delayed = mode != kCastPlain;        // the first pass of a speculation is a delayed-scaling cast
  if (!c || !cfg_ok(cfg) || !src_ok(src_type) || (fmt != FP8LM_E4M3 && fmt != FP8LM_E5M2))
    return FP8LM_ERR_INVALID_ARGUMENT;
  c->fused.valid = false;
  if (fuse && !(beta1 >= 0.0f && beta1 < 1.0f)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!src || !dst || !meta || (fuse && (!m || !m_meta))) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(src) || !aligned16(dst) || (fuse && !aligned16(m))) return FP8LM_ERR_MISALIGNED;
  DeviceGuard guard(c->device);
  hipStream_t s = (hipStream_t)stream;
  const uint32_t fmax_bits = fmt == FP8LM_E4M3 ? kBitsE4M3Max : kBitsE5M2Max;
  if (delayed) {
    Timed tm(c, s, FP8LM_K_SCALARS);
    const dim3 gs((c->n_tensors + 255) / 256), bs(256);
    if (mode == kCastSpeculative)
      hipLaunchKernelGGL(speculate_scale_kernel, gs, bs, 0, s, c->d_desc, meta, c->d_scratch, c->n_tensors, fmax_bits,
                         cfg->hist_window, cfg->margin);
    else
      hipLaunchKernelGGL(delayed_scale_kernel, gs, bs, 0, s, c->d_desc, meta, c->n_tensors, fmax_bits, cfg->hist_window,
                         cfg->margin);
    fp8lm_status st = after_launch();
    if (st != FP8LM_OK) return st;
  }
  CastParams p{};
  p.speculative = mode == kCastSpeculative ? 1 : 0;
  p.fmax_bits = fmax_bits;
  p.margin = cfg->margin;
  p.src = src;
  p.dst = dst;
  p.meta = meta;
  p.rule = rule_of(cfg);
  p.hist_window = cfg->hist_window;
  p.m = m;
  p.m_meta = m_meta;
  p.b1 = beta1;
  p.omb1 = (float)(1.0 - (double)beta1);
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
  if (st == FP8LM_OK && mode == kCastSpeculative) {
    // the tensors whose scale turned out different: their chunk list, then the plain cast over that list
    {
      Timed tm(c, s, FP8LM_K_SCALARS);
      hipLaunchKernelGGL(redo_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, c->d_desc, c->d_scratch, c->d_redo_desc,
                         c->n_tensors, c->d_redo_count, c->d_spec_totals);
      hipLaunchKernelGGL(redo_fill_kernel, dim3(std::min<int>(c->n_tensors, 1024)), dim3(256), 0, s, c->d_redo_desc,
                         c->d_redo_chunk_tensor, c->n_tensors);
      st = after_launch();
    }
    if (st == FP8LM_OK) {
      const Tables rt = redo_tables_of(c);
      p.speculative = 0;
      Timed tm(c, s, FP8LM_K_CAST);
#define FP8LM_REDO_LAUNCH(F, S)                                                                            \
      do {                                                                                                  \
        if (fuse) launch_walk_on<CastOp<F, false, true, S>>(c, s, cast_kernel<F, false, true, S>, p, rt);   \
        else launch_walk_on<CastOp<F, false, false, S>>(c, s, cast_kernel<F, false, false, S>, p, rt);      \
      } while (0)
#define FP8LM_REDO_SRC(S)                                                                                  \
      do {                                                                                                  \
        if (fmt == FP8LM_E4M3) FP8LM_REDO_LAUNCH(kE4M3, S);                                                 \
        else FP8LM_REDO_LAUNCH(kE5M2, S);                                                                   \
      } while (0)
      if (src_type == FP8LM_SRC_F32) FP8LM_REDO_SRC(kSrcF32);
      else if (src_type == FP8LM_SRC_F16) FP8LM_REDO_SRC(kSrcF16);
      else FP8LM_REDO_SRC(kSrcBF16);
#undef FP8LM_REDO_SRC
#undef FP8LM_REDO_LAUNCH
      st = after_launch();
    }
  }
  if (st == FP8LM_OK && fuse) c->fused = {true, dst, m, m_meta, p.b1, fmt};
  return st;
}

fp8lm_status fp8lm_cast_fp8(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                            fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, void* stream) {
  return cast_impl(c, src, src_type, dst, fmt, meta, cfg, kCastPlain, false, nullptr, nullptr, 0.0f, stream);
}

fp8lm_status fp8lm_cast_fp8_delayed(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                                    fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, void* stream) {
  return cast_impl(c, src, src_type, dst, fmt, meta, cfg, kCastDelayed, false, nullptr, nullptr, 0.0f, stream);
}

fp8lm_status fp8lm_cast_fp8_for_adam(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                                     fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, int32_t delayed,
                                     const uint8_t* m, const fp8lm_meta* m_meta, float beta1, void* stream) {
  return cast_impl(c, src, src_type, dst, fmt, meta, cfg, delayed != 0 ? kCastDelayed : kCastPlain, true, m, m_meta, beta1,
                   stream);
}

fp8lm_status fp8lm_quantize_fp8(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                                fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, void* stream) {
  return cast_impl(c, src, src_type, dst, fmt, meta, cfg, kCastSpeculative, false, nullptr, nullptr, 0.0f, stream);
}

fp8lm_status fp8lm_quantize_fp8_for_adam(fp8lm_ctx* c, const void* src, fp8lm_src src_type, uint8_t* dst, fp8lm_fmt fmt,
                                         fp8lm_meta* meta, const fp8lm_autoscale_cfg* cfg, const uint8_t* m,
                                         const fp8lm_meta* m_meta, float beta1, void* stream) {
  return cast_impl(c, src, src_type, dst, fmt, meta, cfg, kCastSpeculative, true, m, m_meta, beta1, stream);
}

fp8lm_status fp8lm_get_speculation_stats(fp8lm_ctx* c, uint64_t* calls, uint64_t* tensors_redone, uint64_t* elems_redone,
                                         void* stream) {
  if (!c || !calls || !tensors_redone || !elems_redone) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  unsigned long long h[3] = {0, 0, 0};
  HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
  HIP_TRY(hipMemcpy(h, c->d_spec_totals, sizeof(h), hipMemcpyDeviceToHost));
  *calls = h[0]; *tensors_redone = h[1]; *elems_redone = h[2];
  return FP8LM_OK;
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
  p.rule = rule_of(cfg);
  DeviceGuard guard(c->device);
  Timed tm(c, (hipStream_t)stream, FP8LM_K_SUM);
  hipStream_t s = (hipStream_t)stream;
#define FP8LM_SUM_N(N)                                                                          \
  case N:                                                                                       \
    if (fmt == FP8LM_E4M3) launch_walk<SumOp<kE4M3, N>>(c, s, sum_fp8_kernel<kE4M3, N>, p);   \
    else launch_walk<SumOp<kE5M2, N>>(c, s, sum_fp8_kernel<kE5M2, N>, p);                     \
    break
  static_assert(kUnrolledRanks == 8, "one case per unrolled rank count");
  switch (n_ranks) {
    FP8LM_SUM_N(1); FP8LM_SUM_N(2); FP8LM_SUM_N(3); FP8LM_SUM_N(4);
    FP8LM_SUM_N(5); FP8LM_SUM_N(6); FP8LM_SUM_N(7); FP8LM_SUM_N(8);
    default:          // any larger number of ranks: the kernel that loops over them
      if (fmt == FP8LM_E4M3) launch_walk<SumOp<kE4M3, 0>>(c, s, sum_fp8_kernel<kE4M3, 0>, p);
      else launch_walk<SumOp<kE5M2, 0>>(c, s, sum_fp8_kernel<kE5M2, 0>, p);
      break;
  }
#undef FP8LM_SUM_N
  return after_launch();
}

fp8lm_status fp8lm_autoscale_broadcast(fp8lm_ctx* c, const fp8lm_meta* from, fp8lm_meta* const* metas, int32_t n_ranks,
                                       void* stream) {
  if (!c || !metas || n_ranks < 1 || n_ranks > kMaxRanks) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_tensors == 0) return FP8LM_OK;
  if (!from) return FP8LM_ERR_INVALID_ARGUMENT;
  RankMetasOut rm{};
  rm.n_ranks = n_ranks;
  for (int r = 0; r < n_ranks; ++r) {
    if (!metas[r] || metas[r] == from) return FP8LM_ERR_INVALID_ARGUMENT;
    rm.m[r] = metas[r];
  }
  DeviceGuard guard(c->device);
  Timed tm(c, (hipStream_t)stream, FP8LM_K_SCALARS);
  hipLaunchKernelGGL(autoscale_broadcast_kernel, dim3((c->n_tensors + 255) / 256), dim3(256), 0, (hipStream_t)stream,
                     from, rm, c->n_tensors);
  return after_launch();
}

fp8lm_status fp8lm_set_mu(fp8lm_ctx* c, fp8lm_meta* meta, int32_t mu_exp, void* stream) {
  if (!c || mu_exp < -64 || mu_exp > 1) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_tensors == 0) return FP8LM_OK;
  if (!meta) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  Timed tm(c, (hipStream_t)stream, FP8LM_K_SCALARS);
  hipLaunchKernelGGL(set_mu_kernel, dim3((c->n_tensors + 255) / 256), dim3(256), 0, (hipStream_t)stream, meta,
                     c->n_tensors, mu_exp);
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

// Validation of everything but the context (shared by the two Adam entry points).
static fp8lm_status adam_args_ok(const uint8_t* grad, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta, uint8_t* m,
                                 fp8lm_meta* m_meta, void* v, fp8lm_meta* v_meta, void* w, fp8lm_meta* w_meta, void* wcopy,
                                 fp8lm_meta* wcopy_meta, const fp8lm_adam_hparams* hp, bool have_chunks) {
  if (!hp || (grad_fmt != FP8LM_E4M3 && grad_fmt != FP8LM_E5M2)) return FP8LM_ERR_INVALID_ARGUMENT;
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
  if (!have_chunks) return FP8LM_OK;
  if (!grad || !grad_meta || !m || !m_meta || !v || !v_meta || !w || !w_meta || !wcopy || !wcopy_meta)
    return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(grad) || !aligned16(m) || !aligned16(v) || !aligned16(w) || !aligned16(wcopy)) return FP8LM_ERR_MISALIGNED;
  // the one pair of buffers that may be the same: an E4M3 weight copy written over the gradient it was computed from
  if (static_cast<const void*>(grad) == wcopy && hp->wcopy != FP8LM_WCOPY_E4M3) return FP8LM_ERR_INVALID_ARGUMENT;
  return FP8LM_OK;
}

static fp8lm_status adam_launch(fp8lm_ctx* c, const uint8_t* grad, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta,
                                uint8_t* m, fp8lm_meta* m_meta, void* v, fp8lm_meta* v_meta, void* w, fp8lm_meta* w_meta,
                                void* wcopy, fp8lm_meta* wcopy_meta, const fp8lm_adam_hparams* hp, hipStream_t s,
                                const uint8_t* m_in = nullptr);

fp8lm_status fp8lm_adam_step_fp8(fp8lm_ctx* c, const uint8_t* grad, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta,
                                 uint8_t* m, fp8lm_meta* m_meta, void* v, fp8lm_meta* v_meta, void* w,
                                 fp8lm_meta* w_meta, void* wcopy, fp8lm_meta* wcopy_meta, const fp8lm_adam_hparams* hp,
                                 void* stream) {
  if (!c) return FP8LM_ERR_INVALID_ARGUMENT;
  const fp8lm_status ok = adam_args_ok(grad, grad_fmt, grad_meta, m, m_meta, v, v_meta, w, w_meta, wcopy, wcopy_meta, hp,
                                       c->n_chunks > 0);
  if (ok != FP8LM_OK) return ok;
  if (c->n_chunks == 0) return FP8LM_OK;
  DeviceGuard guard(c->device);
  return adam_launch(c, grad, grad_fmt, grad_meta, m, m_meta, v, v_meta, w, w_meta, wcopy, wcopy_meta, hp,
                     (hipStream_t)stream);
}

// The launches of one Adam step on the tables `c` points to (a context's own, or the fixed device array).
// m_in: null for the in-place step; otherwise the buffer the first moment is read from, and its scale is speculated.
static fp8lm_status adam_launch(fp8lm_ctx* c, const uint8_t* grad, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta,
                                uint8_t* m, fp8lm_meta* m_meta, void* v, fp8lm_meta* v_meta, void* w, fp8lm_meta* w_meta,
                                void* wcopy, fp8lm_meta* wcopy_meta, const fp8lm_adam_hparams* hp, hipStream_t s,
                                const uint8_t* m_in) {
  const bool variant = hp->master_fmt != FP8LM_STATE_F16 || hp->v_fmt != FP8LM_STATE_F16;
  const bool spec_m = m_in != nullptr;

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
  p.m_in = spec_m ? m_in : m;
  p.speculative_m = spec_m ? 1 : 0;

  const bool stats = hp->stats != 0, fast = hp->exact == 0;
  const Tables tb = tables_of(c);
  const bool e5 = grad_fmt == FP8LM_E5M2, q8 = hp->wcopy == FP8LM_WCOPY_E4M3;
  if (spec_m) {
    Timed tm(c, s, FP8LM_K_SCALARS);
    const dim3 gs((c->n_tensors + 255) / 256), bs(256);
    if (q8) hipLaunchKernelGGL((adam_speculate_scales_kernel<FP8LM_WCOPY_E4M3>), gs, bs, 0, s, tb, p, c->n_tensors);
    else hipLaunchKernelGGL((adam_speculate_scales_kernel<FP8LM_WCOPY_BF16>), gs, bs, 0, s, tb, p, c->n_tensors);
  } else if (hp->m_scale_mode == FP8LM_MSCALE_FROM_CAST) {
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
  st = after_launch();
  if (st != FP8LM_OK || !spec_m) return st;
  // tensors whose first-moment scale turned out different: their chunk list, then the moment once more
  {
    Timed tm(c, s, FP8LM_K_SCALARS);
    hipLaunchKernelGGL(redo_scan_kernel, dim3(1), dim3(kScanThreads), 0, s, c->d_desc, c->d_scratch, c->d_redo_desc,
                       c->n_tensors, c->d_redo_count, c->d_spec_totals + 3);
    hipLaunchKernelGGL(redo_fill_kernel, dim3(std::min<int>(c->n_tensors, 1024)), dim3(256), 0, s, c->d_redo_desc,
                       c->d_redo_chunk_tensor, c->n_tensors);
    st = after_launch();
    if (st != FP8LM_OK) return st;
  }
  {
    const Tables rt = redo_tables_of(c);
    const dim3 g(grid_of(c)), b(kThreads);
    Timed tm(c, s, FP8LM_K_ADAM_AMAX);
    if (e5) hipLaunchKernelGGL((adam_moment_redo_kernel<kE5M2>), g, b, 0, s, rt, p);
    else hipLaunchKernelGGL((adam_moment_redo_kernel<kE4M3>), g, b, 0, s, rt, p);
  }
  return after_launch();
}

fp8lm_status fp8lm_adam_step_fp8_m2(fp8lm_ctx* c, const uint8_t* grad, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta,
                                    const uint8_t* m_in, uint8_t* m_out, fp8lm_meta* m_meta, void* v, fp8lm_meta* v_meta,
                                    void* w, fp8lm_meta* w_meta, void* wcopy, fp8lm_meta* wcopy_meta,
                                    const fp8lm_adam_hparams* hp, void* stream) {
  if (!c) return FP8LM_ERR_INVALID_ARGUMENT;
  const fp8lm_status ok = adam_args_ok(grad, grad_fmt, grad_meta, m_out, m_meta, v, v_meta, w, w_meta, wcopy, wcopy_meta, hp,
                                       c->n_chunks > 0);
  if (ok != FP8LM_OK) return ok;
  // the exact-amax scale only, default storage formats, no element counters (they would have to be recounted)
  if (hp->m_scale_mode != FP8LM_MSCALE_EXACT_PASS || hp->master_fmt != FP8LM_STATE_F16 || hp->v_fmt != FP8LM_STATE_F16 || hp->stats)
    return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks == 0) return FP8LM_OK;
  if (!m_in || m_in == m_out) return FP8LM_ERR_INVALID_ARGUMENT;
  if (!aligned16(m_in)) return FP8LM_ERR_MISALIGNED;
  if (static_cast<const void*>(grad) == wcopy) return FP8LM_ERR_OVERLAP;     // the repair reads the gradient again
  {
    // the two buffers must not share an element of any tensor
    long long extent = 0;
    for (const fp8lm_tensor& T : c->tensors) extent = std::max<long long>(extent, T.numel > 0 ? T.offset + T.numel : 0);
    const uintptr_t a = reinterpret_cast<uintptr_t>(m_in), b = reinterpret_cast<uintptr_t>(m_out);
    if (a < b + (uintptr_t)extent && b < a + (uintptr_t)extent) return FP8LM_ERR_OVERLAP;
  }
  DeviceGuard guard(c->device);
  c->fused.valid = false;
  return adam_launch(c, grad, grad_fmt, grad_meta, m_out, m_meta, v, v_meta, w, w_meta, wcopy, wcopy_meta, hp,
                     (hipStream_t)stream, m_in);
}

fp8lm_status fp8lm_get_moment_speculation_stats(fp8lm_ctx* c, uint64_t* calls, uint64_t* tensors_redone,
                                                uint64_t* elems_redone, void* stream) {
  if (!c || !calls || !tensors_redone || !elems_redone) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  unsigned long long h[3] = {0, 0, 0};
  HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
  HIP_TRY(hipMemcpy(h, c->d_spec_totals + 3, sizeof(h), hipMemcpyDeviceToHost));
  *calls = h[0]; *tensors_redone = h[1]; *elems_redone = h[2];
  return FP8LM_OK;
}

// ---- the Adam step without a context: tables, scales and reduction records in the fixed device array ----------
namespace {

constexpr int kMaxDevices = 64;
struct StaticDevice {
  StaticArena* arena = nullptr;      // device address of `scratch` on this GPU
  int num_cus = 0;
};
std::mutex g_static_mutex;
StaticDevice g_static_dev[kMaxDevices];

// Device address of the fixed array on `device` (which must be current) and that GPU's size; looked up on the
// first call per GPU.  Each GPU holds its own copy of the array at its own address.
fp8lm_status static_arena_of(int device, StaticDevice* out) {
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticDevice& d = g_static_dev[device];
  if (!d.arena) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) { g_hip_error = "hipGetSymbolAddress returned a null address"; return FP8LM_ERR_HIP; }
    int cus = 0;
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device));
    d.num_cus = cus > 0 ? cus : 256;
    d.arena = static_cast<StaticArena*>(ptr);
  }
  *out = d;
  return FP8LM_OK;
}

}  // namespace

fp8lm_status fp8lm_adam_step_fp8_static(int device, const fp8lm_tensor* tensors, int32_t n, const uint32_t* tensor_flags,
                                        const uint8_t* grad, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta, uint8_t* m,
                                        fp8lm_meta* m_meta, void* v, fp8lm_meta* v_meta, void* w, fp8lm_meta* w_meta,
                                        void* wcopy, fp8lm_meta* wcopy_meta, const fp8lm_adam_hparams* hp, void* stream) {
  if (n < 0 || (n > 0 && !tensors) || device < 0 || device >= kMaxDevices) return FP8LM_ERR_INVALID_ARGUMENT;
  if (n > FP8LM_STATIC_MAX_TENSORS) return FP8LM_ERR_TOO_LARGE;
  // the tensor list: same rules as fp8lm_create; everything below lives on this thread's stack
  long long total_chunks = 0;
  {
    std::pair<long long, long long> spans[FP8LM_STATIC_MAX_TENSORS];
    int n_spans = 0;
    for (int t = 0; t < n; ++t) {
      if (tensors[t].numel < 0 || tensors[t].offset < 0) return FP8LM_ERR_INVALID_ARGUMENT;
      if (tensors[t].offset % 16 != 0) return FP8LM_ERR_MISALIGNED;
      if (tensor_flags && (tensor_flags[t] & ~(uint32_t)FP8LM_TENSOR_NO_WEIGHT_DECAY)) return FP8LM_ERR_INVALID_ARGUMENT;
      if (tensors[t].numel > 0) spans[n_spans++] = {tensors[t].offset, tensors[t].offset + tensors[t].numel};
      total_chunks += (tensors[t].numel + kStaticChunkElems - 1) / kStaticChunkElems;
      if (total_chunks > FP8LM_STATIC_MAX_CHUNKS) return FP8LM_ERR_TOO_LARGE;
    }
    std::sort(spans, spans + n_spans);
    for (int i = 1; i < n_spans; ++i)
      if (spans[i].first < spans[i - 1].second) return FP8LM_ERR_OVERLAP;
  }
  const fp8lm_status ok = adam_args_ok(grad, grad_fmt, grad_meta, m, m_meta, v, v_meta, w, w_meta, wcopy, wcopy_meta, hp,
                                       total_chunks > 0);
  if (ok != FP8LM_OK) return ok;
  if (hp->m_scale_mode == FP8LM_MSCALE_FROM_CAST) return FP8LM_ERR_INVALID_ARGUMENT;   // needs the fused cast's context
  int count = 0;
  HIP_TRY(hipGetDeviceCount(&count));
  if (device >= count) return FP8LM_ERR_INVALID_ARGUMENT;
  if (total_chunks == 0) return FP8LM_OK;
  DeviceGuard guard(device);
  if (!guard.ok) { g_hip_error = "hipSetDevice failed"; return FP8LM_ERR_HIP; }
  StaticDevice dev;
  const fp8lm_status got = static_arena_of(device, &dev);
  if (got != FP8LM_OK) return got;
  StaticArena* A = dev.arena;
  hipStream_t s = (hipStream_t)stream;

  // 1. the tensor table, a batch of descriptors per launch, then the chunk table
  DescBatch batch;
  int32_t first_chunk = 0;
  for (int t0 = 0; t0 < n; t0 += kDescBatch) {
    batch.first = t0;
    batch.count = std::min(kDescBatch, n - t0);
    for (int i = 0; i < batch.count; ++i) {
      const fp8lm_tensor& T = tensors[t0 + i];
      const int32_t nc = (int32_t)((T.numel + kStaticChunkElems - 1) / kStaticChunkElems);
      batch.d[i] = TensorDesc{T.offset, T.numel, first_chunk, nc, tensor_flags ? tensor_flags[t0 + i] : 0u, 0u};
      first_chunk += nc;
    }
    for (int i = batch.count; i < kDescBatch; ++i) batch.d[i] = TensorDesc{0, 0, 0, 0, 0u, 0u};
    hipLaunchKernelGGL(static_desc_kernel, dim3(1), dim3(kDescBatch), 0, s, batch, A->desc);
  }
  hipLaunchKernelGGL(static_chunks_kernel, dim3(std::min(n, 1024)), dim3(256), 0, s, A->desc, A->chunk_tensor, A->scratch, n);
  fp8lm_status st = after_launch();
  if (st != FP8LM_OK) return st;

  // 2. the two passes, on a context-shaped view of the array (no vectors in it are ever filled: nothing allocates)
  fp8lm_ctx view;
  view.device = device;
  view.n_tensors = n;
  view.num_cus = dev.num_cus;
  view.chunk_elems = kStaticChunkElems;
  view.blocks_per_cu = std::max(1, std::min<int>(kMaxBlocksPerCu, kStaticMaxGrid / dev.num_cus));   // grid <= kStaticMaxGrid records
  if ((long long)view.num_cus * view.blocks_per_cu > kStaticMaxGrid) return FP8LM_ERR_TOO_LARGE;
  view.single_pass_min_chunks = 1 << 30;     // per-tensor totals in a second launch: no tickets to keep at zero
  view.n_chunks = (int32_t)total_chunks;
  view.d_desc = A->desc;
  view.d_chunk_tensor = A->chunk_tensor;
  view.d_scratch = A->scratch;
  view.d_partials = A->partials;
  return adam_launch(&view, grad, grad_fmt, grad_meta, m, m_meta, v, v_meta, w, w_meta, wcopy, wcopy_meta, hp, s);
}

fp8lm_status fp8lm_quant_error_stats(fp8lm_ctx* c, const void* ref, fp8lm_src ref_type, const uint8_t* q, fp8lm_fmt fmt,
                                     const fp8lm_meta* q_meta, fp8lm_quant_stats* out, void* stream) {
  if (!c || !src_ok(ref_type) || (fmt != FP8LM_E4M3 && fmt != FP8LM_E5M2)) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_tensors == 0) return FP8LM_OK;
  if (!out || (c->n_chunks > 0 && (!ref || !q || !q_meta))) return FP8LM_ERR_INVALID_ARGUMENT;
  if (c->n_chunks > 0 && (!aligned16(ref) || !aligned16(q))) return FP8LM_ERR_MISALIGNED;
  DeviceGuard guard(c->device);
  hipStream_t s = (hipStream_t)stream;
  {
    // entries of empty tensors are never written by the reduction: start from zero
    Timed tm(c, s, FP8LM_K_SCALARS);
    hipLaunchKernelGGL(quant_stats_zero_kernel, dim3((c->n_tensors + 255) / 256), dim3(256), 0, s, out, c->n_tensors);
    fp8lm_status st = after_launch();
    if (st != FP8LM_OK) return st;
  }
  if (c->n_chunks == 0) return FP8LM_OK;
  StatsParams p{ref, q, q_meta, out};
  Timed tm(c, s, FP8LM_K_STATS);
#define FP8LM_STATS_SRC(S)                                                                                   \
  do {                                                                                                       \
    if (fmt == FP8LM_E4M3) launch_walk<QuantStatsOp<kE4M3, S>>(c, s, quant_stats_kernel<kE4M3, S>, p);        \
    else launch_walk<QuantStatsOp<kE5M2, S>>(c, s, quant_stats_kernel<kE5M2, S>, p);                          \
  } while (0)
  if (ref_type == FP8LM_SRC_F32) FP8LM_STATS_SRC(kSrcF32);
  else if (ref_type == FP8LM_SRC_F16) FP8LM_STATS_SRC(kSrcF16);
  else FP8LM_STATS_SRC(kSrcBF16);
#undef FP8LM_STATS_SRC
  return after_launch();
}

// Host only.  Whole-tensor greedy distribution of Sec. 2.3, Alg. 1, with a heap over the GPUs.
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

fp8lm_status fp8lm_memory_skeleton(fp8lm_ctx* c, int32_t shape, void* const* bufs, int64_t n_elems, void* stream) {
  static const int n_bufs[] = {1, 2, 1, 1, 2, 5, 5, 5};
  if (!c || shape < 0 || shape > FP8LM_SKEL_UPDATE_WRITES || !bufs || n_elems < 0 || n_elems % kTile != 0)
    return FP8LM_ERR_INVALID_ARGUMENT;
  for (int i = 0; i < n_bufs[shape]; ++i) {
    if (!bufs[i]) return FP8LM_ERR_INVALID_ARGUMENT;
    if (!aligned16(bufs[i])) return FP8LM_ERR_MISALIGNED;
  }
  if (n_elems == 0) return FP8LM_OK;
  DeviceGuard guard(c->device);
  SkeletonParams p{};
  p.n_tiles = n_elems / kTile;
  p.sink = reinterpret_cast<uint32_t*>(c->d_partials);     // kWaves words per workgroup: far inside the record array
  const long long want = (long long)c->num_cus * c->blocks_per_cu;
  const dim3 g((unsigned)std::max<long long>(1, std::min<long long>(want, p.n_tiles))), b(kThreads);
  hipStream_t s = (hipStream_t)stream;
  Timed tm(c, s, FP8LM_K_SKELETON);
  switch (shape) {
    case FP8LM_SKEL_READ16:
      p.s2[0] = static_cast<const uint16_t*>(bufs[0]);
      hipLaunchKernelGGL((skeleton_kernel<0, 1, 0, 0, FP8LM_UN_READ>), g, b, 0, s, p);
      break;
    case FP8LM_SKEL_READ8X2:
      p.s1[0] = static_cast<const uint8_t*>(bufs[0]); p.s1[1] = static_cast<const uint8_t*>(bufs[1]);
      hipLaunchKernelGGL((skeleton_kernel<2, 0, 0, 0, FP8LM_UN_READ>), g, b, 0, s, p);
      break;
    case FP8LM_SKEL_WRITE16:
      p.d2[0] = static_cast<uint16_t*>(bufs[0]);
      hipLaunchKernelGGL((skeleton_kernel<0, 0, 0, 1, 1>), g, b, 0, s, p);
      break;
    case FP8LM_SKEL_WRITE8:
      p.d1[0] = static_cast<uint8_t*>(bufs[0]);
      hipLaunchKernelGGL((skeleton_kernel<0, 0, 1, 0, 1>), g, b, 0, s, p);
      break;
    case FP8LM_SKEL_CAST:
      p.s2[0] = static_cast<const uint16_t*>(bufs[0]); p.d1[0] = static_cast<uint8_t*>(bufs[1]);
      hipLaunchKernelGGL((skeleton_kernel<0, 1, 1, 0, FP8LM_UN_CAST>), g, b, 0, s, p);
      break;
    default:   // the update shapes: reads g, m, v, w; writes m, v, w in place and the weight copy; or one half of that
      p.s1[0] = static_cast<const uint8_t*>(bufs[0]); p.s1[1] = static_cast<const uint8_t*>(bufs[1]);
      p.s2[0] = static_cast<const uint16_t*>(bufs[2]); p.s2[1] = static_cast<const uint16_t*>(bufs[3]);
      p.d1[0] = static_cast<uint8_t*>(bufs[1]); p.d1[1] = static_cast<uint8_t*>(bufs[4]);
      p.d2[0] = static_cast<uint16_t*>(bufs[2]); p.d2[1] = static_cast<uint16_t*>(bufs[3]);
      if (shape == FP8LM_SKEL_UPDATE) hipLaunchKernelGGL((skeleton_kernel<2, 2, 2, 2, FP8LM_UN_UPDATE>), g, b, 0, s, p);
      else if (shape == FP8LM_SKEL_UPDATE_READS) hipLaunchKernelGGL((skeleton_kernel<2, 2, 0, 0, FP8LM_UN_UPDATE>), g, b, 0, s, p);
      else hipLaunchKernelGGL((skeleton_kernel<0, 0, 2, 2, FP8LM_UN_UPDATE>), g, b, 0, s, p);
      break;
  }
  return after_launch();
}

// ---- device memory piece by piece (HIP virtual memory management); see fp8lm.h ---------------------------------
namespace {
hipMemAllocationProp vmm_prop(int device) {
  hipMemAllocationProp prop = {};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = device;
  return prop;
}
fp8lm_status vmm_granularity_of(int device, size_t* g) {
  const hipMemAllocationProp prop = vmm_prop(device);
  HIP_TRY(hipMemGetAllocationGranularity(g, &prop, hipMemAllocationGranularityRecommended));
  if (*g == 0) *g = 4096;
  return FP8LM_OK;
}
}  // namespace

fp8lm_status fp8lm_vmm_granularity(int device, uint64_t* bytes) {
  if (!bytes || device < 0) return FP8LM_ERR_INVALID_ARGUMENT;
  int ok = 0;
  HIP_TRY(hipDeviceGetAttribute(&ok, hipDeviceAttributeVirtualMemoryManagementSupported, device));
  if (!ok) { g_hip_error = "virtual memory management is not supported on this device"; return FP8LM_ERR_HIP; }
  size_t g = 0;
  const fp8lm_status st = vmm_granularity_of(device, &g);
  if (st == FP8LM_OK) *bytes = g;
  return st;
}

fp8lm_status fp8lm_vmm_reserve(uint64_t bytes, void** va) {
  if (!va || bytes == 0) return FP8LM_ERR_INVALID_ARGUMENT;
  *va = nullptr;
  HIP_TRY(hipMemAddressReserve(va, bytes, 0, nullptr, 0));
  return FP8LM_OK;
}

fp8lm_status fp8lm_vmm_free(void* va, uint64_t bytes) {
  if (!va || bytes == 0) return FP8LM_ERR_INVALID_ARGUMENT;
  HIP_TRY(hipMemAddressFree(va, bytes));
  return FP8LM_OK;
}

fp8lm_status fp8lm_vmm_create(int device, uint64_t bytes, uint64_t* piece) {
  if (!piece || bytes == 0 || device < 0) return FP8LM_ERR_INVALID_ARGUMENT;
  size_t g = 0;
  const fp8lm_status st = vmm_granularity_of(device, &g);
  if (st != FP8LM_OK) return st;
  if (bytes % g != 0) return FP8LM_ERR_INVALID_ARGUMENT;
  const hipMemAllocationProp prop = vmm_prop(device);
  hipMemGenericAllocationHandle_t h{};
  HIP_TRY(hipMemCreate(&h, bytes, &prop, 0));
  static_assert(sizeof(h) <= sizeof(uint64_t), "the handle travels as 64 bits");
  *piece = 0;
  std::memcpy(piece, &h, sizeof(h));
  return FP8LM_OK;
}

fp8lm_status fp8lm_vmm_destroy(uint64_t piece) {
  if (piece == 0) return FP8LM_ERR_INVALID_ARGUMENT;
  hipMemGenericAllocationHandle_t h{};
  std::memcpy(&h, &piece, sizeof(h));
  HIP_TRY(hipMemRelease(h));
  return FP8LM_OK;
}

fp8lm_status fp8lm_vmm_map(void* va, uint64_t bytes, uint64_t piece, int device) {
  if (!va || bytes == 0 || piece == 0 || device < 0) return FP8LM_ERR_INVALID_ARGUMENT;
  hipMemGenericAllocationHandle_t h{};
  std::memcpy(&h, &piece, sizeof(h));
  HIP_TRY(hipMemMap(va, bytes, 0, h, 0));
  hipMemAccessDesc acc = {};
  acc.location.type = hipMemLocationTypeDevice;
  acc.location.id = device;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  const hipError_t e = hipMemSetAccess(va, bytes, &acc, 1);
  if (e != hipSuccess) {
    g_hip_error = std::string("hipMemSetAccess: ") + hipGetErrorString(e);
    (void)hipMemUnmap(va, bytes);
    return FP8LM_ERR_HIP;
  }
  return FP8LM_OK;
}

fp8lm_status fp8lm_vmm_unmap(void* va, uint64_t bytes) {
  if (!va || bytes == 0) return FP8LM_ERR_INVALID_ARGUMENT;
  HIP_TRY(hipDeviceSynchronize());     // no kernel may still be using the mapping
  HIP_TRY(hipMemUnmap(va, bytes));
  return FP8LM_OK;
}

fp8lm_status fp8lm_set_timing(fp8lm_ctx* c, int32_t enable) {
  if (!c) return FP8LM_ERR_INVALID_ARGUMENT;
  DeviceGuard guard(c->device);
  if (enable && c->free_events.empty() && c->stamps.empty()) {
    c->stamps.reserve(4096);           // launches are stamped without touching the host allocator
    c->free_events.reserve(4096);
    for (int i = 0; i < 4096; ++i) {
      hipEvent_t a = nullptr, b = nullptr;
      HIP_TRY(hipEventCreate(&a));
      if (hipError_t e = hipEventCreate(&b); e != hipSuccess) {
        (void)hipEventDestroy(a);
        g_hip_error = std::string("hipEventCreate: ") + hipGetErrorString(e);
        return FP8LM_ERR_HIP;
      }
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
