// Free-running parity of libfp8lm against the CPU oracle, from C++ with nothing but the C ABI of
// include/fp8lm.h and the HIP runtime (no Python, no torch).  Usage:
//   c_abi_parity <path of libfp8lm_oracle.so> [steps]
// The library is linked; the oracle is loaded at run time, its prototypes declared here (it ships no header).
// Inputs are seeded and synthetic: Gaussian bf16 gradients with a per-tensor sigma, Gaussian bf16 weights.
// Both sides start from the same bits and never see each other's state; after every step every payload
// byte and every metadata field must be identical (the division and square root of the weight update are
// the correctly rounded ones on both sides: hp.exact = 1).
#include <dlfcn.h>
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "fp8lm.h"

namespace {

// ---- the oracle's interface (byte layouts equal to those of fp8lm.h where the names match) -----------
struct OracleTensor { int64_t offset, numel; };
struct OracleCfg { int32_t sat_num, sat_den, ramp_steps, hist_window, margin, mu_rule, mu_min_exp; };
struct OracleHparams {
  float lr, beta1, beta2, eps, weight_decay;
  int64_t step;
  int32_t v_scaled, wcopy, m_predict, master_fmt, v_fmt;
};
using MetaInitFn = void (*)(void*, int32_t, const OracleCfg*);
using AmaxFn = void (*)(const uint16_t*, const OracleTensor*, int32_t, int, void*, const OracleCfg*);
using CastFn = void (*)(const uint16_t*, const OracleTensor*, int32_t, uint8_t*, int, void*, const OracleCfg*);
using InitMasterFn = void (*)(const uint16_t*, const OracleTensor*, int32_t, uint16_t*, void*);
using AdamFn = void (*)(const OracleTensor*, int32_t, const uint8_t*, int, const void*, uint8_t*, void*, void*, void*,
                        void*, void*, void*, void*, const OracleHparams*);
using SizeofFn = uint32_t (*)(void);

template <class F> F sym(void* h, const char* name) {
  void* p = dlsym(h, name);
  if (!p) { std::fprintf(stderr, "oracle symbol %s missing\n", name); std::exit(2); }
  return reinterpret_cast<F>(p);
}

// ---- seeded inputs: splitmix64 -> Box-Muller -> bf16 (top half of the fp32 pattern) ---------------------
uint64_t mix(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}
double unit(uint64_t key) { return ((double)(mix(key) >> 11) + 0.5) * (1.0 / 9007199254740992.0); }
uint16_t gaussian_bf16(uint64_t key, double sigma) {
  const double r = std::sqrt(-2.0 * std::log(unit(2 * key))), a = 6.283185307179586 * unit(2 * key + 1);
  const float x = (float)(sigma * r * std::cos(a));
  uint32_t b;
  std::memcpy(&b, &x, 4);
  return (uint16_t)(b >> 16);
}

#define HIP_OK(expr)                                                                             \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #expr, hipGetErrorString(e_)); std::exit(2); } \
  } while (0)
#define LIB_OK(expr)                                                                             \
  do {                                                                                           \
    fp8lm_status s_ = (expr);                                                                    \
    if (s_ != FP8LM_OK) {                                                                        \
      std::fprintf(stderr, "%s: %s (%s)\n", #expr, fp8lm_status_string(s_), fp8lm_last_hip_error());        \
      std::exit(2);                                                                              \
    }                                                                                            \
  } while (0)

template <class T> T* dev_alloc(size_t n) {
  T* p = nullptr;
  HIP_OK(hipMalloc((void**)&p, (n ? n : 1) * sizeof(T)));
  HIP_OK(hipMemset(p, 0, (n ? n : 1) * sizeof(T)));
  return p;
}

int differing(const void* a, const void* b, size_t bytes, const char* what, int step) {
  if (std::memcmp(a, b, bytes) == 0) return 0;
  const uint8_t *pa = static_cast<const uint8_t*>(a), *pb = static_cast<const uint8_t*>(b);
  size_t first = 0, count = 0;
  for (size_t i = 0; i < bytes; ++i)
    if (pa[i] != pb[i]) { if (!count) first = i; ++count; }
  std::printf("step %d: %s differs in %zu of %zu bytes, first at byte %zu (library %u, oracle %u)\n", step, what, count,
              bytes, first, pa[first], pb[first]);
  return 1;
}

}  // namespace

int main(int argc, char** argv) {
  if (argc < 2) { std::fprintf(stderr, "usage: %s <libfp8lm_oracle.so> [steps]\n", argv[0]); return 2; }
  const int steps = argc > 2 ? std::atoi(argv[2]) : 4;
  void* oh = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
  if (!oh) { std::fprintf(stderr, "dlopen: %s\n", dlerror()); return 2; }
  const auto o_meta_init = sym<MetaInitFn>(oh, "oracle_meta_init");
  const auto o_amax = sym<AmaxFn>(oh, "oracle_amax_scale");
  const auto o_cast = sym<CastFn>(oh, "oracle_cast_fp8");
  const auto o_init_master = sym<InitMasterFn>(oh, "oracle_init_master");
  const auto o_adam = sym<AdamFn>(oh, "oracle_adam_step_fp8");
  if (sym<SizeofFn>(oh, "oracle_sizeof_meta")() != sizeof(fp8lm_meta) || fp8lm_sizeof_meta() != sizeof(fp8lm_meta)) {
    std::fprintf(stderr, "metadata layouts disagree\n");
    return 2;
  }

  // ragged tensors: several tiles and a tail, exactly one chunk, a few elements, empty, many chunks
  const int64_t numel[] = {70001, 16384, 17, 0, 300003, 4096, 1};
  const double sigma[] = {1e-4, 3e-2, 1e-6, 1.0, 2e-5, 5.0, 1e-3};
  const int n = (int)(sizeof(numel) / sizeof(numel[0]));
  std::vector<fp8lm_tensor> tensors(n);
  std::vector<OracleTensor> o_tensors(n);
  int64_t total = 0;
  for (int t = 0; t < n; ++t) {
    tensors[t] = fp8lm_tensor{total, numel[t]};
    o_tensors[t] = OracleTensor{total, numel[t]};
    total += (numel[t] + 15) / 16 * 16;
  }
  const size_t T = (size_t)total;

  fp8lm_autoscale_cfg cfg{};
  cfg.sat_num = 1; cfg.sat_den = 100000; cfg.ramp_steps = 4; cfg.hist_window = 2; cfg.margin = 0;
  cfg.mu_rule = FP8LM_MU_SET_HALF; cfg.mu_min_exp = -1;
  const OracleCfg o_cfg{cfg.sat_num, cfg.sat_den, cfg.ramp_steps, cfg.hist_window, cfg.margin, cfg.mu_rule, cfg.mu_min_exp};

  fp8lm_ctx* ctx = nullptr;
  LIB_OK(fp8lm_create(&ctx, tensors.data(), n, 0));
  uint16_t* d_g = dev_alloc<uint16_t>(T);
  uint16_t* d_w0 = dev_alloc<uint16_t>(T);
  // The FP8 gradient lives in device memory put together piece by piece (fp8lm_vmm_*): two pieces mapped one after
  // the other into one reserved range, as a caller would do to make the buffer alternate between HBM regions.
  uint8_t* d_q = nullptr;
  uint64_t gran = 0, piece_bytes = 0, pieces[2] = {0, 0};
  if (fp8lm_vmm_granularity(0, &gran) == FP8LM_OK) {
    piece_bytes = ((T + 1) / 2 + gran - 1) / gran * gran;
    void* va = nullptr;
    LIB_OK(fp8lm_vmm_reserve(2 * piece_bytes, &va));
    for (int k = 0; k < 2; ++k) {
      LIB_OK(fp8lm_vmm_create(0, piece_bytes, &pieces[k]));
      LIB_OK(fp8lm_vmm_map(static_cast<char*>(va) + k * piece_bytes, piece_bytes, pieces[k], 0));
    }
    d_q = static_cast<uint8_t*>(va);
    HIP_OK(hipMemset(d_q, 0, 2 * piece_bytes));
    std::printf("c_abi_parity: FP8 gradient in two mapped pieces of %llu bytes\n", (unsigned long long)piece_bytes);
  } else {
    std::printf("c_abi_parity: no virtual memory management here (%s): plain allocation\n", fp8lm_last_hip_error());
    d_q = dev_alloc<uint8_t>(T);
  }
  uint8_t* d_m = dev_alloc<uint8_t>(T);
  uint16_t* d_v = dev_alloc<uint16_t>(T);
  uint16_t* d_w = dev_alloc<uint16_t>(T);
  uint8_t* d_wq = dev_alloc<uint8_t>(T);
  fp8lm_meta* d_meta[5];   // g, m, v, w, wq
  for (auto& p : d_meta) { p = dev_alloc<fp8lm_meta>(n); LIB_OK(fp8lm_meta_init(ctx, p, &cfg, nullptr)); }

  std::vector<uint16_t> h_g(T, 0), h_w0(T, 0), o_v(T, 0), o_w(T, 0), r_v(T), r_w(T);
  std::vector<uint8_t> o_q(T, 0), o_m(T, 0), o_wq(T, 0), r_q(T), r_m(T), r_wq(T);
  std::vector<fp8lm_meta> o_meta[5], r_meta(n);
  for (auto& m : o_meta) { m.resize(n); o_meta_init(m.data(), n, &o_cfg); }

  for (int t = 0; t < n; ++t)
    for (int64_t i = 0; i < numel[t]; ++i)
      h_w0[tensors[t].offset + i] = gaussian_bf16(((uint64_t)(1000 + t) << 40) + (uint64_t)i, 0.02);
  HIP_OK(hipMemcpy(d_w0, h_w0.data(), T * 2, hipMemcpyHostToDevice));
  LIB_OK(fp8lm_init_master(ctx, d_w0, d_w, d_meta[3], nullptr));
  o_init_master(h_w0.data(), o_tensors.data(), n, o_w.data(), o_meta[3].data());

  int bad = 0, mu_min = 9, mu_max = -9;
  uint64_t sat = 0;
  for (int step = 1; step <= steps && !bad; ++step) {
    std::printf("c_abi_parity: step %d of %d\n", step, steps);
    std::fflush(stdout);
    // the gradient grows by 16x at step 3 so that the history window, saturation and mu all move
    const double growth = step == 3 ? 16.0 : 1.0;
    for (int t = 0; t < n; ++t)
      for (int64_t i = 0; i < numel[t]; ++i)
        h_g[tensors[t].offset + i] = gaussian_bf16(((uint64_t)(step * 64 + t) << 40) + (uint64_t)i, sigma[t] * growth);
    HIP_OK(hipMemcpy(d_g, h_g.data(), T * 2, hipMemcpyHostToDevice));

    fp8lm_adam_hparams hp{};
    hp.lr = 1e-3f; hp.beta1 = 0.9f; hp.beta2 = 0.95f; hp.eps = 1e-8f; hp.weight_decay = 0.1f; hp.step = step;
    hp.v_scaled = 1; hp.wcopy = FP8LM_WCOPY_E4M3; hp.stats = 1; hp.m_scale_mode = FP8LM_MSCALE_EXACT_PASS;
    hp.master_fmt = FP8LM_STATE_F16; hp.v_fmt = FP8LM_STATE_F16; hp.exact = 1;
    LIB_OK(fp8lm_amax_scale(ctx, d_g, FP8LM_SRC_BF16, FP8LM_E5M2, d_meta[0], &cfg, nullptr));
    LIB_OK(fp8lm_cast_fp8(ctx, d_g, FP8LM_SRC_BF16, d_q, FP8LM_E5M2, d_meta[0], &cfg, nullptr));
    LIB_OK(fp8lm_adam_step_fp8(ctx, d_q, FP8LM_E5M2, d_meta[0], d_m, d_meta[1], d_v, d_meta[2], d_w, d_meta[3], d_wq,
                               d_meta[4], &hp, nullptr));
    HIP_OK(hipDeviceSynchronize());

    const OracleHparams o_hp{hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.step, 1, 0, 0, 0, 0};
    o_amax(h_g.data(), o_tensors.data(), n, /*E5M2*/ 1, o_meta[0].data(), &o_cfg);
    o_cast(h_g.data(), o_tensors.data(), n, o_q.data(), 1, o_meta[0].data(), &o_cfg);
    o_adam(o_tensors.data(), n, o_q.data(), 1, o_meta[0].data(), o_m.data(), o_meta[1].data(), o_v.data(),
           o_meta[2].data(), o_w.data(), o_meta[3].data(), o_wq.data(), o_meta[4].data(), &o_hp);

    HIP_OK(hipMemcpy(r_q.data(), d_q, T, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(r_m.data(), d_m, T, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(r_v.data(), d_v, T * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(r_w.data(), d_w, T * 2, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(r_wq.data(), d_wq, T, hipMemcpyDeviceToHost));
    bad += differing(r_q.data(), o_q.data(), T, "FP8 gradient", step);
    bad += differing(r_m.data(), o_m.data(), T, "first moment", step);
    bad += differing(r_v.data(), o_v.data(), T * 2, "second moment", step);
    bad += differing(r_w.data(), o_w.data(), T * 2, "master weights", step);
    bad += differing(r_wq.data(), o_wq.data(), T, "FP8 weight copy", step);
    static const char* names[5] = {"gradient meta", "first-moment meta", "second-moment meta", "master meta", "weight-copy meta"};
    for (int k = 0; k < 5; ++k) {
      HIP_OK(hipMemcpy(r_meta.data(), d_meta[k], n * sizeof(fp8lm_meta), hipMemcpyDeviceToHost));
      for (int t = 0; t < n; ++t) {
        if (numel[t] == 0) continue;   // an empty tensor's metadata is never touched by the library
        bad += differing(&r_meta[t], &o_meta[k][t], sizeof(fp8lm_meta), names[k], step);
      }
    }
    for (int t = 0; t < n; ++t) {
      sat += o_meta[0][t].n_sat;
      if (o_meta[0][t].mu_exp < mu_min) mu_min = o_meta[0][t].mu_exp;
      if (o_meta[0][t].mu_exp > mu_max) mu_max = o_meta[0][t].mu_exp;
    }
  }
  LIB_OK(fp8lm_destroy(ctx));
  if (piece_bytes) {
    LIB_OK(fp8lm_vmm_unmap(d_q, 2 * piece_bytes));
    for (uint64_t h : pieces) LIB_OK(fp8lm_vmm_destroy(h));
    LIB_OK(fp8lm_vmm_free(d_q, 2 * piece_bytes));
  }
  std::printf("c_abi_parity: %s after %d steps, %lld elements in %d tensors (%llu saturated gradient codes in all, log2 mu between %d and %d)\n",
              bad ? "MISMATCH" : "identical", steps, (long long)total, n, (unsigned long long)sat, mu_min, mu_max);
  return bad ? 1 : 0;
}
