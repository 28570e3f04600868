/*
 * fp8lm.h -- C ABI of the MI355X (gfx950) implementation of the optimizer-side hot path of
 * FP8-LM (arXiv 2310.18313): per-tensor automatically scaled FP8 gradient quantisation
 * (Sec. 2.1, Appendix A.2) and the FP8 Adam step (Sec. 2.2).
 *
 * General rules of this boundary
 *   - Plain C.  Every pointer named "device" is a device (HBM) address on the context's GPU; every
 *     pointer named "host" is ordinary host memory that is only read during the call.
 *   - All tensors of a model live in flat buffers.  Tensor t occupies elements
 *     [tensors[t].offset, tensors[t].offset + tensors[t].numel) of EVERY flat buffer passed to a call
 *     (gradient source, FP8 gradient, moments, master weights, weight copy), whatever its element
 *     size.  Offsets are multiples of 16 elements, buffers start on a 16-byte boundary, tensors do not
 *     overlap.  Elements between tensors are padding: never read into a result, never written.
 *   - Each scaled buffer carries one fp8lm_meta per tensor (device memory, caller-owned).  A stored
 *     payload equals value * scale; the value is payload / scale (Sec. 2.1, text before Eq. 4).
 *     Scales are powers of two, so scaling is exact; the one exception is the metadata fp8lm_sum_fp8
 *     writes (scale N * s_g, see there).
 *   - Calls enqueue work on the given HIP stream and return without synchronising.  They allocate no
 *     device memory; only fp8lm_create / fp8lm_destroy, the two calls that rebuild a context's tables
 *     (fp8lm_set_tuning, fp8lm_set_tensor_flags) and the timing aid (fp8lm_set_timing creates its events
 *     up front) touch an allocator.  One context must not be used from two streams at the same time (its
 *     reduction scratch is shared).
 *   - Return value: FP8LM_OK or a negative fp8lm_status.  On an error nothing has been enqueued.
 *     Data-dependent conditions (non-finite inputs, all-zero tensors, saturation) are reported in the
 *     metadata flags and counters on the device, never in the return value.
 *   - Tensors with numel == 0 are skipped: their metadata is left untouched.
 *   - Parameter groups (other hyper-parameters for some tensors): one context per group, over disjoint
 *     tensor lists of the same flat buffers, each with its own metadata arrays (indexed by the position
 *     in its own list) and stepped with its own calls.  The most common case, no weight decay on biases
 *     and normalisation weights, needs no second context: see fp8lm_set_tensor_flags.
 */
#ifndef FP8LM_H
#define FP8LM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fp8lm_ctx fp8lm_ctx;

typedef enum {
  FP8LM_OK = 0,
  FP8LM_ERR_INVALID_ARGUMENT = -1, /* null pointer, bad enum, bad hyper-parameter               */
  FP8LM_ERR_MISALIGNED = -2,       /* offset not a multiple of 16 or buffer not 16-byte aligned  */
  FP8LM_ERR_OVERLAP = -3,          /* two tensors share elements                                 */
  FP8LM_ERR_HIP = -4,              /* a HIP runtime call failed (see fp8lm_last_hip_error)       */
  FP8LM_ERR_TOO_LARGE = -5         /* more chunks / tensors than the 32-bit tables can index     */
} fp8lm_status;

/* Appendix A.1: E4M3 (max 448, NaN, no infinity) and E5M2 (max 57344, infinities and NaN).      */
typedef enum { FP8LM_E4M3 = 0, FP8LM_E5M2 = 1 } fp8lm_fmt;
/* Element type of the high-precision gradient handed to the cast (Sec. 2.1 quantises "high-
 * precision" gradients): bf16 or IEEE half as 2-byte elements, fp32 as 4-byte elements.  Every
 * source is widened to fp32 exactly before it is scaled.                                        */
typedef enum { FP8LM_SRC_BF16 = 0, FP8LM_SRC_F16 = 1, FP8LM_SRC_F32 = 2 } fp8lm_src;
/* Format of the low-precision weight copy written by the optimizer.                             */
typedef enum { FP8LM_WCOPY_E4M3 = 0, FP8LM_WCOPY_BF16 = 1 } fp8lm_wcopy;

/* How fp8lm_adam_step_fp8 chooses the scale of the first moment it stores.
 *   EXACT_PASS : from the exact amax of the new moment, measured by an extra read-only pass over grad
 *                and m inside fp8lm_adam_step_fp8 (just-in-time scaling, Appendix A.2);
 *   PREDICTED  : from the bound fma(beta1, m_meta.amax_deq, (1-beta1) * grad_meta.amax_deq), which no new
 *                |m| exceeds: one pass less, the scale can be a binade or more looser; v, w and the
 *                update itself are unaffected;
 *   FROM_CAST  : the same exact amax as EXACT_PASS, but measured by the immediately preceding
 *                fp8lm_cast_fp8_for_adam call on the same grad, m, m_meta and beta1 (checked; otherwise
 *                INVALID_ARGUMENT).  Only valid when nothing changes grad between the two calls.   */
typedef enum { FP8LM_MSCALE_EXACT_PASS = 0, FP8LM_MSCALE_PREDICTED = 1, FP8LM_MSCALE_FROM_CAST = 2 } fp8lm_mscale;

/* Storage formats of the optimizer state, the precision-decoupling settings of Sec. 3.3 (table of
 * optimizer settings) and Sec. 2.2.  F16 and E4M3 are stored with a per-tensor power-of-two scale and
 * saturate; BF16 and F32 carry no scale (scale 1) and overflow to infinity as IEEE does.
 *   master weight: F16 (setting 2a, the default), BF16 (2b), E4M3 (3), F32 (the alternative of Sec. 2.2);
 *   second moment: F16 (default) or E4M3 (setting 4).                                                  */
typedef enum { FP8LM_STATE_F16 = 0, FP8LM_STATE_BF16 = 1, FP8LM_STATE_E4M3 = 2, FP8LM_STATE_F32 = 3 } fp8lm_state_fmt;

typedef struct {
  int64_t offset; /* first element, multiple of 16 */
  int64_t numel;  /* >= 0                          */
} fp8lm_tensor;

#define FP8LM_HIST 16

#define FP8LM_FLAG_NONFINITE 1u     /* an inf/NaN was seen; scale (and amax history) left unchanged  */
#define FP8LM_FLAG_AMAX_ZERO 2u     /* the magnitude bound was zero; scale left unchanged            */
#define FP8LM_FLAG_SCALE_CLAMPED 4u /* the scale exponent was clamped to [-126, 126]                 */
#define FP8LM_FLAG_SATURATED 8u     /* at least one stored payload sits on the largest finite code   */

/* Per-tensor, per-buffer scaling metadata.  Device resident, plain data, 112 bytes.               */
typedef struct {
  float scale;       /* power of two; stored payload = value * scale                               */
  float inv_scale;   /* 1 / scale: exact for a power-of-two scale; the fp32-rounded reciprocal in the
                        metadata fp8lm_sum_fp8 writes when the number of ranks is not a power of two  */
  float amax;        /* max |value| before quantisation; +inf if a non-finite value was seen       */
  float amax_deq;    /* max |stored payload| / scale over the stored codes that are not NaN        */
  float amax_hist[FP8LM_HIST]; /* ring of recent amax values (Appendix A.2, delayed scaling)       */
  int32_t hist_pos;    /* next ring slot                                                           */
  int32_t mu_exp;      /* log2 of the auto-scaling factor mu of Sec. 2.1, Eq. 3: -1, 0 or +1       */
  int32_t clean_steps; /* consecutive casts without overflow, capped at ramp_steps                 */
  uint32_t flags;      /* FP8LM_FLAG_*                                                             */
  uint64_t n_sat;       /* stored payloads whose magnitude is the largest finite code              */
  uint64_t n_underflow; /* non-zero values stored as zero                                          */
} fp8lm_meta;

/* Auto-scaling configuration (Sec. 2.1, paragraph after Eq. 3).  Defaults in brackets.            */
typedef struct {
  int32_t sat_num;     /* overflow when n_sat * sat_den > numel * sat_num  [1]; 0..2^24            */
  int32_t sat_den;     /*   ... i.e. more than 0.001 % of the payloads on the top code  [100000]; 1..2^24 */
  int32_t ramp_steps;  /* mu climbs from 1/2 to 2 over this many clean steps  [1000]               */
  int32_t hist_window; /* amax values that bound the scale, 1..FP8LM_HIST; 1 = just-in-time  [1]   */
  int32_t margin;      /* extra binades of headroom subtracted from the scale exponent  [0]        */
  int32_t mu_rule;     /* fp8lm_mu_rule: which reading of the garbled sentence of Sec. 2.1  [SET_HALF] */
  int32_t mu_min_exp;  /* FP8LM_MU_HALVE only: lowest log2(mu), -64..-1                             */
} fp8lm_autoscale_cfg;
/* FP8LM_MU_SET_HALF: an overflowing step sets mu to 1/2; mu then depends on the number of clean steps
 * since: 1/2 below ramp_steps/2, 1 below ramp_steps, 2 from there on.  FP8LM_MU_HALVE: every overflowing
 * step halves mu (down to 2^mu_min_exp), every ramp_steps/2 clean steps in a row double it (up to 2);
 * needed when a sum over many ranks outgrows the FP8 range by more than a factor of 2.             */
typedef enum { FP8LM_MU_SET_HALF = 0, FP8LM_MU_HALVE = 1 } fp8lm_mu_rule;

/* Hyper-parameters of one AdamW step (Sec. 3.1.2: beta1 0.9, beta2 0.95, weight decay 0.1).
 * Accepted ranges: 0 <= lr <= 1024, 0 <= beta1, beta2 < 1, 2^-36 <= eps < inf,
 * 0 <= weight_decay <= 1024, step >= 1.                                                            */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  int64_t step;     /* 1 for the first update (bias correction)                                    */
  int32_t v_scaled; /* 1: second moment stored as FP16 with a per-tensor scale; 0: plain FP16      */
  int32_t wcopy;    /* fp8lm_wcopy                                                                 */
  int32_t stats;    /* 1: count n_sat / n_underflow of the four outputs exactly (more ALU work);
                       0: leave them 0; FLAG_SATURATED is still exact (derived from the amax)      */
  int32_t m_scale_mode; /* fp8lm_mscale: where the scale of the stored first moment comes from             */
  int32_t master_fmt; /* fp8lm_state_fmt of w (default F16 with tensor scaling)                            */
  int32_t v_fmt;      /* fp8lm_state_fmt of v: F16 (default) or E4M3.  Any non-default pair requires
                         wcopy = E4M3 and stats = 0, and always uses correctly rounded arithmetic          */
  int32_t exact;    /* 1: correctly rounded sqrt and divide in the weight update (results identical to
                          the scalar definition);
                       0: hardware v_sqrt_f32 / v_rcp_f32, 1 ulp each: m and v are unaffected, the
                          update term is off by a few fp32 ulps, so a new weight is within one FP16
                          ulp of max(|w|, lr * |update|) -- more than one ulp of the result itself
                          where the two nearly cancel.  This setting is therefore OUTSIDE the accuracy
                          bar of this library (master weights within one FP16 ulp of the scalar
                          definition): a faster, looser variant, never the default                 */
} fp8lm_adam_hparams;

/*
 * Creates a context for a fixed tensor list on GPU `device`.
 *   tensors : host array of n entries, copied.  n >= 0.
 * Allocates the device-side tensor/chunk tables and the reduction scratch, and synchronises once.
 * Errors: INVALID_ARGUMENT (null, negative numel/offset), MISALIGNED, OVERLAP, TOO_LARGE, HIP.
 */
fp8lm_status fp8lm_create(fp8lm_ctx** out, const fp8lm_tensor* tensors /*host*/, int32_t n, int device);

/* Frees everything fp8lm_create allocated.  The caller guarantees no enqueued work still uses it. */
fp8lm_status fp8lm_destroy(fp8lm_ctx* ctx);

/*
 * Launch tuning (optional; defaults 16384, 16, 2^30).  chunk_elems: elements per work unit, a multiple of
 * 4096 in [4096, 1048576]; a chunk never spans two tensors and each workgroup walks one contiguous range
 * of chunks.  blocks_per_cu: 256-thread workgroups per compute unit that a launch uses at most, 1..16.
 * single_pass_min_chunks: how the per-tensor statistics of the workgroups are combined.  With at least
 * this many chunks per workgroup, in the same launch (each workgroup bumps a per-tensor ticket, the one
 * that completes it finishes the tensor); with fewer, in a second tiny launch, because the tickets then
 * cost more than the data.  0 = always in the same launch; the default always takes the second launch
 * (measured faster at every size on MI355X); results are identical either way.
 * Rebuilds the chunk table (synchronises the device; not to be called while a stream is being captured).
 * A HIP graph captured from this context before the call holds the old tables and must not be replayed
 * afterwards.  On an error the context keeps its previous tuning and tables.
 */
fp8lm_status fp8lm_set_tuning(fp8lm_ctx* ctx, int32_t chunk_elems, int32_t blocks_per_cu,
                              int32_t single_pass_min_chunks);

/*
 * Per-tensor attributes (optional; all 0 after fp8lm_create).  flags: host array of n = the context's tensor
 * count entries, each a combination of FP8LM_TENSOR_* bits.
 *   FP8LM_TENSOR_NO_WEIGHT_DECAY: fp8lm_adam_step_fp8 updates this tensor as if hp->weight_decay were 0 (the
 *   usual exemption of biases and normalisation weights; Sec. 3.1.2 states one weight decay of 0.1 and is silent
 *   on exemptions).  Every other hyper-parameter stays common to the call; tensors that need another learning rate
 *   or other betas go into a context of their own.
 * Rebuilds the tensor table (synchronises the device; not under stream capture; graphs captured from this context
 * before the call must not be replayed afterwards).  Unknown bits are refused.
 */
#define FP8LM_TENSOR_NO_WEIGHT_DECAY 1u
fp8lm_status fp8lm_set_tensor_flags(fp8lm_ctx* ctx, const uint32_t* flags /*host[n]*/, int32_t n);

/*
 * Initial metadata: scale 1, empty amax history, mu = 1 (clean_steps = ramp_steps / 2; 0 with
 * FP8LM_MU_HALVE), counters 0.
 *   meta : device array of n entries (n = the context's tensor count), overwritten.
 */
fp8lm_status fp8lm_meta_init(fp8lm_ctx* ctx, fp8lm_meta* meta /*device*/, const fp8lm_autoscale_cfg* cfg /*host*/,
                             void* stream);

/*
 * Step 1 of the gradient quantisation (Appendix A.2, just-in-time scaling; Sec. 2.1, Eq. 3).
 * For every tensor: amax = max |src|; the amax is pushed into the history ring; the scale becomes
 * 2^(k + mu_exp - margin) where k is the largest integer with 2^k * amax_eff <= max finite value of
 * `target` and amax_eff is the largest of the last hist_window amax values.  An all-zero history
 * keeps the old scale (FLAG_AMAX_ZERO); a non-finite input keeps scale and history, sets amax = +inf
 * (FLAG_NONFINITE).  Writes meta[t].{scale, inv_scale, amax, amax_hist, hist_pos, flags}.
 *   src  : device, flat gradient buffer of element type src_type (read only, 16-byte aligned).
 *   meta : device array [n_tensors], read and written.
 */
fp8lm_status fp8lm_amax_scale(fp8lm_ctx* ctx, const void* src /*device*/, fp8lm_src src_type, fp8lm_fmt target,
                              fp8lm_meta* meta /*device*/, const fp8lm_autoscale_cfg* cfg /*host*/, void* stream);

/*
 * Step 2 of the gradient quantisation (Sec. 2.1: the scaling tensor (g', s'); Appendix A.1).
 * dst[i] = FP8(meta[t].scale * src[i]), round to nearest even, saturating to the largest finite
 * code (inf included); NaN becomes 0x7F.  Precondition: meta[t].flags is what fp8lm_amax_scale left for
 * this very source (FLAG_NONFINITE routes the tensor to the element-by-element path that knows NaN; with
 * stale flags a NaN in src is stored as an arbitrary finite code).  fp8lm_cast_fp8_delayed has no such
 * precondition.  Also writes meta[t].{n_sat, n_underflow, amax_deq,
 * FLAG_SATURATED} and advances the auto-scaling state of Sec. 2.1: if more than sat_num/sat_den of
 * the payloads sit on the top code the next scale uses mu = 1/2 (clean_steps = 0); otherwise
 * clean_steps grows and mu = 1/2, 1, 2 as it passes 0, ramp_steps/2, ramp_steps.
 *   src : device, flat buffer of element type src_type (read only).
 *   dst : device, flat uint8 (written inside tensors only).
 */
fp8lm_status fp8lm_cast_fp8(fp8lm_ctx* ctx, const void* src /*device*/, fp8lm_src src_type, uint8_t* dst /*device*/,
                            fp8lm_fmt fmt, fp8lm_meta* meta /*device*/, const fp8lm_autoscale_cfg* cfg /*host*/,
                            void* stream);

/*
 * Single-pass gradient quantisation with delayed scaling (Appendix A.2: the scale is chosen from the
 * amax values of preceding iterations).  The scale of every tensor is first set from its history ring
 * as it stands (same rule as fp8lm_amax_scale; an all-zero history keeps the scale in the metadata,
 * FLAG_AMAX_ZERO), then one pass casts src with that scale exactly as fp8lm_cast_fp8 does
 * (saturating: a gradient that outgrew its history clips and is counted in n_sat) and at the same
 * time measures this step's amax, which is stored in meta[t].amax and pushed into the ring for the
 * following steps (a non-finite amax is flagged and not pushed).  The first step of a run should use
 * fp8lm_amax_scale + fp8lm_cast_fp8, which also seeds the history.
 */
fp8lm_status fp8lm_cast_fp8_delayed(fp8lm_ctx* ctx, const void* src /*device*/, fp8lm_src src_type,
                                    uint8_t* dst /*device*/, fp8lm_fmt fmt, fp8lm_meta* meta /*device*/,
                                    const fp8lm_autoscale_cfg* cfg /*host*/, void* stream);

/*
 * fp8lm_cast_fp8 (delayed = 0) or fp8lm_cast_fp8_delayed (delayed = 1) that also measures, in the same
 * pass, the amax of the first moment the following Adam step will produce: max |fma(beta1, m / s_m,
 * (1-beta1) * dst / s_g)| over each tensor, with dst the FP8 gradient just written.  On one GPU, where
 * nothing touches the gradient between quantisation and optimizer, this replaces the Adam step's own
 * read-only pass (19 -> 18 bytes per parameter and step) with identical results: call
 * fp8lm_adam_step_fp8 next with m_scale_mode = FP8LM_MSCALE_FROM_CAST.
 *   m, m_meta : device, the E4M3 first moment and its metadata as they stand (read only).
 */
fp8lm_status fp8lm_cast_fp8_for_adam(fp8lm_ctx* ctx, const void* src /*device*/, fp8lm_src src_type,
                                     uint8_t* dst /*device*/, fp8lm_fmt fmt, fp8lm_meta* meta /*device*/,
                                     const fp8lm_autoscale_cfg* cfg /*host*/, int32_t delayed,
                                     const uint8_t* m /*device*/, const fp8lm_meta* m_meta /*device*/, float beta1,
                                     void* stream);

/*
 * Just-in-time quantisation (Appendix A.2; Sec. 2.1) in one call: the results -- dst and every field of meta -- are
 * those of fp8lm_amax_scale followed by fp8lm_cast_fp8, bit for bit, but a tensor whose scale does not change from
 * one step to the next is read once instead of twice.  The scale is first set as the tensor's amax history predicts
 * it (the rule of fp8lm_cast_fp8_delayed) and one pass casts with it while measuring the true amax; then the scale
 * the true amax demands is computed exactly as fp8lm_amax_scale does, and only the tensors for which it differs
 * from the prediction (the amax crossed a power-of-two boundary, the first step, an inf/NaN in the source) are
 * cast a second time with the right scale.  Per step this moves 3 bytes per element of the tensors whose
 * prediction held and 6 of the others, instead of 5 of all.
 * fp8lm_quantize_fp8_for_adam also measures the amax of the first moment the following Adam step will produce, like
 * fp8lm_cast_fp8_for_adam: call fp8lm_adam_step_fp8 next with m_scale_mode = FP8LM_MSCALE_FROM_CAST.
 * fp8lm_get_speculation_stats synchronises `stream` and returns the context's running totals since fp8lm_create:
 * calls of the two entry points above, tensors cast twice, elements cast twice.
 */
fp8lm_status fp8lm_quantize_fp8(fp8lm_ctx* ctx, const void* src /*device*/, fp8lm_src src_type, uint8_t* dst /*device*/,
                                fp8lm_fmt fmt, fp8lm_meta* meta /*device*/, const fp8lm_autoscale_cfg* cfg /*host*/,
                                void* stream);
fp8lm_status fp8lm_quantize_fp8_for_adam(fp8lm_ctx* ctx, const void* src /*device*/, fp8lm_src src_type,
                                         uint8_t* dst /*device*/, fp8lm_fmt fmt, fp8lm_meta* meta /*device*/,
                                         const fp8lm_autoscale_cfg* cfg /*host*/, const uint8_t* m /*device*/,
                                         const fp8lm_meta* m_meta /*device*/, float beta1, void* stream);
fp8lm_status fp8lm_get_speculation_stats(fp8lm_ctx* ctx, uint64_t* calls /*host*/, uint64_t* tensors_redone /*host*/,
                                         uint64_t* elems_redone /*host*/, void* stream);

/*
 * The three steps around the FP8 gradient all-reduce of Sec. 2.1 (Eq. 4-6), as one GPU can run them;
 * the collectives themselves are not part of this library.  n_ranks <= 128.
 *
 * Eq. 4: shared[t] = min over r of metas[r][t].scale.
 *   metas  : host array of n_ranks device pointers, each to a meta array [n_tensors];
 *   shared : device array [n_tensors], written.
 */
fp8lm_status fp8lm_shared_scale(fp8lm_ctx* ctx, const fp8lm_meta* const* metas /*host -> device*/, int32_t n_ranks,
                                float* shared /*device*/, void* stream);
/*
 * Eq. 5: dst[i] = FP8(shared[t] * (src[i] / src_meta[t].scale)), round to nearest even.  For a source as
 * fp8lm_cast_fp8 leaves it both scales are powers of two and shared <= scale, so this is an exponent shift:
 * nothing saturates, values that fall below the format's range lose bits or become zero (n_underflow).  A
 * source with another scale (say the output of fp8lm_sum_fp8) is multiplied by src_meta[t].inv_scale and
 * by shared[t], two fp32 roundings, and saturates like any cast.  dst may be src (in place);
 * dst_meta must not be src_meta.  Writes dst_meta[t].{scale = shared, inv_scale, amax, amax_deq, n_sat,
 * n_underflow, flags}; the auto-scaling fields are left alone.
 */
fp8lm_status fp8lm_requantize_fp8(fp8lm_ctx* ctx, const uint8_t* src /*device*/, fp8lm_fmt fmt,
                                  const fp8lm_meta* src_meta /*device*/, const float* shared /*device*/,
                                  uint8_t* dst /*device*/, fp8lm_meta* dst_meta /*device*/, void* stream);
/*
 * Eq. 6 as a sum all-reduce would leave it on every rank: dst[i] = FP8(payloads[0][i] + ... +
 * payloads[N-1][i]), added in rank order in fp32 and rounded once (nearest even, saturating).  All
 * payloads carry the shared scale; dst_meta[t].scale = N * shared[t], so dst / scale is the mean
 * gradient.  For N that is not a power of two this scale is not one either and dst_meta[t].inv_scale is the
 * fp32-rounded 1 / (N * shared[t]): fp8lm_adam_step_fp8 dequantises with inv_scale, so it sees the mean
 * gradient to within one fp32 rounding (2^-24 relative) instead of exactly.  Also writes amax (of the sum, in
 * value units), amax_deq, n_sat, n_underflow, flags, and advances the auto-scaling state of dst_meta with
 * n_sat as fp8lm_cast_fp8 does.
 *   payloads : host array of n_ranks device pointers to flat FP8 buffers (read only).
 */
fp8lm_status fp8lm_sum_fp8(fp8lm_ctx* ctx, const uint8_t* const* payloads /*host -> device*/, int32_t n_ranks,
                           fp8lm_fmt fmt, const float* shared /*device*/, uint8_t* dst /*device*/,
                           fp8lm_meta* dst_meta /*device*/, const fp8lm_autoscale_cfg* cfg /*host*/, void* stream);

/*
 * Sec. 2.1 (text after Eq. 3): the auto-scaling factor mu follows the saturation statistic of the summed
 * gradient, and every rank applies it to its own gradient in the next step.  fp8lm_sum_fp8 leaves the state
 * (mu_exp, clean_steps) in the sum's metadata; this call copies those two fields of `from[t]` into
 * metas[r][t] for every rank, where the ranks' next fp8lm_amax_scale reads them.  Nothing else is touched.
 *   from  : device array [n_tensors] (read only);
 *   metas : host array of n_ranks device pointers, each to a meta array [n_tensors].  n_ranks <= 128.
 */
fp8lm_status fp8lm_autoscale_broadcast(fp8lm_ctx* ctx, const fp8lm_meta* from /*device*/,
                                       fp8lm_meta* const* metas /*host -> device*/, int32_t n_ranks, void* stream);
/*
 * Sec. 2.1, Eq. 1-2: the fixed factors the paper compares auto-scaling with -- pre-scaling (mu = 1/N, Eq. 1)
 * and post-scaling (mu = 1, Eq. 2).  Sets meta[t].mu_exp = mu_exp (-64..1) for every tensor; the following
 * fp8lm_amax_scale multiplies the scale with 2^mu_exp.  (A cast afterwards recomputes mu_exp from its own
 * statistic, so a fixed factor is set again before every step.)
 */
fp8lm_status fp8lm_set_mu(fp8lm_ctx* ctx, fp8lm_meta* meta /*device*/, int32_t mu_exp, void* stream);

/*
 * Master-weight initialisation (Sec. 2.2: FP16 master weights with tensor scaling).
 * For every tensor: scale = 2^(k - 1) with k the largest integer such that 2^k * max|w| <= 65504,
 * w_f16[i] = FP16(scale * w_bf16[i]) (round to nearest even, saturating).  A tensor of zeros (biases) or one
 * that holds inf/NaN gets scale 1 (FLAG_AMAX_ZERO / FLAG_NONFINITE).  Writes w_meta[t].{scale, inv_scale,
 * amax, amax_deq, flags, n_sat, n_underflow} whatever the buffer held before; the auto-scaling fields and the
 * amax history are not used by master weights and are left alone.
 */
fp8lm_status fp8lm_init_master(fp8lm_ctx* ctx, const void* w_bf16 /*device*/, uint16_t* w_f16 /*device*/,
                               fp8lm_meta* w_meta /*device*/, void* stream);
/* The same for any master-weight format: F16 / E4M3 with scale 2^(k - 1), k from their largest finite
 * value; BF16 / F32 with scale 1.  w_out holds 2, 2, 1 or 4 bytes per element.                        */
fp8lm_status fp8lm_init_master_as(fp8lm_ctx* ctx, const void* w_bf16 /*device*/, void* w_out /*device*/,
                                  fp8lm_meta* w_meta /*device*/, fp8lm_state_fmt master_fmt, void* stream);

/*
 * One FP8 AdamW step (Sec. 2.2, Eq. 8: FP8 gradient, FP8 first moment, FP16 second moment, scaled FP16
 * master weight; Sec. 3.1.2 for the optimizer).  With g, m, v, w the dequantised inputs, in fp32:
 *     m' = fma(beta1, m, (1-beta1) * g)          v' = fma(beta2, v, (1-beta2) * g*g)
 *     w' = fma(-lr, (m' / (1-beta1^step)) / (sqrt(v' / (1-beta2^step)) + eps), w * (1 - lr*weight_decay))
 * and m', v', w' are stored back in place with refreshed per-tensor scales:
 *     m : E4M3, scale chosen as hp->m_scale_mode says (default: exact amax of m', measured by an extra
 *         read-only pass over grad and m);
 *     v : FP16, scale from the bound fma(beta2, v_meta.amax_deq, (1-beta2) * grad_meta.amax_deq^2), which
 *         no v' exceeds (v_scaled = 0: scale 1);
 *     w : FP16, scale from w_meta.amax_deq before the step, minus one binade;
 *     wcopy : E4M3 with the scale from w_meta.amax_deq before the step (saturating), or bf16 (scale 1).
 * Each meta receives scale, inv_scale, amax, amax_deq and flags; n_sat / n_underflow are counted
 * when hp->stats is set.  grad_meta is read only; its amax_deq and flags must describe `grad` (as left by
 * fp8lm_cast_fp8).  The state buffers must hold what this library (or an equivalent encoder) wrote:
 * non-finite payloads in v or w are only handled when the corresponding meta carries FLAG_NONFINITE.
 * Buffers are either disjoint or, for one pair, the same: an E4M3 weight copy may be written over the FP8 gradient
 * (wcopy == grad, the same address).  The gradient is dead once the step has read it and the copy is only needed
 * after the step, so one buffer can serve both; every thread reads an element's gradient code before it stores that
 * element's copy.  The results are the same bytes as with two buffers, the step moves the same 12 bytes per element
 * in the same time, and the state is 1 byte per element smaller.  A bf16 copy cannot share the gradient's buffer
 * (INVALID_ARGUMENT); buffers that overlap in any other way give undefined results.
 * Errors: INVALID_ARGUMENT for hyper-parameters outside the ranges given at fp8lm_adam_hparams.
 */
fp8lm_status fp8lm_adam_step_fp8(fp8lm_ctx* ctx,
                                 const uint8_t* grad /*device*/, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta /*device*/,
                                 uint8_t* m /*device, in place*/, fp8lm_meta* m_meta /*device*/,
                                 void* v /*device, in place; element type per hp->v_fmt*/, fp8lm_meta* v_meta /*device*/,
                                 void* w /*device, in place; element type per hp->master_fmt*/, fp8lm_meta* w_meta /*device*/,
                                 void* wcopy /*device, write only*/, fp8lm_meta* wcopy_meta /*device*/,
                                 const fp8lm_adam_hparams* hp /*host*/, void* stream);

/*
 * fp8lm_adam_step_fp8 with m_scale_mode = EXACT_PASS, without its read-only first pass: the same results bit for bit
 * -- m_out holds what fp8lm_adam_step_fp8 would have left in m, every metadata field is equal -- for one extra
 * buffer.  The first moment is read from m_in and written to m_out (callers swap the two after every step; m_in is
 * left untouched).  Its scale is first taken as the one already in m_meta (what the previous step's exact amax gave);
 * the update pass measures the exact amax of the new moment anyway, and its epilogue computes the scale that amax
 * demands by the rule of the first pass.  Where it differs from the prediction -- the amax crossed a power-of-two
 * boundary, the first step -- the tensor's moment is computed once more from grad and m_in and stored with the right
 * scale; the second moment, the master weights and the weight copy never depend on that scale.  Per step this moves
 * 12 bytes per element plus 3 for the tensors that are repaired, instead of 14.
 * Restrictions: default storage formats, hp->stats = 0, hp->m_scale_mode = EXACT_PASS (INVALID_ARGUMENT otherwise);
 * m_in and m_out must not overlap over the tensors' extent (OVERLAP); wcopy must not be grad, which the repair
 * reads again (OVERLAP).
 * fp8lm_get_moment_speculation_stats: as fp8lm_get_speculation_stats, for this entry point.
 */
fp8lm_status fp8lm_adam_step_fp8_m2(fp8lm_ctx* ctx,
                                    const uint8_t* grad /*device*/, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta /*device*/,
                                    const uint8_t* m_in /*device, read only*/, uint8_t* m_out /*device, written*/,
                                    fp8lm_meta* m_meta /*device*/,
                                    void* v /*device, in place*/, fp8lm_meta* v_meta /*device*/,
                                    void* w /*device, in place*/, fp8lm_meta* w_meta /*device*/,
                                    void* wcopy /*device, write only*/, fp8lm_meta* wcopy_meta /*device*/,
                                    const fp8lm_adam_hparams* hp /*host*/, void* stream);
fp8lm_status fp8lm_get_moment_speculation_stats(fp8lm_ctx* ctx, uint64_t* calls /*host*/, uint64_t* tensors_redone /*host*/,
                                                uint64_t* elems_redone /*host*/, void* stream);

/*
 * fp8lm_adam_step_fp8 for callers that cannot allocate device memory and therefore cannot hold a context:
 * code under HIP graph capture that must not call hipMalloc, tight serving or training loops, harnesses that
 * forbid allocation.  Same arithmetic, same kernels, same results, bit for bit; what a context keeps in
 * hipMalloc'd memory (tensor and chunk tables, the per-tensor scales that the first pass hands to the second,
 * the per-workgroup reduction records) lives in a fixed array inside the library's device image instead (about
 * 5.4 MiB, held by every GPU the library runs on until the process ends).  Every call rebuilds the tables in
 * that array from `tensors` with small kernels on `stream` (arguments travel as kernel arguments: no copy from
 * host memory), then runs the two passes.  The call itself calls no allocator of any kind.
 *   device       : GPU that owns all buffers; tensors, tensor_flags: host arrays of n entries, read during the
 *                  call (tensor_flags may be NULL: all 0; same meaning as fp8lm_set_tensor_flags).
 *   Limits       : n <= FP8LM_STATIC_MAX_TENSORS and at most FP8LM_STATIC_MAX_CHUNKS chunks of 16384 elements
 *                  (a tensor of k elements takes ceil(k / 16384) of them; about 1.7e10 elements in all):
 *                  FP8LM_ERR_TOO_LARGE beyond either, nothing enqueued.
 *   Not offered  : hp->m_scale_mode = FP8LM_MSCALE_FROM_CAST (needs the context of the fused cast):
 *                  INVALID_ARGUMENT.
 *   Concurrency  : all calls on one GPU share the one array and each leaves its tables and scales in it.  Calls
 *                  on the same stream are ordered and safe; calls that overlap on one GPU (two streams, two
 *                  threads) race and give wrong results.  Nothing in the array has to start at zero: a call
 *                  overwrites every entry before it reads it.
 * Errors otherwise as fp8lm_create (tensor list) and fp8lm_adam_step_fp8 (everything else).
 */
#define FP8LM_STATIC_MAX_TENSORS 4096
#define FP8LM_STATIC_MAX_CHUNKS (1 << 20)
fp8lm_status fp8lm_adam_step_fp8_static(int device, const fp8lm_tensor* tensors /*host*/, int32_t n,
                                        const uint32_t* tensor_flags /*host[n] or NULL*/,
                                        const uint8_t* grad /*device*/, fp8lm_fmt grad_fmt, const fp8lm_meta* grad_meta /*device*/,
                                        uint8_t* m /*device, in place*/, fp8lm_meta* m_meta /*device*/,
                                        void* v /*device, in place*/, fp8lm_meta* v_meta /*device*/,
                                        void* w /*device, in place*/, fp8lm_meta* w_meta /*device*/,
                                        void* wcopy /*device, write only*/, fp8lm_meta* wcopy_meta /*device*/,
                                        const fp8lm_adam_hparams* hp /*host*/, void* stream);

/*
 * Quantisation error of an FP8 gradient against a high-precision reference: the three quantities of
 * the communication ablation (Sec. 3.3, figure comparing pre-, post- and auto-scaling for the FP8
 * gradient all-reduce).  With r the reference and x = payload / scale the value a scaling tensor
 * stands for (Sec. 2.1), per tensor:
 *   signal = sum r^2, noise = sum (r - x)^2 (float64; SNR = 10 log10(signal / noise) is left to the
 *   caller), n_nonzero = #{r != 0}, n_underflow = #{r != 0, payload = +-0}, n_overflow = #{|payload|
 *   is the largest finite code}.  Elements whose reference is inf/NaN or whose payload is a NaN/inf
 *   code are counted in n_nonfinite and in nothing else.
 * The sums are accumulated in an order that depends only on the launch shape (they agree with a
 * sequential sum to about numel * 2^-52 relative and are reproducible from call to call); the counts
 * are exact.
 *   ref  : device, flat buffer of element type ref_type (read only);
 *   q    : device, flat uint8 payloads of format fmt;  q_meta : device [n_tensors], only scale is read;
 *   out  : device [n_tensors], overwritten (entries of empty tensors are zeroed).
 */
typedef struct {
  double signal, noise;
  uint64_t n_nonzero, n_underflow, n_overflow, n_nonfinite;
} fp8lm_quant_stats;
fp8lm_status fp8lm_quant_error_stats(fp8lm_ctx* ctx, const void* ref /*device*/, fp8lm_src ref_type,
                                     const uint8_t* q /*device*/, fp8lm_fmt fmt, const fp8lm_meta* q_meta /*device*/,
                                     fp8lm_quant_stats* out /*device*/, void* stream);

/*
 * Host-only helper: the whole-tensor greedy distribution of Sec. 2.3, Alg. 1 (how this path would be
 * sharded over GPUs: a tensor and its scale always stay together).  Tensors are taken in descending
 * order of sizes[i] (equal sizes in index order); each goes to the GPU with the least memory in use
 * (the lowest-numbered among equals).
 *   sizes : host[n], >= 0.   owner : host[n], written: GPU of tensor i.   usage : host[n_gpus], written.
 */
fp8lm_status fp8lm_greedy_partition(const int64_t* sizes /*host*/, int32_t n, int32_t n_gpus,
                                    int32_t* owner /*host*/, int64_t* usage /*host*/);

/* A plain 128-bit copy kernel over `bytes` bytes (multiple of 16): the measured bandwidth ceiling
 * the streaming kernels are compared with.                                                        */
fp8lm_status fp8lm_copy_bytes(fp8lm_ctx* ctx, const void* src /*device*/, void* dst /*device*/, int64_t bytes,
                              void* stream);

/*
 * Memory-only skeletons of the hot kernels, for measurement: the same grid, tile walk, access widths, access
 * layout and cache policies as the kernel named, with the arithmetic replaced by XORs, so that what they reach
 * is the bandwidth ceiling of that access pattern on this machine.  They move exactly the algorithmic bytes of
 * the kernel they stand for.  Buffers written are overwritten with meaningless data.
 *   READ16   bufs = {src16}                     reads 2 B/element     (fp8lm_amax_scale on a bf16 gradient)
 *   READ8X2  bufs = {a8, b8}                    reads 1 + 1           (first pass of fp8lm_adam_step_fp8)
 *   WRITE16  bufs = {dst16}                     writes 2
 *   WRITE8   bufs = {dst8}                      writes 1
 *   CAST     bufs = {src16, dst8}               reads 2, writes 1     (fp8lm_cast_fp8 from a 16-bit source)
 *   UPDATE   bufs = {g8, m8, v16, w16, q8}      reads g, m, v, w (6), writes m, v, w in place and q (6)
 *                                               (second pass of fp8lm_adam_step_fp8, default formats)
 *   UPDATE_READS / UPDATE_WRITES  same bufs as UPDATE: only its four read streams (6 B/element), only its four
 *                                               write streams (6): what the two directions reach when they do not
 *                                               share the memory with each other
 *   bufs : host array of device pointers, each covering n_elems elements; n_elems a multiple of 4096.
 */
typedef enum { FP8LM_SKEL_READ16 = 0, FP8LM_SKEL_READ8X2 = 1, FP8LM_SKEL_WRITE16 = 2, FP8LM_SKEL_WRITE8 = 3,
               FP8LM_SKEL_CAST = 4, FP8LM_SKEL_UPDATE = 5, FP8LM_SKEL_UPDATE_READS = 6,
               FP8LM_SKEL_UPDATE_WRITES = 7 } fp8lm_skeleton;
fp8lm_status fp8lm_memory_skeleton(fp8lm_ctx* ctx, int32_t shape, void* const* bufs /*host -> device*/,
                                   int64_t n_elems, void* stream);

/*
 * Device memory whose pieces are chosen one by one: thin wrappers of the HIP virtual-memory calls, for callers that
 * lay their flat buffers out over the regions of HBM.  On MI355X a kernel that writes (the update pass, the cast)
 * runs up to 20 % slower while everything it writes lies in one 96 GiB region of the physical address space; a buffer
 * whose address range alternates between pieces from two regions does not have that problem wherever a kernel is in
 * it.  Where a piece lies can only be measured (fp8lm_memory_skeleton across two pieces is faster than inside one
 * region), so the steps are separate: create pieces, map each somewhere, time it against a reference piece, then map
 * the pieces wanted into one reserved range in alternating order and destroy the others.  None of these calls is on
 * the path of a training step; they allocate, and fp8lm_vmm_unmap waits for the device.
 *   fp8lm_vmm_granularity : *bytes = what piece sizes and offsets must be multiples of
 *   fp8lm_vmm_reserve     : reserves an address range of `bytes`; nothing is behind it yet
 *   fp8lm_vmm_create      : physical memory of `bytes` on `device`; *piece is an opaque handle
 *   fp8lm_vmm_map         : puts `piece` behind [va, va + bytes) of a reserved range, readable and writable by `device`
 *   fp8lm_vmm_unmap       : waits for the device, then takes the mapping away (the piece stays)
 *   fp8lm_vmm_destroy     : gives the piece's memory back once it is mapped nowhere
 *   fp8lm_vmm_free        : gives a reserved range back (nothing may be mapped in it)
 * Errors: INVALID_ARGUMENT for null pointers, zero sizes or sizes that are not multiples of the granularity; HIP
 * for whatever the runtime refuses (fp8lm_last_hip_error has the text).
 */
fp8lm_status fp8lm_vmm_granularity(int device, uint64_t* bytes /*host*/);
fp8lm_status fp8lm_vmm_reserve(uint64_t bytes, void** va /*host; receives a device address*/);
fp8lm_status fp8lm_vmm_free(void* va, uint64_t bytes);
fp8lm_status fp8lm_vmm_create(int device, uint64_t bytes, uint64_t* piece /*host*/);
fp8lm_status fp8lm_vmm_destroy(uint64_t piece);
fp8lm_status fp8lm_vmm_map(void* va, uint64_t bytes, uint64_t piece, int device);
fp8lm_status fp8lm_vmm_unmap(void* va, uint64_t bytes);

/* Times the most recent launch of each kernel with HIP events recorded on the launch stream.
 * fp8lm_set_timing(ctx, 1) starts recording event pairs around every kernel launch;
 * fp8lm_get_timing synchronises and returns, per kernel id, the number of launches and the summed
 * duration in milliseconds since timing was enabled, then resets the sums.                       */
enum { FP8LM_K_AMAX = 0, FP8LM_K_CAST = 1, FP8LM_K_ADAM_AMAX = 2, FP8LM_K_ADAM_UPDATE = 3,
       FP8LM_K_INIT_MASTER = 4, FP8LM_K_COPY = 5, FP8LM_K_SCALARS = 6 /* per-tensor scalar kernels */,
       FP8LM_K_REQUANT = 7, FP8LM_K_SUM = 8, FP8LM_K_STATS = 9, FP8LM_K_SKELETON = 10, FP8LM_K_COUNT = 11 };
fp8lm_status fp8lm_set_timing(fp8lm_ctx* ctx, int32_t enable);
fp8lm_status fp8lm_get_timing(fp8lm_ctx* ctx, int32_t* launches /*host[FP8LM_K_COUNT]*/,
                              double* total_ms /*host[FP8LM_K_COUNT]*/);

const char* fp8lm_status_string(fp8lm_status s);
/* Text of the last HIP error seen by this thread's calls ("" if none).                            */
const char* fp8lm_last_hip_error(void);
/* Size of fp8lm_meta as compiled into the library (layout check for bindings).                    */
uint32_t fp8lm_sizeof_meta(void);

#ifdef __cplusplus
}
#endif
#endif /* FP8LM_H */
