"""Thin ctypes binding of libfp8lm.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in include/fp8lm.h; this
module turns torch tensors into raw device pointers and the current torch stream into a HIP stream
handle.  There is no CPU fallback: if the library is missing or fails to load, importing the
functions raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Sequence, Tuple

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libfp8lm.so")

HIST = 16
E4M3, E5M2 = 0, 1
SRC_BF16, SRC_F16, SRC_F32 = 0, 1, 2
WCOPY_E4M3, WCOPY_BF16 = 0, 1
MSCALE_EXACT_PASS, MSCALE_PREDICTED, MSCALE_FROM_CAST = 0, 1, 2
TENSOR_NO_WEIGHT_DECAY = 1
MU_SET_HALF, MU_HALVE = 0, 1
STATE_F16, STATE_BF16, STATE_E4M3, STATE_F32 = 0, 1, 2, 3
STATE_BYTES = {STATE_F16: 2, STATE_BF16: 2, STATE_E4M3: 1, STATE_F32: 4}
FLAG_NONFINITE, FLAG_AMAX_ZERO, FLAG_SCALE_CLAMPED, FLAG_SATURATED = 1, 2, 4, 8
SKEL_READ16, SKEL_READ8X2, SKEL_WRITE16, SKEL_WRITE8, SKEL_CAST, SKEL_UPDATE, SKEL_UPDATE_READS, SKEL_UPDATE_WRITES = range(8)
SKEL_BYTES_PER_ELEM = {SKEL_READ16: 2, SKEL_READ8X2: 2, SKEL_WRITE16: 2, SKEL_WRITE8: 1, SKEL_CAST: 3, SKEL_UPDATE: 12,
                       SKEL_UPDATE_READS: 6, SKEL_UPDATE_WRITES: 6}
K_AMAX, K_CAST, K_ADAM_AMAX, K_ADAM_UPDATE, K_INIT_MASTER, K_COPY, K_SCALARS, K_REQUANT, K_SUM, K_STATS, K_SKELETON, K_COUNT = range(12)
KERNEL_NAMES = ["amax", "cast", "adam_amax", "adam_update", "init_master", "copy", "scalars", "requantize", "sum", "quant_stats", "skeleton"]

EXPORTS = [
    "fp8lm_create", "fp8lm_destroy", "fp8lm_set_tuning", "fp8lm_set_tensor_flags", "fp8lm_meta_init", "fp8lm_amax_scale",
    "fp8lm_cast_fp8", "fp8lm_cast_fp8_delayed", "fp8lm_cast_fp8_for_adam", "fp8lm_shared_scale", "fp8lm_requantize_fp8", "fp8lm_sum_fp8",
    "fp8lm_quant_error_stats", "fp8lm_autoscale_broadcast", "fp8lm_set_mu", "fp8lm_memory_skeleton", "fp8lm_adam_step_fp8_static",
    "fp8lm_quantize_fp8", "fp8lm_quantize_fp8_for_adam", "fp8lm_get_speculation_stats", "fp8lm_adam_step_fp8_m2",
    "fp8lm_get_moment_speculation_stats", "fp8lm_vmm_granularity", "fp8lm_vmm_reserve", "fp8lm_vmm_free", "fp8lm_vmm_create",
    "fp8lm_vmm_destroy", "fp8lm_vmm_map", "fp8lm_vmm_unmap",
    "fp8lm_init_master", "fp8lm_init_master_as", "fp8lm_greedy_partition", "fp8lm_adam_step_fp8", "fp8lm_copy_bytes", "fp8lm_set_timing",
    "fp8lm_get_timing", "fp8lm_status_string", "fp8lm_last_hip_error", "fp8lm_sizeof_meta",
]


QUANT_STATS_DTYPE = np.dtype([("signal", "<f8"), ("noise", "<f8"), ("n_nonzero", "<u8"), ("n_underflow", "<u8"),
                              ("n_overflow", "<u8"), ("n_nonfinite", "<u8")])


class Tensor(C.Structure):
    _fields_ = [("offset", C.c_int64), ("numel", C.c_int64)]


class Meta(C.Structure):
    _fields_ = [
        ("scale", C.c_float), ("inv_scale", C.c_float), ("amax", C.c_float), ("amax_deq", C.c_float),
        ("amax_hist", C.c_float * HIST), ("hist_pos", C.c_int32), ("mu_exp", C.c_int32),
        ("clean_steps", C.c_int32), ("flags", C.c_uint32), ("n_sat", C.c_uint64),
        ("n_underflow", C.c_uint64),
    ]


META_DTYPE = np.dtype([
    ("scale", "<f4"), ("inv_scale", "<f4"), ("amax", "<f4"), ("amax_deq", "<f4"),
    ("amax_hist", "<f4", (HIST,)), ("hist_pos", "<i4"), ("mu_exp", "<i4"), ("clean_steps", "<i4"),
    ("flags", "<u4"), ("n_sat", "<u8"), ("n_underflow", "<u8"),
])


class AutoscaleCfg(C.Structure):
    _fields_ = [("sat_num", C.c_int32), ("sat_den", C.c_int32), ("ramp_steps", C.c_int32),
                ("hist_window", C.c_int32), ("margin", C.c_int32), ("mu_rule", C.c_int32), ("mu_min_exp", C.c_int32)]


class AdamHparams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("step", C.c_int64), ("v_scaled", C.c_int32),
                ("wcopy", C.c_int32), ("stats", C.c_int32), ("m_scale_mode", C.c_int32), ("master_fmt", C.c_int32),
                ("v_fmt", C.c_int32), ("exact", C.c_int32)]


def autoscale_cfg(ramp_steps=1000, hist_window=1, margin=0, sat_num=1, sat_den=100000, mu_rule=0,
                  mu_min_exp=-1) -> AutoscaleCfg:
    """mu_rule: MU_SET_HALF (the reading taken by default) or MU_HALVE (halve on every overflowing step down to
    2^mu_min_exp, double after ramp_steps / 2 clean ones)."""
    return AutoscaleCfg(sat_num, sat_den, ramp_steps, hist_window, margin, mu_rule, mu_min_exp)


def adam_hparams(lr, step, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, v_scaled=1,
                 wcopy=WCOPY_E4M3, stats=0, exact=1, m_scale_mode=MSCALE_EXACT_PASS, master_fmt=STATE_F16,
                 v_fmt=STATE_F16) -> AdamHparams:
    return AdamHparams(lr, beta1, beta2, eps, weight_decay, step, v_scaled, wcopy, stats, m_scale_mode, master_fmt,
                       v_fmt, exact)


class Fp8lmError(RuntimeError):
    def __init__(self, status: int, where: str):
        L = lib()
        msg = L.fp8lm_status_string(status).decode()
        hip = L.fp8lm_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({status})" + (f" [{hip}]" if hip and status == -4 else ""))
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Loads libfp8lm.so (built in-tree by paper_2310_18313_amd.build); raises if it is absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2310_18313_amd.build` "
                              "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.fp8lm_create.argtypes = [C.POINTER(vp), vp, i32, C.c_int]
        L.fp8lm_destroy.argtypes = [vp]
        L.fp8lm_set_tuning.argtypes = [vp, i32, i32, i32]
        L.fp8lm_set_tensor_flags.argtypes = [vp, vp, i32]
        L.fp8lm_meta_init.argtypes = [vp, vp, vp, vp]
        L.fp8lm_amax_scale.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp, vp]
        L.fp8lm_cast_fp8.argtypes = [vp, vp, C.c_int, vp, C.c_int, vp, vp, vp]
        L.fp8lm_cast_fp8_delayed.argtypes = [vp, vp, C.c_int, vp, C.c_int, vp, vp, vp]
        L.fp8lm_cast_fp8_for_adam.argtypes = [vp, vp, C.c_int, vp, C.c_int, vp, vp, i32, vp, vp, C.c_float, vp]
        L.fp8lm_quantize_fp8.argtypes = [vp, vp, C.c_int, vp, C.c_int, vp, vp, vp]
        L.fp8lm_quantize_fp8_for_adam.argtypes = [vp, vp, C.c_int, vp, C.c_int, vp, vp, vp, vp, C.c_float, vp]
        L.fp8lm_get_speculation_stats.argtypes = [vp, vp, vp, vp, vp]
        L.fp8lm_get_moment_speculation_stats.argtypes = [vp, vp, vp, vp, vp]
        L.fp8lm_adam_step_fp8_m2.argtypes = [vp, vp, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fp8lm_init_master.argtypes = [vp, vp, vp, vp, vp]
        L.fp8lm_init_master_as.argtypes = [vp, vp, vp, vp, C.c_int, vp]
        L.fp8lm_shared_scale.argtypes = [vp, vp, i32, vp, vp]
        L.fp8lm_requantize_fp8.argtypes = [vp, vp, C.c_int, vp, vp, vp, vp, vp]
        L.fp8lm_sum_fp8.argtypes = [vp, vp, i32, C.c_int, vp, vp, vp, vp, vp]
        L.fp8lm_quant_error_stats.argtypes = [vp, vp, C.c_int, vp, C.c_int, vp, vp, vp]
        L.fp8lm_autoscale_broadcast.argtypes = [vp, vp, vp, i32, vp]
        L.fp8lm_set_mu.argtypes = [vp, vp, i32, vp]
        L.fp8lm_memory_skeleton.argtypes = [vp, i32, vp, i64, vp]
        L.fp8lm_adam_step_fp8.argtypes = [vp, vp, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fp8lm_adam_step_fp8_static.argtypes = [C.c_int, vp, i32, vp, vp, C.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fp8lm_copy_bytes.argtypes = [vp, vp, vp, i64, vp]
        u64 = C.c_uint64
        L.fp8lm_vmm_granularity.argtypes = [C.c_int, vp]
        L.fp8lm_vmm_reserve.argtypes = [u64, vp]
        L.fp8lm_vmm_free.argtypes = [vp, u64]
        L.fp8lm_vmm_create.argtypes = [C.c_int, u64, vp]
        L.fp8lm_vmm_destroy.argtypes = [u64]
        L.fp8lm_vmm_map.argtypes = [vp, u64, u64, C.c_int]
        L.fp8lm_vmm_unmap.argtypes = [vp, u64]
        L.fp8lm_greedy_partition.argtypes = [vp, i32, i32, vp, vp]
        L.fp8lm_set_timing.argtypes = [vp, i32]
        L.fp8lm_get_timing.argtypes = [vp, vp, vp]
        for name in EXPORTS:
            getattr(L, name).restype = C.c_int
        L.fp8lm_status_string.restype = C.c_char_p
        L.fp8lm_status_string.argtypes = [C.c_int]
        L.fp8lm_last_hip_error.restype = C.c_char_p
        L.fp8lm_last_hip_error.argtypes = []
        L.fp8lm_sizeof_meta.restype = C.c_uint32
        L.fp8lm_sizeof_meta.argtypes = []
        if L.fp8lm_sizeof_meta() != C.sizeof(Meta) or C.sizeof(Meta) != META_DTYPE.itemsize:
            raise ImportError("fp8lm_meta layout mismatch between the library and the binding")
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != 0:
        raise Fp8lmError(status, where)


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t) -> int:
    if t is None:
        return 0
    assert t.is_cuda and t.is_contiguous()
    return t.data_ptr()


def src_type_of(t: torch.Tensor) -> int:
    """The library's source type for a gradient tensor; 16-bit integer tensors count as bf16 bit patterns."""
    kinds = {torch.bfloat16: SRC_BF16, torch.int16: SRC_BF16, torch.uint16: SRC_BF16, torch.float16: SRC_F16,
             torch.float32: SRC_F32}
    if t.dtype not in kinds:
        raise TypeError(f"no FP8 cast from {t.dtype}: the gradient must be bf16, fp16 or fp32")
    return kinds[t.dtype]


class Context:
    """Owns one fp8lm_ctx: a fixed list of (offset, numel) tensors inside flat device buffers."""

    def __init__(self, tensors: Sequence[Tuple[int, int]], device: int = 0):
        self.n_tensors = len(tensors)
        arr = (Tensor * max(1, self.n_tensors))()
        for i, (off, n) in enumerate(tensors):
            arr[i].offset, arr[i].numel = int(off), int(n)
        h = C.c_void_p()
        _check(lib().fp8lm_create(C.byref(h), C.cast(arr, C.c_void_p), self.n_tensors, device), "fp8lm_create")
        self._h = h
        self.device = device
        # the C ABI takes bare pointers: the extent every flat buffer must cover is checked here
        self.required_elems = max([int(o) + int(n) for o, n in tensors if n > 0], default=0)

    def _fits(self, *bufs):
        for t in bufs:
            if t.numel() < self.required_elems:
                raise ValueError(f"flat buffer of {t.numel()} elements is shorter than the tensor list needs "
                                 f"({self.required_elems})")
            if t.device.index != self.device:
                raise ValueError("buffer is on another device than the context")

    def _fits_meta(self, *metas):
        for t in metas:
            if t.numel() * t.element_size() < self.n_tensors * C.sizeof(Meta):
                raise ValueError("meta array is shorter than the tensor list")

    def close(self):
        if getattr(self, "_h", None):
            lib().fp8lm_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:  # interpreter shutdown
            pass

    def set_tuning(self, chunk_elems=16384, blocks_per_cu=16, single_pass_min_chunks=1 << 30):
        _check(lib().fp8lm_set_tuning(self._h, chunk_elems, blocks_per_cu, single_pass_min_chunks), "fp8lm_set_tuning")

    def set_tensor_flags(self, flags) -> None:
        """One combination of TENSOR_* bits per tensor of the context (TENSOR_NO_WEIGHT_DECAY: the Adam step treats
        the tensor as if weight_decay were 0)."""
        arr = np.ascontiguousarray(flags, dtype=np.uint32)
        _check(lib().fp8lm_set_tensor_flags(self._h, arr.ctypes.data, len(arr)), "fp8lm_set_tensor_flags")

    def new_meta(self, cfg: AutoscaleCfg, stream=None) -> torch.Tensor:
        """Device array of fp8lm_meta (as raw bytes, [n_tensors, 112]) in its initial state."""
        meta = torch.empty((max(1, self.n_tensors), C.sizeof(Meta)), dtype=torch.uint8, device=f"cuda:{self.device}")
        _check(lib().fp8lm_meta_init(self._h, _ptr(meta), C.addressof(cfg), _stream(stream)), "fp8lm_meta_init")
        return meta

    def amax_scale(self, src, target_fmt, meta, cfg, stream=None):
        self._fits(src)
        self._fits_meta(meta)
        _check(lib().fp8lm_amax_scale(self._h, _ptr(src), src_type_of(src), target_fmt, _ptr(meta), C.addressof(cfg),
                                      _stream(stream)), "fp8lm_amax_scale")

    def cast_fp8(self, src, dst, fmt, meta, cfg, stream=None):
        assert dst.element_size() == 1
        self._fits(src, dst)
        self._fits_meta(meta)
        _check(lib().fp8lm_cast_fp8(self._h, _ptr(src), src_type_of(src), _ptr(dst), fmt, _ptr(meta), C.addressof(cfg),
                                    _stream(stream)), "fp8lm_cast_fp8")

    def cast_fp8_delayed(self, src, dst, fmt, meta, cfg, stream=None):
        assert dst.element_size() == 1
        self._fits(src, dst)
        self._fits_meta(meta)
        _check(lib().fp8lm_cast_fp8_delayed(self._h, _ptr(src), src_type_of(src), _ptr(dst), fmt, _ptr(meta),
                                            C.addressof(cfg), _stream(stream)), "fp8lm_cast_fp8_delayed")

    def cast_fp8_for_adam(self, src, dst, fmt, meta, cfg, m, m_meta, beta1, delayed=False, stream=None):
        assert dst.element_size() == 1 and m.element_size() == 1
        self._fits(src, dst, m)
        self._fits_meta(meta, m_meta)
        _check(lib().fp8lm_cast_fp8_for_adam(self._h, _ptr(src), src_type_of(src), _ptr(dst), fmt, _ptr(meta), C.addressof(cfg),
                                             1 if delayed else 0, _ptr(m), _ptr(m_meta), beta1, _stream(stream)),
               "fp8lm_cast_fp8_for_adam")

    def quantize_fp8(self, src, dst, fmt, meta, cfg, stream=None):
        """amax + scale + cast with the results of amax_scale followed by cast_fp8, reading unchanged-scale tensors once."""
        assert dst.element_size() == 1
        self._fits(src, dst)
        self._fits_meta(meta)
        _check(lib().fp8lm_quantize_fp8(self._h, _ptr(src), src_type_of(src), _ptr(dst), fmt, _ptr(meta), C.addressof(cfg),
                                        _stream(stream)), "fp8lm_quantize_fp8")

    def quantize_fp8_for_adam(self, src, dst, fmt, meta, cfg, m, m_meta, beta1, stream=None):
        assert dst.element_size() == 1 and m.element_size() == 1
        self._fits(src, dst, m)
        self._fits_meta(meta, m_meta)
        _check(lib().fp8lm_quantize_fp8_for_adam(self._h, _ptr(src), src_type_of(src), _ptr(dst), fmt, _ptr(meta),
                                                 C.addressof(cfg), _ptr(m), _ptr(m_meta), beta1, _stream(stream)),
               "fp8lm_quantize_fp8_for_adam")

    def speculation_stats(self, stream=None, moment: bool = False) -> dict:
        """Running totals of quantize_fp8 / quantize_fp8_for_adam on this context, or with `moment` of
        adam_step_fp8_m2 (synchronises the stream)."""
        vals = (C.c_uint64 * 3)()
        fn = lib().fp8lm_get_moment_speculation_stats if moment else lib().fp8lm_get_speculation_stats
        _check(fn(self._h, C.addressof(vals), C.addressof(vals) + 8, C.addressof(vals) + 16, _stream(stream)),
               "fp8lm_get_speculation_stats")
        return {"calls": int(vals[0]), "tensors_redone": int(vals[1]), "elems_redone": int(vals[2])}

    def adam_step_fp8_m2(self, grad, grad_fmt, grad_meta, m_in, m_out, m_meta, v, v_meta, w, w_meta, wcopy, wcopy_meta,
                         hp: AdamHparams, stream=None):
        """adam_step_fp8 (exact first-moment scale) without its first pass: m is read from m_in and written to m_out."""
        assert grad.element_size() == 1 and m_in.element_size() == 1 and m_out.element_size() == 1
        assert v.element_size() == 2 and w.element_size() == 2
        assert wcopy.element_size() == (1 if hp.wcopy == WCOPY_E4M3 else 2)
        self._fits(grad, m_in, m_out, v, w, wcopy)
        self._fits_meta(grad_meta, m_meta, v_meta, w_meta, wcopy_meta)
        _check(lib().fp8lm_adam_step_fp8_m2(self._h, _ptr(grad), grad_fmt, _ptr(grad_meta), _ptr(m_in), _ptr(m_out),
                                            _ptr(m_meta), _ptr(v), _ptr(v_meta), _ptr(w), _ptr(w_meta), _ptr(wcopy),
                                            _ptr(wcopy_meta), C.addressof(hp), _stream(stream)), "fp8lm_adam_step_fp8_m2")

    def shared_scale(self, metas, stream=None) -> torch.Tensor:
        """Eq. 4: per-tensor minimum of the ranks' scales; returns a device fp32 array [n_tensors]."""
        self._fits_meta(*metas)
        out = torch.empty(max(1, self.n_tensors), dtype=torch.float32, device=f"cuda:{self.device}")
        ptrs = (C.c_void_p * len(metas))(*[_ptr(m) for m in metas])
        _check(lib().fp8lm_shared_scale(self._h, C.cast(ptrs, C.c_void_p), len(metas), _ptr(out), _stream(stream)),
               "fp8lm_shared_scale")
        return out

    def requantize_fp8(self, src, fmt, src_meta, shared, dst, dst_meta, stream=None):
        assert src.element_size() == 1 and dst.element_size() == 1 and shared.dtype == torch.float32
        self._fits(src, dst)
        self._fits_meta(src_meta, dst_meta)
        assert shared.numel() >= self.n_tensors
        _check(lib().fp8lm_requantize_fp8(self._h, _ptr(src), fmt, _ptr(src_meta), _ptr(shared), _ptr(dst),
                                          _ptr(dst_meta), _stream(stream)), "fp8lm_requantize_fp8")

    def sum_fp8(self, payloads, fmt, shared, dst, dst_meta, cfg, stream=None):
        assert all(p.element_size() == 1 for p in payloads) and dst.element_size() == 1
        self._fits(dst, *payloads)
        self._fits_meta(dst_meta)
        assert shared.dtype == torch.float32 and shared.numel() >= self.n_tensors
        ptrs = (C.c_void_p * len(payloads))(*[_ptr(p) for p in payloads])
        _check(lib().fp8lm_sum_fp8(self._h, C.cast(ptrs, C.c_void_p), len(payloads), fmt, _ptr(shared), _ptr(dst),
                                   _ptr(dst_meta), C.addressof(cfg), _stream(stream)), "fp8lm_sum_fp8")

    def autoscale_broadcast(self, from_meta, metas, stream=None):
        """Copies the auto-scaling state (mu_exp, clean_steps) of `from_meta` into every meta array of `metas`."""
        self._fits_meta(from_meta, *metas)
        ptrs = (C.c_void_p * len(metas))(*[_ptr(m) for m in metas])
        _check(lib().fp8lm_autoscale_broadcast(self._h, _ptr(from_meta), C.cast(ptrs, C.c_void_p), len(metas),
                                               _stream(stream)), "fp8lm_autoscale_broadcast")

    def set_mu(self, meta, mu_exp: int, stream=None):
        """Fixed auto-scaling factor 2^mu_exp for the next scale computation of every tensor."""
        self._fits_meta(meta)
        _check(lib().fp8lm_set_mu(self._h, _ptr(meta), mu_exp, _stream(stream)), "fp8lm_set_mu")

    def quant_error_stats(self, ref, q, fmt, q_meta, stream=None) -> np.ndarray:
        """Per-tensor signal and noise energies and underflow / overflow counts of the FP8 tensor `q` against the
        high-precision reference `ref` (Sec. 3.3, communication ablation).  Synchronises and returns a host array
        of QUANT_STATS_DTYPE (the signal-to-noise ratio is signal / noise)."""
        assert q.element_size() == 1
        self._fits(ref, q)
        self._fits_meta(q_meta)
        out = torch.empty((max(1, self.n_tensors), QUANT_STATS_DTYPE.itemsize), dtype=torch.uint8,
                          device=f"cuda:{self.device}")
        _check(lib().fp8lm_quant_error_stats(self._h, _ptr(ref), src_type_of(ref), _ptr(q), fmt, _ptr(q_meta), _ptr(out),
                                             _stream(stream)), "fp8lm_quant_error_stats")
        return out.cpu().numpy().view(QUANT_STATS_DTYPE).reshape(-1)[:self.n_tensors].copy()

    def init_master(self, w_bf16, w_out, w_meta, master_fmt=STATE_F16, stream=None):
        assert w_bf16.element_size() == 2 and w_out.element_size() == STATE_BYTES[master_fmt]
        self._fits(w_bf16, w_out)
        self._fits_meta(w_meta)
        _check(lib().fp8lm_init_master_as(self._h, _ptr(w_bf16), _ptr(w_out), _ptr(w_meta), master_fmt,
                                          _stream(stream)), "fp8lm_init_master_as")

    def adam_step_fp8(self, grad, grad_fmt, grad_meta, m, m_meta, v, v_meta, w, w_meta, wcopy, wcopy_meta,
                      hp: AdamHparams, stream=None):
        assert grad.element_size() == 1 and m.element_size() == 1
        assert v.element_size() == STATE_BYTES[hp.v_fmt] and w.element_size() == STATE_BYTES[hp.master_fmt]
        assert wcopy.element_size() == (1 if hp.wcopy == WCOPY_E4M3 else 2)
        self._fits(grad, m, v, w, wcopy)
        self._fits_meta(grad_meta, m_meta, v_meta, w_meta, wcopy_meta)
        _check(lib().fp8lm_adam_step_fp8(self._h, _ptr(grad), grad_fmt, _ptr(grad_meta), _ptr(m), _ptr(m_meta),
                                         _ptr(v), _ptr(v_meta), _ptr(w), _ptr(w_meta), _ptr(wcopy),
                                         _ptr(wcopy_meta), C.addressof(hp), _stream(stream)), "fp8lm_adam_step_fp8")

    def copy_bytes(self, src, dst, nbytes, stream=None):
        assert src.numel() * src.element_size() >= nbytes and dst.numel() * dst.element_size() >= nbytes
        _check(lib().fp8lm_copy_bytes(self._h, _ptr(src), _ptr(dst), nbytes, _stream(stream)), "fp8lm_copy_bytes")

    def memory_skeleton(self, shape: int, bufs, n_elems: int, stream=None):
        """Memory-only stand-in of one hot kernel over the first n_elems elements of `bufs` (see fp8lm.h); buffers
        that the shape writes are overwritten with meaningless data."""
        sizes = {SKEL_READ16: (2,), SKEL_READ8X2: (1, 1), SKEL_WRITE16: (2,), SKEL_WRITE8: (1,), SKEL_CAST: (2, 1),
                 SKEL_UPDATE: (1, 1, 2, 2, 1), SKEL_UPDATE_READS: (1, 1, 2, 2, 1), SKEL_UPDATE_WRITES: (1, 1, 2, 2, 1)}[shape]
        assert len(bufs) == len(sizes)
        for t, sz in zip(bufs, sizes):
            assert t.element_size() == sz and t.numel() >= n_elems
        ptrs = (C.c_void_p * len(bufs))(*[_ptr(t) for t in bufs])
        _check(lib().fp8lm_memory_skeleton(self._h, shape, C.cast(ptrs, C.c_void_p), n_elems, _stream(stream)),
               "fp8lm_memory_skeleton")

    def set_timing(self, enable: bool):
        _check(lib().fp8lm_set_timing(self._h, 1 if enable else 0), "fp8lm_set_timing")

    def get_timing(self):
        """{kernel name: (launches, total ms)} since timing was enabled or last read (synchronises)."""
        n = (C.c_int32 * K_COUNT)()
        ms = (C.c_double * K_COUNT)()
        _check(lib().fp8lm_get_timing(self._h, C.cast(n, C.c_void_p), C.cast(ms, C.c_void_p)), "fp8lm_get_timing")
        return {KERNEL_NAMES[k]: (int(n[k]), float(ms[k])) for k in range(K_COUNT)}


STATIC_MAX_TENSORS, STATIC_MAX_CHUNKS, STATIC_CHUNK_ELEMS = 4096, 1 << 20, 16384


def adam_step_fp8_static(tensors: Sequence[Tuple[int, int]], grad, grad_fmt, grad_meta, m, m_meta, v, v_meta, w, w_meta,
                         wcopy, wcopy_meta, hp: AdamHparams, tensor_flags=None, device: int = 0, stream=None) -> None:
    """fp8lm_adam_step_fp8 without a context, for callers that cannot allocate device memory (see fp8lm.h): the
    tensor list travels with every call."""
    n = len(tensors)
    arr = (Tensor * max(1, n))()
    for i, (off, k) in enumerate(tensors):
        arr[i].offset, arr[i].numel = int(off), int(k)
    need = max([int(o) + int(k) for o, k in tensors if k > 0], default=0)
    for t in (grad, m, v, w, wcopy):
        if t.numel() < need:
            raise ValueError(f"flat buffer of {t.numel()} elements is shorter than the tensor list needs ({need})")
    for t in (grad_meta, m_meta, v_meta, w_meta, wcopy_meta):
        if t.numel() * t.element_size() < n * C.sizeof(Meta):
            raise ValueError("meta array is shorter than the tensor list")
    flags = None
    if tensor_flags is not None:
        flags = np.ascontiguousarray(tensor_flags, dtype=np.uint32)
        assert len(flags) == n
    _check(lib().fp8lm_adam_step_fp8_static(device, C.cast(arr, C.c_void_p), n, flags.ctypes.data if flags is not None else None,
                                            _ptr(grad), grad_fmt, _ptr(grad_meta), _ptr(m), _ptr(m_meta), _ptr(v),
                                            _ptr(v_meta), _ptr(w), _ptr(w_meta), _ptr(wcopy), _ptr(wcopy_meta),
                                            C.addressof(hp), _stream(stream)), "fp8lm_adam_step_fp8_static")


# ---- device memory piece by piece (see fp8lm.h): argument marshalling only ------------------------------------------
def vmm_granularity(device: int = 0) -> int:
    out = C.c_uint64(0)
    _check(lib().fp8lm_vmm_granularity(device, C.addressof(out)), "fp8lm_vmm_granularity")
    return int(out.value)


def vmm_reserve(nbytes: int) -> int:
    out = C.c_void_p(0)
    _check(lib().fp8lm_vmm_reserve(nbytes, C.addressof(out)), "fp8lm_vmm_reserve")
    return int(out.value)


def vmm_free(va: int, nbytes: int) -> None:
    _check(lib().fp8lm_vmm_free(va, nbytes), "fp8lm_vmm_free")


def vmm_create(nbytes: int, device: int = 0) -> int:
    out = C.c_uint64(0)
    _check(lib().fp8lm_vmm_create(device, nbytes, C.addressof(out)), "fp8lm_vmm_create")
    return int(out.value)


def vmm_destroy(piece: int) -> None:
    _check(lib().fp8lm_vmm_destroy(piece), "fp8lm_vmm_destroy")


def vmm_map(va: int, nbytes: int, piece: int, device: int = 0) -> None:
    _check(lib().fp8lm_vmm_map(va, nbytes, piece, device), "fp8lm_vmm_map")


def vmm_unmap(va: int, nbytes: int) -> None:
    _check(lib().fp8lm_vmm_unmap(va, nbytes), "fp8lm_vmm_unmap")


def greedy_partition(sizes, n_gpus: int):
    """Alg. 1 of the paper on the host: returns (owner[n], usage[n_gpus]) as numpy arrays."""
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    owner = np.zeros(max(1, len(sizes)), dtype=np.int32)
    usage = np.zeros(n_gpus, dtype=np.int64)
    _check(lib().fp8lm_greedy_partition(sizes.ctypes.data, len(sizes), n_gpus, owner.ctypes.data, usage.ctypes.data),
           "fp8lm_greedy_partition")
    return owner[:len(sizes)], usage


def meta_to_numpy(meta: torch.Tensor, n: int) -> np.ndarray:
    """Host copy of a device meta array as a numpy structured array."""
    return meta.detach().cpu().numpy().reshape(-1).view(META_DTYPE)[:n].copy()


def meta_from_numpy(arr: np.ndarray, device) -> torch.Tensor:
    raw = np.ascontiguousarray(arr).view(np.uint8).reshape(len(arr), META_DTYPE.itemsize)
    return torch.from_numpy(raw.copy()).to(device)
