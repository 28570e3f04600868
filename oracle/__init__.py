"""CPU oracle of the FP8 gradient cast + FP8 Adam step (test infrastructure only).

Nothing in the product package imports this.  Allowed callers: ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg.  The arithmetic lives in ``fp8lm_oracle.cpp``; this module only
builds it with g++ and marshals numpy arrays into it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fp8lm_oracle.cpp")
_LIB = os.path.join(_HERE, "_build", "libfp8lm_oracle.so")

HIST = 16
E4M3, E5M2 = 0, 1
WCOPY_E4M3, WCOPY_BF16 = 0, 1
ST_F16, ST_BF16, ST_E4M3, ST_F32 = 0, 1, 2, 3
FLAG_NONFINITE, FLAG_AMAX_ZERO, FLAG_SCALE_CLAMPED, FLAG_SATURATED = 1, 2, 4, 8


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
                ("wcopy", C.c_int32), ("m_predict", C.c_int32), ("master_fmt", C.c_int32), ("v_fmt", C.c_int32)]


MU_SET_HALF, MU_HALVE = 0, 1


def default_cfg(ramp_steps=1000, hist_window=1, margin=0, sat_num=1, sat_den=100000, mu_rule=MU_SET_HALF, mu_min_exp=-1):
    return AutoscaleCfg(sat_num, sat_den, ramp_steps, hist_window, margin, mu_rule, mu_min_exp)


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        subprocess.check_call([
            "g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra",
            "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.oracle_decode_e4m3.restype = C.c_float
        L.oracle_decode_e4m3.argtypes = [C.c_uint8]
        L.oracle_decode_e5m2.restype = C.c_float
        L.oracle_decode_e5m2.argtypes = [C.c_uint8]
        L.oracle_decode_f16.restype = C.c_float
        L.oracle_decode_f16.argtypes = [C.c_uint16]
        L.oracle_decode_bf16.restype = C.c_float
        L.oracle_decode_bf16.argtypes = [C.c_uint16]
        L.oracle_encode_e4m3.restype = C.c_uint8
        L.oracle_encode_e4m3.argtypes = [C.c_float]
        L.oracle_encode_e5m2.restype = C.c_uint8
        L.oracle_encode_e5m2.argtypes = [C.c_float]
        L.oracle_encode_f16_sat.restype = C.c_uint16
        L.oracle_encode_f16_sat.argtypes = [C.c_float]
        L.oracle_encode_bf16.restype = C.c_uint16
        L.oracle_encode_bf16.argtypes = [C.c_float]
        L.oracle_encode_fp8_nearest.restype = C.c_uint8
        L.oracle_encode_fp8_nearest.argtypes = [C.c_int, C.c_float]
        L.oracle_pow2_exp.restype = C.c_int
        L.oracle_pow2_exp.argtypes = [C.c_float, C.c_float]
        L.oracle_sizeof_meta.restype = C.c_uint32
        for name in ("oracle_encode_fp8_array", "oracle_encode_fp8_nearest_array"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_int64]
        for name in ("oracle_encode_f16_sat_array", "oracle_encode_bf16_array"):
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        L.oracle_meta_init.restype = None
        L.oracle_meta_init.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.oracle_amax_scale.restype = None
        L.oracle_amax_scale.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int, C.c_void_p, C.c_void_p]
        L.oracle_cast_fp8.restype = None
        L.oracle_cast_fp8.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int,
                                      C.c_void_p, C.c_void_p]
        L.oracle_cast_fp8_delayed.restype = None
        L.oracle_cast_fp8_delayed.argtypes = L.oracle_cast_fp8.argtypes
        for name in ("oracle_amax_scale_src", "oracle_cast_fp8_src", "oracle_cast_fp8_delayed_src"):
            base = getattr(L, name[:-4])
            getattr(L, name).restype = None
            getattr(L, name).argtypes = [C.c_void_p, C.c_int] + list(base.argtypes[1:])
        L.oracle_quant_error_stats.restype = None
        L.oracle_quant_error_stats.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                                               C.c_int32, C.c_void_p]
        L.oracle_shared_scale.restype = None
        L.oracle_shared_scale.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.oracle_requantize_fp8.restype = None
        L.oracle_requantize_fp8.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                            C.c_void_p, C.c_void_p]
        L.oracle_sum_fp8.restype = None
        L.oracle_sum_fp8.argtypes = [C.c_void_p, C.c_int32, C.c_int, C.c_void_p, C.c_void_p, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_greedy_partition.restype = None
        L.oracle_greedy_partition.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.oracle_init_master.restype = None
        L.oracle_init_master.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
        L.oracle_init_master_as.restype = None
        L.oracle_init_master_as.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int]
        L.oracle_adam_step_fp8.restype = None
        L.oracle_adam_step_fp8.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int, C.c_void_p] + \
            [C.c_void_p] * 8 + [C.c_void_p]
        L.oracle_derive_hparams.restype = None
        L.oracle_derive_hparams.argtypes = [C.c_void_p, C.c_void_p]
        assert L.oracle_sizeof_meta() == C.sizeof(Meta) == META_DTYPE.itemsize
        _lib = L
    return _lib


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def tensors_array(tensors) -> np.ndarray:
    """[(offset, numel), ...] -> int64 array [n, 2] with the oracle_tensor layout."""
    return np.ascontiguousarray(np.asarray(tensors, dtype=np.int64).reshape(-1, 2))


def new_meta(n: int, cfg: AutoscaleCfg) -> np.ndarray:
    meta = np.zeros(n, dtype=META_DTYPE)
    lib().oracle_meta_init(_p(meta), n, C.byref(cfg))
    return meta


# source types of a cast: bf16 and IEEE half arrive as their uint16 bit patterns, fp32 as float32
SRC_BF16, SRC_F16, SRC_F32 = 0, 1, 2


def _src_ok(src: np.ndarray, src_type: int) -> bool:
    return src.dtype == (np.float32 if src_type == SRC_F32 else np.uint16)


def amax_scale(src: np.ndarray, tensors: np.ndarray, target_fmt: int, meta: np.ndarray,
               cfg: AutoscaleCfg, src_type: int = SRC_BF16) -> None:
    assert _src_ok(src, src_type)
    lib().oracle_amax_scale_src(_p(src), src_type, _p(tensors), len(tensors), target_fmt, _p(meta), C.byref(cfg))


def cast_fp8(src: np.ndarray, tensors: np.ndarray, dst: np.ndarray, fmt: int, meta: np.ndarray,
             cfg: AutoscaleCfg, src_type: int = SRC_BF16) -> None:
    assert _src_ok(src, src_type) and dst.dtype == np.uint8
    lib().oracle_cast_fp8_src(_p(src), src_type, _p(tensors), len(tensors), _p(dst), fmt, _p(meta), C.byref(cfg))


def cast_fp8_delayed(src: np.ndarray, tensors: np.ndarray, dst: np.ndarray, fmt: int, meta: np.ndarray,
                     cfg: AutoscaleCfg, src_type: int = SRC_BF16) -> None:
    assert _src_ok(src, src_type) and dst.dtype == np.uint8
    lib().oracle_cast_fp8_delayed_src(_p(src), src_type, _p(tensors), len(tensors), _p(dst), fmt, _p(meta),
                                      C.byref(cfg))


QUANT_STATS_DTYPE = np.dtype([("signal", np.float64), ("noise", np.float64), ("n_nonzero", np.uint64),
                              ("n_underflow", np.uint64), ("n_overflow", np.uint64), ("n_nonfinite", np.uint64)])


def quant_error_stats(ref: np.ndarray, q: np.ndarray, fmt: int, meta: np.ndarray, tensors: np.ndarray,
                      ref_type: int = SRC_F32) -> np.ndarray:
    """Per-tensor signal / noise energies and underflow / overflow counts of an FP8 gradient (Sec. 3.3)."""
    assert _src_ok(ref, ref_type) and q.dtype == np.uint8
    out = np.zeros(len(tensors), dtype=QUANT_STATS_DTYPE)
    lib().oracle_quant_error_stats(_p(ref), ref_type, _p(q), fmt, _p(meta), _p(tensors), len(tensors), _p(out))
    return out


def _ptr_array(arrays):
    arr = (C.c_void_p * len(arrays))(*[a.ctypes.data for a in arrays])
    return arr


def shared_scale(metas, n_tensors: int) -> np.ndarray:
    """Eq. 4: per tensor, the smallest scale among the ranks' meta arrays."""
    out = np.zeros(n_tensors, dtype=np.float32)
    lib().oracle_shared_scale(_ptr_array(metas), len(metas), n_tensors, _p(out))
    return out


def requantize_fp8(src, fmt, src_meta, shared, tensors, dst, dst_meta) -> None:
    assert src.dtype == np.uint8 and dst.dtype == np.uint8 and shared.dtype == np.float32
    lib().oracle_requantize_fp8(_p(src), fmt, _p(src_meta), _p(shared), _p(tensors), len(tensors), _p(dst), _p(dst_meta))


def sum_fp8(payloads, fmt, shared, tensors, dst, dst_meta, cfg) -> None:
    assert all(a.dtype == np.uint8 for a in payloads) and dst.dtype == np.uint8
    lib().oracle_sum_fp8(_ptr_array(payloads), len(payloads), fmt, _p(shared), _p(tensors), len(tensors), _p(dst),
                         _p(dst_meta), C.byref(cfg))


def greedy_partition(sizes, n_gpus: int):
    """Alg. 1: (owner[n], usage[n_gpus])."""
    sizes = np.ascontiguousarray(sizes, dtype=np.int64)
    owner = np.zeros(len(sizes), dtype=np.int32)
    usage = np.zeros(n_gpus, dtype=np.int64)
    lib().oracle_greedy_partition(_p(sizes), len(sizes), n_gpus, _p(owner), _p(usage))
    return owner, usage


def init_master(w_bf16: np.ndarray, tensors: np.ndarray, w_f16: np.ndarray, w_meta: np.ndarray) -> None:
    assert w_bf16.dtype == np.uint16 and w_f16.dtype == np.uint16
    lib().oracle_init_master(_p(w_bf16), _p(tensors), len(tensors), _p(w_f16), _p(w_meta))


STATE_DTYPE = {ST_F16: np.uint16, ST_BF16: np.uint16, ST_E4M3: np.uint8, ST_F32: np.uint32}


def init_master_as(w_bf16: np.ndarray, tensors: np.ndarray, w_out: np.ndarray, w_meta: np.ndarray, master_fmt: int) -> None:
    assert w_bf16.dtype == np.uint16 and w_out.dtype == STATE_DTYPE[master_fmt]
    lib().oracle_init_master_as(_p(w_bf16), _p(tensors), len(tensors), _p(w_out), _p(w_meta), master_fmt)


def adam_step_fp8(tensors, grad, grad_fmt, grad_meta, m, m_meta, v, v_meta, w, w_meta, wcopy,
                  wcopy_meta, hp: AdamHparams) -> None:
    assert grad.dtype == np.uint8 and m.dtype == np.uint8
    assert v.dtype == STATE_DTYPE[hp.v_fmt] and w.dtype == STATE_DTYPE[hp.master_fmt]
    assert wcopy.dtype == (np.uint8 if hp.wcopy == WCOPY_E4M3 else np.uint16)
    lib().oracle_adam_step_fp8(_p(tensors), len(tensors), _p(grad), grad_fmt, _p(grad_meta),
                               _p(m), _p(m_meta), _p(v), _p(v_meta), _p(w), _p(w_meta),
                               _p(wcopy), _p(wcopy_meta), C.byref(hp))


def derive_hparams(hp: AdamHparams) -> np.ndarray:
    """[b1, 1-b1, 1/(1-b1^t), b2, 1-b2, 1/(1-b2^t), 1-lr*wd] as the oracle uses them."""
    out = np.zeros(7, dtype=np.float32)
    lib().oracle_derive_hparams(C.byref(hp), _p(out))
    return out


def encode_fp8(fmt: int, x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    lib().oracle_encode_fp8_array(fmt, _p(x), _p(out), x.size)
    return out


def encode_fp8_nearest(fmt: int, x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    lib().oracle_encode_fp8_nearest_array(fmt, _p(x), _p(out), x.size)
    return out


def encode_f16_sat(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().oracle_encode_f16_sat_array(_p(x), _p(out), x.size)
    return out


def encode_bf16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().oracle_encode_bf16_array(_p(x), _p(out), x.size)
    return out


def decode_table(fmt: int) -> np.ndarray:
    f = lib().oracle_decode_e4m3 if fmt == E4M3 else lib().oracle_decode_e5m2
    return np.array([f(c) for c in range(256)], dtype=np.float32)
