"""The Adam step for callers that cannot allocate (fp8lm_adam_step_fp8_static) against fp8lm_adam_step_fp8.

Two states start from the same seeded weights and see the same FP8 gradients; one is stepped through its context,
the other through the entry point that keeps tables, scales and reduction records in the library's fixed device
array.  Every payload byte and every metadata byte must be equal after each call.  Two calls in a row, the second
on a smaller tensor list (the array still holds the first call's tables), then a third on the first list again
with weight-decay exemptions and the predicted moment scale, a fourth with hardware sqrt, a fifth on E4M3 gradients.
"""
import ctypes as C

import numpy as np
import pytest
import torch

import parity as P
from conftest import say
from paper_2310_18313_amd import binding as B
from paper_2310_18313_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
NAMES = ("m", "v", "w", "wq")
METAS = ("m_meta", "v_meta", "w_meta", "q_meta")


def _pair(wl, seed):
    a, w0 = P.make_state(wl, seed)
    b, _ = P.make_state(wl, seed)
    return a, b, w0


def _assert_same(a, b, what):
    for k in NAMES + METAS:
        assert torch.equal(getattr(a, k), getattr(b, k)), f"{what}: {k} differs"


def _step_both(a, b, grad, hp, flags=None, what=""):
    """a: through its context; b: through the entry point without a context (same FP8 gradient for both)."""
    a.quantize_grad(grad)
    say(f"no-alloc entry point: {what}")
    a.adam(hp)
    B.adam_step_fp8_static(b.tensors, a.g8, a.grad_fmt, a.g_meta, b.m, b.m_meta, b.v, b.v_meta, b.w, b.w_meta, b.wq,
                           b.q_meta, hp, tensor_flags=flags)
    torch.cuda.synchronize()
    _assert_same(a, b, what)


def test_the_entry_point_without_a_context_steps_like_the_one_with():
    big = synth.Workload("noalloc-big", synth.Layout(["a", "b", "c", "d", "e", "f", "g"],
                                                      [70001, 1, 4096, 333, 0, 16385, 300000]), lr=1e-3, sigma=None)
    small = synth.Workload("noalloc-small", synth.Layout(["a", "b", "c"], [5000, 17, 40000]), lr=1e-3, sigma=None)
    A1, B1, _ = _pair(big, 41)
    A2, B2, _ = _pair(small, 42)
    g1 = torch.zeros(max(big.layout.total, 16), dtype=torch.bfloat16, device=DEV)
    g2 = torch.zeros(max(small.layout.total, 16), dtype=torch.bfloat16, device=DEV)
    # first call: the larger list
    synth.fill_gradients(g1, big, 41, 1)
    _step_both(A1, B1, g1, B.adam_hparams(big.lr, 1), what="first call, 7 tensors")
    # second call, directly after: a smaller list; the array still holds the tables of the first
    synth.fill_gradients(g2, small, 42, 1)
    _step_both(A2, B2, g2, B.adam_hparams(small.lr, 1, stats=1), what="second call, 3 tensors")
    # back to the first list: exemptions from weight decay, predicted moment scale
    flags = [0, 1, 0, 1, 0, 0, 1]
    A1.ctx.set_tensor_flags(flags)
    synth.fill_gradients(g1, big, 41, 2)
    _step_both(A1, B1, g1, B.adam_hparams(big.lr, 2, m_scale_mode=B.MSCALE_PREDICTED), flags=flags, what="third call, flags")
    synth.fill_gradients(g2, small, 42, 2)
    _step_both(A2, B2, g2, B.adam_hparams(small.lr, 2, exact=0), what="fourth call, hardware sqrt")
    # a fifth call with the just-in-time moment scale again, E4M3 gradients
    A3, B3, _ = [x for x in (P.make_state(small, 43, B.E4M3)[0], P.make_state(small, 43, B.E4M3)[0], None)]
    synth.fill_gradients(g2, small, 43, 1)
    _step_both(A3, B3, g2, B.adam_hparams(small.lr, 1), what="fifth call, E4M3 gradient")


def test_limits_and_errors_of_the_entry_point_without_a_context():
    wl = synth.Workload("noalloc-err", synth.Layout(["a", "b"], [4096, 4096]), lr=1e-3, sigma=None)
    st, _ = P.make_state(wl, 1)
    hp = B.adam_hparams(1e-3, 1)
    args = (st.g8, st.grad_fmt, st.g_meta, st.m, st.m_meta, st.v, st.v_meta, st.w, st.w_meta, st.wq, st.q_meta)

    def status_of(tensors, hp=hp, flags=None):
        try:
            B.adam_step_fp8_static(tensors, *args, hp, tensor_flags=flags)
        except B.Fp8lmError as e:
            return e.status
        return 0

    lib = B.lib()
    # too many tensors / too many chunks: refused before anything is enqueued (checked on the raw ABI: the binding
    # would refuse the short buffers first)
    many = (B.Tensor * (B.STATIC_MAX_TENSORS + 1))()
    raw = lambda arr, n: lib.fp8lm_adam_step_fp8_static(0, C.cast(arr, C.c_void_p), n, None, *[B._ptr(t) if hasattr(t, "data_ptr") else t for t in args],
                                                        C.addressof(hp), 0)
    assert raw(many, B.STATIC_MAX_TENSORS + 1) == -5
    one = (B.Tensor * 1)()
    one[0].offset, one[0].numel = 0, B.STATIC_MAX_CHUNKS * B.STATIC_CHUNK_ELEMS + 1
    assert raw(one, 1) == -5
    assert status_of([(8, 100)]) == -2                                   # offset not a multiple of 16
    assert status_of([(0, 100), (96, 100)]) == -3                        # overlap
    assert status_of([(0, 4096)], flags=[2]) == -1                       # unknown tensor flag
    assert status_of([(0, 4096)], hp=B.adam_hparams(1e-3, 1, m_scale_mode=B.MSCALE_FROM_CAST)) == -1
    assert status_of([(0, 4096)], hp=B.adam_hparams(1e-3, 0)) == -1       # step < 1
    assert status_of([]) == 0 and status_of([(0, 0)]) == 0               # nothing to do
    torch.cuda.synchronize()
