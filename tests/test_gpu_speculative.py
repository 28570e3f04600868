"""Just-in-time quantisation in one call (fp8lm_quantize_fp8): the same bytes as fp8lm_amax_scale + fp8lm_cast_fp8.

Two sets of payloads and metadata see the same gradients step after step, one through the two calls, one through
the speculative call; every payload byte and every metadata byte must agree after every step, whether the
speculation held (scale unchanged: one pass) or not (amax crossed a power-of-two boundary, first step, all-zero
tensor, inf/NaN: second cast).  The two-call path is itself held to the oracle by the other GPU tests; one case
here also runs the oracle directly.
"""
import numpy as np
import pytest
import torch

import parity as P
from conftest import say
from paper_2310_18313_amd import binding as B
from paper_2310_18313_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _layout():
    return synth.Layout(["a", "b", "c", "d", "e", "f", "g", "h"], [70001, 1, 4096, 333, 0, 16385, 300000, 17])


# per step: the factor every tensor's gradient is multiplied with (a power of two moves the scale by design, a
# factor near 1 usually leaves it), and what is planted
STEPS = [(1.0, None), (1.0, None), (1.03, None), (0.97, None), (4.0, None), (4.0, "nan"), (4.0, None), (0.25, "zero"),
         (0.25, None), (1.0, "inf"), (1.0, None), (1.0, None)]


@pytest.mark.parametrize("fmt", [B.E5M2, B.E4M3])
@pytest.mark.parametrize("dtype,hist", [(torch.bfloat16, 1), (torch.float32, 3), (torch.float16, 2)])
def test_quantize_fp8_equals_amax_scale_then_cast(fmt, dtype, hist):
    lay = _layout()
    wl = synth.Workload("spec", lay, lr=1e-3, sigma=None, ramp_steps=4, hist_window=hist)
    cfg = B.autoscale_cfg(ramp_steps=4, hist_window=hist)
    ctx = B.Context(lay.tensors())
    size = max(lay.total, 16)
    grad = torch.zeros(size, dtype=dtype, device=DEV)
    two = dict(q=torch.zeros(size, dtype=torch.uint8, device=DEV), meta=ctx.new_meta(cfg))
    one = dict(q=torch.zeros(size, dtype=torch.uint8, device=DEV), meta=ctx.new_meta(cfg))
    held_any = redone_any = False
    for step, (factor, plant) in enumerate(STEPS, 1):
        synth.fill_gradients(grad, wl, 7, min(step, 3))           # from step 3 on the same draw: only `factor` moves the amax
        grad *= factor
        off6, n6 = lay.tensors()[6]
        if plant == "nan":
            grad[off6 + 12345] = float("nan")
        elif plant == "inf":
            grad[off6 + 5] = float("-inf")
        elif plant == "zero":
            grad[off6:off6 + n6] = 0
        before = ctx.speculation_stats()
        ctx.amax_scale(grad, fmt, two["meta"], cfg)
        ctx.cast_fp8(grad, two["q"], fmt, two["meta"], cfg)
        say(f"speculative quantisation fmt={fmt} dtype={dtype} H={hist} step={step} factor={factor} plant={plant}")
        ctx.quantize_fp8(grad, one["q"], fmt, one["meta"], cfg)
        torch.cuda.synchronize()
        after = ctx.speculation_stats()
        redone = after["tensors_redone"] - before["tensors_redone"]
        assert after["calls"] == before["calls"] + 1 and 0 <= redone <= 7
        held_any |= redone < 7
        redone_any |= redone > 0
        if step == 1:
            assert redone == 7                                      # nothing to predict from yet
        a, b = B.meta_to_numpy(two["meta"], lay.n_tensors), B.meta_to_numpy(one["meta"], lay.n_tensors)
        for t, (off, n) in enumerate(lay.tensors()):
            assert torch.equal(two["q"][off:off + n], one["q"][off:off + n]), (step, t)
            if n:
                assert a[t].tobytes() == b[t].tobytes(), (step, t, a[t], b[t])
    assert held_any and redone_any


def test_speculative_path_matches_the_oracle_and_the_fused_adam_step():
    """The whole step through quantize_fp8_for_adam + Adam with the moment amax taken from the cast, lock-step against
    the oracle, next to the same state stepped through the three plain calls."""
    wl = synth.Workload("spec-adam", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None, hist_window=2)
    plain, _ = P.make_state(wl, 9)
    spec, _ = P.make_state(wl, 9)
    ids = list(range(wl.layout.n_tensors))
    grad = torch.zeros(max(wl.layout.total, 16), dtype=torch.bfloat16, device=DEV)
    for step in range(1, 7):
        synth.fill_gradients(grad, wl, 9, step)
        if step == 4:
            off0, n0 = wl.layout.tensors()[0]
            grad[off0 + 3] = float("nan")
        mode = B.MSCALE_FROM_CAST if step % 2 else B.MSCALE_EXACT_PASS
        snaps = [P.Snapshot(spec, grad, t) for t in ids]
        say(f"speculative path, whole step {step}, moment-scale mode {mode}")
        plain.step(grad, B.adam_hparams(wl.lr, step))
        spec.step(grad, B.adam_hparams(wl.lr, step, m_scale_mode=mode), speculative=True)
        torch.cuda.synchronize()
        P.check_step(spec, snaps, B.adam_hparams(wl.lr, step, m_scale_mode=mode), what=f"speculative step {step}")
        for k in ("g8", "m", "v", "w", "wq", "g_meta", "m_meta", "v_meta", "w_meta", "q_meta"):
            a, b = getattr(plain, k), getattr(spec, k)
            if a.element_size() == 2:                      # bit patterns: a NaN is not equal to itself
                a, b = a.view(torch.int16), b.view(torch.int16)
            assert torch.equal(a, b), (step, k)
    s = spec.ctx.speculation_stats()
    assert s["calls"] == 6 and 0 < s["tensors_redone"] < 6 * wl.layout.n_tensors


def test_speculation_with_many_small_tensors_and_every_launch_shape():
    """More tensors than one scan block, many of them failing at once, under the ticket form and odd launch shapes."""
    rng = np.random.default_rng(3)
    numels = np.minimum(40000, (rng.pareto(1.2, 3000) * 60).astype(np.int64)).tolist()
    numels[5], numels[2999] = 0, 1
    lay = synth.Layout([f"t{i}" for i in range(len(numels))], numels)
    wl = synth.Workload("spec-many", lay, lr=1e-3, sigma=None)
    cfg = B.autoscale_cfg()
    for tuning in ((16384, 16, 1 << 30), (4096, 3, 0), (65536, 16, 0)):
        ctx = B.Context(lay.tensors())
        ctx.set_tuning(*tuning)
        size = max(lay.total, 16)
        grad = torch.zeros(size, dtype=torch.bfloat16, device=DEV)
        qa, qb = (torch.zeros(size, dtype=torch.uint8, device=DEV) for _ in range(2))
        ma, mb = ctx.new_meta(cfg), ctx.new_meta(cfg)
        sig = torch.ones(size, device=DEV)
        for step in range(1, 5):
            synth.fill_gradients(grad, wl, 11, 1)
            if step > 1:                                     # a third of the tensors move by a binade each step
                for t in range(step % 3, lay.n_tensors, 3):
                    off, n = lay.tensors()[t]
                    sig[off:off + n] = 2.0 ** (step - 2)
                grad = (grad.float() * sig).to(torch.bfloat16)
            ctx.amax_scale(grad, B.E5M2, ma, cfg)
            ctx.cast_fp8(grad, qa, B.E5M2, ma, cfg)
            say(f"speculation over {lay.n_tensors} tensors, tuning {tuning}, step {step}")
            ctx.quantize_fp8(grad, qb, B.E5M2, mb, cfg)
            torch.cuda.synchronize()
            assert torch.equal(qa, qb), (tuning, step)
            assert torch.equal(ma, mb), (tuning, step)
        s = ctx.speculation_stats()
        assert s["calls"] == 4 and lay.n_tensors < s["tensors_redone"] < 4 * lay.n_tensors


@pytest.mark.parametrize("grad_fmt,wcopy,exact", [(B.E5M2, B.WCOPY_E4M3, 1), (B.E4M3, B.WCOPY_BF16, 1), (B.E5M2, B.WCOPY_E4M3, 0)])
def test_adam_step_with_a_pair_of_moment_buffers_equals_the_two_pass_step(grad_fmt, wcopy, exact):
    """fp8lm_adam_step_fp8_m2 (speculated first-moment scale, repaired where it fails) against fp8lm_adam_step_fp8 with
    the exact pass: every payload byte and every metadata byte, over steps whose gradients jump by factors of 8 and
    1/16 (the moment's amax crosses binades: repairs), stay put (no repair), vanish, and carry a NaN; the first
    state is also held to the oracle lock-step."""
    from paper_2310_18313_amd.state import OptimizerState
    lay = _layout()
    wl = synth.Workload("pair-m", lay, lr=1e-3, sigma=None, ramp_steps=4)
    plain, w0 = P.make_state(wl, 23, grad_fmt, wcopy)
    cfg = plain.cfg
    pair = OptimizerState(lay.tensors(), lay.total, cfg, 0, grad_fmt, wcopy, second_m=True)
    pair.init_master(w0)
    ids = list(range(lay.n_tensors))
    grad = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    factors = [1.0, 1.0, 1.0, 8.0, 8.0, 1.0 / 16, 1.0, 0.0, 1.0, 1.0, 1.0, 1.0]
    repaired_any = held_any = False
    for step, f in enumerate(factors, 1):
        synth.fill_gradients(grad, wl, 23, min(step, 3))
        grad *= f
        if step == 10:
            off6, n6 = lay.tensors()[6]
            grad[off6 + 777] = float("nan")
        hp = B.adam_hparams(wl.lr, step, wcopy=wcopy, exact=exact)
        snaps = [P.Snapshot(plain, grad, t) for t in ids]
        before = pair.ctx.speculation_stats(moment=True)
        say(f"pair of moment buffers: fmt={grad_fmt} wcopy={wcopy} exact={exact} step={step} factor={f}")
        plain.step(grad, hp)
        pair.step(grad, hp, pair_m=True, speculative=bool(step % 2))
        torch.cuda.synchronize()
        after = pair.ctx.speculation_stats(moment=True)
        redone = after["tensors_redone"] - before["tensors_redone"]
        assert after["calls"] == before["calls"] + 1 and 0 <= redone <= 7
        repaired_any |= redone > 0
        held_any |= redone == 0
        if step in (1, 4):
            assert redone > 0, step                      # zero state; the jump up (a drop only decays the moment by 10 % a step)
        if exact:
            P.check_step(plain, snaps, hp, what=f"plain step {step}")
        for k in ("g8", "m", "v", "w", "wq", "g_meta", "m_meta", "v_meta", "w_meta", "q_meta"):
            a, b = getattr(plain, k), getattr(pair, k)
            if a.element_size() == 2:
                a, b = a.view(torch.int16), b.view(torch.int16)
            assert torch.equal(a, b), (step, k)
    assert repaired_any and held_any
    # argument errors: the same buffer twice, overlapping buffers, the element counters, another scale mode
    hp = B.adam_hparams(wl.lr, 99, wcopy=wcopy)
    args = lambda mi, mo, h: pair.ctx.adam_step_fp8_m2(pair.g8, grad_fmt, pair.g_meta, mi, mo, pair.m_meta, pair.v, pair.v_meta,
                                                        pair.w, pair.w_meta, pair.wq, pair.q_meta, h)
    for mi, mo, h in ((pair.m, pair.m, hp), (pair.m, pair.m[16:], hp), (pair.m, pair.m_other, B.adam_hparams(wl.lr, 99, wcopy=wcopy, stats=1)),
                      (pair.m, pair.m_other, B.adam_hparams(wl.lr, 99, wcopy=wcopy, m_scale_mode=B.MSCALE_PREDICTED))):
        with pytest.raises((B.Fp8lmError, ValueError)):
            args(mi, mo, h)
