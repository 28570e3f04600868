"""GPU parity tests: the HIP path behind the C ABI against the CPU oracle, element by element."""
import ctypes as C
import os

import numpy as np
import pytest
import torch

import oracle as O
import parity as P
from conftest import say
from paper_2310_18313_amd import binding as B
from paper_2310_18313_amd import synth
from paper_2310_18313_amd.state import OptimizerState

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bf16_tensor_from_bits(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)


# ---- hardware convert semantics: every bf16 pattern times many power-of-two scales --------------------
@pytest.mark.parametrize("fmt", [B.E5M2, B.E4M3])
def test_cast_every_bf16_pattern_under_many_scales(fmt):
    pats = np.arange(65536, dtype=np.uint16)
    finite = pats[(pats & 0x7F80) != 0x7F80]                  # 65280 patterns, no inf/NaN: fast path
    exps = list(range(-126, 127, 6)) + [-20, -17, -16, -15, -10, -9, -8, -1, 0, 1, 7, 8, 15, 16]
    n_fast = len(exps)
    numels = [finite.size] * n_fast + [pats.size] * 3          # three tensors with inf/NaN: careful path
    lay = synth.Layout([f"t{i}" for i in range(len(numels))], numels)
    src = np.zeros(lay.total, dtype=np.uint16)
    for i, (off, n) in enumerate(lay.tensors()):
        src[off:off + n] = finite if i < n_fast else pats
    cfg = B.autoscale_cfg()
    ctx = B.Context(lay.tensors())
    meta = B.meta_to_numpy(ctx.new_meta(cfg), lay.n_tensors)
    scales = exps + [0, -12, 9]
    for i, e in enumerate(scales):
        meta["scale"][i] = 2.0 ** e
        meta["inv_scale"][i] = 2.0 ** -e
        if i >= n_fast:
            meta["flags"][i] = B.FLAG_NONFINITE              # as the amax pass would have left it
    ref_meta = meta.copy()
    d_meta = B.meta_from_numpy(meta, DEV)
    d_src = bf16_tensor_from_bits(src)
    d_dst = torch.zeros(lay.total, dtype=torch.uint8, device=DEV)
    say(f"cast sweep fmt={fmt} tensors={lay.n_tensors}")
    ctx.cast_fp8(d_src, d_dst, fmt, d_meta, cfg)
    torch.cuda.synchronize()
    ref = np.zeros(lay.total, dtype=np.uint8)
    O.cast_fp8(src, O.tensors_array(lay.tensors()), ref, fmt, ref_meta, P.oracle_cfg(cfg))
    got = d_dst.cpu().numpy()
    bad = np.flatnonzero(got != ref)
    assert bad.size == 0, f"{bad.size} codes differ, first at {bad[:5]}: gpu {got[bad[:5]]} oracle {ref[bad[:5]]} src {src[bad[:5]]}"
    got_meta = B.meta_to_numpy(d_meta, lay.n_tensors)
    for t in range(lay.n_tensors):
        diff = P.meta_equal(got_meta[t], ref_meta[t], P.ALL_FIELDS)
        assert not diff, (t, diff, got_meta[t], ref_meta[t])


@pytest.mark.parametrize("gfmt", [B.E5M2, B.E4M3])
@pytest.mark.parametrize("finite_only", [True, False])
def test_fp8_decode_of_every_code_matches_the_oracle_through_adam(gfmt, finite_only):
    """Every gradient code x every moment code goes through the Adam kernels (all 256 x 256 codes on the
    careful path, the finite ones on the fast path); the results must equal the oracle's, which pins
    the hardware decoders."""
    g_codes = np.repeat(np.arange(256, dtype=np.uint8), 256)
    m_codes = np.tile(np.arange(256, dtype=np.uint8), 256)
    if finite_only:
        g_fin = np.isfinite(O.decode_table(gfmt))[g_codes]
        m_fin = np.isfinite(O.decode_table(O.E4M3))[m_codes]
        g_codes, m_codes = g_codes[g_fin & m_fin], m_codes[g_fin & m_fin]
    n = g_codes.size
    lay = synth.flat_layout(n)
    cfg = B.autoscale_cfg()
    st = OptimizerState(lay.tensors(), lay.total, cfg, 0, gfmt, B.WCOPY_E4M3)
    st.g8[:n] = torch.from_numpy(g_codes).to(DEV)
    st.m[:n] = torch.from_numpy(m_codes).to(DEV)
    gm = B.meta_to_numpy(st.g_meta, 1)
    gm["scale"][0], gm["inv_scale"][0], gm["amax_deq"][0] = 4.0, 0.25, (57344.0 if gfmt == B.E5M2 else 448.0) / 4
    st.g_meta = B.meta_from_numpy(gm, DEV)
    hp = B.adam_hparams(1e-3, 3, stats=1, exact=1)
    pad = lay.total
    pre_m = np.zeros(pad, np.uint8)
    pre_m[:n] = m_codes
    g_pad = np.zeros(pad, np.uint8)
    g_pad[:n] = g_codes
    pre_v, pre_w, wq = np.zeros(pad, np.uint16), np.zeros(pad, np.uint16), np.zeros(pad, np.uint8)
    metas = {k: B.meta_to_numpy(getattr(st, k), 1) for k in ("g_meta", "m_meta", "v_meta", "w_meta", "q_meta")}
    say(f"decode sweep gfmt={gfmt} finite_only={finite_only} n={n}")
    st.adam(hp)
    torch.cuda.synchronize()
    O.adam_step_fp8(O.tensors_array(lay.tensors()), g_pad, gfmt, metas["g_meta"], pre_m, metas["m_meta"],
                    pre_v, metas["v_meta"], pre_w, metas["w_meta"], wq, metas["q_meta"], P.oracle_hp(hp))
    assert np.array_equal(st.m[:n].cpu().numpy(), pre_m[:n])
    assert np.array_equal(synth.bits16(st.v[:n]), pre_v[:n])
    assert np.array_equal(synth.bits16(st.w[:n]), pre_w[:n])
    assert np.array_equal(st.wq[:n].cpu().numpy(), wq[:n])
    for k in ("m_meta", "v_meta", "w_meta", "q_meta"):
        got = B.meta_to_numpy(getattr(st, k), 1)[0]
        diff = P.meta_equal(got, metas[k][0], ["scale", "inv_scale", "amax", "amax_deq", "flags", "n_sat", "n_underflow"])
        assert not diff, (k, diff, got, metas[k][0])


@pytest.mark.parametrize("finite_only", [True, False])
def test_fp16_decode_of_every_pattern_matches_the_oracle_through_adam(finite_only):
    """Every FP16 pattern as a stored master weight, every non-negative one as a stored second moment (subnormals
    included): the finite ones on the fast path, all of them (inf and NaN too) on the careful path."""
    pats = np.arange(65536, dtype=np.uint16)
    w_bits = pats[(pats & 0x7C00) != 0x7C00] if finite_only else pats
    n = w_bits.size
    v_bits = (np.arange(n, dtype=np.uint32) * 7 % 0x7C00).astype(np.uint16)        # finite, non-negative, all exponents
    lay = synth.flat_layout(n)
    cfg = B.autoscale_cfg()
    st = OptimizerState(lay.tensors(), lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3)
    rng = np.random.default_rng(8)
    g_codes = rng.integers(0, 0x7C, n).astype(np.uint8) | (rng.integers(0, 2, n).astype(np.uint8) << 7)
    m_codes = rng.integers(0, 0x7F, n).astype(np.uint8) | (rng.integers(0, 2, n).astype(np.uint8) << 7)
    pad = lay.total
    host = {k: np.zeros(pad, dt) for k, dt in (("g8", np.uint8), ("m", np.uint8), ("v", np.uint16), ("w", np.uint16))}
    host["g8"][:n], host["m"][:n], host["v"][:n], host["w"][:n] = g_codes, m_codes, v_bits, w_bits
    st.g8.copy_(torch.from_numpy(host["g8"]).to(DEV))
    st.m.copy_(torch.from_numpy(host["m"]).to(DEV))
    st.v.copy_(torch.from_numpy(host["v"].view(np.int16)).to(DEV).view(torch.float16))
    st.w.copy_(torch.from_numpy(host["w"].view(np.int16)).to(DEV).view(torch.float16))
    metas = {k: B.meta_to_numpy(getattr(st, k), 1) for k in ("g_meta", "m_meta", "v_meta", "w_meta", "q_meta")}
    metas["g_meta"]["scale"], metas["g_meta"]["inv_scale"], metas["g_meta"]["amax_deq"] = 2.0 ** 20, 2.0 ** -20, 57344.0 * 2.0 ** -20
    metas["m_meta"]["scale"], metas["m_meta"]["inv_scale"], metas["m_meta"]["amax_deq"] = 2.0 ** 12, 2.0 ** -12, 448.0 * 2.0 ** -12
    metas["v_meta"]["scale"], metas["v_meta"]["inv_scale"], metas["v_meta"]["amax_deq"] = 2.0 ** 30, 2.0 ** -30, 65504.0 * 2.0 ** -30
    metas["w_meta"]["scale"], metas["w_meta"]["inv_scale"], metas["w_meta"]["amax_deq"] = 2.0 ** 14, 2.0 ** -14, 65504.0 * 2.0 ** -14
    if not finite_only:
        metas["w_meta"]["flags"] = B.FLAG_NONFINITE             # as the step that stored the inf / NaN left it
    for k, mt in metas.items():
        setattr(st, k, B.meta_from_numpy(mt, DEV))
    hp = B.adam_hparams(1e-2, 5, stats=1)
    say(f"FP16 decode sweep finite_only={finite_only} n={n}")
    st.adam(hp)
    torch.cuda.synchronize()
    wq = np.zeros(pad, np.uint8)
    O.adam_step_fp8(O.tensors_array(lay.tensors()), host["g8"], B.E5M2, metas["g_meta"], host["m"], metas["m_meta"],
                    host["v"], metas["v_meta"], host["w"], metas["w_meta"], wq, metas["q_meta"], P.oracle_hp(hp))
    assert np.array_equal(st.m[:n].cpu().numpy(), host["m"][:n])
    assert np.array_equal(synth.bits16(st.v[:n]), host["v"][:n])
    assert np.array_equal(synth.bits16(st.w[:n]), host["w"][:n])
    assert np.array_equal(st.wq[:n].cpu().numpy(), wq[:n])
    for k in ("m_meta", "v_meta", "w_meta", "q_meta"):
        got = B.meta_to_numpy(getattr(st, k), 1)[0]
        diff = P.meta_equal(got, metas[k][0], ["scale", "inv_scale", "amax", "amax_deq", "flags", "n_sat", "n_underflow"])
        assert not diff, (k, diff, got, metas[k][0])


# ---- whole-path lock-step parity ------------------------------------------------------------------------
def run_lockstep(wl, seed, steps, ids=None, grad_fmt=B.E5M2, wcopy=B.WCOPY_E4M3, v_scaled=1, stats=0, exact=1,
                 check_steps=None, tuning=None, lr=None):
    st, w0 = P.make_state(wl, seed, grad_fmt, wcopy)
    if tuning:
        st.ctx.set_tuning(*tuning)
    ids = list(range(wl.layout.n_tensors)) if ids is None else ids
    P.check_init_master(st, w0, ids)
    del w0
    grad = torch.zeros(max(wl.layout.total, 16), dtype=torch.bfloat16, device=DEV)
    tot = dict(elements=0, m_diff=0, w_diff=0, q_diff=0, w_amax_ulp=0)
    for step in range(1, steps + 1):
        synth.fill_gradients(grad, wl, seed, step)
        hp = B.adam_hparams(lr or wl.lr, step, v_scaled=v_scaled, wcopy=wcopy, stats=stats, exact=exact)
        checked = check_steps is None or step in check_steps
        snaps = [P.Snapshot(st, grad, t) for t in ids] if checked else []
        say(f"{wl.name} seed={seed} step={step} fmt={grad_fmt} wcopy={wcopy} v_scaled={v_scaled} stats={stats} exact={exact} checked={checked}"
            + ("" if exact else "  [exact=0: checked against the documented looser contract, outside the 1-ulp bar by design]"))
        st.step(grad, hp)
        torch.cuda.synchronize()
        if checked:
            r = P.check_step(st, snaps, hp, what=f"{wl.name} step {step}")
            for k in tot:
                tot[k] = max(tot[k], r[k]) if k == "w_amax_ulp" else tot[k] + r[k]
    say(f"  -> {tot}")
    return st, tot


@pytest.mark.parametrize("grad_fmt", [B.E5M2, B.E4M3])
@pytest.mark.parametrize("wcopy", [B.WCOPY_E4M3, B.WCOPY_BF16])
@pytest.mark.parametrize("exact", [0, 1])
def test_ragged_tensors_every_variant(grad_fmt, wcopy, exact):
    wl = synth.workload("tiny")
    for v_scaled, stats in ((1, 1), (0, 0)):
        _, tot = run_lockstep(wl, seed=3, steps=3, grad_fmt=grad_fmt, wcopy=wcopy, v_scaled=v_scaled, stats=stats, exact=exact)
        assert tot["m_diff"] == 0
        if exact:
            assert tot["w_diff"] == 0 and tot["q_diff"] == 0


def test_config1_flat_1m():
    wl = synth.workload("flat1m")
    for exact in (1, 0):
        _, tot = run_lockstep(wl, seed=0, steps=1, exact=exact, stats=1)
        assert tot["m_diff"] == 0
        assert tot["w_diff"] <= 0.01 * tot["elements"]


def test_config2_gpt125m_ten_steps():
    wl = synth.workload("gpt125m")
    _, tot = run_lockstep(wl, seed=1, steps=10, check_steps={1, 10})      # the free-running test below compares every byte after 10
    assert tot["m_diff"] == 0
    assert tot["w_diff"] <= 0.01 * tot["elements"]


@pytest.mark.parametrize("name,steps", [("flat1m", 3), ("gpt125m", 10)])
def test_free_running_oracle_and_gpu_end_in_the_same_state(name, steps):
    """Both sides start from the same seeded weights, see the same seeded gradients and never exchange state."""
    wl = synth.workload(name)
    st, w0 = P.make_state(wl, seed=4)
    fr = P.FreeRunningOracle(wl.layout, st.cfg, synth.bits16(w0), threads=16)
    grad = torch.zeros(max(wl.layout.total, 16), dtype=torch.bfloat16, device=DEV)
    for step in range(1, steps + 1):
        synth.fill_gradients(grad, wl, 4, step)
        hp = B.adam_hparams(wl.lr, step)
        say(f"free-running {name} step {step}")
        st.step(grad, hp)
        fr.step(synth.bits16(grad), hp)
    torch.cuda.synchronize()
    fr.assert_equal_to(st, f"{name} after {steps} free-running steps")


@pytest.mark.parametrize("mu_rule", [B.MU_SET_HALF, B.MU_HALVE])
def test_three_hundred_free_running_steps_with_heavy_tails(mu_rule):
    """A long run without any exchange of state: heavy-tailed gradients and a ramp of 20 steps take mu through many
    overflow / recovery cycles, the amax history (window 3) and every scale move all the time; the two sides must
    still hold the same bytes at steps 50, 150 and 300."""
    wl = synth.Workload("long", synth.gpt_layout(128, 2, 512, 1000), lr=1e-3, grad_kind="student_t", sigma=None,
                        hist_window=3, ramp_steps=20)
    cfg = B.autoscale_cfg(ramp_steps=20, hist_window=3, mu_rule=mu_rule, mu_min_exp=-4)
    st = OptimizerState(wl.layout.tensors(), wl.layout.total, cfg, 0, B.E5M2, B.WCOPY_E4M3)
    w0 = torch.zeros(max(wl.layout.total, 16), dtype=torch.bfloat16, device=DEV)
    synth.fill_weights(w0, wl.layout, 21)
    st.init_master(w0)
    fr = P.FreeRunningOracle(wl.layout, cfg, synth.bits16(w0), threads=16)
    grad = torch.zeros(max(wl.layout.total, 16), dtype=torch.bfloat16, device=DEV)
    mus = set()
    for step in range(1, 301):
        synth.fill_gradients(grad, wl, 21, step)
        hp = B.adam_hparams(wl.lr, step)
        st.step(grad, hp)
        fr.step(synth.bits16(grad), hp)
        if step in (50, 150, 300):
            say(f"long free-running run, mu rule {mu_rule}: comparing at step {step}")
            torch.cuda.synchronize()
            fr.assert_equal_to(st, f"step {step} of the long free-running run")
            mus.update(int(x) for x in B.meta_to_numpy(st.g_meta, wl.layout.n_tensors)["mu_exp"])
    assert len(mus) >= 2, mus


@pytest.mark.parametrize("single_pass", [0, 1 << 30])
def test_twenty_thousand_small_tensors(single_pass):
    """Many tensors per workgroup: 20 000 tensors of 0 to 6000 elements (a workgroup crosses a dozen of them per launch,
    leaves a record for each, and every tensor is a chunk of its own), three free-running steps, both forms of the
    grid-wide reduction."""
    rng = np.random.default_rng(77)
    numels = np.minimum(6000, (rng.pareto(1.2, 20000) * 40).astype(np.int64)).tolist()
    numels[17], numels[18], numels[19999] = 0, 0, 1
    lay = synth.Layout([f"t{i}" for i in range(len(numels))], numels)
    wl = synth.Workload("many", lay, lr=1e-3, sigma=None, ramp_steps=4, hist_window=2)
    cfg = B.autoscale_cfg(ramp_steps=4, hist_window=2)
    st = OptimizerState(lay.tensors(), lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3)
    st.ctx.set_tuning(16384, 16, single_pass)
    say(f"{lay.n_tensors} tensors, {lay.n_params} parameters, reduction form {single_pass}")
    gw = torch.Generator(device=DEV)
    gw.manual_seed(5)
    w0 = torch.randn(lay.total, device=DEV, generator=gw).mul_(0.02).to(torch.bfloat16)
    st.init_master(w0)
    fr = P.FreeRunningOracle(lay, cfg, synth.bits16(w0), threads=16)
    sig_host = np.zeros(lay.total, dtype=np.float32)
    for (off, n), sg in zip(lay.tensors(), 10.0 ** rng.uniform(-5, -2, lay.n_tensors)):
        sig_host[off:off + n] = sg
    sig = torch.from_numpy(sig_host).to(DEV)
    g = torch.Generator(device=DEV)
    for step in (1, 2, 3):
        g.manual_seed(1000 + step)
        grad = (torch.randn(lay.total, device=DEV, generator=g) * sig * (20.0 if step == 3 else 1.0)).to(torch.bfloat16)
        hp = B.adam_hparams(wl.lr, step)
        st.step(grad, hp)
        fr.step(synth.bits16(grad), hp)
    torch.cuda.synchronize()
    say("comparing 20 000 tensors")
    fr.assert_equal_to(st, "20 000 tensors after 3 steps")


# chunk size, workgroups per CU, and both forms of the cross-workgroup reduction (third entry 0: tickets in the
# same launch; large: a second launch finishes the tensors)
@pytest.mark.parametrize("tuning", [(4096, 1, 0), (4096, 16, 0), (65536, 4, 0), (1048576, 2, 0), (16384, 16, 0),
                                    (4096, 16, 1 << 20), (16384, 3, 1 << 20), (262144, 16, 1 << 20)])
def test_launch_shapes_give_identical_results(tuning):
    wl = synth.workload("tiny")
    run_lockstep(wl, seed=5, steps=2, exact=1, stats=1, tuning=tuning)
    wl2 = synth.Workload("mid", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None)
    run_lockstep(wl2, seed=5, steps=2, exact=1, tuning=tuning)


# ---- special values and degenerate tensors ------------------------------------------------------------
def test_nonfinite_zero_and_extreme_gradients():
    lay = synth.Layout(["nan", "inf", "zero", "huge", "tiny", "ok", "one"], [5000, 4099, 777, 20000, 20000, 33333, 1])
    wl = synth.Workload("special", lay, lr=1e-3, sigma=1e-3)
    st, w0 = P.make_state(wl, 4)
    rng = np.random.default_rng(0)
    ids = list(range(lay.n_tensors))
    for step in range(1, 4):
        bits = np.zeros(lay.total, dtype=np.uint16)
        for i, (off, n) in enumerate(lay.tensors()):
            x = rng.standard_normal(n).astype(np.float32) * 1e-3
            if lay.names[i] == "huge":
                x *= 1e35 if step != 2 else 1e20
            if lay.names[i] == "tiny":
                x *= 1e-34
            b = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
            if lay.names[i] == "zero":
                b[:] = 0
                b[5] = 0x8000
            if lay.names[i] == "nan" and step == 1:
                b[17] = 0x7FC0
                b[4000] = 0xFFFF
            if lay.names[i] == "inf" and step <= 2:
                b[0] = 0x7F80
                b[4098] = 0xFF80
            bits[off:off + n] = b
        grad = bf16_tensor_from_bits(bits)
        hp = B.adam_hparams(1e-3, step, stats=1, exact=1)
        snaps = [P.Snapshot(st, grad, t) for t in ids]
        say(f"special step {step}")
        st.step(grad, hp)
        torch.cuda.synchronize()
        P.check_step(st, snaps, hp, what=f"special step {step}")
    gm = B.meta_to_numpy(st.g_meta, lay.n_tensors)
    assert gm["flags"][2] & B.FLAG_AMAX_ZERO
    mm = B.meta_to_numpy(st.m_meta, lay.n_tensors)
    assert mm["flags"][0] & B.FLAG_NONFINITE          # the NaN of step 1 lives on in the moment


def test_empty_layouts_and_empty_tensors():
    cfg = B.autoscale_cfg()
    ctx = B.Context([])
    z = torch.zeros(16, dtype=torch.bfloat16, device=DEV)
    meta = ctx.new_meta(cfg)
    ctx.amax_scale(z, B.E5M2, meta, cfg)
    ctx.cast_fp8(z, torch.zeros(16, dtype=torch.uint8, device=DEV), B.E5M2, meta, cfg)
    ctx2 = B.Context([(0, 0), (16, 0)])
    meta2 = ctx2.new_meta(cfg)
    before = meta2.clone()
    ctx2.amax_scale(z, B.E5M2, meta2, cfg)
    torch.cuda.synchronize()
    assert torch.equal(before, meta2)


def test_tensor_lists_beyond_the_tables_are_refused():
    """The chunk table is indexed with 32 bits: a list that needs more chunks is refused at creation, before
    anything is allocated; so are overlapping and misaligned lists."""
    for tensors, status in (([(0, 1 << 46)], -5), ([(0, 1 << 45), (1 << 45, 1 << 45)], -5),
                            ([(0, 100), (96, 100)], -3), ([(8, 100)], -2), ([(0, -1)], -1)):
        with pytest.raises(B.Fp8lmError) as e:
            B.Context(tensors)
        assert e.value.status == status, (tensors, e.value.status)
    big = B.Context([(0, (1 << 31) + 16), ((1 << 33), 4096)])     # sizes and offsets past 32 bits are fine
    assert big.required_elems == (1 << 33) + 4096
    big.close()


def test_argument_errors_are_reported_not_launched():
    lay = synth.flat_layout(1024)
    cfg = B.autoscale_cfg()
    st = OptimizerState(lay.tensors(), lay.total, cfg)
    grad = torch.zeros(lay.total + 16, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.Fp8lmError) as e:
        st.ctx.amax_scale(grad[1:], B.E5M2, st.g_meta, cfg)          # 2-byte offset: misaligned
    assert e.value.status == -2
    for bad in (dict(eps=0.0), dict(beta1=1.0), dict(lr=-1.0), dict(step=0), dict(weight_decay=float("nan"))):
        kw = dict(lr=1e-3, step=1)
        kw.update(bad)
        with pytest.raises(B.Fp8lmError) as e:
            st.adam(B.adam_hparams(**kw))
        assert e.value.status == -1
    with pytest.raises(B.Fp8lmError) as e:      # no fused cast came before
        st.adam(B.adam_hparams(1e-3, 1, m_scale_mode=B.MSCALE_FROM_CAST))
    assert e.value.status == -1
    st.ctx.cast_fp8_for_adam(grad, st.g8, B.E5M2, st.g_meta, cfg, st.m, st.m_meta, 0.9)
    with pytest.raises(B.Fp8lmError):           # another beta1 than the cast measured for
        st.adam(B.adam_hparams(1e-3, 1, beta1=0.8, m_scale_mode=B.MSCALE_FROM_CAST))
    with pytest.raises(B.Fp8lmError):
        st.ctx.set_tuning(1000, 8, 8)
    for bad_cfg in (B.autoscale_cfg(hist_window=17), B.autoscale_cfg(sat_den=(1 << 24) + 1), B.autoscale_cfg(sat_den=0),
                    B.autoscale_cfg(ramp_steps=1), B.autoscale_cfg(mu_rule=2), B.autoscale_cfg(mu_rule=B.MU_HALVE, mu_min_exp=-65)):
        with pytest.raises(B.Fp8lmError) as e:
            st.ctx.amax_scale(grad, B.E5M2, st.g_meta, bad_cfg)
        assert e.value.status == -1


# ---- auto-scaling over many steps with heavy tails ----------------------------------------------------
def test_heavy_tailed_gradients_drive_the_mu_state_machine():
    """A scaled-down transformer layer with Student-t gradients and rare huge outliers, short ramp:
    overflow -> mu = 1/2 -> ramp -> saturation at mu = 2, metadata bit-exact along the way."""
    wl = synth.Workload("layer_small", synth.gpt_layout(384, 1, 1536, 0), lr=3e-5, grad_kind="student_t",
                        sigma=1e-4, steps=60, ramp_steps=20)
    st, tot = run_lockstep(wl, seed=7, steps=60, check_steps={1, 2, 3, 10, 11, 20, 21, 22, 23, 24, 40, 59, 60})
    gm = B.meta_to_numpy(st.g_meta, wl.layout.n_tensors)
    assert tot["m_diff"] == 0
    assert set(np.unique(gm["mu_exp"])) <= {-1, 0, 1}


def test_amax_history_window_carries_across_steps():
    wl = synth.Workload("hist", synth.gpt_layout(128, 2, 512, 500), lr=3e-4, sigma=None, hist_window=4)
    run_lockstep(wl, seed=9, steps=6)


# ---- single-pass variants: delayed gradient scaling and predicted first-moment scale ------------------
@pytest.mark.parametrize("grad_fmt", [B.E5M2, B.E4M3])
@pytest.mark.parametrize("m_scale_mode", [B.MSCALE_EXACT_PASS, B.MSCALE_PREDICTED, B.MSCALE_FROM_CAST])
def test_delayed_scaling_and_moment_scale_modes(grad_fmt, m_scale_mode):
    for wl in (synth.workload("tiny"), synth.Workload("mid", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None,
                                                      hist_window=2, ramp_steps=6)):
        st, w0 = P.make_state(wl, 11, grad_fmt)
        ids = list(range(wl.layout.n_tensors))
        grad = torch.zeros(max(wl.layout.total, 16), dtype=torch.bfloat16, device=DEV)
        for step in range(1, 8):
            synth.fill_gradients(grad, wl, 11, step)
            if step == 4:
                grad *= 4                                    # outgrows the history: the delayed cast clips
            if step == 6:
                bits = synth.bits16(grad).copy()
                off0, n0 = wl.layout.tensors()[0]
                bits[off0 + 5] = 0x7FC0                      # a NaN and an infinity nobody announced
                bits[off0 + n0 - 1] = 0xFF80
                grad = bf16_tensor_from_bits(bits)
            delayed = step > 1                               # the first step seeds the history just in time
            hp = B.adam_hparams(wl.lr, step, stats=1, m_scale_mode=m_scale_mode)
            snaps = [P.Snapshot(st, grad, t) for t in ids]
            say(f"{wl.name} fmt={grad_fmt} m_scale_mode={m_scale_mode} step={step} delayed={delayed}")
            st.step(grad, hp, delayed=delayed)
            torch.cuda.synchronize()
            r = P.check_step(st, snaps, hp, what=f"{wl.name} variants step {step}", delayed=delayed)
            assert r["m_diff"] == 0 and r["w_diff"] == 0 and r["q_diff"] == 0
            if step == 4:
                assert B.meta_to_numpy(st.g_meta, len(ids))["n_sat"].sum() > 0


# ---- shared-scale re-quantisation and the FP8 sum (Sec. 2.1, Eq. 4-6) on one GPU -------------------------
@pytest.mark.parametrize("fmt", [B.E5M2, B.E4M3])
def test_shared_scale_requantize_and_sum(fmt):
    n_ranks = 4
    wl = synth.Workload("ranks", synth.Layout(["a", "b", "c", "d", "e", "f", "g"], [70001, 1, 4096, 333, 0, 16385, 300000]),
                        lr=1e-3, sigma=None)
    lay = wl.layout
    cfg = B.autoscale_cfg(ramp_steps=20)
    ocfg = P.oracle_cfg(cfg)
    ctx = B.Context(lay.tensors())
    tens = O.tensors_array(lay.tensors())
    nt = lay.n_tensors
    d_q, d_meta, h_q, h_meta = [], [], [], []
    for r in range(n_ranks):
        grad = torch.zeros(lay.total, dtype=torch.bfloat16, device=DEV)
        synth.fill_gradients(grad, wl, 20 + r, 1)
        grad *= [1.0, 0.25, 8.0, 0.01][r]
        if r == 2:
            bits = synth.bits16(grad).copy()
            bits[lay.offsets[0] + 9] = 0x7FC0            # rank 2 contributes a NaN in tensor 0
            grad = bf16_tensor_from_bits(bits)
        meta = ctx.new_meta(cfg)
        q = torch.zeros(lay.total, dtype=torch.uint8, device=DEV)
        ctx.amax_scale(grad, fmt, meta, cfg)
        ctx.cast_fp8(grad, q, fmt, meta, cfg)
        d_q.append(q); d_meta.append(meta)
    torch.cuda.synchronize()
    h_q = [q.cpu().numpy() for q in d_q]
    h_meta = [B.meta_to_numpy(m, nt) for m in d_meta]
    say(f"requantize/sum fmt={fmt}")
    shared = ctx.shared_scale(d_meta)
    ref_shared = O.shared_scale(h_meta, nt)
    assert np.array_equal(shared.cpu().numpy()[:nt], ref_shared)
    d_rq, h_rq = [], []
    for r in range(n_ranks):
        out_meta = ctx.new_meta(cfg)
        before = B.meta_to_numpy(out_meta, nt)
        dst = d_q[r].clone() if r % 2 else torch.zeros_like(d_q[r])
        ctx.requantize_fp8(dst if r % 2 else d_q[r], fmt, d_meta[r], shared, dst, out_meta)     # odd ranks: in place
        torch.cuda.synchronize()
        ref = np.zeros(lay.total, dtype=np.uint8)
        ref_meta = before.copy()
        O.requantize_fp8(h_q[r], fmt, h_meta[r], ref_shared, tens, ref, ref_meta)
        got = dst.cpu().numpy()
        for t, (off, n) in enumerate(lay.tensors()):
            assert np.array_equal(got[off:off + n], ref[off:off + n]), (r, t)
            diff = P.meta_equal(B.meta_to_numpy(out_meta, nt)[t], ref_meta[t], P.ALL_FIELDS)
            assert not diff, (r, t, diff, B.meta_to_numpy(out_meta, nt)[t], ref_meta[t])
        d_rq.append(dst); h_rq.append(ref)
    for ranks in (n_ranks, 1, 3):
        out = torch.zeros(lay.total, dtype=torch.uint8, device=DEV)
        out_meta = ctx.new_meta(cfg)
        ref_meta = B.meta_to_numpy(out_meta, nt)
        ctx.sum_fp8(d_rq[:ranks], fmt, shared, out, out_meta, cfg)
        torch.cuda.synchronize()
        ref = np.zeros(lay.total, dtype=np.uint8)
        O.sum_fp8(h_rq[:ranks], fmt, ref_shared, tens, ref, ref_meta, ocfg)
        got = out.cpu().numpy()
        gm = B.meta_to_numpy(out_meta, nt)
        for t, (off, n) in enumerate(lay.tensors()):
            assert np.array_equal(got[off:off + n], ref[off:off + n]), (ranks, t)
            diff = P.meta_equal(gm[t], ref_meta[t], P.ALL_FIELDS)
            assert not diff, (ranks, t, diff, gm[t], ref_meta[t])
        if ranks >= 3:
            assert gm["flags"][0] & B.FLAG_NONFINITE


@pytest.mark.parametrize("fmt", [B.E5M2, B.E4M3])
@pytest.mark.parametrize("n_ranks", [9, 13, 128])
def test_sum_of_many_ranks(fmt, n_ranks):
    """More ranks than have a kernel of their own (the paper's communication study uses 128): shared scale and
    sum go through the kernels that loop over the ranks."""
    wl = synth.Workload("manyranks", synth.Layout(["a", "b", "c", "d"], [20001, 4096, 17, 50000]), lr=1e-3, sigma=None)
    lay = wl.layout
    cfg = B.autoscale_cfg(ramp_steps=20)
    ocfg = P.oracle_cfg(cfg)
    ctx = B.Context(lay.tensors())
    tens = O.tensors_array(lay.tensors())
    nt = lay.n_tensors
    size = max(lay.total, 16)
    d_q, d_meta = [], []
    grad = torch.zeros(size, dtype=torch.bfloat16, device=DEV)
    for r in range(n_ranks):
        synth.fill_gradients(grad, wl, 300 + r, 1)
        grad *= float(2.0 ** ((r * 7) % 5 - 2))               # ranks with different scales
        if r == n_ranks - 2:
            grad[lay.offsets[3] + 5] = float("nan")
        meta, q = ctx.new_meta(cfg), torch.zeros(size, dtype=torch.uint8, device=DEV)
        ctx.amax_scale(grad, fmt, meta, cfg)
        ctx.cast_fp8(grad, q, fmt, meta, cfg)
        d_q.append(q); d_meta.append(meta)
    say(f"sum of {n_ranks} ranks fmt={fmt}")
    shared = ctx.shared_scale(d_meta)
    h_meta = [B.meta_to_numpy(m, nt) for m in d_meta]
    ref_shared = O.shared_scale(h_meta, nt)
    assert np.array_equal(shared.cpu().numpy()[:nt], ref_shared)
    d_rq, h_rq = [], []
    for r in range(n_ranks):
        dst, out_meta = torch.zeros(size, dtype=torch.uint8, device=DEV), ctx.new_meta(cfg)
        ctx.requantize_fp8(d_q[r], fmt, d_meta[r], shared, dst, out_meta)
        ref, ref_meta = np.zeros(size, dtype=np.uint8), O.new_meta(nt, ocfg)
        O.requantize_fp8(d_q[r].cpu().numpy(), fmt, h_meta[r], ref_shared, tens, ref, ref_meta)
        d_rq.append(dst); h_rq.append(ref)
    out, out_meta = torch.zeros(size, dtype=torch.uint8, device=DEV), ctx.new_meta(cfg)
    ref_meta = B.meta_to_numpy(out_meta, nt)
    ctx.sum_fp8(d_rq, fmt, shared, out, out_meta, cfg)
    torch.cuda.synchronize()
    for r in range(n_ranks):
        assert np.array_equal(d_rq[r].cpu().numpy(), h_rq[r]), r
    ref = np.zeros(size, dtype=np.uint8)
    O.sum_fp8(h_rq, fmt, ref_shared, tens, ref, ref_meta, ocfg)
    got, gm = out.cpu().numpy(), B.meta_to_numpy(out_meta, nt)
    for t, (off, n) in enumerate(lay.tensors()):
        assert np.array_equal(got[off:off + n], ref[off:off + n]), t
        diff = P.meta_equal(gm[t], ref_meta[t], P.ALL_FIELDS)
        assert not diff, (t, diff, gm[t], ref_meta[t])
    assert gm["flags"][3] & B.FLAG_NONFINITE
    with pytest.raises(B.Fp8lmError):
        ctx.sum_fp8(d_rq + d_rq[:129 - n_ranks] if n_ranks == 128 else [d_rq[0]] * 129, fmt, shared, out, out_meta, cfg)


@pytest.mark.parametrize("n_ranks", [3, 4])
def test_summed_gradient_feeds_the_adam_step(n_ranks):
    """The data-parallel chain end to end on one GPU (Sec. 2.1 Eq. 4-6, then Sec. 2.2): every rank casts its own
    gradient, shared scale, re-quantisation, FP8 sum with scale N * s_g (no power of two for N = 3, so the Adam
    kernels dequantise with a rounded reciprocal), Adam step on the sum with the sum's metadata, and the sum's
    auto-scaling state handed back to the ranks for the next step.  Three steps, every byte against the same chain
    on the oracle."""
    fmt = B.E5M2
    wl = synth.Workload("join", synth.Layout(["a", "b", "c", "d", "e", "f"], [70001, 1, 4096, 333, 0, 16385]), lr=1e-3,
                        sigma=None, ramp_steps=4)
    lay = wl.layout
    nt, size = lay.n_tensors, max(lay.total, 16)
    st, w0 = P.make_state(wl, 17, fmt, ramp_steps=4)
    cfg, ocfg, ctx = st.cfg, P.oracle_cfg(st.cfg), st.ctx
    tens = O.tensors_array(lay.tensors())
    # the oracle's own state
    o = dict(m=np.zeros(size, np.uint8), v=np.zeros(size, np.uint16), w=np.zeros(size, np.uint16), wq=np.zeros(size, np.uint8),
             g8=np.zeros(size, np.uint8))
    om = {k: O.new_meta(nt, ocfg) for k in ("sum", "m", "v", "w", "q")}
    O.init_master(synth.bits16(w0), tens, o["w"], om["w"])
    o_rank_meta = [O.new_meta(nt, ocfg) for _ in range(n_ranks)]
    d_rank_meta = [ctx.new_meta(cfg) for _ in range(n_ranks)]
    d_sum_meta = ctx.new_meta(cfg)
    d_pay = [torch.zeros(size, dtype=torch.uint8, device=DEV) for _ in range(n_ranks)]
    scratch_meta = ctx.new_meta(cfg)
    grad = torch.zeros(size, dtype=torch.bfloat16, device=DEV)
    for step in range(1, 4):
        hp = B.adam_hparams(wl.lr, step)
        o_pay = []
        ctx.autoscale_broadcast(d_sum_meta, d_rank_meta)
        for r in range(n_ranks):
            synth.fill_gradients(grad, wl, 170 + r, step)
            grad *= [1.0, 0.25, 8.0, 0.5][r]
            ctx.amax_scale(grad, fmt, d_rank_meta[r], cfg)
            ctx.cast_fp8(grad, d_pay[r], fmt, d_rank_meta[r], cfg)
            bits = synth.bits16(grad)
            o_rank_meta[r]["mu_exp"], o_rank_meta[r]["clean_steps"] = om["sum"]["mu_exp"], om["sum"]["clean_steps"]
            q = np.zeros(size, np.uint8)
            O.amax_scale(bits, tens, fmt, o_rank_meta[r], ocfg)
            O.cast_fp8(bits, tens, q, fmt, o_rank_meta[r], ocfg)
            o_pay.append(q)
        say(f"join of Eq. 4-6 and the Adam step: {n_ranks} ranks, step {step}")
        shared = ctx.shared_scale(d_rank_meta)
        for r in range(n_ranks):
            ctx.requantize_fp8(d_pay[r], fmt, d_rank_meta[r], shared, d_pay[r], scratch_meta)
        ctx.sum_fp8(d_pay, fmt, shared, st.g8, d_sum_meta, cfg)
        if step == 1:
            with pytest.raises(B.Fp8lmError):            # no fused cast has seen this gradient
                ctx.adam_step_fp8(st.g8, fmt, d_sum_meta, st.m, st.m_meta, st.v, st.v_meta, st.w, st.w_meta, st.wq, st.q_meta,
                                  B.adam_hparams(wl.lr, step, m_scale_mode=B.MSCALE_FROM_CAST))
        ctx.adam_step_fp8(st.g8, fmt, d_sum_meta, st.m, st.m_meta, st.v, st.v_meta, st.w, st.w_meta, st.wq, st.q_meta, hp)
        torch.cuda.synchronize()
        o_shared = O.shared_scale(o_rank_meta, nt)
        for r in range(n_ranks):
            O.requantize_fp8(o_pay[r], fmt, o_rank_meta[r], o_shared, tens, o_pay[r], O.new_meta(nt, ocfg))
        O.sum_fp8(o_pay, fmt, o_shared, tens, o["g8"], om["sum"], ocfg)
        O.adam_step_fp8(tens, o["g8"], fmt, om["sum"], o["m"], om["m"], o["v"], om["v"], o["w"], om["w"], o["wq"], om["q"],
                        P.oracle_hp(hp))
        if n_ranks == 3:
            assert not np.any(np.log2(om["sum"]["scale"][[0, 2, 3, 5]]) % 1 == 0)       # not powers of two
        got_meta = {k: B.meta_to_numpy(t, nt) for k, t in (("sum", d_sum_meta), ("m", st.m_meta), ("v", st.v_meta),
                                                           ("w", st.w_meta), ("q", st.q_meta))}
        for t, (off, n) in enumerate(lay.tensors()):
            for name, dev_buf in (("g8", st.g8), ("m", st.m), ("v", st.v), ("w", st.w), ("wq", st.wq)):
                assert np.array_equal(P._host_bits(dev_buf, off, n), o[name][off:off + n]), (step, t, name)
            if n:
                bad = P.meta_equal(got_meta["sum"][t], om["sum"][t], P.ALL_FIELDS)
                assert not bad, (step, t, bad, got_meta["sum"][t], om["sum"][t])
                for k in ("m", "v", "w", "q"):
                    bad = P.meta_equal(got_meta[k][t], om[k][t], ["scale", "inv_scale", "amax", "amax_deq", "flags"])
                    assert not bad, (step, t, k, bad, got_meta[k][t], om[k][t])
    # the hand-over moved the state of the sum into every rank, and only that
    rm = B.meta_to_numpy(d_rank_meta[0], nt)
    assert np.array_equal(rm["scale"], o_rank_meta[0]["scale"]) and np.array_equal(rm["amax_hist"], o_rank_meta[0]["amax_hist"])


# ---- storage formats of the precision-decoupling study (Sec. 2.2; Sec. 3.3) ----------------------------
# every pair but the default one (scaled FP16 for both), which all the other tests cover
@pytest.mark.parametrize("master_fmt,v_fmt", [(mf, vf) for vf in (B.STATE_F16, B.STATE_E4M3)
                                              for mf in (B.STATE_F16, B.STATE_BF16, B.STATE_E4M3, B.STATE_F32)
                                              if (mf, vf) != (B.STATE_F16, B.STATE_F16)])
def test_master_weight_and_second_moment_formats(master_fmt, v_fmt):
    for wl, grad_fmt in ((synth.workload("tiny"), B.E5M2),
                         (synth.Workload("mid", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None), B.E4M3)):
        st, w0 = P.make_state(wl, 13, grad_fmt, master_fmt=master_fmt, v_fmt=v_fmt)
        ids = list(range(wl.layout.n_tensors))
        P.check_init_master(st, w0, ids)
        grad = torch.zeros(max(wl.layout.total, 16), dtype=torch.bfloat16, device=DEV)
        for step in range(1, 5):
            synth.fill_gradients(grad, wl, 13, step)
            if step == 3:                                    # a NaN and an infinity: the careful path of every format
                bits = synth.bits16(grad).copy()
                off0, n0 = wl.layout.tensors()[0]
                bits[off0 + 3] = 0x7FC0
                bits[off0 + n0 - 2] = 0x7F80
                grad = bf16_tensor_from_bits(bits)
            mode = [B.MSCALE_EXACT_PASS, B.MSCALE_PREDICTED, B.MSCALE_FROM_CAST][step % 3]
            hp = B.adam_hparams(wl.lr, step, master_fmt=master_fmt, v_fmt=v_fmt, m_scale_mode=mode)
            snaps = [P.Snapshot(st, grad, t) for t in ids]
            say(f"{wl.name} master_fmt={master_fmt} v_fmt={v_fmt} step={step} mode={mode}")
            st.step(grad, hp)
            torch.cuda.synchronize()
            P.check_step(st, snaps, hp, what=f"{wl.name} formats step {step}")
    with pytest.raises(B.Fp8lmError):                        # counters are not available for these formats
        st.adam(B.adam_hparams(1e-3, 9, master_fmt=master_fmt, v_fmt=v_fmt, stats=1))


# ---- fp16 and fp32 gradient sources ---------------------------------------------------------------------
def _interesting_f32(fmt):
    """fp32 values that decide roundings: every FP8 value, every midpoint between neighbours, each one fp32
    step up and down, the same around the saturation point, zeros, subnormals and the largest floats."""
    table = O.decode_table(fmt)
    vals = np.unique(np.abs(table[np.isfinite(table)])).astype(np.float32)
    mids = ((vals[:-1].astype(np.float64) + vals[1:].astype(np.float64)) / 2).astype(np.float32)
    top = vals[-1]
    base = np.concatenate([vals, mids, [top * 1.03125, top * 1.0625, top * 2, 3.0e38, 1e-45, 1e-40, 1.17549435e-38]])
    base = base.astype(np.float32)
    up = np.nextafter(base, np.float32(np.inf))
    down = np.nextafter(base, np.float32(0))
    mag = np.concatenate([base, up, down])
    return np.concatenate([mag, -mag]).astype(np.float32)


@pytest.mark.parametrize("fmt", [B.E5M2, B.E4M3])
@pytest.mark.parametrize("kind", [B.SRC_F16, B.SRC_F32])
def test_cast_wide_sources_under_many_scales(fmt, kind):
    rng = np.random.default_rng(5)
    if kind == B.SRC_F16:
        pats = np.arange(65536, dtype=np.uint16)
        finite = pats[(pats & 0x7C00) != 0x7C00]
        everything = pats
        exps = [-126, -60, -24, -15, -14, -9, -8, -3, -1, 0, 1, 2, 7, 8, 9, 15, 16, 17, 24, 25, 40, 126]
        np_dtype, t_dtype = np.uint16, torch.float16
    else:
        special = _interesting_f32(fmt)
        rnd = rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32)
        everything = np.concatenate([special.view(np.uint32), rnd, np.array([0x7F800000, 0xFF800000, 0x7FC00000, 0xFFFFFFFF], np.uint32)])
        finite = everything[(everything & 0x7F800000) != 0x7F800000]
        exps = [-126, -100, -30, -9, -8, -1, 0, 1, 3, 8, 15, 16, 30, 100, 126]
        np_dtype, t_dtype = np.uint32, torch.float32
    n_fast = len(exps)
    numels = [finite.size] * n_fast + [everything.size] * 3
    lay = synth.Layout([f"t{i}" for i in range(len(numels))], numels)
    src = np.zeros(lay.total, dtype=np_dtype)
    for i, (off, n) in enumerate(lay.tensors()):
        src[off:off + n] = finite if i < n_fast else everything
    cfg = B.autoscale_cfg()
    ctx = B.Context(lay.tensors())
    meta = B.meta_to_numpy(ctx.new_meta(cfg), lay.n_tensors)
    for i, e in enumerate(exps + [0, -12, 9]):
        meta["scale"][i] = 2.0 ** e
        meta["inv_scale"][i] = 2.0 ** -e
        if i >= n_fast:
            meta["flags"][i] = B.FLAG_NONFINITE
    d_src = torch.from_numpy(src.view(np.int16 if kind == B.SRC_F16 else np.int32).copy()).to(DEV).view(t_dtype)
    o_src = src.view(np.float32) if kind == B.SRC_F32 else src
    tens = O.tensors_array(lay.tensors())
    # 1. the cast alone with the scales planted above (fast path and careful path)
    ref_meta = meta.copy()
    d_meta = B.meta_from_numpy(meta, DEV)
    d_dst = torch.zeros(lay.total, dtype=torch.uint8, device=DEV)
    say(f"wide-source cast sweep fmt={fmt} kind={kind} tensors={lay.n_tensors} elements={lay.total}")
    ctx.cast_fp8(d_src, d_dst, fmt, d_meta, cfg)
    torch.cuda.synchronize()
    ref = np.zeros(lay.total, dtype=np.uint8)
    O.cast_fp8(o_src, tens, ref, fmt, ref_meta, P.oracle_cfg(cfg), src_type=kind)
    got = d_dst.cpu().numpy()
    bad = np.flatnonzero(got != ref)
    assert bad.size == 0, f"{bad.size} codes differ, first at {bad[:5]}: gpu {got[bad[:5]]} oracle {ref[bad[:5]]} src {src[bad[:5]]}"
    got_meta = B.meta_to_numpy(d_meta, lay.n_tensors)
    for t in range(lay.n_tensors):
        diff = P.meta_equal(got_meta[t], ref_meta[t], P.ALL_FIELDS)
        assert not diff, (t, diff, got_meta[t], ref_meta[t])
    # 2. amax + scale + cast, and the delayed single pass, from fresh metadata
    for delayed in (False, True):
        ref_meta = B.meta_to_numpy(ctx.new_meta(cfg), lay.n_tensors)
        d_meta = B.meta_from_numpy(ref_meta, DEV)
        for rep in range(2):
            say(f"  delayed={delayed} rep={rep}")
            if delayed:
                ctx.cast_fp8_delayed(d_src, d_dst, fmt, d_meta, cfg)
                O.cast_fp8_delayed(o_src, tens, ref, fmt, ref_meta, P.oracle_cfg(cfg), src_type=kind)
            else:
                ctx.amax_scale(d_src, fmt, d_meta, cfg)
                ctx.cast_fp8(d_src, d_dst, fmt, d_meta, cfg)
                O.amax_scale(o_src, tens, fmt, ref_meta, P.oracle_cfg(cfg), src_type=kind)
                O.cast_fp8(o_src, tens, ref, fmt, ref_meta, P.oracle_cfg(cfg), src_type=kind)
            torch.cuda.synchronize()
            assert np.array_equal(d_dst.cpu().numpy(), ref)
            got_meta = B.meta_to_numpy(d_meta, lay.n_tensors)
            for t in range(lay.n_tensors):
                diff = P.meta_equal(got_meta[t], ref_meta[t], P.ALL_FIELDS)
                assert not diff, (delayed, rep, t, diff, got_meta[t], ref_meta[t])


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("grad_fmt", [B.E5M2, B.E4M3])
def test_whole_path_from_fp16_and_fp32_gradients(dtype, grad_fmt):
    for wl in (synth.workload("tiny"), synth.Workload("mid", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None)):
        st, w0 = P.make_state(wl, 21, grad_fmt, hist_window=2)
        ids = list(range(wl.layout.n_tensors))
        grad = torch.zeros(max(wl.layout.total, 16), dtype=dtype, device=DEV)
        for step in range(1, 7):
            synth.fill_gradients(grad, wl, 21, step)
            if step == 4:                                        # inf and NaN in the first tensor
                off0, n0 = wl.layout.tensors()[0]
                grad[off0 + 1] = float("inf")
                grad[off0 + n0 - 1] = float("nan")
            delayed = step in (3, 4, 6)
            mode = [B.MSCALE_EXACT_PASS, B.MSCALE_PREDICTED, B.MSCALE_FROM_CAST][step % 3]
            hp = B.adam_hparams(wl.lr, step, m_scale_mode=mode)
            snaps = [P.Snapshot(st, grad, t) for t in ids]
            say(f"{wl.name} dtype={dtype} fmt={grad_fmt} step={step} delayed={delayed} mode={mode}")
            st.step(grad, hp, delayed=delayed)
            torch.cuda.synchronize()
            P.check_step(st, snaps, hp, what=f"{wl.name} {dtype} step {step}", delayed=delayed)


# ---- quantisation-error statistics and the three all-reduce scaling strategies (Sec. 3.3) -------------------
def _stats_close(got, ref, n):
    for k in ("n_nonzero", "n_underflow", "n_overflow", "n_nonfinite"):
        assert got[k] == ref[k], (k, got, ref)
    tol = max(n, 1) * 2.0 ** -52 * 4                          # float64 sums of non-negative terms in another order
    for k in ("signal", "noise"):
        assert abs(got[k] - ref[k]) <= tol * abs(ref[k]), (k, got, ref)


@pytest.mark.parametrize("fmt", [B.E5M2, B.E4M3])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16, torch.float32])
def test_quant_error_stats_match_the_oracle(fmt, dtype):
    wl = synth.workload("tiny")
    lay = wl.layout
    cfg = B.autoscale_cfg()
    ctx = B.Context(lay.tensors())
    ref = torch.zeros(max(lay.total, 16), dtype=dtype, device=DEV)
    synth.fill_gradients(ref, wl, 3, 1)
    off0, n0 = next((o, n) for o, n in lay.tensors() if n > 40)
    ref[off0 + 2] = float("nan")
    ref[off0 + 5] = float("inf")
    ref[off0 + 9: off0 + 20] = 0
    meta = ctx.new_meta(cfg)
    q = torch.zeros(max(lay.total, 16), dtype=torch.uint8, device=DEV)
    src = ref.clone()
    src[off0 + 2] = 1.0                                       # the payload differs from the reference here
    src[off0 + 30] = float("nan")                             # ... and is a NaN code here
    ctx.amax_scale(src, fmt, meta, cfg)
    hm = B.meta_to_numpy(meta, lay.n_tensors)
    hm["mu_exp"][:] = 1                                       # mu = 2: some payloads sit on the top code
    meta = B.meta_from_numpy(hm, DEV)
    ctx.amax_scale(src, fmt, meta, cfg)
    ctx.cast_fp8(src, q, fmt, meta, cfg)
    say(f"quant stats fmt={fmt} dtype={dtype}")
    got = ctx.quant_error_stats(ref, q, fmt, meta)
    again = ctx.quant_error_stats(ref, q, fmt, meta)
    assert got.tobytes() == again.tobytes()                   # the float64 sums are reproducible, bit for bit
    kind = B.src_type_of(ref)
    h_ref = P._host_bits(ref, 0, ref.numel())
    if kind == B.SRC_F32:
        h_ref = h_ref.view(np.float32)
    want = O.quant_error_stats(h_ref, q.cpu().numpy(), fmt, B.meta_to_numpy(meta, lay.n_tensors),
                               O.tensors_array(lay.tensors()), ref_type=kind)
    for t, (_, n) in enumerate(lay.tensors()):
        _stats_close(got[t], want[t], n)
    assert got["n_overflow"].sum() > 0 and got["n_nonfinite"].sum() == 3 and got["n_underflow"].sum() >= 0


@pytest.mark.parametrize("fmt", [B.E4M3, B.E5M2])
def test_allreduce_strategies_match_the_oracle_and_order_as_the_ablation_says(fmt):
    from paper_2310_18313_amd.allreduce_study import Fp8AllReduce, report
    n_ranks, steps = 4, 6
    lay = synth.Layout(["a", "b", "c", "d"], [70001, 4096, 333, 150000])
    wl = synth.Workload("study", lay, lr=1e-3, sigma=1e-3, grad_kind="student_t", ramp_steps=4)
    cfg = B.autoscale_cfg(ramp_steps=4)
    ocfg = P.oracle_cfg(cfg)
    tens = O.tensors_array(lay.tensors())
    ctx = B.Context(lay.tensors())
    size = max(lay.total, 16)
    grads = [torch.zeros(size, dtype=torch.float32, device=DEV) for _ in range(n_ranks)]
    final = {}
    for strategy in ("pre", "post", "auto"):
        ar = Fp8AllReduce(ctx, n_ranks, lay.total, fmt, cfg, strategy)
        o_meta = [O.new_meta(lay.n_tensors, ocfg) for _ in range(n_ranks)]
        o_sum_meta = O.new_meta(lay.n_tensors, ocfg)
        for step in range(1, steps + 1):
            for r in range(n_ranks):
                synth.fill_gradients(grads[r], wl, 100 + r, step)
            mean = torch.stack(grads).sum(dim=0) / n_ranks
            say(f"all-reduce study fmt={fmt} strategy={strategy} step={step}")
            ar.step(grads)
            got = ar.error_stats(mean)
            torch.cuda.synchronize()
            # the same sequence on the oracle
            h = [g.cpu().numpy() for g in grads]
            o_pay, o_shared_pay, o_shared_meta = [], [], []
            for r in range(n_ranks):
                if strategy == "auto":
                    o_meta[r]["mu_exp"], o_meta[r]["clean_steps"] = o_sum_meta["mu_exp"], o_sum_meta["clean_steps"]
                else:
                    o_meta[r]["mu_exp"] = -2 if strategy == "pre" else 0
                qr = np.zeros(size, dtype=np.uint8)
                O.amax_scale(h[r], tens, fmt, o_meta[r], ocfg, src_type=O.SRC_F32)
                O.cast_fp8(h[r], tens, qr, fmt, o_meta[r], ocfg, src_type=O.SRC_F32)
                o_pay.append(qr)
            shared = O.shared_scale(o_meta, lay.n_tensors)
            for r in range(n_ranks):
                q2, m2 = np.zeros(size, dtype=np.uint8), O.new_meta(lay.n_tensors, ocfg)
                O.requantize_fp8(o_pay[r], fmt, o_meta[r], shared, tens, q2, m2)
                o_shared_pay.append(q2)
            o_sum = np.zeros(size, dtype=np.uint8)
            O.sum_fp8(o_shared_pay, fmt, shared, tens, o_sum, o_sum_meta, ocfg)
            want = O.quant_error_stats(mean.cpu().numpy(), o_sum, fmt, o_sum_meta, tens)
            assert np.array_equal(ar.summed.cpu().numpy(), o_sum), f"{strategy} step {step}: summed payload differs"
            gm = B.meta_to_numpy(ar.summed_meta, lay.n_tensors)
            for t, (_, n) in enumerate(lay.tensors()):
                bad = P.meta_equal(gm[t], o_sum_meta[t], ["scale", "inv_scale", "amax_deq", "mu_exp", "clean_steps", "n_sat", "flags"])
                assert not bad, (strategy, step, t, bad, gm[t], o_sum_meta[t])
                _stats_close(got[t], want[t], n)
        final[strategy] = report(got, lay.numels)
        say(f"  {strategy}: {final[strategy]}")
    # what the ablation observes: dividing first loses small entries, summing first clips.  E5M2 spans 32
    # binades, so with these inputs nothing leaves its range at the bottom: the zeros it stores for non-zero
    # means are ranks cancelling exactly after rounding to two mantissa bits, the same under every strategy.
    if fmt == B.E4M3:
        assert final["pre"]["underflow_rate"] > final["post"]["underflow_rate"]
    assert final["pre"]["underflow_rate"] >= final["post"]["underflow_rate"]
    assert final["post"]["overflow_rate"] >= final["pre"]["overflow_rate"]
    assert final["pre"]["underflow_rate"] >= final["auto"]["underflow_rate"]


# ---- the entry points can be recorded into a HIP graph ---------------------------------------------------------
@pytest.mark.parametrize("grad_fmt,route", [(B.E5M2, "jit"), (B.E4M3, "spec"), (B.E5M2, "static"), (B.E5M2, "predicted")])
def test_weight_copy_written_over_the_fp8_gradient(grad_fmt, route):
    """wcopy == grad (the E4M3 weight copy takes the place of the gradient it was computed from): the buffer must hold
    the bytes that a separate copy buffer holds, everything else must be untouched by the sharing; the state with
    two buffers is held to the oracle lock-step.  Ragged sizes (tails, one-element and empty tensors), a careful
    tensor (NaN planted), every route into the update pass."""
    from paper_2310_18313_amd.state import OptimizerState
    lay = synth.Layout(["a", "b", "c", "d", "e", "f", "g"], [70001, 1, 4096, 333, 0, 16385, 300017])
    wl = synth.Workload("alias", lay, lr=1e-3, sigma=None, ramp_steps=4)
    two, w0 = P.make_state(wl, 31, grad_fmt, B.WCOPY_E4M3)
    one = OptimizerState(lay.tensors(), lay.total, two.cfg, 0, grad_fmt, B.WCOPY_E4M3, wcopy_over_grad=True)
    assert one.wq.data_ptr() == one.g8.data_ptr()
    one.init_master(w0)
    ids = list(range(lay.n_tensors))
    grad = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    mode = B.MSCALE_PREDICTED if route == "predicted" else B.MSCALE_EXACT_PASS
    for step in range(1, 6):
        synth.fill_gradients(grad, wl, 31, step)
        if step == 3:
            grad[lay.tensors()[5][0] + 99] = float("nan")
        hp = B.adam_hparams(wl.lr, step, stats=step % 2, m_scale_mode=mode)
        snaps = [P.Snapshot(two, grad, t) for t in ids]
        say(f"weight copy over the gradient: fmt={grad_fmt} route={route} step={step}")
        two.step(grad, hp, speculative=(route == "spec"))
        if route == "static":
            one.quantize_grad(grad)
            B.adam_step_fp8_static(lay.tensors(), one.g8, grad_fmt, one.g_meta, one.m, one.m_meta, one.v, one.v_meta,
                                   one.w, one.w_meta, one.g8, one.q_meta, hp)
        else:
            one.step(grad, hp, speculative=(route == "spec"))
        torch.cuda.synchronize()
        P.check_step(two, snaps, hp, what=f"two buffers, step {step}")
        for k in ("m", "v", "w", "wq", "g_meta", "m_meta", "v_meta", "w_meta", "q_meta"):
            a, b = getattr(two, k), getattr(one, k)
            if a.element_size() == 2:
                a, b = a.view(torch.int16), b.view(torch.int16)
            assert torch.equal(a, b), (step, k)
    # a bf16 copy does not fit the gradient's buffer; the step with a pair of moment buffers reads the gradient twice
    big = torch.zeros(2 * one.g8.numel(), dtype=torch.uint8, device=DEV)
    with pytest.raises(B.Fp8lmError):
        one.ctx.adam_step_fp8(big[:one.g8.numel()], grad_fmt, one.g_meta, one.m, one.m_meta, one.v, one.v_meta, one.w,
                              one.w_meta, big.view(torch.bfloat16), one.q_meta, B.adam_hparams(wl.lr, 9, wcopy=B.WCOPY_BF16))
    with pytest.raises(B.Fp8lmError):
        one.ctx.adam_step_fp8_m2(one.g8, grad_fmt, one.g_meta, one.m, two.m, one.m_meta, one.v, one.v_meta, one.w,
                                 one.w_meta, one.g8, one.q_meta, B.adam_hparams(wl.lr, 9))


def test_region_aware_placement_changes_no_result():
    """OptimizerState(spread=True): where the buffers lie is decided by timing (placement.RegionAllocator); what the
    kernels compute must not depend on it.  A state of 0.5e9 parameters placed that way and one carved out of a plain
    arena step side by side and must hold the same bytes; if the allocator reports the two groups apart, the check
    that bench.py prints must agree."""
    from paper_2310_18313_amd.placement import verify_spread
    from paper_2310_18313_amd.state import OptimizerState
    lay = synth.Layout(["a", "b", "c"], [250_000_017, 4097, 250_000_000])
    wl = synth.Workload("placed", lay, lr=1e-3, sigma=None, ramp_steps=4)
    cfg = B.autoscale_cfg(ramp_steps=4)
    placed = OptimizerState(lay.tensors(), lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3, spread=True, grad_buffer=True)
    say(f"region-aware placement: {placed.placement}")
    for t in (placed.v, placed.w, placed.m, placed.g8, placed.wq, placed.grad):
        assert int(t.view(torch.uint8).max()) == 0              # handed over as zeros, whatever the probes wrote
    if placed.spread:
        where = placed.placement["where"]
        assert placed.placement["traffic_share_busiest"] <= 0.8 + 1e-6
        if set(where["v"]) == {"0"} and set(where["w"]) == {"1"}:      # v and w as wholes in different regions
            chk = verify_spread(placed.ctx, placed.v, placed.w)
            assert chk["distinct"], chk
            placed.v.zero_()
            placed.w.zero_()
    plain = OptimizerState(lay.tensors(), lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3)
    synth.fill_weights(placed.grad, lay, 3)
    placed.init_master(placed.grad)
    plain.init_master(placed.grad)
    for step in (1, 2):
        synth.fill_gradients(placed.grad, wl, 3, step)
        hp = B.adam_hparams(wl.lr, step)
        placed.step(placed.grad, hp, speculative=True)
        plain.step(placed.grad, hp, speculative=True)
        torch.cuda.synchronize()
        for k in ("g8", "m", "v", "w", "wq", "g_meta", "m_meta", "v_meta", "w_meta", "q_meta"):
            a, b = getattr(placed, k), getattr(plain, k)
            if a.element_size() == 2:
                a, b = a.view(torch.int16), b.view(torch.int16)
            assert torch.equal(a, b), (step, k)


def test_striped_arena_is_ordinary_memory_and_gives_it_back():
    """placement.StripedArena (pieces of device memory mapped into one address range in alternating order): what it
    hands out must behave like any allocation -- zeroed, writable through views, usable by the kernels -- and the
    device must have its memory back once the last view is gone.  Whether two regions could be found depends on what
    the process holds already; if not, the constructor must say so with a RuntimeError and leave nothing behind."""
    import gc
    from paper_2310_18313_amd.placement import StripedArena
    gc.collect()
    torch.cuda.empty_cache()
    lay = synth.Layout(["a"], [1 << 20])
    ctx = B.Context(lay.tensors())
    free0 = torch.cuda.mem_get_info(0)[0]
    nbytes = 6 << 30
    try:
        arena = StripedArena(ctx, nbytes)
    except RuntimeError as e:
        say(f"striped arena not built: {e}")
        assert str(e)
        gc.collect()
        assert torch.cuda.mem_get_info(0)[0] >= free0 - (64 << 20)
        return
    say(f"striped arena: {arena.log}")
    assert arena.nbytes >= nbytes and 0.25 <= arena.log["share_outside_first_region"] <= 0.75
    a, b = arena.tensor(0, 1 << 30), arena.tensor((3 << 30) - 4096, 8192, torch.int16)       # b lies across two pieces
    assert int(arena.bytes.max()) == 0
    b.fill_(-2)
    a[:16] = 7
    assert int(arena.bytes[(3 << 30) - 4096:(3 << 30) + 4096].view(torch.int16).min()) == -2
    assert int(arena.bytes[:16].sum()) == 112 and int(arena.bytes[16:(3 << 30) - 4096].max()) == 0
    # the kernels take it like any buffer: a cast into it equals a cast into a plain buffer
    wl = synth.Workload("striped", lay, lr=1e-3, sigma=None, ramp_steps=4)
    cfg = B.autoscale_cfg()
    grad = torch.zeros(lay.total, dtype=torch.bfloat16, device=DEV)
    synth.fill_gradients(grad, wl, 5, 1)
    q_plain, m_plain = torch.zeros(lay.total, dtype=torch.uint8, device=DEV), ctx.new_meta(cfg)
    q_striped, m_striped = arena.tensor((1 << 30) - (1 << 19), lay.total), ctx.new_meta(cfg)
    for q, m in ((q_plain, m_plain), (q_striped, m_striped)):
        ctx.amax_scale(grad, B.E5M2, m, cfg)
        ctx.cast_fp8(grad, q, B.E5M2, m, cfg)
    torch.cuda.synchronize()
    assert torch.equal(q_plain, q_striped) and torch.equal(m_plain, m_striped)
    held = free0 - torch.cuda.mem_get_info(0)[0]
    assert held >= nbytes
    del a, b, q, q_striped, arena                      # every view keeps the mappings alive
    gc.collect()
    assert torch.cuda.mem_get_info(0)[0] >= free0 - (64 << 20) - 2 * lay.total - (1 << 20)


def test_a_step_replayed_from_a_hip_graph_equals_the_eager_step():
    """None of the hot-path calls synchronises, allocates or clears memory with a memset, so a whole step can be
    captured once and replayed; the hyper-parameters are baked in at capture, so every replay is the same step."""
    wl = synth.Workload("mid", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None)
    st, _ = P.make_state(wl, 31)
    grad = torch.zeros(max(wl.layout.total, 16), dtype=torch.bfloat16, device=DEV)
    for step in (1, 2):                                          # some history first
        synth.fill_gradients(grad, wl, 31, step)
        st.step(grad, B.adam_hparams(wl.lr, step))
    synth.fill_gradients(grad, wl, 31, 3)
    hp = B.adam_hparams(wl.lr, 3)
    names = ("g8", "m", "v", "w", "wq", "g_meta", "m_meta", "v_meta", "w_meta", "q_meta")
    before = {k: getattr(st, k).clone() for k in names}
    st.step(grad, hp)                                            # eager reference
    torch.cuda.synchronize()
    want = {k: getattr(st, k).clone() for k in names}

    def restore():
        for k in names:
            getattr(st, k).copy_(before[k])

    restore()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    say("capturing one step into a HIP graph")
    with torch.cuda.graph(graph, stream=side):
        st.step(grad, hp)
    torch.cuda.synchronize()
    for rep in range(3):
        restore()                                                # eager work between the replays
        torch.cuda.synchronize()
        say(f"graph replay {rep}")
        graph.replay()
        torch.cuda.synchronize()
        for k in names:
            assert torch.equal(getattr(st, k), want[k]), f"replay {rep}: {k} differs from the eager step"


# ---- parameter groups: one context per group over the same flat buffers ---------------------------------------
def test_parameter_groups_share_the_flat_buffers():
    """Weight decay on the matrices, none on biases and LayerNorm weights: two tensor lists, two contexts, the
    same buffers.  Every tensor must come out as the oracle computes it with its own group's hyper-parameters,
    and no group may touch the other's elements."""
    wl = synth.Workload("groups", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None)
    lay = wl.layout
    decay = [i for i, nm in enumerate(lay.names) if nm.endswith(".w") and "ln" not in nm or nm == "emb"]
    plain = [i for i in range(lay.n_tensors) if i not in decay]
    assert decay and plain
    cfg = B.autoscale_cfg()
    tens = lay.tensors()
    st_d = OptimizerState([tens[i] for i in decay], lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3)
    st_p = OptimizerState([tens[i] for i in plain], lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3, share_with=st_d)
    w0 = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    synth.fill_weights(w0, lay, 17)
    st_d.init_master(w0)
    st_p.init_master(w0)
    grad = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    for step in (1, 2, 3):
        synth.fill_gradients(grad, wl, 17, step)
        hp_d = B.adam_hparams(wl.lr, step, weight_decay=0.1)
        hp_p = B.adam_hparams(wl.lr, step, weight_decay=0.0)
        snaps_d = [P.Snapshot(st_d, grad, t) for t in range(len(decay))]
        snaps_p = [P.Snapshot(st_p, grad, t) for t in range(len(plain))]
        say(f"parameter groups step {step}: {len(decay)} + {len(plain)} tensors")
        st_d.step(grad, hp_d)
        st_p.step(grad, hp_p)
        torch.cuda.synchronize()
        P.check_step(st_d, snaps_d, hp_d, what=f"decay group step {step}")
        P.check_step(st_p, snaps_p, hp_p, what=f"no-decay group step {step}")


@pytest.mark.parametrize("master_fmt,exact", [(B.STATE_F16, 1), (B.STATE_F16, 0), (B.STATE_BF16, 1)])
def test_weight_decay_exemption_by_tensor_flag(master_fmt, exact):
    """One context, one launch: tensors flagged TENSOR_NO_WEIGHT_DECAY (biases, LayerNorm weights) must come out as
    the oracle computes them with weight_decay = 0, all others with the call's weight decay; with the flags cleared
    again every tensor decays."""
    wl = synth.Workload("flags", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-2, sigma=None)
    lay = wl.layout
    exempt = [i for i, nm in enumerate(lay.names) if not (nm.endswith(".w") and "ln" not in nm or nm == "emb")]
    decays = [i for i in range(lay.n_tensors) if i not in exempt]
    assert exempt and decays
    st, _ = P.make_state(wl, 31, master_fmt=master_fmt)
    flags = np.zeros(lay.n_tensors, dtype=np.uint32)
    flags[exempt] = B.TENSOR_NO_WEIGHT_DECAY
    st.ctx.set_tensor_flags(flags)
    grad = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    for step in (1, 2, 3):
        if step == 3:
            st.ctx.set_tensor_flags(np.zeros(lay.n_tensors, dtype=np.uint32))
        synth.fill_gradients(grad, wl, 31, step)
        kw = dict(weight_decay=0.5, exact=exact, master_fmt=master_fmt)
        hp = B.adam_hparams(wl.lr, step, **kw)
        hp0 = B.adam_hparams(wl.lr, step, **dict(kw, weight_decay=0.0))
        with_decay = decays if step < 3 else decays + exempt
        snaps_d = [P.Snapshot(st, grad, t) for t in with_decay]
        snaps_e = [P.Snapshot(st, grad, t) for t in exempt] if step < 3 else []
        say(f"tensor flags (master {master_fmt}, exact {exact}) step {step}: {len(with_decay)} decaying, {len(snaps_e)} exempt")
        st.step(grad, hp)
        torch.cuda.synchronize()
        P.check_step(st, snaps_d, hp, what=f"decaying tensors step {step}")
        if snaps_e:
            P.check_step(st, snaps_e, hp0, what=f"exempt tensors step {step}")
    with pytest.raises(B.Fp8lmError):
        st.ctx.set_tensor_flags(np.full(lay.n_tensors, 2, dtype=np.uint32))      # unknown bit
    with pytest.raises(B.Fp8lmError):
        st.ctx.set_tensor_flags(np.zeros(lay.n_tensors + 1, dtype=np.uint32))    # wrong length


def test_two_contexts_on_two_streams_at_once():
    """One context per stream is the rule; two contexts on two streams may run at the same time (each has its own
    records and scratch).  Two halves of a layout are stepped concurrently and each must match the oracle."""
    wl = synth.Workload("streams", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None)
    lay, tens = wl.layout, wl.layout.tensors()
    halves = [list(range(0, lay.n_tensors, 2)), list(range(1, lay.n_tensors, 2))]
    cfg = B.autoscale_cfg()
    st = [OptimizerState([tens[t] for t in halves[0]], lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3)]
    st.append(OptimizerState([tens[t] for t in halves[1]], lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3, share_with=st[0]))
    w0 = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    synth.fill_weights(w0, lay, 29)
    for x in st:
        x.init_master(w0)
    grad = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    streams = [torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)]
    for step in (1, 2, 3):
        synth.fill_gradients(grad, wl, 29, step)
        hp = B.adam_hparams(wl.lr, step)
        snaps = [[P.Snapshot(x, grad, t) for t in range(len(h))] for x, h in zip(st, halves)]
        torch.cuda.synchronize()
        say(f"two streams step {step}")
        for x, s in zip(st, streams):
            with torch.cuda.stream(s):
                x.step(grad, hp)
        torch.cuda.synchronize()
        for k, x in enumerate(st):
            P.check_step(x, snaps[k], hp, what=f"stream {k} step {step}")


def test_shards_of_the_greedy_distribution_step_like_the_whole_model():
    """Sec. 2.3, Alg. 1 on one GPU: the tensors are dealt to eight owners by the greedy rule; every owner steps only
    its own tensors (a context over its tensor list, its own metadata) inside the shared flat buffers.  The union of
    the shards must hold the bytes and the scales of the whole model stepped by one context, which in turn is checked
    against the free-running oracle."""
    wl = synth.Workload("shards", synth.gpt_layout(256, 2, 1024, 1000), lr=1e-3, sigma=None)
    lay, tens = wl.layout, wl.layout.tensors()
    owner, usage = B.greedy_partition(np.array(lay.numels, dtype=np.int64) * 7, 8)
    assert usage.max() <= usage.sum() / 8 + max(lay.numels) * 7
    cfg = B.autoscale_cfg(ramp_steps=4, hist_window=2)
    whole = OptimizerState(tens, lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3)
    ids = [[t for t in range(lay.n_tensors) if owner[t] == r] for r in range(8)]
    assert all(ids)
    shards = [OptimizerState([tens[t] for t in ids[0]], lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3)]
    shards += [OptimizerState([tens[t] for t in ids[r]], lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3, share_with=shards[0])
               for r in range(1, 8)]
    w0 = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    synth.fill_weights(w0, lay, 23)
    whole.init_master(w0)
    for sh in shards:
        sh.init_master(w0)
    fr = P.FreeRunningOracle(lay, cfg, synth.bits16(w0), threads=8)
    grad = torch.zeros(max(lay.total, 16), dtype=torch.bfloat16, device=DEV)
    for step in range(1, 7):
        synth.fill_gradients(grad, wl, 23, step)
        if step == 4:
            grad.mul_(32.0)                       # a jump the amax history and mu have to follow
        hp = B.adam_hparams(wl.lr, step)
        say(f"greedy shards step {step}")
        whole.step(grad, hp)
        for sh in shards:
            sh.step(grad, hp)
        fr.step(synth.bits16(grad), hp)
    torch.cuda.synchronize()
    fr.assert_equal_to(whole, "whole model after 6 steps")
    for name in ("g8", "m", "v", "w", "wq"):
        assert torch.equal(getattr(shards[0], name), getattr(whole, name)), f"{name}: union of the shards differs"
    for k in ("g_meta", "m_meta", "v_meta", "w_meta", "q_meta"):
        ref = B.meta_to_numpy(getattr(whole, k), lay.n_tensors)
        for r, sh in enumerate(shards):
            got = B.meta_to_numpy(getattr(sh, k), len(ids[r]))
            assert got.tobytes() == ref[ids[r]].tobytes(), f"{k} of owner {r} differs from the whole model's rows"


# ---- randomised differential test -----------------------------------------------------------------------------
def test_random_layouts_and_hyper_parameters_match_the_oracle():
    """Sixty seeded random cases: ragged tensor sizes, gradient scales over forty binades, hyper-parameters at and
    between the ends of their ranges, every format, source type, moment-scale mode, both gradient scalings (the
    just-in-time one also through the speculative call) and both auto-scaling rules.  FP8LM_RANDOM_CASES / FP8LM_RANDOM_SEED in the environment run more cases or other ones."""
    n_cases = int(os.environ.get("FP8LM_RANDOM_CASES", "60"))
    rng = np.random.default_rng(int(os.environ.get("FP8LM_RANDOM_SEED", "20231018")))
    rng2 = np.random.default_rng(int(os.environ.get("FP8LM_RANDOM_SEED", "20231018")) + 1)    # draws added later: the cases above stay what they were
    dtypes = [torch.bfloat16, torch.float16, torch.float32]
    for case in range(n_cases):
        n_t = int(rng.integers(1, 7))
        numels = [int(rng.choice([0, 1, 15, 16, 17, 255, 4095, 4096, 4097, int(rng.integers(1, 70000))])) for _ in range(n_t)]
        if sum(numels) == 0:
            numels[0] = 33
        lay = synth.Layout([f"t{i}" for i in range(n_t)], numels)
        dtype = dtypes[case % 3]
        lo = -6 if dtype == torch.float16 else -20
        sig = float(2.0 ** rng.integers(lo, 6))
        wl = synth.Workload(f"rnd{case}", lay, lr=1e-3, sigma=sig, grad_kind=["normal", "student_t"][case % 2],
                            ramp_steps=int(rng.choice([2, 4, 20])), hist_window=int(rng.choice([1, 1, 3, 16])))
        grad_fmt = [B.E5M2, B.E4M3][int(rng.integers(0, 2))]
        wcopy = [B.WCOPY_E4M3, B.WCOPY_BF16][int(rng.integers(0, 2))]
        master_fmt, v_fmt = B.STATE_F16, B.STATE_F16
        if wcopy == B.WCOPY_E4M3 and rng.random() < 0.4:
            master_fmt = int(rng.choice([B.STATE_F16, B.STATE_BF16, B.STATE_E4M3, B.STATE_F32]))
            v_fmt = int(rng.choice([B.STATE_F16, B.STATE_E4M3]))
        mu_rule = int(rng.integers(0, 2))
        st, _ = P.make_state(wl, case, grad_fmt, wcopy, master_fmt=master_fmt, v_fmt=v_fmt, mu_rule=mu_rule,
                             mu_min_exp=int(rng.integers(-5, 0)), second_m=True)
        flags = rng.integers(0, 2, n_t).astype(np.uint32) if rng.random() < 0.3 else np.zeros(n_t, dtype=np.uint32)
        st.ctx.set_tensor_flags(flags)               # before the tuning call: the flags must survive the table rebuild
        if rng.random() < 0.5:
            st.ctx.set_tuning(int(rng.choice([4096, 16384])), int(rng.integers(1, 17)), int(rng.choice([0, 1 << 30])))
        ids = list(range(n_t))
        grad = torch.zeros(max(lay.total, 16), dtype=dtype, device=DEV)
        step0 = int(rng.choice([1, 1, 2, 1000, 10 ** 6]))
        for k in range(3):
            synth.fill_gradients(grad, wl, case, k + 1)
            hp = B.adam_hparams(lr=float(rng.choice([0.0, 1e-5, 1e-3, 0.5, 1024.0])), step=step0 + k,
                                beta1=float(rng.choice([0.0, 0.5, 0.9, 0.999])), beta2=float(rng.choice([0.0, 0.5, 0.95, 0.9999])),
                                eps=float(rng.choice([2.0 ** -36, 1e-8, 1e-3, 1.0])), weight_decay=float(rng.choice([0.0, 0.1, 10.0])),
                                v_scaled=int(rng.integers(0, 2)) if (master_fmt, v_fmt) == (B.STATE_F16, B.STATE_F16) else 1,
                                wcopy=wcopy, stats=int(rng.integers(0, 2)) if (master_fmt, v_fmt) == (B.STATE_F16, B.STATE_F16) else 0,
                                m_scale_mode=int(rng.integers(0, 3)), master_fmt=master_fmt, v_fmt=v_fmt)
            delayed = bool(rng.integers(0, 2)) and k > 0
            speculative = bool(rng2.integers(0, 2)) and not delayed      # same results as just in time, by another route
            # ... and so has the Adam step with the exact moment scale: through the pair of first-moment buffers
            pair_m = (bool(rng2.integers(0, 2)) and not delayed and (master_fmt, v_fmt) == (B.STATE_F16, B.STATE_F16)
                      and hp.stats == 0 and hp.m_scale_mode == B.MSCALE_EXACT_PASS)
            snaps = [P.Snapshot(st, grad, t) for t in ids]
            say(f"random case {case} step {k}: numels={numels} dtype={dtype} sigma={sig:g} fmt={grad_fmt} wcopy={wcopy} "
                f"master={master_fmt} v={v_fmt} lr={hp.lr:g} b1={hp.beta1:g} b2={hp.beta2:g} eps={hp.eps:g} wd={hp.weight_decay:g} "
                f"t={hp.step} v_scaled={hp.v_scaled} stats={hp.stats} mode={hp.m_scale_mode} delayed={delayed} speculative={speculative} pair_m={pair_m} mu_rule={mu_rule} "
                f"exempt={flags.tolist()}")
            st.step(grad, hp, delayed=delayed, speculative=speculative, pair_m=pair_m)
            torch.cuda.synchronize()
            P.check_step(st, [x for x in snaps if not flags[x.t]], hp, what=f"random case {case} step {k}", delayed=delayed)
            if flags.any():
                hp0 = B.AdamHparams.from_buffer_copy(hp)
                hp0.weight_decay = 0.0
                P.check_step(st, [x for x in snaps if flags[x.t]], hp0, what=f"random case {case} step {k}, exempt tensors",
                             delayed=delayed)


# ---- the alternative reading of the auto-scaling rule ------------------------------------------------------------
@pytest.mark.parametrize("fmt", [B.E5M2, B.E4M3])
def test_halving_rule_follows_the_oracle_through_cast_and_sum(fmt):
    """mu_rule = MU_HALVE: eight ranks whose sum outgrows the range by far more than 2.  The summed gradient's
    statistic drives mu (fed back to the ranks' casts), step after step, on both sides."""
    from paper_2310_18313_amd.allreduce_study import Fp8AllReduce
    n_ranks, steps = 8, 14
    lay = synth.Layout(["a", "b", "c"], [30001, 4096, 200])
    wl = synth.Workload("halve", lay, lr=1e-3, sigma=1e-2, ramp_steps=6)
    cfg = B.autoscale_cfg(ramp_steps=6, mu_rule=B.MU_HALVE, mu_min_exp=-6)
    ocfg = P.oracle_cfg(cfg)
    assert ocfg.mu_rule == 1 and ocfg.mu_min_exp == -6
    tens = O.tensors_array(lay.tensors())
    ctx = B.Context(lay.tensors())
    size = max(lay.total, 16)
    common = torch.zeros(size, dtype=torch.float32, device=DEV)
    grads = [torch.zeros(size, dtype=torch.float32, device=DEV) for _ in range(n_ranks)]
    ar = Fp8AllReduce(ctx, n_ranks, lay.total, fmt, cfg, "auto")
    o_meta = [O.new_meta(lay.n_tensors, ocfg) for _ in range(n_ranks)]
    o_sum_meta = O.new_meta(lay.n_tensors, ocfg)
    assert np.array_equal(B.meta_to_numpy(ar.summed_meta, lay.n_tensors)["clean_steps"], o_sum_meta["clean_steps"])
    seen = set()
    for step in range(1, steps + 1):
        synth.fill_gradients(common, wl, 77, step)
        for r in range(n_ranks):
            synth.fill_gradients(grads[r], wl, 500 + r, step)
            grads[r].mul_(0.05).add_(common)                   # almost the same gradient on every rank: the sum is 8x
        say(f"halving rule fmt={fmt} step={step}")
        ar.step(grads)
        torch.cuda.synchronize()
        h = [g.cpu().numpy() for g in grads]
        pay = []
        for r in range(n_ranks):
            o_meta[r]["mu_exp"], o_meta[r]["clean_steps"] = o_sum_meta["mu_exp"], o_sum_meta["clean_steps"]
            q = np.zeros(size, dtype=np.uint8)
            O.amax_scale(h[r], tens, fmt, o_meta[r], ocfg, src_type=O.SRC_F32)
            O.cast_fp8(h[r], tens, q, fmt, o_meta[r], ocfg, src_type=O.SRC_F32)
            pay.append(q)
        shared = O.shared_scale(o_meta, lay.n_tensors)
        rq = []
        for r in range(n_ranks):
            q2, m2 = np.zeros(size, dtype=np.uint8), O.new_meta(lay.n_tensors, ocfg)
            O.requantize_fp8(pay[r], fmt, o_meta[r], shared, tens, q2, m2)
            rq.append(q2)
        o_sum = np.zeros(size, dtype=np.uint8)
        O.sum_fp8(rq, fmt, shared, tens, o_sum, o_sum_meta, ocfg)
        assert np.array_equal(ar.summed.cpu().numpy(), o_sum), f"step {step}: summed payload differs"
        gm = B.meta_to_numpy(ar.summed_meta, lay.n_tensors)
        for t in range(lay.n_tensors):
            bad = P.meta_equal(gm[t], o_sum_meta[t], ["scale", "inv_scale", "amax_deq", "mu_exp", "clean_steps", "n_sat", "flags"])
            assert not bad, (step, t, bad, gm[t], o_sum_meta[t])
            rm = B.meta_to_numpy(ar.meta[0], lay.n_tensors)[t]
            bad = P.meta_equal(rm, o_meta[0][t], P.ALL_FIELDS)
            assert not bad, (step, t, bad, rm, o_meta[0][t])
        seen.update(int(x) for x in gm["mu_exp"])
    assert min(seen) <= -3, seen                               # mu went well below the 1/2 floor of the default rule
    bad_cfg = B.autoscale_cfg(mu_rule=B.MU_HALVE, mu_min_exp=0)
    with pytest.raises(B.Fp8lmError):
        ctx.new_meta(bad_cfg)


def test_c_program_steps_identically_to_the_oracle_through_the_c_abi():
    """No Python between the caller and the library: a C++ program (built beforehand) drives five free-running steps
    through include/fp8lm.h on ragged tensors and compares every byte and metadata field with the oracle."""
    import subprocess
    import c_abi_build
    exe = c_abi_build.build()          # a host-only compile of two seconds, and only if the program is missing or stale
    assert os.path.exists(exe)
    say("c_abi_parity: 5 steps")
    r = subprocess.run([exe, O.build(), "5"], capture_output=True, text=True, timeout=120)
    say(r.stdout.strip().splitlines()[-1] if r.stdout.strip() else r.stderr[-300:])
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
    assert "identical after 5 steps" in r.stdout
    assert "log2 mu between -1 and 1" in r.stdout          # the auto-scaling state went through all three values
