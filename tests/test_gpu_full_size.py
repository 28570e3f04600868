"""GPU parity at the full sizes of the benchmark configurations, on sampled tensors.

The whole model steps on the GPU in the launch configuration bench.py times (default tuning, the buffers
carved out of one allocation); before a checked step the inputs of the sampled tensors are copied to
the host and the oracle recomputes those tensors completely.  Every small tensor (LayerNorm weights,
biases) is sampled, plus one tensor of every distinct large shape.
"""
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
SMALL = 1 << 20


def sample_ids(layout):
    small = [t for t, n in enumerate(layout.numels) if 0 < n <= SMALL]
    seen, big = set(), []
    # one tensor per distinct large shape, taken from the middle of the model
    order = sorted(range(layout.n_tensors), key=lambda t: abs(t - layout.n_tensors // 2))
    for t in order:
        n = layout.numels[t]
        kind = layout.names[t].split(".", 1)[-1]
        if n > SMALL and (kind, n) not in seen:
            seen.add((kind, n))
            big.append(t)
    return small, sorted(big)


def run(wl, seed, steps, small_steps, big_steps, big_ids=None, track_mu=False, paths=None, tuning=None, spread=False,
        speculative=False, pair_steps=()):
    lay = wl.layout
    cfg = B.autoscale_cfg(ramp_steps=wl.ramp_steps, hist_window=wl.hist_window)
    st = OptimizerState(lay.tensors(), lay.total, cfg, 0, B.E5M2, B.WCOPY_E4M3, grad_buffer=True, spread=spread,
                        second_m=bool(pair_steps))
    if tuning:
        st.ctx.set_tuning(*tuning)
    say(f"{wl.name}: {lay.n_tensors} tensors, {lay.n_params} params, placement={st.placement}, tuning={tuning}")
    grad = st.grad
    synth.fill_weights(grad, lay, seed)
    st.init_master(grad)
    torch.cuda.synchronize()
    small, big = sample_ids(lay)
    if big_ids is not None:
        big = big_ids
    P.check_init_master(st, grad, small + big[:2])
    grad.zero_()
    tot = dict(elements=0, m_diff=0, w_diff=0, q_diff=0, w_amax_ulp=0)
    mus = []
    for step in range(1, steps + 1):
        synth.fill_gradients(grad, wl, seed, step)
        mode, delayed = (paths or {}).get(step, (B.MSCALE_EXACT_PASS, False))
        hp = B.adam_hparams(wl.lr, step, m_scale_mode=mode)
        ids = (small if step in small_steps else []) + (big if step in big_steps else [])
        snaps = [P.Snapshot(st, grad, t) for t in ids]
        st.step(grad, hp, delayed=delayed, speculative=speculative and not delayed, pair_m=step in pair_steps)
        torch.cuda.synchronize()
        if ids:
            say(f"{wl.name} step {step} (moment-scale mode {mode}, delayed {delayed}): checking {len(ids)} tensors, "
                f"{sum(lay.numels[t] for t in ids)} elements")
            r = P.check_step(st, snaps, hp, what=f"{wl.name} step {step}", delayed=delayed)
            for k in tot:
                tot[k] = max(tot[k], r[k]) if k == "w_amax_ulp" else tot[k] + r[k]
        if track_mu:
            mus.append(B.meta_to_numpy(st.g_meta, lay.n_tensors)["mu_exp"].copy())
    say(f"{wl.name}: {tot}")
    # exact arithmetic is the default: nothing may differ
    assert tot["m_diff"] == 0 and tot["w_diff"] == 0 and tot["q_diff"] == 0
    return st, tot, mus


def lay_tensors_with_elements(wl) -> int:
    return sum(1 for n in wl.layout.numels if n > 0)


def test_gpt13b_in_the_benchmark_configuration():
    wl = synth.workload("gpt13b")
    # as bench.py runs it by default: region-aware placement, just-in-time quantisation through fp8lm_quantize_fp8
    st, tot, _ = run(wl, seed=0, steps=2, small_steps={1, 2}, big_steps={1}, spread=True, speculative=True)
    spec = st.ctx.speculation_stats()
    say(f"placement {st.placement}; speculation {spec}")
    assert spec["calls"] == 2 and lay_tensors_with_elements(wl) <= spec["tensors_redone"] < 2 * lay_tensors_with_elements(wl)
    assert st.state_bytes_per_param == 6          # Sec. 2.2, Eq. 8
    assert tot["elements"] > 5e8


def test_gpt7b_five_steps_with_amax_history():
    wl = synth.workload("gpt7b")
    assert wl.hist_window == 4
    # steps 1-2 on the two-pass path, then the one-GPU fused cast, then the single-pass path (delayed gradient
    # scale + predicted moment scale): the three paths bench.py times, at full size and default tuning
    paths = {3: (B.MSCALE_FROM_CAST, False), 4: (B.MSCALE_PREDICTED, True), 5: (B.MSCALE_FROM_CAST, True)}
    # every small tensor at every step; the five large shapes at steps 2, 3 and 4, one per path.  Step 2
    # goes through fp8lm_adam_step_fp8_m2 (first moment read from one buffer of a pair, written to the other).
    st, _, _ = run(wl, seed=2, steps=5, small_steps={1, 2, 3, 4, 5}, big_steps={2, 3, 4}, paths=paths, pair_steps={2})
    assert st.ctx.speculation_stats(moment=True)["calls"] == 1


def test_gpt175b_layer_heavy_tails_hundred_steps():
    wl = synth.workload("gpt175b_layer")
    lay = wl.layout
    proj = lay.names.index("l0.proj.w")
    checked = {1, 2, 3, 10, 11, 20, 21, 22, 23, 24, 50, 99, 100}
    # this one combines the workgroups' statistics through tickets in the same launch (third tuning entry 0);
    # the other two use the default, a second launch
    st, tot, mus = run(wl, seed=5, steps=100, small_steps=checked, big_steps={1, 100}, big_ids=[proj],
                       track_mu=True, tuning=(16384, 16, 0))
    mus = np.array(mus)                            # [step, tensor]
    # Large matrices: the amax is set by a rare outlier, so even mu = 2 clips far fewer than 0.001 % of
    # the elements and mu climbs to 2 and stays.  Small tensors (< 100 000 elements) overflow whenever
    # their largest element lands on the top code, so they keep cycling 1/2 -> 1 -> 2.
    big = [t for t, n in enumerate(lay.numels) if n > SMALL]
    small = [t for t, n in enumerate(lay.numels) if 0 < n <= SMALL]
    assert (mus[-1, big] == 1).all() and (mus[0, big] == 0).all()
    assert (mus[:, small] == -1).any() and (mus[:, small] == 0).any() and (mus[:, small] == 1).any()
    gm = B.meta_to_numpy(st.g_meta, lay.n_tensors)
    assert gm["n_sat"].sum() > 0


def test_gpt175b_layer_with_the_papers_ramp_of_a_thousand_steps():
    """Same layer and gradients with the ramp length the paper states (Sec. 2.1: back up over 1000 steps): within a
    dozen steps nothing can climb, so a tensor that overflowed sits at mu = 1/2 and the others stay at mu = 1."""
    wl = synth.workload("gpt175b_layer")
    wl.ramp_steps = 1000
    lay = wl.layout
    st, tot, mus = run(wl, seed=5, steps=12, small_steps=set(range(1, 13)), big_steps={12},
                       big_ids=[lay.names.index("l0.proj.w")], track_mu=True)
    mus = np.array(mus)
    big = [t for t, n in enumerate(lay.numels) if n > SMALL]
    small = [t for t, n in enumerate(lay.numels) if 0 < n <= SMALL]
    assert (mus[:, big] == 0).all()                                    # mu = 1 throughout
    assert set(np.unique(mus[:, small])) <= {-1, 0}                    # mu = 1 until the first overflow, then 1/2
    gm = B.meta_to_numpy(st.g_meta, lay.n_tensors)
    overflowed = [t for t in small if (mus[:, t] == -1).any()]
    assert overflowed, "no small tensor put its largest element on the top code in 12 steps"
    for t in overflowed:
        first = int(np.argmax(mus[:, t] == -1))
        assert (mus[first:, t] == -1).all() and gm["clean_steps"][t] < 500


@pytest.mark.parametrize("fmt,scale_exp", [(B.E5M2, 3), (B.E4M3, -2)])
def test_cast_of_every_fp32_bit_pattern(fmt, scale_exp):
    """All 2^32 fp32 inputs through the cast kernel (hardware clamp + convert on the fast path, the explicit NaN
    handling on the careful path) against the oracle's encoder, 2^28 patterns at a time, under one scale per
    format; scales that push the product through fp32 overflow and into the subnormals (2^-126 .. 2^126) are
    covered on the values that decide roundings by test_cast_wide_sources_under_many_scales."""
    from concurrent.futures import ThreadPoolExecutor
    piece, parts = 1 << 28, 16
    sub = piece // parts                                            # 2^24 patterns per tensor: one top byte each
    tensors = [(i * sub, sub) for i in range(parts)]
    cfg = B.autoscale_cfg()
    ctx = B.Context(tensors)
    tens = O.tensors_array(tensors)
    src = torch.empty(piece, dtype=torch.int32, device=DEV)
    dst = torch.zeros(piece, dtype=torch.uint8, device=DEV)
    base = torch.arange(piece, dtype=torch.int64, device=DEV)
    pool = ThreadPoolExecutor(parts)
    # scales other than 1, so that the multiply is exercised too; the large ones push part of the inputs through
    # fp32 overflow and subnormal products
    for k in range(16):
        src.copy_(((base + (k << 28)) & 0xFFFFFFFF).to(torch.int32) if k < 8 else (base + (k << 28) - (1 << 32)).to(torch.int32))
        meta = B.meta_to_numpy(ctx.new_meta(cfg), parts)
        meta["scale"], meta["inv_scale"] = 2.0 ** scale_exp, 2.0 ** -scale_exp
        for i in range(parts):
            top_byte = (k << 4) | i
            if top_byte in (0x7F, 0xFF):                           # holds the infinities and NaNs
                meta["flags"][i] = B.FLAG_NONFINITE
        ref_meta = meta.copy()
        d_meta = B.meta_from_numpy(meta, DEV)
        say(f"fp32 sweep fmt={fmt} scale=2^{scale_exp}: patterns {k << 28:#010x} .. {((k + 1) << 28) - 1:#010x}")
        ctx.cast_fp8(src.view(torch.float32), dst, fmt, d_meta, cfg)
        torch.cuda.synchronize()
        h_src = src.cpu().numpy().view(np.float32)
        ref = np.zeros(piece, dtype=np.uint8)

        def one(i):
            O.cast_fp8(h_src, tens[i:i + 1], ref, fmt, ref_meta[i:i + 1], P.oracle_cfg(cfg), src_type=O.SRC_F32)

        list(pool.map(one, range(parts)))
        got = dst.cpu().numpy()
        bad = np.flatnonzero(got != ref)
        assert bad.size == 0, f"{bad.size} codes differ, first {h_src.view(np.uint32)[bad[:4]]} -> gpu {got[bad[:4]]} oracle {ref[bad[:4]]}"
        gm = B.meta_to_numpy(d_meta, parts)
        for i in range(parts):
            diff = P.meta_equal(gm[i], ref_meta[i], ["n_sat", "n_underflow", "amax_deq", "flags", "mu_exp", "clean_steps"])
            assert not diff, (k, i, diff, gm[i], ref_meta[i])


def test_one_tensor_with_more_than_two_to_the_31_elements():
    """Element indices that do not fit 32 bits.  One tensor of 16 x (2^27 + 12368) elements is stepped twice; the
    same flat range cut into 16 tensors is stepped beside it.  Every piece carries the same planted extremes (the
    largest gradient, the largest weight), so all sixteen pieces and the one huge tensor choose the same scales and
    their payloads must be equal element by element, the huge tensor's counters the sum of the pieces'.  Three of
    the pieces are recomputed by the oracle."""
    pieces, piece = 16, (1 << 27) + 3 * 4096 + 5 * 16
    total = pieces * piece
    assert total > (1 << 31) and piece % 16 == 0
    cfg = B.autoscale_cfg()
    huge = OptimizerState([(0, total)], total, cfg, 0, B.E5M2, B.WCOPY_E4M3)
    split = OptimizerState([(k * piece, piece) for k in range(pieces)], total, cfg, 0, B.E5M2, B.WCOPY_E4M3)
    buf = torch.zeros(total, dtype=torch.bfloat16, device=DEV)
    starts = torch.arange(pieces, device=DEV, dtype=torch.int64) * piece

    def fill(seed, sigma, at0, at1):
        g = torch.Generator(device=DEV)
        g.manual_seed(seed)
        for p0 in range(0, total, 1 << 26):
            n = min(1 << 26, total - p0)
            buf[p0:p0 + n] = (torch.randn(n, generator=g, device=DEV, dtype=torch.float32) * sigma).to(torch.bfloat16)
        buf[starts] = at0           # element 0 of every piece
        buf[starts + 1] = at1       # element 1 of every piece

    say(f"huge tensor: {total} elements; weights")
    fill(31, 0.02, 0.01, 0.5)       # the largest weight of every piece: 0.5, on an element whose gradient stays zero
    huge.init_master(buf)
    split.init_master(buf)
    torch.cuda.synchronize()
    checked = [0, 7, 15]
    P.check_init_master(split, buf, checked)
    for step in (1, 2):
        say(f"huge tensor: gradients of step {step}")
        fill(40 + step, 1e-4, 1.0 if step == 1 else -0.75, 0.0)   # the largest gradient of every piece, same place
        hp = B.adam_hparams(3e-4, step, stats=1)
        snaps = [P.Snapshot(split, buf, t) for t in checked]
        huge.step(buf, hp)
        split.step(buf, hp)
        torch.cuda.synchronize()
        say(f"huge tensor step {step}: oracle on pieces {checked}")
        r = P.check_step(split, snaps, hp, what=f"pieces, step {step}")
        assert r["m_diff"] == 0 and r["w_diff"] == 0 and r["q_diff"] == 0
        say(f"huge tensor step {step}: comparing {total} elements of five buffers")
        for name in ("g8", "m", "v", "w", "wq"):
            assert torch.equal(getattr(huge, name), getattr(split, name)), f"step {step}: {name} differs"
        for k in ("g_meta", "m_meta", "v_meta", "w_meta", "q_meta"):
            one = B.meta_to_numpy(getattr(huge, k), 1)[0]
            many = B.meta_to_numpy(getattr(split, k), pieces)
            assert (many["scale"] == one["scale"]).all(), (k, one["scale"], many["scale"])
            assert one["amax"] == many["amax"].max() and one["amax_deq"] == many["amax_deq"].max(), k
            assert int(one["n_sat"]) == int(many["n_sat"].sum()) and int(one["n_underflow"]) == int(many["n_underflow"].sum()), k
            assert int(one["flags"]) == int(np.bitwise_or.reduce(many["flags"])), k
        gm = B.meta_to_numpy(huge.g_meta, 1)[0]
        assert gm["amax"] == (1.0 if step == 1 else 0.75) and gm["n_underflow"] > 0
