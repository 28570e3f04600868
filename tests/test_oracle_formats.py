"""Pins for the oracle's number formats and the scale rule (CPU only).

Every check here compares the oracle with something that is not the oracle: values the paper
prints (Appendix A.1 range table, under tests/golden/), numpy's IEEE half, torch's CPU bfloat16 /
float8 casts, exact rational arithmetic, or a brute-force search.
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle as O
from conftest import read_golden_table

TABLE = read_golden_table("range_table.txt")
CONST = read_golden_table("paper_constants.txt")


def _finite_positive_values(fmt):
    tab = O.decode_table(fmt)
    vals = tab[:128]
    return vals[np.isfinite(vals)]


# ---- decode tables vs the paper's printed numbers ------------------------------------------------
@pytest.mark.parametrize("fmt,name,first_normal_code", [(O.E4M3, "E4M3", 0x08), (O.E5M2, "E5M2", 0x04)])
def test_decode_matches_paper_range_table(fmt, name, first_normal_code):
    mx, min_normal, min_sub, rn0, rn1, rs0, rs1 = TABLE[name]
    vals = _finite_positive_values(fmt)
    assert vals.max() == mx == CONST[name.lower() + "_max"][0]
    assert vals[first_normal_code] == pytest.approx(min_normal, rel=5e-3)
    assert vals[1] == pytest.approx(min_sub, rel=5e-3)
    # codes are monotone in value
    assert np.all(np.diff(vals) > 0)
    normals = vals[first_normal_code:]
    subs = vals[1:first_normal_code]
    assert (normals[1] - normals[0]) / normals[1] == pytest.approx(rn0, rel=5e-3)
    assert (normals[-1] - normals[-2]) / normals[-2] == pytest.approx(rn1, rel=5e-3)
    assert (subs[1] - subs[0]) / subs[1] == pytest.approx(rs0, rel=5e-3)
    assert (subs[-1] - subs[-2]) / subs[-2] == pytest.approx(rs1, rel=5e-3)


def test_e4m3_has_nan_but_no_inf_and_e5m2_has_both():
    e4 = O.decode_table(O.E4M3)
    e5 = O.decode_table(O.E5M2)
    assert not np.isinf(e4).any()
    assert set(np.flatnonzero(np.isnan(e4))) == {0x7F, 0xFF}
    assert set(np.flatnonzero(np.isinf(e5))) == {0x7C, 0xFC}
    assert set(np.flatnonzero(np.isnan(e5))) == {0x7D, 0x7E, 0x7F, 0xFD, 0xFE, 0xFF}
    assert e4[0x7E] == 448.0 and e4[0xFE] == -448.0
    assert e5[0x7B] == 57344.0 and e5[0xFB] == -57344.0


def test_f16_decode_matches_paper_and_numpy():
    mx, min_normal, min_sub, rn0, rn1, rs0, rs1 = TABLE["FP16"]
    L = O.lib()
    codes = np.arange(65536, dtype=np.uint16)
    mine = np.array([L.oracle_decode_f16(int(c)) for c in codes], dtype=np.float32)
    ref = codes.view(np.float16).astype(np.float32)
    assert np.array_equal(np.isnan(mine), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(mine[ok].view(np.uint32), ref[ok].view(np.uint32))
    assert mine[0x7BFF] == mx
    assert mine[0x0400] == pytest.approx(min_normal, rel=5e-3)
    assert mine[0x0001] == pytest.approx(min_sub, rel=5e-3)
    assert (mine[0x0401] - mine[0x0400]) / mine[0x0401] == pytest.approx(rn0, rel=5e-3)
    assert (mine[0x7BFF] - mine[0x7BFE]) / mine[0x7BFE] == pytest.approx(rn1, rel=5e-3)
    assert (mine[0x03FF] - mine[0x03FE]) / mine[0x03FE] == pytest.approx(rs1, rel=5e-3)


def test_e5m2_decode_is_the_top_byte_of_ieee_half():
    codes = np.arange(256, dtype=np.uint16)
    ref = (codes << 8).astype(np.uint16).view(np.float16).astype(np.float32)
    mine = O.decode_table(O.E5M2)
    assert np.array_equal(np.isnan(mine), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(mine[ok].view(np.uint32), ref[ok].view(np.uint32))


def test_fp8_decode_matches_torch_cpu_views():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    for fmt, tdt in ((O.E4M3, torch.float8_e4m3fn), (O.E5M2, torch.float8_e5m2)):
        ref = codes.view(tdt).to(torch.float32).numpy()
        mine = O.decode_table(fmt)
        assert np.array_equal(np.isnan(mine), np.isnan(ref))
        ok = ~np.isnan(ref)
        assert np.array_equal(mine[ok].view(np.uint32), ref[ok].view(np.uint32))


def test_bf16_decode_and_encode_match_torch_and_paper():
    mx, min_normal, min_sub, rn0, rn1, rs0, rs1 = TABLE["BF16"]
    L = O.lib()
    codes = np.arange(65536, dtype=np.uint16)
    mine = np.array([L.oracle_decode_bf16(int(c)) for c in codes], dtype=np.float32)
    ref = torch.from_numpy(codes.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    ok = ~np.isnan(ref)
    assert np.array_equal(np.isnan(mine), np.isnan(ref))
    assert np.array_equal(mine[ok].view(np.uint32), ref[ok].view(np.uint32))
    assert mine[0x7F7F] == pytest.approx(mx, rel=5e-3)
    assert mine[0x0080] == pytest.approx(min_normal, rel=5e-3)
    assert mine[0x0001] == pytest.approx(min_sub, rel=5e-3)
    assert (mine[0x0081] - mine[0x0080]) / mine[0x0081] == pytest.approx(rn0, rel=5e-3)
    # encode: RNE as torch's CPU cast does it
    rng = np.random.default_rng(5)
    x = rng.standard_normal(200000).astype(np.float32) * np.exp2(rng.integers(-40, 40, 200000)).astype(np.float32)
    x = np.concatenate([x, np.array([0.0, -0.0, np.inf, -np.inf, 3.3e38, 3.4e38, 1e-40, -1e-40], np.float32)])
    # add exact ties
    base = rng.integers(0, 0x7F00, 20000).astype(np.uint32) << 16
    ties = (base | 0x8000).view(np.float32)
    x = np.concatenate([x, ties, -ties])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.encode_bf16(x), ref)
    assert O.lib().oracle_encode_bf16(float("nan")) == 0x7FC0


# ---- encoders ------------------------------------------------------------------------------------
@pytest.mark.parametrize("fmt", [O.E4M3, O.E5M2])
def test_encode_roundtrips_every_finite_code(fmt):
    tab = O.decode_table(fmt)
    finite = np.isfinite(tab)
    codes = np.arange(256, dtype=np.uint8)
    back = O.encode_fp8(fmt, np.where(finite, tab, 0.0))
    assert np.array_equal(back[finite], codes[finite])
    assert finite.sum() == (254 if fmt == O.E4M3 else 248)


def _all_bf16_times_pow2(exps):
    pats = np.arange(65536, dtype=np.uint32) << 16
    base = pats.view(np.float32)
    base = base[np.isfinite(base)]
    out = []
    for e in exps:
        with np.errstate(over="ignore", under="ignore"):
            out.append(base * np.float32(2.0 ** e))
    return np.concatenate(out)


@pytest.mark.parametrize("fmt", [O.E4M3, O.E5M2])
def test_bit_level_encoder_equals_brute_force_nearest(fmt):
    tab = O.decode_table(fmt)
    pos = tab[:128][np.isfinite(tab[:128])].astype(np.float64)
    # every midpoint between adjacent codes, and one fp32 ulp either side of it
    mids = ((pos[1:] + pos[:-1]) / 2).astype(np.float32)
    assert np.array_equal(mids.astype(np.float64), (pos[1:] + pos[:-1]) / 2)  # exactly representable
    around = np.concatenate([mids, np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(0))])
    fmax = np.float32(pos[-1])
    edge = np.array([0.0, -0.0, fmax, np.nextafter(fmax, np.float32(np.inf)), np.nextafter(fmax, np.float32(0)),
                     np.inf, -np.inf, 1e-45, 1e-38, 3e38, pos[1] / 2, np.nextafter(np.float32(pos[1] / 2), np.float32(1))],
                    dtype=np.float32)
    rng = np.random.default_rng(11)
    rnd = (rng.integers(0, 2 ** 32, 1_000_000, dtype=np.uint64).astype(np.uint32)).view(np.float32)
    rnd = rnd[~np.isnan(rnd)]
    sweep = _all_bf16_times_pow2(range(-24, 25, 3))
    x = np.concatenate([around, -around, edge, -edge, rnd, sweep])
    a = O.encode_fp8(fmt, x)
    b = O.encode_fp8_nearest(fmt, x)
    bad = np.flatnonzero(a != b)
    assert bad.size == 0, (x[bad[:5]], a[bad[:5]], b[bad[:5]])
    # ties go to the even code
    tie_codes = O.encode_fp8(fmt, mids)
    assert np.all(tie_codes % 2 == 0)
    # NaN
    assert O.encode_fp8(fmt, np.array([np.nan], np.float32))[0] == 0x7F
    assert O.encode_fp8_nearest(fmt, np.array([np.nan], np.float32))[0] == 0x7F


@pytest.mark.parametrize("fmt,tdt", [(O.E4M3, torch.float8_e4m3fn), (O.E5M2, torch.float8_e5m2)])
def test_encoder_equals_torch_cpu_cast_inside_the_range(fmt, tdt):
    """torch's CPU float8 casts round to nearest even but do not saturate: compare where the
    rounded result stays finite."""
    tab = O.decode_table(fmt)
    fmax = float(np.nanmax(np.where(np.isfinite(tab), tab, -np.inf)))
    x = _all_bf16_times_pow2(range(-20, 12, 1))
    rng = np.random.default_rng(3)
    rnd = (rng.standard_normal(500000) * np.exp2(rng.uniform(-20, 9, 500000))).astype(np.float32)
    x = np.concatenate([x, rnd])
    x = x[np.abs(x) <= fmax]
    ref = torch.from_numpy(x).to(tdt).view(torch.uint8).numpy()
    mine = O.encode_fp8(fmt, x)
    assert np.array_equal(mine, ref)


@pytest.mark.parametrize("fmt", [O.E4M3, O.E5M2])
def test_encoder_saturates_instead_of_overflowing(fmt):
    top = 0x7E if fmt == O.E4M3 else 0x7B
    fmax = 448.0 if fmt == O.E4M3 else 57344.0
    x = np.array([fmax, fmax * 1.0001, fmax * 2, 1e30, np.inf], np.float32)
    assert np.all(O.encode_fp8(fmt, x) == top)
    assert np.all(O.encode_fp8(fmt, -x) == (0x80 | top))


def test_f16_encoder_equals_numpy_and_saturates():
    rng = np.random.default_rng(9)
    x = (rng.standard_normal(1_000_000) * np.exp2(rng.uniform(-30, 16, 1_000_000))).astype(np.float32)
    sweep = _all_bf16_times_pow2(range(-8, 9, 4))
    halves = np.arange(0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)
    mids = ((halves[1:].astype(np.float64) + halves[:-1]) / 2).astype(np.float32)   # exact in fp32
    x = np.concatenate([x, sweep, halves, -halves, mids, -mids,
                        np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(0))])
    inr = np.abs(x) < 65520.0
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    mine = O.encode_f16_sat(x)
    assert np.array_equal(mine[inr], ref[inr])
    big = ~inr
    assert np.all((mine[big] & 0x7FFF) == 0x7BFF)
    assert np.array_equal(mine[big] >> 15, (x[big] < 0).astype(np.uint16))
    edge = O.encode_f16_sat(np.array([65519.996, 65520.0, np.inf, -np.inf, np.nan, -0.0], np.float32))
    assert list(edge) == [0x7BFF, 0x7BFF, 0x7BFF, 0xFBFF, 0x7E00, 0x8000]


# ---- the power-of-two scale rule -------------------------------------------------------------------
@pytest.mark.parametrize("fmax", [448.0, 57344.0, 65504.0])
def test_pow2_rule_is_the_largest_power_of_two_that_fits(fmax):
    L = O.lib()
    rng = np.random.default_rng(2)
    A = (rng.uniform(1, 2, 3000) * np.exp2(rng.integers(-148, 127, 3000))).astype(np.float32)
    # exact boundaries: A = fmax * 2^-j, and its two fp32 neighbours
    j = np.arange(-100, 130)
    with np.errstate(over="ignore", under="ignore"):
        exact = (np.float32(fmax) * np.exp2(-j.astype(np.float64))).astype(np.float32)
    exact = exact[np.isfinite(exact) & (exact > 0)]
    A = np.concatenate([A, exact, np.nextafter(exact, np.float32(np.inf)), np.nextafter(exact, np.float32(0)),
                        np.array([1e-45, 1.17549435e-38, 3.4028235e38], np.float32)])
    A = A[(A > 0) & np.isfinite(A)]
    F = Fraction(fmax)
    for a in A:
        k = L.oracle_pow2_exp(fmax, float(a))
        fa = Fraction(float(a))
        assert Fraction(2) ** k * fa <= F < Fraction(2) ** (k + 1) * fa, (a, k)


def test_hparam_derivation_matches_float64():
    for step in (1, 2, 10, 1000, 100000):
        hp = O.AdamHparams(3e-4, 0.9, 0.95, 1e-8, 0.1, step, 1, 0)
        d = O.derive_hparams(hp)
        b1, b2 = float(np.float32(0.9)), float(np.float32(0.95))
        lr, wd = float(np.float32(3e-4)), float(np.float32(0.1))
        want = [b1, 1 - b1, 1 / (1 - b1 ** step), b2, 1 - b2, 1 / (1 - b2 ** step), 1 - lr * wd]
        assert np.array_equal(d, np.array(want, dtype=np.float32))
    assert CONST["beta1"][0] == 0.9 and CONST["beta2"][0] == 0.95 and CONST["weight_decay"][0] == 0.1
    assert math.isclose(O.derive_hparams(O.AdamHparams(1e-4, 0.9, 0.95, 1e-8, 0.1, 1, 1, 0))[2], 10.0, rel_tol=1e-6)
