"""Whole-tensor greedy distribution (Sec. 2.3, Alg. 1): the oracle against a hand-worked example and the
guarantees of largest-first list scheduling; the library's host implementation against the oracle."""
import numpy as np
import pytest

import oracle as O
from paper_2310_18313_amd import binding as B
from paper_2310_18313_amd import synth


def test_hand_worked_example():
    # sorted 5,4,3,3,3 on two GPUs: 5->G0, 4->G1, 3->G1 (4<5), 3->G0 (5<7), 3->G1 (7<8)
    owner, usage = O.greedy_partition([3, 5, 3, 4, 3], 2)
    assert list(owner) == [1, 0, 0, 1, 1]
    assert list(usage) == [8, 10]
    # equal loads: the lowest-numbered GPU receives; equal sizes: index order
    owner, usage = O.greedy_partition([2, 2, 2, 2], 4)
    assert list(owner) == [0, 1, 2, 3]


@pytest.mark.parametrize("name", ["gpt125m", "gpt7b", "gpt13b", "gpt175b_layer"])
@pytest.mark.parametrize("n_gpus", [2, 8, 32])
def test_properties_on_the_model_layouts(name, n_gpus):
    sizes = np.array(synth.workload(name).layout.numels, dtype=np.int64)
    owner, usage = O.greedy_partition(sizes, n_gpus)
    assert owner.min() >= 0 and owner.max() < n_gpus
    assert np.array_equal(np.bincount(owner, weights=sizes, minlength=n_gpus).astype(np.int64), usage)
    lower = max(int(np.ceil(sizes.sum() / n_gpus)), int(sizes.max()))
    assert usage.max() <= (4 / 3 - 1 / (3 * n_gpus)) * lower + 1e-9      # Graham's bound for largest-first
    assert usage.max() - usage.min() <= sizes.max()
    # when a tensor is placed, no GPU is emptier than its receiver: replay in sorted order
    order = sorted(range(len(sizes)), key=lambda i: (-sizes[i], i))
    u = np.zeros(n_gpus, dtype=np.int64)
    for i in order:
        assert u[owner[i]] == u.min()
        u[owner[i]] += sizes[i]


def test_library_host_function_equals_the_oracle():
    rng = np.random.default_rng(0)
    for trial in range(50):
        n = int(rng.integers(0, 300))
        m = int(rng.integers(1, 40))
        sizes = rng.integers(0, 50, n) * rng.integers(1, 1000, n) if trial % 2 else rng.integers(0, 6, n)
        a_owner, a_usage = O.greedy_partition(sizes, m)
        b_owner, b_usage = B.greedy_partition(sizes, m)
        assert np.array_equal(a_owner, b_owner) and np.array_equal(a_usage, b_usage)
    for name in ("gpt13b", "gpt175b_layer"):
        sizes = synth.workload(name).layout.numels
        assert np.array_equal(O.greedy_partition(sizes, 8)[0], B.greedy_partition(sizes, 8)[0])
    assert B.lib().fp8lm_greedy_partition(None, 3, 2, None, None) == -1
