"""Pins for the oracle's mask construction (no GPU).

Each test checks the oracle against something other than itself: exhaustive
enumeration of the optimisation problems the paper states (Eq. 2 for the
column-vector mask, the 2:4 constraint of Eq. 3), exact structural counts, the
sparsity formula of Section 1, and crafted ties for the stated tie-breaks.
"""
import itertools

import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc


def _ints_to_bits(A, dtype):
    return synth.to_bits(np.asarray(A, dtype=np.float32), dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("V,K,Kv", [(1, 8, 4), (2, 8, 4), (4, 8, 4), (4, 8, 2), (2, 10, 6)])
def test_vector_mask_is_eq2_argmax_by_enumeration(V, K, Kv, dtype):
    # Eq. 2 with identity order: the kept set maximises the retained saliency
    # among all C(K, Kv) column subsets of each tile.
    rng = np.random.default_rng(V * 100 + K * 10 + Kv)
    T = 3
    W = rng.standard_normal((T * V, K)).astype(np.float32)
    Wb = synth.to_bits(W, dtype)
    Wd = orc.decode(Wb, dtype)
    vec = orc.vector_index(Wb, dtype, V, Kv)
    for t in range(T):
        col_sal = (Wd[t * V:(t + 1) * V] ** 2).sum(axis=0)
        best = max(sum(col_sal[list(S)]) for S in itertools.combinations(range(K), Kv))
        got = col_sal[vec[t]].sum()
        assert got == pytest.approx(best, rel=1e-12)
        assert len(set(vec[t].tolist())) == Kv
        assert np.all(np.diff(vec[t]) > 0)          # strictly ascending


def test_vector_mask_tie_goes_to_lower_column():
    # columns 1, 3, 5 tie at the boundary; two slots left -> columns 1 and 3
    W = np.array([[3, 1, 0, 1, 2, -1, 0, 0],
                  [0, 1, 0, -1, 2, 1, 0, 0]], dtype=np.float32)
    vec = orc.vector_index(_ints_to_bits(W, "f16"), "f16", 2, 4)
    assert vec.tolist() == [[0, 1, 3, 4]]
    # all columns equal: the first Kv columns win
    W = np.ones((2, 8), dtype=np.float32)
    assert orc.vector_index(_ints_to_bits(W, "bf16"), "bf16", 2, 4).tolist() == [[0, 1, 2, 3]]


def test_vector_mask_lexicographically_first_among_maximisers():
    # with ties, the oracle's subset is the lexicographically first of all
    # subsets that attain the maximum of Eq. 2
    rng = np.random.default_rng(5)
    for trial in range(20):
        W = rng.integers(-2, 3, size=(2, 8)).astype(np.float32)
        sal = (W ** 2).sum(axis=0)
        best = max(sal[list(S)].sum() for S in itertools.combinations(range(8), 4))
        first = min(S for S in itertools.combinations(range(8), 4) if sal[list(S)].sum() == best)
        vec = orc.vector_index(_ints_to_bits(W, "f16"), "f16", 2, 4)
        assert tuple(vec[0].tolist()) == first


def test_vector_scores_sum_order_is_sequential_binary64():
    # sequential ascending-row summation differs from pairwise summation on
    # this input; the oracle must produce the sequential result.
    V = 4
    col = np.array([1.0, 2.0 ** -27, 2.0 ** -27, 2.0 ** -27], dtype=np.float32)  # exact in bf16
    W = np.stack([col, col], axis=1)
    s = orc.vector_scores(synth.to_bits(W, "bf16"), "bf16", V)
    seq = 0.0
    for v in col.astype(np.float64):
        seq = seq + v * v
    assert s[0, 0] == seq
    # magnitude check of the score itself against exact rational arithmetic
    from fractions import Fraction
    exact = sum(Fraction(float(v)) ** 2 for v in col)
    assert abs(Fraction(s[0, 0]) - exact) <= Fraction(2) ** -52 * exact * 4


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_nm_positions_is_best_pair_by_enumeration(dtype):
    rng = np.random.default_rng(7)
    C = orc.decode(synth.to_bits(rng.standard_normal((50, 6, 4)).astype(np.float32), dtype), dtype)
    p0, p1 = orc.nm_positions(C)
    assert np.all(p0 < p1)
    for idx in np.ndindex(50, 6):
        mags = np.abs(C[idx])
        best = max(mags[a] + mags[b] for a, b in itertools.combinations(range(4), 2))
        assert mags[p0[idx]] + mags[p1[idx]] == best


@pytest.mark.parametrize("group,expect", [
    ([1, -1, 1, 1], (0, 1)),        # four-way tie -> the two lowest positions
    ([0, 0, 0, 0], (0, 1)),         # all zero: still exactly two kept
    ([0, 0, 0, 5], (0, 3)),
    ([2, 3, -3, 2], (1, 2)),
    ([-0.0, 0.0, 1, -0.0], (0, 2)),  # +0 and -0 tie
    ([1, 2, 2, 2], (1, 2)),
    ([2, 1, 1, 2], (0, 3)),
    ([1, 2, 1, 2], (1, 3)),
])
def test_nm_positions_ties(group, expect):
    p0, p1 = orc.nm_positions(np.array(group, dtype=np.float64).reshape(1, 4))
    assert (int(p0[0]), int(p1[0])) == expect


@pytest.mark.parametrize("case", [
    synth.small_case(64, 96, 16, 48, 4, "f16", 1),
    synth.small_case(128, 64, 32, 16, 4, "bf16", 2),
    synth.small_case(64, 64, 64, 64, 4, "bf16", 3),      # s_v = 0: plain 2:4
])
def test_structural_counts_and_sparsity_formula(case):
    Wb = case.weights()
    vals, nm, vec = orc.pack(Wb, case.dtype, case.V, case.Kv)
    m = orc.mask(nm, vec, case.M, case.K, case.V)
    # exactly Kv columns per tile survive vector pruning, the same for all rows of a tile
    for t in range(case.T):
        cols_used = np.nonzero(m[t * case.V:(t + 1) * case.V].any(axis=0))[0]
        assert set(cols_used.tolist()) <= set(vec[t].tolist())
        # exactly two per group of four kept columns, in every row
        sub = m[t * case.V:(t + 1) * case.V][:, vec[t]].reshape(case.V, -1, 4)
        assert np.all(sub.sum(axis=-1) == 2)
    # Section 1: total sparsity 1 - (1 - s_v) * 0.5
    s_v = 1.0 - case.Kv / case.K
    assert 1.0 - m.sum() / m.size == pytest.approx(1.0 - (1.0 - s_v) * 0.5, abs=0)
    assert vals.shape == (case.M, case.Kv // 2)


def test_sparsity_75_and_875_percent():
    # the two ratios the workloads use: s_v = 50 % -> 75 %, s_v = 75 % -> 87.5 %
    for Kv, want in ((64, 0.75), (32, 0.875)):
        case = synth.small_case(32, 128, 16, Kv, 1, "bf16", 4)
        _, nm, vec = orc.pack(case.weights(), "bf16", 16, Kv)
        m = orc.mask(nm, vec, 32, 128, 16)
        assert 1.0 - m.mean() == want
