"""Pins for the oracle's pack / unpack (no GPU)."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc


def test_hand_example_pack(hand_example):
    ex = hand_example
    for dtype in ("f16", "bf16"):
        Wb = synth.to_bits(ex["W"].astype(np.float32), dtype)
        vals, nm, vec = orc.pack(Wb, dtype, 4, 8)
        assert vec.tolist() == ex["vec_idx"].tolist()
        assert orc.decode(vals, dtype).tolist() == ex["vals"].astype(np.float64).tolist()
        assert nm.reshape(-1).tolist() == ex["nm_idx"].reshape(-1).tolist()
        scores = orc.vector_scores(Wb, dtype, 4)
        assert scores[0].tolist() == [22, 18, 18, 2, 39, 7, 21, 18, 2, 66, 3, 3, 26, 2, 64, 3]


@pytest.mark.parametrize("case", [
    synth.small_case(64, 96, 16, 48, 4, "f16", 11),
    synth.small_case(128, 128, 32, 32, 4, "bf16", 12),
])
def test_unpack_is_masked_w_bit_for_bit(case):
    Wb = case.weights()
    vals, nm, vec = orc.pack(Wb, case.dtype, case.V, case.Kv)
    Wh = orc.unpack(vals, nm, vec, case.M, case.K, case.V)
    m = orc.mask(nm, vec, case.M, case.K, case.V)
    assert np.array_equal(Wh, np.where(m, Wb, np.uint16(0)))
    assert np.array_equal(orc.unpack_fast(vals, nm, vec, case.M, case.K, case.V), Wh)


def test_signed_zero_is_a_bit_copy():
    W = np.zeros((4, 8), dtype=np.float32)
    Wb = synth.to_bits(W, "f16")
    Wb[:, 1] = 0x8000                         # -0.0
    vals, nm, vec = orc.pack(Wb, "f16", 4, 8)
    assert vec.tolist() == [list(range(8))]
    assert vals[:, 0].tolist() == [0] * 4 and vals[:, 1].tolist() == [0x8000] * 4


def test_repack_is_a_fixed_point_when_kept_entries_dominate():
    # continuous random data: no ties, so packing the pruned matrix again must
    # reproduce the same three arrays
    case = synth.small_case(64, 64, 16, 32, 4, "f16", 13)
    Wb = case.weights()
    a = orc.pack(Wb, "f16", 16, 32)
    Wh = orc.unpack(*a, 64, 64, 16)
    b = orc.pack(Wh, "f16", 16, 32)
    # pruned columns now score 0 < every kept column's score
    assert np.array_equal(a[2], b[2])
    # inside kept columns the two survivors are the only non-zeros of their group
    assert np.array_equal(orc.unpack(*b, 64, 64, 16), Wh)


def test_nibble_layout_low_nibble_first():
    # one row, two groups: group 0 keeps positions (0, 3), group 1 keeps (1, 2)
    W = np.array([[9, 0, 0, 8, 0, 7, 6, 0]], dtype=np.float32)
    vals, nm, vec = orc.pack(synth.to_bits(W, "f16"), "f16", 1, 8)
    assert nm.tolist() == [[(0 | 3 << 2) | ((1 | 2 << 2) << 4)]]
    assert orc.decode(vals, "f16").tolist() == [[9, 8, 7, 6]]


def test_rounding_helpers_match_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0, 1e-8, -1e-8,
                                  3.0e38, np.inf, -np.inf], dtype=np.float32)])
    t = torch.from_numpy(x)
    want_bf = t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    want_h = t.to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.round_to_storage(x, "bf16"), want_bf)
    assert np.array_equal(orc.round_to_storage(x, "f16"), want_h)
    assert np.array_equal(synth.to_bits(x[:20000], "bf16"), want_bf[:20000])
    back = torch.from_numpy(want_bf.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.decode(want_bf, "bf16"), back, equal_nan=True)


# ---- tile-wise order of the kept column vectors (Section 3.2; sigma_i^t of Section 4.2) ------------------

def test_hand_example_with_tile_order(hand_example):
    from tests.conftest import load_golden
    ex, so = hand_example, load_golden("hand_example_v4_tile_order.txt")
    for dtype in ("f16", "bf16"):
        Wb = synth.to_bits(ex["W"].astype(np.float32), dtype)
        vals, nm, vec = orc.pack(Wb, dtype, 4, 8, sigma=so["sigma"])
        assert vec.tolist() == so["vec_idx"].tolist()
        assert orc.decode(vals, dtype).tolist() == so["vals"].astype(np.float64).tolist()
        assert nm.reshape(-1).tolist() == so["nm_idx"].reshape(-1).tolist()
        Wh = orc.unpack(vals, nm, vec, 4, 16, 4)
        Xb = synth.to_bits(ex["X"].astype(np.float32), dtype)
        Y = orc.spmm(Wh, Xb, dtype, ex["pi_in"].reshape(-1), ex["pi_out"].reshape(-1))
        assert orc.decode(Y, dtype).tolist() == so["Y"].astype(np.float64).tolist()


def test_ascending_tile_order_is_the_plain_pack():
    c = synth.small_case(64, 96, 16, 48, 4, "f16", 21)
    Wb = c.weights()
    ident = np.tile(np.arange(c.K), (c.T, 1))
    for a, b in zip(orc.pack(Wb, c.dtype, c.V, c.Kv), orc.pack(Wb, c.dtype, c.V, c.Kv, sigma=ident)):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_tile_order_keeps_the_vector_mask_and_regroups(dtype):
    c = synth.small_case(48, 40, 16, 24, 4, dtype, 22)
    Wb = c.weights()
    rng = np.random.default_rng(5)
    sigma = np.stack([rng.permutation(c.K) for _ in range(c.T)])
    _, _, plain = orc.pack(Wb, dtype, c.V, c.Kv)
    vals, nm, vec = orc.pack(Wb, dtype, c.V, c.Kv, sigma=sigma)
    W = orc.decode(Wb, dtype)
    for t in range(c.T):
        # the same columns survive, arranged as a subsequence of sigma[t]
        assert sorted(vec[t].tolist()) == plain[t].tolist()
        where = {ch: i for i, ch in enumerate(sigma[t].tolist())}
        pos = [where[ch] for ch in vec[t].tolist()]
        assert pos == sorted(pos)
    # every group of four consecutive kept vectors (in that order) keeps its two largest magnitudes:
    # brute force over the six pairs, the retained magnitude must be the maximum
    m = orc.mask(nm, vec, c.M, c.K, c.V)
    for r in range(c.M):
        t = r // c.V
        for g in range(c.Kv // 4):
            cols = vec[t, 4 * g:4 * g + 4]
            mags = np.abs(W[r, cols])
            kept = m[r, cols]
            assert kept.sum() == 2
            best = max(mags[i] + mags[j] for i in range(4) for j in range(i + 1, 4))
            assert mags[kept].sum() == best
    # and unpack is still the masked matrix, bit for bit
    assert np.array_equal(orc.unpack(vals, nm, vec, c.M, c.K, c.V), np.where(m, Wb, np.uint16(0)))


# ---- caller-given saliency rho (Section 4.1, Eq. 1-3; Section 5.1) and the vector-only state (Section 5.1.2) ----

def test_order_from_arrangement_by_hand_and_round_trip():
    # by hand: K = 6, tile keeps channels 4, 1, 3 in that arrangement -> 4 1 3 then the others ascending 0 2 5
    assert orc.order_from_arrangement(np.array([[4, 1, 3]]), 6).tolist() == [[4, 1, 3, 0, 2, 5]]
    assert orc.order_from_arrangement(np.array([[0, 1]]), 2).tolist() == [[0, 1]]          # everything kept
    # round trip through tile_order (pinned by the hand example above): the order reproduces the arrangement
    rng = np.random.default_rng(5)
    T, K, Kv = 3, 40, 12
    kept = np.stack([np.sort(rng.permutation(K)[:Kv]) for _ in range(T)])
    arr = np.stack([rng.permutation(kept[t]) for t in range(T)])
    sigma = orc.order_from_arrangement(arr, K)
    assert all(sorted(sigma[t].tolist()) == list(range(K)) for t in range(T))
    assert np.array_equal(orc.tile_order(kept, sigma, K), arr)
    assert all(np.all(np.diff(sigma[t, Kv:]) > 0) for t in range(T))                      # pruned ones ascending
    with pytest.raises(AssertionError):
        orc.order_from_arrangement(np.array([[1, 1, 2]]), 6)


def test_hand_example_with_scores(hand_example):
    from tests.conftest import load_golden
    ex, sc = hand_example, load_golden("hand_example_v4_scores.txt")
    rho = sc["rho"].astype(np.float32)
    pin, pout = ex["pi_in"].reshape(-1), ex["pi_out"].reshape(-1)
    for dtype in ("f16", "bf16"):
        Wb = synth.to_bits(ex["W"].astype(np.float32), dtype)
        Xb = synth.to_bits(ex["X"].astype(np.float32), dtype)
        assert orc.vector_scores_rho(rho, 4)[0].tolist() == [4, 2, 4, 10, 2, 4, 8, 1, 12, 2, 0, 8, 3, 2, 8, 16]
        vals, nm, vec = orc.pack(Wb, dtype, 4, 8, rho=rho)
        assert vec.tolist() == sc["vec_idx"].tolist()
        assert orc.decode(vals, dtype).tolist() == sc["vals"].astype(np.float64).tolist()
        assert nm.reshape(-1).tolist() == sc["nm_idx"].reshape(-1).tolist()
        Y = orc.spmm(orc.unpack(vals, nm, vec, 4, 16, 4), Xb, dtype, pin, pout)
        assert orc.decode(Y, dtype).tolist() == sc["Y"].astype(np.float64).tolist()
        vals_v, vec_v = orc.pack_vectors(Wb, dtype, 4, 8, rho=rho)
        assert vec_v.tolist() == sc["vec_idx"].tolist()
        assert orc.decode(vals_v, dtype).tolist() == sc["vals_v"].astype(np.float64).tolist()
        Yv = orc.spmm(orc.unpack_vectors(vals_v, vec_v, 4, 16, 4), Xb, dtype, pin, pout)
        assert orc.decode(Yv, dtype).tolist() == sc["Y_v"].astype(np.float64).tolist()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_squared_weights_as_scores_give_the_plain_pack(dtype):
    # w^2 is exact in float32 for 16-bit w, so summed rho is the L2 vector saliency and the order of
    # rho inside a group is the order of |w|, ties included
    c = synth.small_case(64, 96, 16, 48, 4, dtype, 31)
    Wb = c.weights()
    w = orc.decode(Wb, dtype).astype(np.float32)
    rho = w * w
    assert np.array_equal(rho.astype(np.float64), orc.decode(Wb, dtype) ** 2)
    for a, b in zip(orc.pack(Wb, dtype, c.V, c.Kv), orc.pack(Wb, dtype, c.V, c.Kv, rho=rho)):
        assert np.array_equal(a, b)


def test_scores_select_by_brute_force():
    # Eq. 2 and Eq. 3 with an independent rho: enumerate all column subsets of a tile and all pairs of a
    # group; the kept set must retain the maximal summed rho (small integers, so sums are exact)
    import itertools
    rng = np.random.default_rng(32)
    M, K, V, Kv = 8, 10, 4, 8
    Wb = synth.to_bits(rng.standard_normal((M, K)).astype(np.float32), "f16")
    rho = rng.integers(-3, 9, size=(M, K)).astype(np.float32)
    vals, nm, vec = orc.pack(Wb, "f16", V, Kv, rho=rho)
    m = orc.mask(nm, vec, M, K, V)
    for t in range(M // V):
        col = rho[t * V:(t + 1) * V].astype(np.float64).sum(axis=0)
        best = max(itertools.combinations(range(K), Kv), key=lambda s: (col[list(s)].sum(), [-x for x in s]))
        assert vec[t].tolist() == list(best)      # with ties the lexicographically first maximiser
    for r in range(M):
        for g in range(Kv // 4):
            cols = vec[r // V, 4 * g:4 * g + 4]
            sc = rho[r, cols].astype(np.float64)
            kept = m[r, cols]
            assert kept.sum() == 2
            assert sc[kept].sum() == max(sc[i] + sc[j] for i in range(4) for j in range(i + 1, 4))
    assert np.array_equal(orc.unpack(vals, nm, vec, M, K, V), np.where(m, Wb, np.uint16(0)))


def test_scores_ties_signed_zero_and_negative_sums():
    # one tile of two rows: column sums 0 (from +1 and -1), -0.0 + -0.0 (= +0 from the +0 start), 0, -2, 5 ...
    rho = np.array([[1, -0.0, 0, -1, 5, 2, 2, 2, 0, 0, 0, 0],
                    [-1, -0.0, 0, -1, 0, 2, 2, 2, 0, 0, 0, -4]], dtype=np.float32)
    Wb = synth.to_bits(np.arange(24, dtype=np.float32).reshape(2, 12) + 1, "f16")
    s = orc.vector_scores_rho(rho, 2)
    assert s[0].tolist() == [0, 0, 0, -2, 5, 4, 4, 4, 0, 0, 0, -4] and not np.signbit(s[0][s[0] == 0]).any()
    vals, nm, vec = orc.pack(Wb, "f16", 2, 8, rho=rho)
    # 5, the three 4s, then four of the six zero sums by lower column; the negative sums lose against zero
    assert vec[0].tolist() == [0, 1, 2, 4, 5, 6, 7, 8]
    # row 0, group (c0 c1 c2 c4): rho 1 -0 0 5 -> positions 0 3; group (c5 c6 c7 c8): 2 2 2 0 -> positions 0 1
    # row 1, group (c0 c1 c2 c4): rho -1 -0 0 0 -> -0 ties with +0: positions 1 2; second group as in row 0
    assert nm.reshape(-1).tolist() == [(0 | 3 << 2) | (0 | 1 << 2) << 4, (1 | 2 << 2) | (0 | 1 << 2) << 4]
    assert orc.decode(vals, "f16").tolist() == [[1, 5, 6, 7], [14, 15, 18, 19]]


def test_single_row_tiles_with_scores_are_plain_top_k():
    # V = 1: a vector is one weight, so the vector mask keeps the Kv largest rho of every row
    rng = np.random.default_rng(33)
    M, K, Kv = 6, 24, 8
    Wb = synth.to_bits(rng.standard_normal((M, K)).astype(np.float32), "bf16")
    rho = rng.permutation(M * K).reshape(M, K).astype(np.float32)      # all distinct
    _, vec = orc.pack_vectors(Wb, "bf16", 1, Kv, rho=rho)
    for r in range(M):
        assert vec[r].tolist() == sorted(np.argsort(-rho[r])[:Kv].tolist())


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_two_to_four_on_the_vector_only_state_completes_the_pack(dtype):
    # Section 3.1: the 2:4 step works on what vector pruning left, so pruning the rows of vals_v in groups
    # of four must give the packed layer; and the vector-only matrix is W under the column mask
    c = synth.small_case(64, 96, 16, 48, 4, dtype, 34)
    Wb = c.weights()
    rng = np.random.default_rng(34)
    sigma = np.stack([rng.permutation(c.K) for _ in range(c.T)])
    vals, nm, vec = orc.pack(Wb, dtype, c.V, c.Kv, sigma=sigma)
    vals_v, vec_v = orc.pack_vectors(Wb, dtype, c.V, c.Kv, sigma=sigma)
    assert np.array_equal(vec, vec_v)
    Wv = orc.unpack_vectors(vals_v, vec_v, c.M, c.K, c.V)
    colmask = np.zeros((c.M, c.K), dtype=bool)
    for t in range(c.T):
        colmask[t * c.V:(t + 1) * c.V, vec[t]] = True
    assert np.array_equal(Wv, np.where(colmask, Wb, np.uint16(0)))
    mag = np.abs(orc.decode(vals_v, dtype)).reshape(c.M, c.Kv // 4, 4)
    for r in range(c.M):
        for g in range(c.Kv // 4):
            order = sorted(range(4), key=lambda q: (-mag[r, g, q], q))[:2]
            p0, p1 = min(order), max(order)
            assert vals[r, 2 * g] == vals_v[r, 4 * g + p0] and vals[r, 2 * g + 1] == vals_v[r, 4 * g + p1]
            assert (nm[r, g >> 1] >> (4 * (g & 1))) & 15 == p0 | p1 << 2
