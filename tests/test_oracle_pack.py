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
