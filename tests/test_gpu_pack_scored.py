"""GPU parity of hinm_pack_scored (caller-given saliency scores, Section 4.1 of the paper), of
hinm_pack_vectors and of hinm_spmm_vectors (the vector-only state of gradual pruning, Section 5.1.2)
against the CPU oracle: packing bit-exact, products within the product tolerance."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu


def _sigma(T, K, seed):
    rng = np.random.default_rng(seed)
    return np.stack([rng.permutation(K) for _ in range(T)]).astype(np.int32)


def _rho(M, K, seed, kind="halfnormal"):
    rng = np.random.default_rng(seed)
    if kind == "halfnormal":        # like second-order scores: non-negative, wide range
        return np.abs(rng.standard_normal((M, K))).astype(np.float32) ** 2
    if kind == "signed":
        return rng.standard_normal((M, K)).astype(np.float32)
    if kind == "coarse":            # few distinct values: ties everywhere, in both selections
        return rng.integers(0, 3, size=(M, K)).astype(np.float32)
    raise ValueError(kind)


def _check_pack(Wb, dtype, V, Kv, rho, sigma=None, tiles=None):
    from tests import gpu_util as gu
    p = gu.gpu_pack(Wb, dtype, V, Kv, sigma=sigma, rho=rho)
    vals, nm, vec = p.host()
    for t in (range(Wb.shape[0] // V) if tiles is None else tiles):
        rows = slice(t * V, (t + 1) * V)
        o_vals, o_nm, o_vec = orc.pack(Wb[rows], dtype, V, Kv, rho=rho[rows],
                                       sigma=None if sigma is None else sigma[t:t + 1])
        assert np.array_equal(vec[t], o_vec[0]), f"vector index differs in tile {t}"
        assert np.array_equal(nm[rows], o_nm), f"NM index differs in tile {t}"
        assert np.array_equal(vals[rows], o_vals), f"packed values differ in tile {t}"
    return p


def test_hand_example_with_scores_on_gpu(hand_example):
    from tests.conftest import load_golden
    from tests import gpu_util as gu
    sc = load_golden("hand_example_v4_scores.txt")
    rho = sc["rho"].astype(np.float32)
    for dtype in ("f16", "bf16"):
        Wb = synth.to_bits(hand_example["W"].astype(np.float32), dtype)
        vals, nm, vec = gu.gpu_pack(Wb, dtype, 4, 8, rho=rho).host()
        assert vec.tolist() == sc["vec_idx"].tolist()
        assert orc.decode(vals, dtype).tolist() == sc["vals"].astype(np.float64).tolist()
        assert nm.reshape(-1).tolist() == sc["nm_idx"].reshape(-1).tolist()
        pv = gu.gpu_pack_vectors(Wb, dtype, 4, 8, rho=rho)
        vals_v, vec_v = pv.host()
        assert vec_v.tolist() == sc["vec_idx"].tolist()
        assert orc.decode(vals_v, dtype).tolist() == sc["vals_v"].astype(np.float64).tolist()
        Xb = synth.to_bits(hand_example["X"].astype(np.float32), dtype)
        Y = gu.gpu_spmm_vectors(pv, Xb, hand_example["pi_in"].reshape(-1), hand_example["pi_out"].reshape(-1))
        assert orc.decode(Y, dtype).tolist() == sc["Y_v"].astype(np.float64).tolist()


@pytest.mark.parametrize("M,K,V,Kv,dtype,kind,ordered", [
    (64, 96, 16, 48, "f16", "halfnormal", False),
    (128, 1001, 32, 504, "bf16", "signed", True),        # odd K: scalar loads of rho, negative sums
    (256, 4096, 128, 2048, "f16", "coarse", False),      # rows through LDS, ties in both selections
    (64, 5000, 64, 4096, "bf16", "halfnormal", True),    # rows through LDS with a tile order
    (32, 20000, 32, 2048, "f16", "signed", False),       # K beyond the LDS row kernel with scores
    (8, 16, 4, 16, "f16", "coarse", True),               # everything kept
])
def test_pack_scored_small_cases(M, K, V, Kv, dtype, kind, ordered):
    c = synth.small_case(M, K, V, Kv, 4, dtype, 41)
    _check_pack(c.weights(), dtype, V, Kv, _rho(M, K, 42, kind), _sigma(M // V, K, 43) if ordered else None)


def test_pack_scored_signed_zero_scores():
    # -0 and +0 scores are equal in both selections
    rng = np.random.default_rng(44)
    M, K, V, Kv = 32, 64, 16, 32
    rho = rng.integers(0, 2, size=(M, K)).astype(np.float32)
    rho[rng.random((M, K)) < 0.5] *= -1.0          # -1, -0, +0, +1
    assert np.signbit(rho[rho == 0]).any()
    c = synth.small_case(M, K, V, Kv, 4, "bf16", 44)
    _check_pack(c.weights(), "bf16", V, Kv, rho)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_pack_scored_with_squared_weights_is_pack(dtype):
    from tests import gpu_util as gu
    c = synth.small_case(128, 512, 32, 256, 4, dtype, 45)
    Wb = c.weights()
    w = orc.decode(Wb, dtype).astype(np.float32)
    for a, b in zip(gu.gpu_pack(Wb, dtype, c.V, c.Kv).host(), gu.gpu_pack(Wb, dtype, c.V, c.Kv, rho=w * w).host()):
        assert np.array_equal(a, b)


def test_pack_scored_c2_full_and_c5_sampled_tiles():
    c = synth.c2()
    _check_pack(c.weights(), c.dtype, c.V, c.Kv, _rho(c.M, c.K, 46))
    c = synth.c5()
    _check_pack(c.weights(), c.dtype, c.V, c.Kv, _rho(c.M, c.K, 47), sigma=_sigma(c.T, c.K, 48), tiles=[0, 77, 127])


def test_product_of_a_layer_packed_by_scores():
    from tests import gpu_util as gu
    c = synth.small_case(128, 512, 64, 256, 200, "f16", 49)
    Wb, Xb = c.weights(), c.activations()
    rho = _rho(c.M, c.K, 50)
    p = _check_pack(Wb, c.dtype, c.V, c.Kv, rho)
    vals, nm, vec = orc.pack(Wb, c.dtype, c.V, c.Kv, rho=rho)
    Wh = orc.unpack(vals, nm, vec, c.M, c.K, c.V)
    assert np.array_equal(gu.gpu_unpack(p), Wh)
    pin, pout = c.pi_in(), c.pi_out()
    want = orc.product(Wh, Xb, c.dtype, pin, pout, acc=np.float64)
    got = gu.gpu_spmm_prepared(gu.gpu_prepare(p, pin, pout), Xb, 2).astype(np.float64)
    gu.check_close(got, want, what="prepared kernels on a layer packed by scores")


# ---- the vector-only state ------------------------------------------------------------------------------

@pytest.mark.parametrize("M,K,V,Kv,dtype,scored,ordered", [
    (64, 96, 16, 48, "f16", False, False),
    (128, 1000, 32, 504, "bf16", True, True),
    (256, 4096, 128, 2048, "f16", False, True),       # rows through LDS
    (64, 40000, 64, 2048, "bf16", True, False),       # K beyond the LDS row kernel
])
def test_pack_vectors(M, K, V, Kv, dtype, scored, ordered):
    from tests import gpu_util as gu
    c = synth.small_case(M, K, V, Kv, 4, dtype, 51)
    Wb = c.weights()
    rho = _rho(M, K, 52) if scored else None
    sigma = _sigma(M // V, K, 53) if ordered else None
    vals_v, vec = gu.gpu_pack_vectors(Wb, dtype, V, Kv, sigma=sigma, rho=rho).host()
    o_vals_v, o_vec = orc.pack_vectors(Wb, dtype, V, Kv, sigma=sigma, rho=rho)
    assert np.array_equal(vec, o_vec)
    assert np.array_equal(vals_v, o_vals_v)


@pytest.mark.parametrize("M,K,V,Kv,N,dtype,flags", [
    (128, 512, 32, 256, 300, "f16", 0),         # two column blocks, ragged
    (128, 512, 64, 200, 256, "bf16", 0),        # Kv not a multiple of the 32-column step
    (192, 640, 96, 320, 100, "f16", 2),         # fp32 output
    (256, 1024, 128, 512, 520, "bf16", 1),      # ReLU
    (128, 512, 128, 512, 64, "f16", 0),         # nothing pruned: a plain dense product
    (64, 96, 16, 48, 24, "bf16", 0),            # V = 16: plain kernel
    (128, 512, 64, 256, 1, "f16", 0),           # a single column
    (128, 512, 64, 256, 72, "bf16", 0x100),     # plain kernel forced
])
def test_spmm_vectors_matches_the_oracle(M, K, V, Kv, N, dtype, flags):
    from tests import gpu_util as gu
    c = synth.small_case(M, K, V, Kv, N, dtype, 54)
    Wb, Xb = c.weights(), c.activations()
    sigma = _sigma(M // V, K, 55)
    pv = gu.gpu_pack_vectors(Wb, dtype, V, Kv, sigma=sigma)
    o_vals_v, o_vec = orc.pack_vectors(Wb, dtype, V, Kv, sigma=sigma)
    Wv = orc.unpack_vectors(o_vals_v, o_vec, M, K, V)
    pin, pout = c.pi_in(), c.pi_out()
    relu = bool(flags & 1)
    want = orc.product(Wv, Xb, dtype, pin, pout, acc=np.float32, relu=relu).astype(np.float64)
    got32 = gu.gpu_spmm_vectors(pv, Xb, pin, pout, flags=flags | 2)
    gu.check_close(got32.astype(np.float64), want, what="vector-only product, fp32 accumulators")
    if not flags & 2:
        # 16-bit outputs must be the correctly rounded accumulators
        got = gu.gpu_spmm_vectors(pv, Xb, pin, pout, flags=flags)
        assert np.array_equal(got, orc.round_to_storage(got32, dtype))
    # every tile kernel that fits the shape, pinned through the variant bits
    if V % 32 == 0 and N > 1 and not flags & 0x100:
        for variant in (1, 2, 3, 4, 5):
            if variant >= 2 and Kv % 64:
                continue
            g = gu.gpu_spmm_vectors(pv, Xb, pin, pout, flags=(flags & 1) | 2 | variant << 16)
            gu.check_close(g.astype(np.float64), want, what=f"vector-only product, kernel variant {variant}")
    # identity orders reduce to W_v @ X
    got_id = gu.gpu_spmm_vectors(pv, Xb, None, None, flags=2 | (flags & 0x100)).astype(np.float64)
    gu.check_close(got_id, orc.product(Wv, Xb, dtype, None, None, acc=np.float64), what="identity orders")


@pytest.mark.parametrize("M,K,V,Kv,N,dtype", [
    (4096, 256, 32, 128, 1030, "bf16"),     # 512-column blocks, ragged last block, 32-row tiles
    (4096, 512, 64, 256, 2048, "f16"),      # 512-column blocks, 64-row tiles
    (3072, 640, 96, 320, 1536, "bf16"),     # 96-row tiles
    (2048, 1024, 128, 64, 4096, "f16"),     # a single stage
])
def test_spmm_vectors_wide_blocks_sampled_outputs(M, K, V, Kv, N, dtype):
    from tests import gpu_util as gu
    c = synth.small_case(M, K, V, Kv, N, dtype, 57)
    Wb, Xb = c.weights(), c.activations()
    sigma = _sigma(M // V, K, 58)
    pv = gu.gpu_pack_vectors(Wb, dtype, V, Kv, sigma=sigma)
    o_vals_v, o_vec = orc.pack_vectors(Wb, dtype, V, Kv, sigma=sigma)
    assert np.array_equal(pv.host()[0], o_vals_v)
    Wv = orc.unpack_vectors(o_vals_v, o_vec, M, K, V)
    pin, pout = c.pi_in(), c.pi_out()
    got = gu.gpu_spmm_vectors(pv, Xb, pin, pout, flags=2).astype(np.float64)
    rng = np.random.default_rng(59)
    rows = rng.choice(M, 64, replace=False)
    cols = np.unique(np.concatenate([rng.choice(N, 96, replace=False), [0, 511, 512, N - 1]]))
    want = orc.product_entries(Wv, Xb, dtype, pin, pout, rows, cols)
    gu.check_close(got[np.asarray(pout)[rows]][:, cols], want, what="vector-only product, wide blocks")
    got16 = gu.gpu_spmm_vectors(pv, Xb, pin, pout, flags=0)
    assert np.array_equal(got16, orc.round_to_storage(got.astype(np.float32), dtype))


def test_spmm_vectors_c2_sampled_outputs():
    from tests import gpu_util as gu
    c = synth.c2()
    Wb, Xb = c.weights(), c.activations()
    pv = gu.gpu_pack_vectors(Wb, c.dtype, c.V, c.Kv)
    o_vals_v, o_vec = orc.pack_vectors(Wb, c.dtype, c.V, c.Kv)
    assert np.array_equal(pv.host()[0], o_vals_v)
    Wv = orc.unpack_vectors(o_vals_v, o_vec, c.M, c.K, c.V)
    pin, pout = c.pi_in(), c.pi_out()
    got = gu.gpu_spmm_vectors(pv, Xb, pin, pout, flags=2).astype(np.float64)
    rng = np.random.default_rng(56)
    rows = rng.choice(c.M, 48, replace=False)
    cols = rng.choice(c.N, 64, replace=False)
    want = orc.product_entries(Wv, Xb, c.dtype, pin, pout, rows, cols)
    gu.check_close(got[np.asarray(pout)[rows]][:, cols], want, what="C2 vector-only, sampled outputs")
