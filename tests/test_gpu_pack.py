"""GPU parity of hinm_pack / hinm_unpack against the CPU oracle: bit-exact."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu


def _compare(case_or_W, dtype, V, Kv, tiles=None):
    from tests import gpu_util as gu
    Wb = case_or_W
    p = gu.gpu_pack(Wb, dtype, V, Kv)
    vals, nm, vec = p.host()
    if tiles is None:
        o_vals, o_nm, o_vec = orc.pack(Wb, dtype, V, Kv)
        assert np.array_equal(vec, o_vec), "vector index differs"
        assert np.array_equal(nm, o_nm), "NM index differs"
        assert np.array_equal(vals, o_vals), "packed values differ"
    else:
        for t in tiles:
            rows = slice(t * V, (t + 1) * V)
            o_vals, o_nm, o_vec = orc.pack(Wb[rows], dtype, V, Kv)
            assert np.array_equal(vec[t], o_vec[0]), f"vector index differs in tile {t}"
            assert np.array_equal(nm[rows], o_nm), f"NM index differs in tile {t}"
            assert np.array_equal(vals[rows], o_vals), f"packed values differ in tile {t}"
    return p


@pytest.mark.parametrize("M,K,V,Kv,dtype", [
    (64, 96, 16, 48, "f16"),
    (128, 136, 32, 72, "bf16"),      # K, Kv multiples of 8 only
    (96, 100, 8, 40, "f16"),         # K not a multiple of 8: scalar score path
    (64, 64, 64, 64, "bf16"),        # nothing pruned by vectors
    (48, 2056, 4, 8, "f16"),         # very high vector sparsity, K > one select sweep
    (256, 4104, 128, 2048, "bf16"),  # several select sweeps with a ragged last one
])
def test_pack_small_cases(M, K, V, Kv, dtype):
    case = synth.small_case(M, K, V, Kv, 1, dtype, 40 + V)
    _compare(case.weights(), dtype, V, Kv)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_pack_with_many_ties(dtype):
    # small integers: equal vector scores and equal magnitudes everywhere
    rng = np.random.default_rng(77)
    W = rng.integers(-2, 3, size=(128, 256)).astype(np.float32)
    _compare(synth.to_bits(W, dtype), dtype, 16, 128)
    W[:] = 1.0
    _compare(synth.to_bits(W, dtype), dtype, 32, 64)
    W[:] = 0.0
    W[:, ::3] = -0.0
    _compare(synth.to_bits(W, dtype), dtype, 32, 64)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_pack_subnormal_and_extreme_magnitudes(dtype):
    rng = np.random.default_rng(78)
    expo = rng.integers(-30 if dtype == "bf16" else -24, 15, size=(64, 128))
    W = (rng.standard_normal((64, 128)) * np.exp2(expo)).astype(np.float32)
    Wb = synth.to_bits(W, dtype)
    if dtype == "f16":
        Wb[0, :8] = np.array([1, 2, 3, 0x8001, 0x03FF, 0x0400, 0x7BFF, 0xFBFF], dtype=np.uint16)  # subnormals, max
    _compare(Wb, dtype, 16, 64)


def test_pack_c1_and_round_trip():
    from tests import gpu_util as gu
    c = synth.c1()
    Wb = c.weights()
    p = _compare(Wb, c.dtype, c.V, c.Kv)
    vals, nm, vec = p.host()
    Wh = gu.gpu_unpack(p)
    assert np.array_equal(Wh, orc.unpack(vals, nm, vec, c.M, c.K, c.V))
    m = orc.mask(nm, vec, c.M, c.K, c.V)
    assert np.array_equal(Wh, np.where(m, Wb, np.uint16(0)))
    assert 1.0 - m.mean() == 0.75


def test_pack_c2_full():
    c = synth.c2()
    _compare(c.weights(), c.dtype, c.V, c.Kv)


def test_pack_c4_layers_sampled_tiles():
    c = synth.c4()
    for layer in (0, 1):
        _compare(c.weights(layer), c.dtype, c.V, c.Kv, tiles=[0, 31, 63])


@pytest.mark.parametrize("idx", [0, 3, 6, 9])
def test_pack_c3_sampled_tiles(idx):
    c = synth.c3_cases()[idx]
    _compare(c.weights(), c.dtype, c.V, c.Kv, tiles=[0, c.T // 2, c.T - 1])


def test_pack_c5_sampled_tiles():
    c = synth.c5()
    _compare(c.weights(), c.dtype, c.V, c.Kv, tiles=[0, 77, 127])
