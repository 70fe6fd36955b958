"""The permutation search end to end on the GPU (paper_2407_20496_amd.gyro.gyro_permute: output-channel search
with clustering, vector pruning, tile-wise search, 2:4 packing) on a layer with planted structure: the search
must recover most of the saliency an unpermuted layer loses, and the packed result must be exactly what the
packing oracle gives for the row order and tile order found."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import gyro_oracle as gyro
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu


def _planted_layer(M, K, V, Kv, seed):
    """Channels of M / V kinds, every kind strong on its own Kv input channels, shuffled over the tiles."""
    rng = np.random.default_rng(seed)
    T = M // V
    W = rng.standard_normal((M, K)).astype(np.float32) * 0.01
    kind = rng.permutation(np.repeat(np.arange(T), V))
    for r in range(M):
        strong = (np.arange(Kv) + kind[r] * (K - Kv) // max(1, T - 1)) % K      # a window that moves with the kind
        W[r, strong] += rng.standard_normal(Kv).astype(np.float32)
    return W, kind


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_pipeline_on_a_planted_layer(dtype):
    import torch
    from paper_2407_20496_amd import gyro as g
    from tests import gpu_util as gu
    M, K, V, Kv = 256, 128, 32, 64
    W, kind = _planted_layer(M, K, V, Kv, 110)
    Wb = synth.to_bits(W, dtype)
    S = gyro.saliency_matrix(Wb, dtype, None)
    T = M // V
    before_vec = sum(gyro.vector_pruned_saliency(S[t * V:(t + 1) * V], Kv) for t in range(T))
    out = g.gyro_permute(gu.dev_bits(Wb), V, Kv, dtype, ocp_iters=24, icp_iters=6, seed=1)
    order = out["row_order"].cpu().numpy()
    assert sorted(order.tolist()) == list(range(M))
    after_vec = sum(gyro.vector_pruned_saliency(S[order[t * V:(t + 1) * V]], Kv) for t in range(T))
    trace = out["vector_pruned_saliency"]
    assert after_vec == pytest.approx(trace[-1], rel=1e-9)
    assert after_vec < 0.8 * before_vec, (before_vec, after_vec)       # the planted grouping is largely recovered
    # packed arrays = the packing oracle on W's rows in that order with the tile order found
    sigma = out["tile_order"].cpu().numpy()
    vals, nm, vec = orc.pack(Wb[order], dtype, V, Kv, sigma=sigma)
    assert np.array_equal(out["vec_idx"].cpu().numpy(), vec)
    assert np.array_equal(gu.host_bits(out["vals"]), vals)
    assert np.array_equal(out["nm_idx"].cpu().numpy(), nm)
    # the tile-wise search lowered what 2:4 prunes, and the last value is what the packed layer really lost
    nm_trace = out["nm_pruned_saliency"]
    _, _, plain_vec = orc.pack(Wb[order], dtype, V, Kv)
    start = sum(gyro.pruned_saliency(gyro.kept_saliency(Wb[order], dtype, None, V, plain_vec[t], t)) for t in range(T))
    assert nm_trace[-1] <= start and all(b <= a * (1 + 1e-12) for a, b in zip(nm_trace, nm_trace[1:]))
    kept = np.abs(orc.decode(vals, dtype)).sum()
    surviving = sum(S[order[t * V:(t + 1) * V]][:, vec[t]].sum() for t in range(T))
    assert surviving - kept == pytest.approx(nm_trace[-1], rel=1e-9)
    # the product with pi_out = row_order puts every channel back at its own place
    c = synth.small_case(M, K, V, Kv, 72, dtype, 111)
    Xb = c.activations()
    p = gu.Packed(M, K, V, Kv, dtype, out["vals"].reshape(-1), out["nm_idx"].reshape(-1), out["vec_idx"].reshape(-1))
    got = gu.gpu_spmm_prepared(gu.gpu_prepare(p, None, order), Xb, 2).astype(np.float64)
    Wh = orc.unpack(vals, nm, vec, M, K, V)
    want = orc.product(Wh, Xb, dtype, None, order, acc=np.float64)
    gu.check_close(got, want, what="product of the permuted layer")
    masked_in_place = np.zeros_like(Wh)
    masked_in_place[order] = Wh
    gu.check_close(got, orc.product(masked_in_place, Xb, dtype, None, None, acc=np.float64), what="rows back in place")
