"""GPU parity of hinm_pack_ordered (tile-wise order of the kept column vectors, Section 3.2 of the
paper) against the CPU oracle: packing bit-exact; products from a vector index that is not ascending,
through every kernel family, within the product tolerance."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu


def _sigma(T, K, seed):
    rng = np.random.default_rng(seed)
    return np.stack([rng.permutation(K) for _ in range(T)]).astype(np.int32)


def _check_pack(Wb, dtype, V, Kv, sigma, tiles=None):
    from tests import gpu_util as gu
    p = gu.gpu_pack(Wb, dtype, V, Kv, sigma=sigma)
    vals, nm, vec = p.host()
    for t in (range(Wb.shape[0] // V) if tiles is None else tiles):
        rows = slice(t * V, (t + 1) * V)
        o_vals, o_nm, o_vec = orc.pack(Wb[rows], dtype, V, Kv, sigma=sigma[t:t + 1])
        assert np.array_equal(vec[t], o_vec[0]), f"vector index differs in tile {t}"
        assert np.array_equal(nm[rows], o_nm), f"NM index differs in tile {t}"
        assert np.array_equal(vals[rows], o_vals), f"packed values differ in tile {t}"
    return p


def test_hand_example_with_tile_order_on_gpu(hand_example):
    from tests.conftest import load_golden
    from tests import gpu_util as gu
    so = load_golden("hand_example_v4_tile_order.txt")
    for dtype in ("f16", "bf16"):
        Wb = synth.to_bits(hand_example["W"].astype(np.float32), dtype)
        vals, nm, vec = gu.gpu_pack(Wb, dtype, 4, 8, sigma=so["sigma"].astype(np.int32)).host()
        assert vec.tolist() == so["vec_idx"].tolist()
        assert orc.decode(vals, dtype).tolist() == so["vals"].astype(np.float64).tolist()
        assert nm.reshape(-1).tolist() == so["nm_idx"].reshape(-1).tolist()


@pytest.mark.parametrize("M,K,V,Kv,dtype", [
    (64, 96, 16, 48, "f16"),
    (128, 1000, 32, 504, "bf16"),      # K not a multiple of 32 (bitmap tail), K < one sweep of the workgroup
    (256, 4096, 128, 1024, "f16"),     # several sweeps of 1024 channels
    (64, 5000, 64, 4096, "bf16"),      # Kv larger than one sweep
    (8, 16, 4, 16, "f16"),             # everything kept: the order is sigma itself
])
def test_pack_ordered_small_cases(M, K, V, Kv, dtype):
    c = synth.small_case(M, K, V, Kv, 4, dtype, 31)
    _check_pack(c.weights(), dtype, V, Kv, _sigma(M // V, K, 7))


def test_pack_ordered_with_ascending_order_is_pack():
    from tests import gpu_util as gu
    c = synth.small_case(128, 512, 32, 256, 4, "bf16", 32)
    Wb = c.weights()
    ident = np.tile(np.arange(c.K, dtype=np.int32), (c.T, 1))
    for a, b in zip(gu.gpu_pack(Wb, c.dtype, c.V, c.Kv).host(), gu.gpu_pack(Wb, c.dtype, c.V, c.Kv, sigma=ident).host()):
        assert np.array_equal(a, b)


def test_pack_ordered_many_ties():
    # equal scores everywhere: which columns survive is decided by the tie rule, their order by sigma
    W = np.ones((32, 64), dtype=np.float32)
    Wb = synth.to_bits(W, "f16")
    _check_pack(Wb, "f16", 16, 32, _sigma(2, 64, 8))


def test_pack_ordered_c2_full_and_c5_sampled_tiles():
    c = synth.c2()
    _check_pack(c.weights(), c.dtype, c.V, c.Kv, _sigma(c.T, c.K, 9))
    c = synth.c5()
    _check_pack(c.weights(), c.dtype, c.V, c.Kv, _sigma(c.T, c.K, 10), tiles=[0, 63, 127])


def test_rows_that_are_not_permutations_stay_in_range():
    from tests import gpu_util as gu
    c = synth.small_case(64, 256, 32, 128, 4, "f16", 33)
    Wb = c.weights()
    sigma = _sigma(c.T, c.K, 11)
    sigma[0, :40] = -5          # out of range: skipped
    sigma[1, :] = sigma[1, 0]   # one channel repeated
    _, _, vec = gu.gpu_pack(Wb, c.dtype, c.V, c.Kv, sigma=sigma).host()
    _, _, plain = orc.pack(Wb, c.dtype, c.V, c.Kv)
    for t in range(c.T):
        assert set(vec[t].tolist()) <= set(plain[t].tolist())   # only surviving columns, all in [0, K)


@pytest.mark.parametrize("M,K,V,Kv,N,dtype", [
    (128, 512, 64, 256, 200, "f16"),     # panel / tile kernels
    (256, 4096, 128, 2048, 16, "bf16"),  # few-column kernel
    (128, 2048, 32, 1024, 1, "f16"),
    (64, 96, 16, 48, 24, "bf16"),        # V = 16: canonical kernels only
])
def test_products_follow_an_unordered_vector_index(M, K, V, Kv, N, dtype):
    from tests import gpu_util as gu
    c = synth.small_case(M, K, V, Kv, N, dtype, 34)
    Wb, Xb = c.weights(), c.activations()
    sigma = _sigma(c.T, K, 12)
    p = _check_pack(Wb, dtype, V, Kv, sigma)
    vals, nm, vec = orc.pack(Wb, dtype, V, Kv, sigma=sigma)
    Wh = orc.unpack(vals, nm, vec, M, K, V)
    assert np.array_equal(gu.gpu_unpack(p), Wh)
    pin, pout = c.pi_in(), c.pi_out()
    want = orc.product(Wh, Xb, dtype, pin, pout, acc=np.float64)
    got = gu.gpu_spmm(p, Xb, pin, pout, flags=2).astype(np.float64)          # canonical arrays, fp32 out
    gu.check_close(got, want, what="canonical kernels, ordered vector index")
    if V % 32 == 0:
        pr = gu.gpu_prepare(p, pin, pout)
        got = gu.gpu_spmm_prepared(pr, Xb, 2).astype(np.float64)
        gu.check_close(got, want, what="prepared kernels, ordered vector index")


@pytest.mark.parametrize("T,K,Kv", [(4, 96, 48), (3, 1000, 504), (2, 4096, 1024), (1, 5000, 4096), (2, 16, 16),
                                     (5, 11008, 5504)])
def test_tile_order_from_an_arrangement(T, K, Kv):
    """hinm_tile_order: kept channels as arranged, then the pruned ones ascending, bit for bit; and the order it
    returns makes hinm_pack_ordered reproduce the arrangement."""
    import torch
    import paper_2407_20496_amd as hinm
    rng = np.random.default_rng(K + Kv)
    arr = np.stack([rng.permutation(K)[:Kv] for _ in range(T)]).astype(np.int32)
    want = orc.order_from_arrangement(arr, K)
    vec = torch.from_numpy(arr).cuda()
    out = torch.full((T, K), -7, dtype=torch.int32, device="cuda")
    hinm.hinm_tile_order(T * 4, K, 4, Kv, "f16", vec, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want)


def test_tile_order_round_trip_through_pack_ordered():
    from tests import gpu_util as gu
    import torch
    import paper_2407_20496_amd as hinm
    c = synth.small_case(128, 1000, 32, 504, 4, "bf16", 33)
    Wb = c.weights()
    plain = gu.gpu_pack(Wb, c.dtype, c.V, c.Kv)
    kept = plain.host()[2]
    rng = np.random.default_rng(9)
    arr = np.stack([rng.permutation(kept[t]) for t in range(c.T)]).astype(np.int32)
    sigma = torch.empty((c.T, c.K), dtype=torch.int32, device="cuda")
    hinm.hinm_tile_order(c.M, c.K, c.V, c.Kv, c.dtype, torch.from_numpy(arr).cuda(), sigma)
    torch.cuda.synchronize()
    again = gu.gpu_pack(Wb, c.dtype, c.V, c.Kv, sigma=sigma.cpu().numpy()).host()[2]
    assert np.array_equal(again, arr)


def test_apply_row_order_is_a_row_gather():
    import torch
    import paper_2407_20496_amd as hinm
    rng = np.random.default_rng(3)
    for rows, row_bytes in ((37, 4), (256, 2000), (1000, 8192 * 2)):
        src = rng.integers(0, 256, size=(rows, row_bytes), dtype=np.uint8)
        order = rng.permutation(rows).astype(np.int32)
        d_src = torch.from_numpy(src).cuda()
        d_dst = torch.zeros_like(d_src)
        hinm.hinm_apply_row_order(d_src, d_dst, torch.from_numpy(order).cuda(), rows, row_bytes)
        torch.cuda.synchronize()
        assert np.array_equal(d_dst.cpu().numpy(), src[order])
