"""Oracle parity of the entry points and launch configurations that bench.py times, at their own sizes:
hinm_spmm_prepared (kernel chosen by shape) on C5 and on the four C3 prefill cases, hinm_chain with prepared
layers on C4, and hinm_pack on every tile of C5.

Tolerances as in test_gpu_spmm.py: the fp32 accumulators (HINM_OUT_F32) against the oracle with the literal
thresholds (relative Frobenius error <= 1e-3, max abs error <= 1e-2); 16-bit outputs must be the RNE
rounding of the kernel's own accumulators; bf16 outputs against the oracle rounded to bf16 within
max(1e-2, one ulp)."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu

OUT_F32, RELU = 2, 1


def _ulp_bf16(y):
    e = np.floor(np.log2(np.maximum(np.abs(y), 2.0 ** -14)))
    return np.exp2(e - 7)


@pytest.mark.parametrize("idx", [2, 5, 8, 11])
def test_prepared_c3_prefill_full(idx):
    """All M x 2048 outputs of the four C3 prefill cases through hinm_spmm_prepared with the kernel chosen by
    shape (512-column blocks, and for 11008 x 4096 the second launch on the remaining tiles)."""
    from tests import gpu_util as gu
    c = synth.c3_cases()[idx]
    assert c.N == 2048
    Wb = c.weights()
    p = gu.gpu_pack(Wb, c.dtype, c.V, c.Kv)
    vals, nm, vec = p.host()
    o_vals, o_nm, o_vec = orc.pack(Wb, c.dtype, c.V, c.Kv)
    assert np.array_equal(vec, o_vec) and np.array_equal(nm, o_nm) and np.array_equal(vals, o_vals)
    Wh = orc.unpack_fast(o_vals, o_nm, o_vec, c.M, c.K, c.V)
    Xb = c.activations()
    pin, pout = c.pi_in(), c.pi_out()
    want = orc.product(Wh, Xb, c.dtype, pin, pout).astype(np.float64)
    pr = gu.gpu_prepare(p, pin, pout)
    got32 = gu.gpu_spmm_prepared(pr, Xb, OUT_F32)
    gu.check_close(got32.astype(np.float64), want, what=f"{c.name} fp32 accumulators")
    got = gu.gpu_spmm_prepared(pr, Xb, 0)
    assert np.array_equal(got, orc.round_to_storage(got32, c.dtype)), "output is not the rounded accumulator"
    want_b = orc.decode(orc.round_to_storage(want.astype(np.float32), c.dtype), c.dtype)
    gotd = orc.decode(got, c.dtype)
    assert np.all(np.abs(gotd - want_b) <= np.maximum(1e-2, _ulp_bf16(want_b)))
    gu.check_close(gotd, want_b, max_abs=np.inf, what=f"{c.name} bf16 output")


def test_c4_chain_with_prepared_layers_full():
    """hinm_chain on layers that carry their hinm_prepare buffer (the branch bench.py --workload c4 times):
    all 4096 x 1024 outputs and the intermediate against the oracle's chain."""
    import torch
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    c = synth.c4()
    layers, host_layers, keep = [], [], []
    for l in (0, 1):
        p = gu.gpu_pack(c.weights(l), c.dtype, c.V, c.Kv)
        vals, nm, vec = p.host()
        o_vals, o_nm, o_vec = orc.pack(c.weights(l), c.dtype, c.V, c.Kv)
        assert np.array_equal(vec, o_vec) and np.array_equal(nm, o_nm) and np.array_equal(vals, o_vals)
        Wh = orc.unpack_fast(o_vals, o_nm, o_vec, c.M, c.K, c.V)
        pin, pout = c.pi_in(l), c.pi_out(l)
        host_layers.append((Wh, pin, pout, l == 0))
        pr = gu.gpu_prepare(p, pin, pout)
        keep.append(pr)
        # no canonical arrays, no permutations: everything the layer needs is in its prepared buffer
        layers.append(hinm.Layer(c.M, c.K, c.V, c.Kv, c.dtype, None, None, None, None, None,
                                 RELU if l == 0 else 0, pr.buf))
    Xb = c.activations()
    H = orc.spmm(host_layers[0][0], Xb, c.dtype, host_layers[0][1], host_layers[0][2], relu=True)
    want_acc = orc.product(host_layers[1][0], H, c.dtype, host_layers[1][1], host_layers[1][2]).astype(np.float64)
    want_bits = orc.chain(host_layers, Xb, c.dtype)
    nbytes = hinm.hinm_chain_sizes(layers, c.N)
    assert nbytes == c.M * c.N * 2
    scratch = torch.full((nbytes,), 0x7B, dtype=torch.uint8, device=gu.DEV)
    Y = torch.full((c.M, c.N), 0x7B7B, dtype=torch.int16, device=gu.DEV)
    hinm.hinm_chain(layers, c.N, gu.dev_bits(Xb), c.N, Y, c.N, scratch, nbytes)
    torch.cuda.synchronize()
    got = gu.host_bits(Y)
    gu.check_close(orc.decode(got, c.dtype), want_acc, what="C4 chain, prepared layers")
    # against the oracle's own rounded chain (its intermediate is rounded from another summation order, so
    # single fp16 roundings may flip): the stated tolerance again
    gu.check_close(orc.decode(got, c.dtype), orc.decode(want_bits, c.dtype), what="C4 chain vs rounded oracle chain")
    Hg = gu.host_bits(scratch.view(torch.int16).reshape(c.M, c.N))
    gu.check_close(orc.decode(Hg, c.dtype), orc.decode(H, c.dtype), what="C4 intermediate, prepared layers")
    assert (orc.decode(Hg, c.dtype) >= 0).all()
    # fp32 accumulators of the last layer through the same entry point
    layers[1].flags = OUT_F32
    Yf = torch.full((c.M, c.N), float("nan"), dtype=torch.float32, device=gu.DEV)
    hinm.hinm_chain(layers, c.N, gu.dev_bits(Xb), c.N, Yf, c.N, scratch, nbytes)
    torch.cuda.synchronize()
    acc = Yf.cpu().numpy()
    gu.check_close(acc.astype(np.float64), want_acc, what="C4 chain accumulators")
    assert np.array_equal(got, orc.round_to_storage(acc, c.dtype))


def test_c5_pack_every_tile_and_prepared_product_sampled():
    """C5 at full size.  hinm_pack against the oracle on all 128 tiles; then hinm_spmm_prepared (kernel chosen by
    shape: 128 x 512 blocks) against the oracle on two whole tiles plus eight rows of every tile (1280 rows), all
    8192 columns of each: every tile and every column block of the launch is covered."""
    import torch
    from tests import gpu_util as gu
    c = synth.c5()
    Wb = c.weights()
    p = gu.gpu_pack(Wb, c.dtype, c.V, c.Kv)
    vals, nm, vec = p.host()
    rng = np.random.default_rng(20496)
    whole = [37, 101]
    rows = []
    for t in range(c.T):
        rows.extend(t * c.V + (np.arange(c.V) if t in whole else np.sort(rng.choice(c.V, 8, replace=False))))
    rows = np.array(rows)
    Wh_rows = np.zeros((len(rows), c.K), dtype=np.uint16)
    for t in range(c.T):
        sl = slice(t * c.V, (t + 1) * c.V)
        ov, on, oc = orc.pack(Wb[sl], c.dtype, c.V, c.Kv)
        assert np.array_equal(vec[t], oc[0]), f"vector index of tile {t}"
        assert np.array_equal(nm[sl], on), f"NM index of tile {t}"
        assert np.array_equal(vals[sl], ov), f"stored values of tile {t}"
        Wh_t = orc.unpack_fast(ov, on, oc, c.V, c.K, c.V)
        sel = (rows // c.V) == t
        Wh_rows[sel] = Wh_t[rows[sel] - t * c.V]
    del Wb
    Xb = c.activations()
    pin, pout = c.pi_in(), c.pi_out()
    want = orc.product_rows(Wh_rows, Xb, c.dtype, pin)                   # binary64, [1280, 8192]
    pr = gu.gpu_prepare(p, pin, pout)
    X_dev = gu.dev_bits(Xb)
    got32 = gu.gpu_spmm_prepared(pr, Xb, OUT_F32, X_dev=X_dev)
    assert np.isfinite(got32).all()                                      # every output written (poison is NaN)
    sub = got32[pout[rows]].astype(np.float64)
    gu.check_close(sub, want, what="C5 prepared, fp32 accumulators on 1280 rows x 8192 columns")
    got = gu.gpu_spmm_prepared(pr, Xb, 0, X_dev=X_dev)
    assert np.array_equal(got, orc.round_to_storage(got32, c.dtype)), "output is not the rounded accumulator"
    want_b = orc.decode(orc.round_to_storage(want.astype(np.float32), c.dtype), c.dtype)
    gotd = orc.decode(got[pout[rows]], c.dtype)
    assert np.all(np.abs(gotd - want_b) <= np.maximum(1e-2, _ulp_bf16(want_b)))
    gu.check_close(gotd, want_b, max_abs=np.inf, what="C5 prepared, bf16 output")
    del got32, got
    torch.cuda.empty_cache()
