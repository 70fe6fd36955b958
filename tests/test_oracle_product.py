"""Pins for the oracle's product with channel orders and the chain (no GPU)."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc


def _packed(case):
    Wb = case.weights()
    vals, nm, vec = orc.pack(Wb, case.dtype, case.V, case.Kv)
    Wh = orc.unpack_fast(vals, nm, vec, case.M, case.K, case.V)
    return Wb, vals, nm, vec, Wh


def test_hand_example_product(hand_example):
    ex = hand_example
    for dtype in ("f16", "bf16"):
        Wb = synth.to_bits(ex["W"].astype(np.float32), dtype)
        Xb = synth.to_bits(ex["X"].astype(np.float32), dtype)
        vals, nm, vec = orc.pack(Wb, dtype, 4, 8)
        Wh = orc.unpack(vals, nm, vec, 4, 16, 4)
        pi_in, pi_out = ex["pi_in"][0], ex["pi_out"][0]
        for kw in (dict(), dict(acc=np.float64), dict(naive=True)):
            Y = orc.product(Wh, Xb, dtype, pi_in, pi_out, **kw)
            assert Y.tolist() == ex["Y"].astype(np.float64).tolist()
        assert orc.decode(orc.spmm(Wh, Xb, dtype, pi_in, pi_out), dtype).tolist() == ex["Y"].tolist()


def test_permutation_matrices_definitions():
    pi = np.array([2, 0, 3, 1])
    X = np.arange(8.0).reshape(4, 2)
    assert np.array_equal(orc.perm_matrix_in(pi, 4, np.float64) @ X, X[pi])           # gather
    Z = np.arange(8.0).reshape(4, 2)
    Y = orc.perm_matrix_out(pi, 4, np.float64) @ Z
    for r in range(4):
        assert np.array_equal(Y[pi[r]], Z[r])                                         # scatter
    # both are permutation matrices
    for P in (orc.perm_matrix_in(pi, 4), orc.perm_matrix_out(pi, 4)):
        assert np.array_equal(P.sum(0), np.ones(4)) and np.array_equal(P.sum(1), np.ones(4))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_identity_permutations_reduce_to_plain_matmul(dtype):
    case = synth.small_case(64, 96, 16, 48, 24, dtype, 21)
    _, _, _, _, Wh = _packed(case)
    Xb = case.activations()
    Y = orc.product(Wh, Xb, dtype, None, None, acc=np.float64)
    ref = orc.decode(Wh, dtype) @ orc.decode(Xb, dtype)
    assert np.array_equal(Y, ref)
    ident_in, ident_out = np.arange(case.K), np.arange(case.M)
    assert np.array_equal(orc.product(Wh, Xb, dtype, ident_in, ident_out, acc=np.float64), ref)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_permutation_algebra_with_index_ops(dtype):
    # matrices in the oracle, plain indexing here
    case = synth.small_case(64, 96, 16, 48, 24, dtype, 22)
    _, _, _, _, Wh = _packed(case)
    Xb = case.activations()
    pi_in, pi_out = case.pi_in(), case.pi_out()
    Y = orc.product(Wh, Xb, dtype, pi_in, pi_out, acc=np.float64)
    Z = orc.decode(Wh, dtype) @ orc.decode(Xb, dtype)[pi_in]
    want = np.empty_like(Z)
    want[pi_out] = Z
    assert np.array_equal(Y, want)
    # fp32 product stays within the textbook error bound of the fp64 one
    Y32 = orc.product(Wh, Xb, dtype, pi_in, pi_out)
    bound = case.Kv / 2 * 2.0 ** -24 * (np.abs(orc.decode(Wh, dtype)) @ np.abs(orc.decode(Xb, dtype)[pi_in])).max() * 2
    assert np.abs(Y32 - want).max() <= bound


def test_naive_loop_agrees_with_library_matmul():
    case = synth.small_case(16, 16, 4, 8, 3, "f16", 23)
    _, _, _, _, Wh = _packed(case)
    Xb = case.activations()
    a = orc.product(Wh, Xb, "f16", case.pi_in(), case.pi_out(), naive=True)
    b = orc.product(Wh, Xb, "f16", case.pi_in(), case.pi_out(), acc=np.float64)
    assert a.dtype == np.float32
    assert np.abs(a - b).max() <= 1e-5


def test_full_keep_is_plain_two_four_gemm():
    # s_v = 0: every column survives, vec_idx is the identity, result is an
    # ordinary 2:4-sparse GEMM
    case = synth.small_case(32, 64, 32, 64, 8, "bf16", 24)
    Wb, vals, nm, vec, Wh = _packed(case)
    assert vec.tolist() == [list(range(64))]
    Wd = orc.decode(Wb, "bf16").reshape(32, 16, 4)
    keep = np.zeros_like(Wd, dtype=bool)
    order = np.argsort(-np.abs(Wd), axis=-1, kind="stable")[..., :2]
    np.put_along_axis(keep, order, True, axis=-1)
    ref = (Wd * keep).reshape(32, 64) @ orc.decode(case.activations(), "bf16")
    assert np.array_equal(orc.product(Wh, case.activations(), "bf16", acc=np.float64), ref)


def test_tile_order_invariance():
    # Section 3.2: tiles are independent, so re-ordering whole 4-groups of the
    # vector index (together with their values and nibbles) inside a tile
    # leaves the product unchanged.
    case = synth.small_case(32, 64, 16, 32, 8, "f16", 25)
    Wb, vals, nm, vec, Wh = _packed(case)
    rng = np.random.default_rng(1)
    G = case.Kv // 4
    vals2, vec2 = vals.copy(), vec.copy()
    nib = np.stack([nm & 0xF, nm >> 4], axis=-1).reshape(case.M, G)
    nib2 = nib.copy()
    for t in range(case.T):
        perm = rng.permutation(G)
        vec2[t] = vec[t].reshape(G, 4)[perm].reshape(-1)
        rows = slice(t * case.V, (t + 1) * case.V)
        vals2[rows] = vals[rows].reshape(case.V, G, 2)[:, perm].reshape(case.V, -1)
        nib2[rows] = nib[rows][:, perm]
    nm2 = (nib2[:, 0::2] | (nib2[:, 1::2] << 4)).astype(np.uint8)
    Wh2 = orc.unpack(vals2, nm2, vec2, case.M, case.K, case.V)
    assert np.array_equal(Wh2, Wh)
    Xb = case.activations()
    assert np.array_equal(orc.product(Wh2, Xb, "f16", case.pi_in(), case.pi_out()),
                          orc.product(Wh, Xb, "f16", case.pi_in(), case.pi_out()))


def test_product_entries_matches_matrix_form():
    case = synth.small_case(64, 96, 16, 48, 24, "bf16", 26)
    _, _, _, _, Wh = _packed(case)
    Xb = case.activations()
    pi_in, pi_out = case.pi_in(), case.pi_out()
    Y = orc.product(Wh, Xb, "bf16", pi_in, pi_out, acc=np.float64)
    rows, cols = [0, 5, 17, 63], [0, 3, 23]
    got = orc.product_entries(Wh, Xb, "bf16", pi_in, pi_out, rows, cols)
    for a, r in enumerate(rows):
        assert np.allclose(got[a], Y[pi_out[r], cols], rtol=1e-13, atol=1e-13)
    Yr = orc.product(Wh, Xb, "bf16", pi_in, pi_out, acc=np.float64, relu=True)
    got = orc.product_entries(Wh, Xb, "bf16", pi_in, pi_out, rows, cols, relu=True)
    for a, r in enumerate(rows):
        assert np.allclose(got[a], Yr[pi_out[r], cols], rtol=1e-13, atol=1e-13)
    assert Yr.min() == 0.0


def test_product_rows_matches_matrix_form_and_entry_form():
    # the row-subset form used for sampled checks of large layers: against the explicit permutation
    # matrices (binary64) and against the element-by-element sum, with orders that are not involutions
    case = synth.small_case(64, 96, 16, 48, 24, "bf16", 29)
    _, _, _, _, Wh = _packed(case)
    Xb = case.activations()
    pi_in, pi_out = case.pi_in(), case.pi_out()
    assert not np.array_equal(pi_in[pi_in], np.arange(case.K))
    Y = orc.product(Wh, Xb, "bf16", pi_in, pi_out, acc=np.float64)
    rows = np.array([0, 5, 17, 40, 63])
    got = orc.product_rows(Wh[rows], Xb, "bf16", pi_in)
    assert got.dtype == np.float64 and got.shape == (5, 24)
    assert np.allclose(got, Y[pi_out[rows]], rtol=1e-13, atol=1e-13)
    ent = orc.product_entries(Wh, Xb, "bf16", pi_in, pi_out, rows, np.arange(24))
    assert np.allclose(got, ent, rtol=1e-13, atol=1e-13)
    # a swapped direction of pi_in (scatter instead of gather) must not pass
    inv = np.argsort(pi_in)
    assert not np.allclose(orc.product_rows(Wh[rows], Xb, "bf16", inv), Y[pi_out[rows]], rtol=1e-6, atol=1e-6)
    # identity order and ReLU
    Y0 = orc.product(Wh, Xb, "bf16", None, None, acc=np.float64, relu=True)
    assert np.allclose(orc.product_rows(Wh[rows], Xb, "bf16", None, relu=True), Y0[rows], rtol=1e-13, atol=1e-13)


def test_chain_equals_composition_and_identity_case():
    case = synth.small_case(64, 64, 16, 32, 12, "f16", 27)
    Wh1 = _packed(case)[4]
    W2b = case.weights(layer=1)
    v2 = orc.pack(W2b, "f16", 16, 32)
    Wh2 = orc.unpack_fast(*v2, 64, 64, 16)
    Xb = case.activations()
    p1i, p1o, p2i, p2o = case.pi_in(0), case.pi_out(0), case.pi_in(1), case.pi_out(1)
    got = orc.chain([(Wh1, p1i, p1o, True), (Wh2, p2i, p2o, False)], Xb, "f16")
    H = orc.spmm(Wh1, Xb, "f16", p1i, p1o, relu=True)
    assert np.array_equal(got, orc.spmm(Wh2, H, "f16", p2i, p2o))
    # all orders identity: W2 relu(W1 X) with the intermediate rounded to fp16
    got = orc.chain([(Wh1, None, None, True), (Wh2, None, None, False)], Xb, "f16", acc=np.float64)
    H = np.maximum(orc.decode(Wh1, "f16") @ orc.decode(Xb, "f16"), 0).astype(np.float16)
    want = (orc.decode(Wh2, "f16") @ H.astype(np.float64)).astype(np.float16)
    assert np.array_equal(got, want.view(np.uint16))


def test_independent_orders_need_no_permute_pass():
    # Section 3.2, "maintaining layer consistency": layer 2 may read layer 1's
    # output in layer 1's own output order if its input order absorbs it:
    # using pi_in' = pi_out1[pi_in2] on the scattered H equals using pi_in2 on
    # the un-scattered H.
    case = synth.small_case(64, 64, 16, 32, 12, "f16", 28)
    Wh1 = _packed(case)[4]
    Wh2 = orc.unpack_fast(*orc.pack(case.weights(layer=1), "f16", 16, 32), 64, 64, 16)
    Xb = case.activations()
    p1o, p2i = case.pi_out(0), case.pi_in(1)
    H_plain = orc.spmm(Wh1, Xb, "f16", None, None, relu=True)
    H_scat = orc.spmm(Wh1, Xb, "f16", None, p1o, relu=True)
    a = orc.spmm(Wh2, H_plain, "f16", p2i, None)
    b = orc.spmm(Wh2, H_scat, "f16", p1o[p2i], None)
    assert np.array_equal(a, b)
