"""The launch configuration that bench.py times: several launches captured once into a HIP graph and
replayed.  Every entry point on the timed path is captured here (two launches per graph, on two
buffer sets), replayed three times with eager work and a synchronisation between the replays, and
every replay is compared bit for bit with the eager result, which is itself checked against the CPU
oracle.  The library records kernels only (no memset, copy or allocation nodes)."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu

POISON = 0x7B7B


def _capture(torch, launch_all):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        launch_all()                      # warm-up on the capture stream (first-call set-up happens here)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            launch_all()
    torch.cuda.current_stream().wait_stream(side)
    return graph


def _replays(torch, graph, outputs, eager_bits, what):
    for rep in range(3):
        for Y in outputs:
            Y.fill_(POISON)               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, Y in enumerate(outputs):
            got = Y.cpu().numpy().view(np.uint16)
            assert np.array_equal(got, eager_bits), f"{what}: replay {rep}, buffer set {k} differs from the eager launch"


def _oracle_acc(case, host):
    vals, nm, vec = host
    W = orc.unpack_fast(vals, nm, vec, case.M, case.K, case.V)
    return orc.product(W, case.activations(), case.dtype, case.pi_in(), case.pi_out()).astype(np.float64)


def _check_vs_oracle(case, eager_bits, want_acc):
    from tests import gpu_util as gu
    got = orc.decode(eager_bits, case.dtype)
    if case.dtype == "f16":
        gu.check_close(got, want_acc, what=case.name)
    else:   # bf16 outputs carry their own rounding step: compare with the rounded oracle
        want = orc.decode(orc.round_to_storage(want_acc.astype(np.float32), "bf16"), "bf16")
        gu.check_close(got, want, max_abs=np.inf, what=case.name)


def _prepared_case(case, N, variant=0):
    import torch
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    p = gu.gpu_pack(case.weights(), case.dtype, case.V, case.Kv)
    pr = gu.gpu_prepare(p, case.pi_in(), case.pi_out())
    Xb = case.activations()
    ld = N if N == 1 else (N + 7) // 8 * 8
    Xp = np.zeros((case.K, ld), dtype=np.uint16)
    Xp[:, :N] = Xb
    eager = gu.gpu_spmm_prepared(pr, Xb, variant=variant)
    _check_vs_oracle(case, eager, _oracle_acc(case, p.host()))
    sets = [(pr.buf if k == 0 else pr.buf.clone(), gu.dev_bits(Xp),
             torch.full((case.M, ld), POISON, dtype=torch.int16, device=gu.DEV)) for k in range(2)]

    def launch_all():
        for buf, X, Y in sets:
            hinm.hinm_spmm_prepared(case.M, case.K, case.V, case.Kv, case.dtype, N, buf, X, ld, Y, ld, variant << 16, None, 0)
    graph = _capture(torch, launch_all)
    full = np.full((case.M, ld), POISON, dtype=np.uint16)
    full[:, :N] = eager
    _replays(torch, graph, [Y for _, _, Y in sets], full, case.name)


def test_graph_replay_c2_panel_kernel():
    c = synth.c2()
    _prepared_case(c, c.N)


@pytest.mark.parametrize("idx", [1, 6])   # 16 columns; one column with the input vector staged in LDS
def test_graph_replay_decode(idx):
    c = synth.c3_cases()[idx]
    _prepared_case(c, c.N)


@pytest.mark.parametrize("variant", [3, 16, 14])   # 512-column blocks (copies in chunks), 16 waves, 256-column blocks
def test_graph_replay_tile_kernel_ragged(variant):
    import paper_2407_20496_amd as hinm
    c = synth.small_case(384, 2048, 128, 1024, 1100, "bf16", 97)
    ld = (c.N + 7) // 8 * 8
    assert "spmm_tile_prepared_kernel" in hinm.hinm_spmm_prepared_plan(c.M, c.K, c.V, c.Kv, c.dtype, c.N, ld, ld, variant << 16)[0]
    _prepared_case(c, c.N, variant)


def test_graph_replay_canonical_arrays():
    import torch
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    c = synth.small_case(256, 1024, 64, 512, 520, "f16", 98)
    p = gu.gpu_pack(c.weights(), c.dtype, c.V, c.Kv)
    Xb = c.activations()
    eager = gu.gpu_spmm(p, Xb, c.pi_in(), c.pi_out())
    _check_vs_oracle(c, eager, _oracle_acc(c, p.host()))
    ld = (c.N + 7) // 8 * 8
    X = gu.dev_bits(Xb)
    pin, pout = gu.dev_i32(c.pi_in()), gu.dev_i32(c.pi_out())
    Ys = [torch.full((c.M, ld), POISON, dtype=torch.int16, device=gu.DEV) for _ in range(2)]

    def launch_all():
        for Y in Ys:
            hinm.hinm_spmm(c.M, c.K, c.V, c.Kv, c.dtype, c.N, p.vals, p.nm_idx, p.vec_idx, pin, pout, X, ld, Y, ld, 0)
    graph = _capture(torch, launch_all)
    _replays(torch, graph, Ys, eager, c.name)


def test_graph_replay_chain_and_pack():
    """hinm_chain (two launches, the intermediate in the caller's scratch) and hinm_pack (three kernels and a
    workspace) in one graph: the chain reads what the pack of the same replay wrote."""
    import torch
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    M = K = 512
    V, Kv, N, dtype = 64, 256, 200, "f16"
    cases = [synth.small_case(M, K, V, Kv, N, dtype, 99 + l) for l in (0, 1)]
    Xb = cases[0].activations()
    ld = (N + 7) // 8 * 8
    Xp = np.zeros((K, ld), dtype=np.uint16)
    Xp[:, :N] = Xb
    X = gu.dev_bits(Xp)
    Wd = [gu.dev_bits(c.weights()) for c in cases]
    vb, nb, cb, wb = hinm.hinm_pack_sizes(M, K, V, Kv, dtype)
    packed = [(torch.empty(vb // 2, dtype=torch.int16, device=gu.DEV), torch.empty(nb, dtype=torch.uint8, device=gu.DEV),
               torch.empty(cb // 4, dtype=torch.int32, device=gu.DEV)) for _ in cases]
    ws = torch.empty(wb // 8, dtype=torch.float64, device=gu.DEV)
    pis = [(gu.dev_i32(c.pi_in()), gu.dev_i32(c.pi_out())) for c in cases]
    layers = [hinm.Layer(M, K, V, Kv, dtype, v, n, ve, pi, po, 1 if l == 0 else 0)
              for l, ((v, n, ve), (pi, po)) in enumerate(zip(packed, pis))]
    nbytes = hinm.hinm_chain_sizes(layers, N)
    scratch = torch.empty(nbytes, dtype=torch.uint8, device=gu.DEV)
    Y = torch.full((M, ld), POISON, dtype=torch.int16, device=gu.DEV)

    def launch_all():
        for W, (v, n, ve) in zip(Wd, packed):
            hinm.hinm_pack(M, K, V, Kv, dtype, W, v, n, ve, ws, wb)
        hinm.hinm_chain(layers, N, X, ld, Y, ld, scratch, nbytes)
    launch_all()
    torch.cuda.synchronize()
    eager = Y.cpu().numpy().view(np.uint16).copy()
    # the eager result against the oracle: pack each layer, then the chain with ReLU between
    host_layers = []
    for l, c in enumerate(cases):
        vals, nm, vec = orc.pack(c.weights(), dtype, V, Kv)
        assert np.array_equal(vals, packed[l][0].cpu().numpy().view(np.uint16).reshape(M, Kv // 2))
        assert np.array_equal(vec, packed[l][2].cpu().numpy().reshape(M // V, Kv))
        host_layers.append((orc.unpack_fast(vals, nm, vec, M, K, V), c.pi_in(), c.pi_out(), l == 0))
    H = orc.spmm(host_layers[0][0], Xb, dtype, host_layers[0][1], host_layers[0][2], relu=True)
    want = orc.product(host_layers[1][0], H, dtype, host_layers[1][1], host_layers[1][2]).astype(np.float64)
    gu.check_close(orc.decode(eager[:, :N], dtype), want, what="chain of two packed layers")
    graph = _capture(torch, launch_all)
    outputs = [Y]
    for rep in range(3):
        Y.fill_(POISON)
        for v, n, ve in packed:           # the packed arrays are rewritten by every replay
            v.fill_(POISON)
            ve.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(Y.cpu().numpy().view(np.uint16), eager), f"replay {rep}"
    del outputs
