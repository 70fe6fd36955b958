"""GPU parity of hinm_icp_search (tile-wise input-channel permutation search, Section 4.2 of the paper)
against the CPU oracle.  Several assignments can reach the minimal cost, so what is compared is what is
unique: the cost of the assignment the GPU took, bit for bit against the oracle's cost matrix for the same
state, and its optimality against the oracle's solver; the rest (a valid move of one sample per partition)
is checked for validity.  Later iterations start from the GPU's own arrangement."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import gyro_oracle as gyro
from oracle import hinm_oracle as orc

pytestmark = pytest.mark.gpu


def _gpu_search(c, Wb, rho, vec, samples):
    import torch
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    iters, T, P = samples.shape
    wsb = hinm.hinm_icp_sizes(c.M, c.K, c.V, c.Kv, c.dtype)
    ws = torch.empty(wsb, dtype=torch.uint8, device=gu.DEV)
    vec_d = gu.dev_i32(vec)
    smp_d = torch.from_numpy(np.ascontiguousarray(samples, dtype=np.uint8)).to(gu.DEV)
    obj_d = torch.full((iters, T), float("nan"), dtype=torch.float64, device=gu.DEV)
    hinm.hinm_icp_search(c.M, c.K, c.V, c.Kv, c.dtype, gu.dev_bits(Wb), None if rho is None else gu.dev_f32(rho),
                         vec_d, smp_d, iters, obj_d, ws, wsb)
    torch.cuda.synchronize()
    return vec_d.cpu().numpy().reshape(T, c.Kv), obj_d.cpu().numpy()


def _check_iteration(c, Wb, rho, before, after, sampled, obj, tiles):
    """One iteration from `before` to `after` (both [T, Kv]) against the oracle."""
    P = c.Kv // 4
    for t in tiles:
        S = gyro.kept_saliency(Wb, c.dtype, rho, c.V, before[t], t)
        cost = gyro.icp_cost_fast(S, sampled[t])
        # the move the GPU made: slot 4 i + sampled[i] of partition i now holds the sample of partition assign[i]
        where = {int(before[t][4 * j + sampled[t][j]]): j for j in range(P)}
        assign = np.empty(P, dtype=np.int64)
        for i in range(P):
            for m in range(4):
                if m != sampled[t][i]:
                    assert after[t][4 * i + m] == before[t][4 * i + m], "a vector that was not sampled moved"
            assign[i] = where[int(after[t][4 * i + sampled[t][i]])]
        assert sorted(assign.tolist()) == list(range(P))
        assert obj[t] == gyro.assignment_cost(cost, assign), "reported cost is not the cost of the move made"
        best = gyro.assignment_cost(cost, gyro.icp_assign(cost))
        assert obj[t] <= best + 1e-9 * max(1.0, abs(best)), f"tile {t}: {obj[t]} is not the minimum {best}"


def test_hand_example_on_gpu():
    from tests.conftest import load_golden
    ex = load_golden("hand_example_icp.txt")
    c = synth.small_case(2, 8, 2, 8, 1, "f16", 0)
    Wb = synth.to_bits((ex["rho"] * np.array([[1], [-1]])).astype(np.float32), "f16")
    for rho in (None, ex["rho"].astype(np.float32)):
        vec, obj = _gpu_search(c, Wb, rho, ex["vec_idx"], ex["samples"].reshape(1, 1, 2))
        assert vec.tolist() == ex["vec_idx_after"].tolist()
        assert obj.tolist() == [[21.0]]


@pytest.mark.parametrize("M,K,V,Kv,dtype,scored", [
    (32, 48, 8, 24, "f16", False),
    (64, 200, 16, 104, "bf16", True),       # 26 partitions
    (96, 1200, 32, 1032, "f16", True),      # 258 partitions: more than one column per thread in the solver
    (16, 64, 1, 64, "bf16", False),         # single-row tiles
    (8, 4200, 4, 4096, "f16", True),        # 1024 partitions: the largest tile the solver takes
])
def test_every_iteration_against_the_oracle(M, K, V, Kv, dtype, scored):
    c = synth.small_case(M, K, V, Kv, 1, dtype, 90)
    Wb = c.weights()
    rng = np.random.default_rng(91)
    rho = (rng.standard_normal((M, K)) ** 2).astype(np.float32) if scored else None
    vec = orc.vector_index(Wb, dtype, V, Kv, rho)
    iters = 3
    samples = rng.integers(0, 4, size=(iters, c.T, Kv // 4))
    state = vec.copy()
    trace = []
    for it in range(iters):
        after, obj = _gpu_search(c, Wb, rho, state, samples[it:it + 1])
        _check_iteration(c, Wb, rho, state, after, samples[it], obj[0], range(c.T))
        trace.append(obj[0])
        state = after
    # one call with all iterations gives the same arrangement and the same objectives
    vec_all, obj_all = _gpu_search(c, Wb, rho, vec, samples)
    assert np.array_equal(vec_all, state) and np.array_equal(obj_all, np.stack(trace))
    # the objective never increases, from the starting arrangement on
    for t in range(c.T):
        start = gyro.pruned_saliency(gyro.kept_saliency(Wb, dtype, rho, V, vec[t], t))
        seq = [start] + [o[t] for o in trace]
        assert all(b <= a + 1e-9 * max(1.0, abs(a)) for a, b in zip(seq, seq[1:]))


def test_ties_everywhere():
    # integer scores with few distinct values: many assignments share the minimum; sums are exact
    c = synth.small_case(32, 96, 8, 48, 1, "f16", 92)
    Wb = c.weights()
    rng = np.random.default_rng(93)
    rho = rng.integers(0, 3, size=(c.M, c.K)).astype(np.float32)
    vec = orc.vector_index(Wb, c.dtype, c.V, c.Kv, rho)
    samples = rng.integers(0, 4, size=(1, c.T, c.Kv // 4))
    after, obj = _gpu_search(c, Wb, rho, vec, samples)
    _check_iteration(c, Wb, rho, vec, after, samples[0], obj[0], range(c.T))


def test_c2_layer_two_iterations_and_pack_with_the_result():
    from tests import gpu_util as gu
    c = synth.c2()
    Wb = c.weights()
    rng = np.random.default_rng(94)
    p0 = gu.gpu_pack(Wb, c.dtype, c.V, c.Kv)
    vec = p0.host()[2]
    samples = rng.integers(0, 4, size=(2, c.T, c.Kv // 4))
    mid, obj0 = _gpu_search(c, Wb, None, vec, samples[:1])
    _check_iteration(c, Wb, None, vec, mid, samples[0], obj0[0], [0, 17, 47])
    after, obj1 = _gpu_search(c, Wb, None, mid, samples[1:])
    _check_iteration(c, Wb, None, mid, after, samples[1], obj1[0], [3, 30])
    assert np.all(obj1[0] <= obj0[0] * (1 + 1e-12))
    # pack with the arrangement found: the vector index is the arrangement, and what 2:4 prunes is the objective
    sigma = np.stack([np.concatenate([after[t], np.setdiff1d(np.arange(c.K), after[t])]) for t in range(c.T)])
    vals, nm, pvec = gu.gpu_pack(Wb, c.dtype, c.V, c.Kv, sigma=sigma).host()
    assert np.array_equal(pvec, after)
    mag = np.abs(orc.decode(Wb, c.dtype))
    kept = np.abs(orc.decode(vals, c.dtype))
    for t in (0, 17, 47):
        rows = slice(t * c.V, (t + 1) * c.V)
        pruned = mag[rows][:, after[t]].sum() - kept[rows].sum()
        assert pruned == pytest.approx(obj1[0][t], rel=1e-9)
    # and it is an improvement over the ascending arrangement
    start = [gyro.pruned_saliency(gyro.kept_saliency(Wb, c.dtype, None, c.V, vec[t], t)) for t in (0, 17, 47)]
    assert all(obj1[0][t] < s for t, s in zip((0, 17, 47), start))


def test_costs_that_are_not_finite_leave_the_arrangement():
    c = synth.small_case(16, 32, 8, 16, 1, "f16", 95)
    Wb = c.weights()
    rho = np.full((c.M, c.K), np.nan, dtype=np.float32)
    vec = np.tile(np.arange(16, dtype=np.int32), (c.T, 1))
    samples = np.zeros((1, c.T, 4), dtype=np.uint8)
    after, _ = _gpu_search(c, Wb, rho, vec, samples)
    assert np.array_equal(after, vec)
