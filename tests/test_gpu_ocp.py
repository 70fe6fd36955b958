"""GPU parity of hinm_ocp_search (output-channel permutation search, Section 4.1 Eq. 2 / Section 4.2 of the
paper) against the CPU oracle.  As for the tile-wise search, several assignments can reach the minimum, so the
move the GPU made is checked for validity and its cost for optimality; the costs are binary64 sums whose
order differs between the two sides, so they are compared within 1e-11 relative (exactly for integer scores)."""
import numpy as np
import pytest

import hinm_synth as synth
from oracle import gyro_oracle as gyro

pytestmark = pytest.mark.gpu


def _gpu_search(c, Wb, rho, row_order, samples, clusters):
    import torch
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    iters, T, n = samples.shape
    wsb = hinm.hinm_ocp_sizes(c.M, c.K, c.V, c.Kv, c.dtype, n)
    ws = torch.empty(wsb, dtype=torch.uint8, device=gu.DEV)
    order_d = gu.dev_i32(row_order)
    obj_d = torch.full((iters,), float("nan"), dtype=torch.float64, device=gu.DEV)
    hinm.hinm_ocp_search(c.M, c.K, c.V, c.Kv, c.dtype, gu.dev_bits(Wb), None if rho is None else gu.dev_f32(rho),
                         order_d, gu.dev_i32(samples), None if clusters is None else gu.dev_i32(clusters), n, iters,
                         obj_d, ws, wsb)
    torch.cuda.synchronize()
    return order_d.cpu().numpy(), obj_d.cpu().numpy()


def _check_iteration(c, S, before, after, sampled, clusters, obj, exact):
    T, V, n = c.T, c.V, sampled.shape[1]
    rows0, rows1 = before.reshape(T, V), after.reshape(T, V)
    cost = gyro.ocp_cost(S, rows0, sampled, clusters, c.Kv)
    cl = np.arange(T * n).reshape(T, n) if clusters is None else clusters
    pool = [int(rows0[q // n, sampled[q // n, q % n]]) for q in range(T * n)]
    members = {tuple(pool[int(q)] for q in cl[j]): j for j in range(T)}
    assign = np.empty(T, dtype=np.int64)
    for i in range(T):
        stay = [p for p in range(V) if p not in set(sampled[i].tolist())]
        assert np.array_equal(rows1[i, stay], rows0[i, stay]), "a channel that was not sampled moved"
        assign[i] = members[tuple(int(x) for x in rows1[i, sampled[i]])]
    assert sorted(assign.tolist()) == list(range(T))
    assert sorted(after.tolist()) == list(range(c.M))
    took = gyro.assignment_cost(cost, assign)
    best = gyro.assignment_cost(cost, gyro.icp_assign(cost))
    if exact:
        assert obj == took and took == best
    else:
        assert obj == pytest.approx(took, rel=1e-11)
        assert took <= best * (1 + 1e-9) + 1e-12


def test_hand_example_on_gpu():
    # the example of tests/golden/hand_example_ocp.txt with every input channel repeated four times (K = 16,
    # Kv = 8: the ABI wants Kv % 8 == 0): all costs are four times those of the file, the move is the same
    from tests.conftest import load_golden
    ex = load_golden("hand_example_ocp.txt")
    rho = np.repeat(ex["rho"], 4, axis=1).astype(np.float32)
    c = synth.small_case(4, 16, 2, 8, 1, "bf16", 0)
    Wb = synth.to_bits(rho, "bf16")
    for r in (rho, None):
        order, obj = _gpu_search(c, Wb, r, ex["row_order"].reshape(-1), ex["samples"].reshape(1, 2, 1).astype(np.int32), None)
        assert order.tolist() == ex["row_order_after"].reshape(-1).tolist()
        assert obj.tolist() == [4.0 * float(ex["objective"][0, 0])]


@pytest.mark.parametrize("M,K,V,Kv,n,dtype,scored,clustered", [
    (48, 40, 8, 16, 3, "f16", False, False),
    (64, 72, 16, 32, 5, "bf16", True, True),
    (64, 2000, 16, 1000, 2, "f16", True, True),       # 16 scores per thread in the cost kernel
    (32, 5000, 8, 2504, 1, "bf16", False, False),     # 64 scores per thread; one sample per tile
    (40, 24, 1, 8, 1, "f16", True, True),             # single-channel tiles
])
def test_every_iteration_against_the_oracle(M, K, V, Kv, n, dtype, scored, clustered):
    c = synth.small_case(M, K, V, Kv, 1, dtype, 96)
    Wb = c.weights()
    rng = np.random.default_rng(97)
    rho = (rng.standard_normal((M, K)) ** 2).astype(np.float32) if scored else None
    S = gyro.saliency_matrix(Wb, dtype, rho)
    iters = 3
    samples = np.stack([np.stack([rng.permutation(V)[:n] for _ in range(c.T)]) for _ in range(iters)]).astype(np.int32)
    clusters = (np.stack([rng.permutation(c.T * n).reshape(c.T, n) for _ in range(iters)]).astype(np.int32)
                if clustered else None)
    start = rng.permutation(M).astype(np.int32)
    state, trace = start.copy(), []
    for it in range(iters):
        cl = None if clusters is None else clusters[it:it + 1]
        after, obj = _gpu_search(c, Wb, rho, state, samples[it:it + 1], cl)
        _check_iteration(c, S, state, after, samples[it], None if clusters is None else clusters[it], obj[0], exact=False)
        trace.append(obj[0])
        state = after
    all_order, all_obj = _gpu_search(c, Wb, rho, start, samples, clusters)
    assert np.array_equal(all_order, state) and np.array_equal(all_obj, np.array(trace))
    if not clustered:      # the identity assignment is always available: the objective cannot rise
        first = sum(gyro.vector_pruned_saliency(S[start[t * V:(t + 1) * V]], Kv) for t in range(c.T))
        seq = [first] + trace
        assert all(b <= a * (1 + 1e-11) for a, b in zip(seq, seq[1:]))
    final = sum(gyro.vector_pruned_saliency(S[state[t * V:(t + 1) * V]], Kv) for t in range(c.T))
    assert final == pytest.approx(trace[-1], rel=1e-11)


def test_integer_scores_are_exact_and_ties_are_handled():
    c = synth.small_case(96, 64, 8, 24, 1, "f16", 98)
    Wb = c.weights()
    rng = np.random.default_rng(99)
    rho = rng.integers(0, 4, size=(c.M, c.K)).astype(np.float32)      # many equal column scores at the threshold
    S = gyro.saliency_matrix(Wb, c.dtype, rho)
    samples = np.stack([rng.permutation(c.V)[:2] for _ in range(c.T)])[None].astype(np.int32)
    start = np.arange(c.M, dtype=np.int32)
    after, obj = _gpu_search(c, Wb, rho, start, samples, None)
    _check_iteration(c, S, start, after, samples[0], None, obj[0], exact=True)


def test_c2_layer_one_iteration():
    c = synth.c2()
    Wb = c.weights()
    rng = np.random.default_rng(100)
    S = gyro.saliency_matrix(Wb, c.dtype, None)
    n = 8
    samples = np.stack([rng.permutation(c.V)[:n] for _ in range(c.T)])[None].astype(np.int32)
    clusters = rng.permutation(c.T * n).reshape(1, c.T, n).astype(np.int32)
    start = np.arange(c.M, dtype=np.int32)
    after, obj = _gpu_search(c, Wb, None, start, samples, clusters)
    _check_iteration(c, S, start, after, samples[0], clusters[0], obj[0], exact=False)


# ---- clustering phase: balanced K-means over the sampled channels -----------------------------------------

def _gpu_cluster(c, Wb, rho, row_order, sampled, rounds, centroids=None):
    import torch
    import paper_2407_20496_amd as hinm
    from tests import gpu_util as gu
    T, n = sampled.shape
    wsb = hinm.hinm_ocp_cluster_sizes(c.M, c.K, c.V, c.Kv, c.dtype, n)
    ws = torch.empty(wsb, dtype=torch.uint8, device=gu.DEV)
    cen = (torch.full((T, c.K), float("nan"), dtype=torch.float64, device=gu.DEV) if centroids is None
           else torch.from_numpy(np.ascontiguousarray(centroids)).to(gu.DEV))
    clusters = torch.full((T, n), -1, dtype=torch.int32, device=gu.DEV)
    obj = torch.full((rounds,), float("nan"), dtype=torch.float64, device=gu.DEV)
    hinm.hinm_ocp_cluster(c.M, c.K, c.V, c.Kv, c.dtype, gu.dev_bits(Wb), None if rho is None else gu.dev_f32(rho),
                          gu.dev_i32(row_order), gu.dev_i32(sampled), n, rounds, cen, centroids is None, clusters, obj,
                          ws, wsb)
    torch.cuda.synchronize()
    return clusters.cpu().numpy(), cen.cpu().numpy(), obj.cpu().numpy()


@pytest.mark.parametrize("M,K,V,Kv,n,dtype,scored", [
    (48, 40, 8, 16, 3, "f16", False),
    (64, 300, 16, 152, 5, "bf16", True),
    (40, 24, 1, 8, 1, "f16", True),
])
def test_balanced_kmeans_round_by_round(M, K, V, Kv, n, dtype, scored):
    c = synth.small_case(M, K, V, Kv, 1, dtype, 101)
    Wb = c.weights()
    rng = np.random.default_rng(102)
    rho = (rng.standard_normal((M, K)) ** 2).astype(np.float32) if scored else None
    S = gyro.saliency_matrix(Wb, dtype, rho)
    row_order = rng.permutation(M).astype(np.int32)
    sampled = np.stack([rng.permutation(V)[:n] for _ in range(c.T)]).astype(np.int32)
    F = gyro.sampled_features(S, row_order.reshape(c.T, V), sampled)
    cen, trace = None, []
    for r in range(3):
        start = gyro.kmeans_initial_centroids(F, n) if cen is None else cen
        clusters, cen_new, obj = _gpu_cluster(c, Wb, rho, row_order, sampled, 1, cen)
        assert sorted(clusters.reshape(-1).tolist()) == list(range(c.T * n))          # every item once: n per cluster
        assert all(clusters[k].tolist() == sorted(clusters[k].tolist()) for k in range(c.T))
        label = np.empty(c.T * n, dtype=np.int64)
        for k in range(c.T):
            label[clusters[k]] = k
        d = gyro.kmeans_distances(F, start)
        assert obj[0] == gyro.kmeans_objective(d, label)                               # same distances, same order
        best = gyro.kmeans_objective(d, gyro.kmeans_balanced_assignment(d, n))
        assert obj[0] <= best * (1 + 1e-9) + 1e-300
        assert np.array_equal(cen_new, gyro.kmeans_centroids(F, label, c.T, n))
        trace.append(obj[0])
        cen = cen_new
    assert all(b <= a * (1 + 1e-12) for a, b in zip(trace, trace[1:]))
    # three rounds in one call: the same clusters, centroids and objectives
    clusters3, cen3, obj3 = _gpu_cluster(c, Wb, rho, row_order, sampled, 3, None)
    assert np.array_equal(clusters3, clusters) and np.array_equal(cen3, cen) and np.array_equal(obj3, np.array(trace))


def test_clusters_feed_the_search_on_the_c2_layer():
    c = synth.c2()
    Wb = c.weights()
    rng = np.random.default_rng(103)
    S = gyro.saliency_matrix(Wb, c.dtype, None)
    n = 8
    sampled = np.stack([rng.permutation(c.V)[:n] for _ in range(c.T)]).astype(np.int32)
    start = np.arange(c.M, dtype=np.int32)
    clusters, cen, obj = _gpu_cluster(c, Wb, None, start, sampled, 2, None)
    assert sorted(clusters.reshape(-1).tolist()) == list(range(c.T * n)) and obj[1] <= obj[0]
    F = gyro.sampled_features(S, start.reshape(c.T, c.V), sampled)
    d0 = gyro.kmeans_distances(F, gyro.kmeans_initial_centroids(F, n))
    assert obj[0] <= gyro.kmeans_objective(d0, gyro.kmeans_balanced_assignment(d0, n)) * (1 + 1e-9)
    after, sobj = _gpu_search(c, Wb, None, start, sampled[None], clusters[None].astype(np.int32))
    _check_iteration(c, S, start, after, sampled, clusters, sobj[0], exact=False)
