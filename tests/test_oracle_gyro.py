"""Pins for the oracle of the tile-wise input-channel permutation search (no GPU)."""
import itertools

import numpy as np
import pytest

import hinm_synth as synth
from oracle import gyro_oracle as gyro
from oracle import hinm_oracle as orc
from tests.conftest import load_golden


def test_hand_example():
    ex = load_golden("hand_example_icp.txt")
    S = ex["rho"].astype(np.float64)
    sampled = ex["samples"].reshape(-1)
    cost = gyro.icp_cost(S, sampled)
    assert cost.tolist() == ex["cost"].astype(np.float64).tolist()
    assign = gyro.icp_assign(cost)
    assert assign.tolist() == ex["assign"].reshape(-1).tolist()
    assert gyro.assignment_cost(cost, assign) == float(ex["objective"][0, 0])
    after = gyro.icp_apply(ex["vec_idx"].reshape(-1), sampled, assign)
    assert after.tolist() == ex["vec_idx_after"].reshape(-1).tolist()
    assert gyro.pruned_saliency(S[:, after]) == float(ex["objective"][0, 0])
    # the same through the search on a weight matrix whose magnitudes are these scores
    Wb = synth.to_bits((ex["rho"] * np.array([[1], [-1]])).astype(np.float32), "f16")
    vec, obj = gyro.icp_search(Wb, "f16", None, 2, ex["vec_idx"], sampled.reshape(1, 1, 2))
    assert vec.tolist() == ex["vec_idx_after"].tolist() and obj.tolist() == [[21.0]]


def _integer_tile(V, Kv, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, 20, size=(V, Kv)).astype(np.float64), rng.integers(0, 4, size=Kv // 4)


@pytest.mark.parametrize("P", [2, 3, 5, 6])
def test_assignment_is_the_brute_force_minimum(P):
    S, sampled = _integer_tile(3, 4 * P, 70 + P)
    cost = gyro.icp_cost(S, sampled)
    best = min(sum(cost[i, perm[i]] for i in range(P)) for perm in itertools.permutations(range(P)))
    assign = gyro.icp_assign(cost)
    assert sorted(assign.tolist()) == list(range(P))
    assert gyro.assignment_cost(cost, assign) == best


def test_cost_is_the_pruned_saliency_of_the_arrangement_it_describes():
    # integer scores: every sum is exact, so the identities hold bit for bit
    S, sampled = _integer_tile(5, 24, 81)
    P = 6
    cost = gyro.icp_cost(S, sampled)
    arrangement = np.arange(24)
    ident = np.arange(P)
    assert gyro.assignment_cost(cost, ident) == gyro.pruned_saliency(S)          # nothing moves
    for perm in ([1, 0, 2, 3, 4, 5], [5, 4, 3, 2, 1, 0], [2, 0, 1, 4, 5, 3]):
        after = gyro.icp_apply(arrangement, sampled, np.array(perm))
        assert sorted(after.tolist()) == list(range(24))
        assert gyro.assignment_cost(cost, np.array(perm)) == gyro.pruned_saliency(S[:, after])
    # brute force of one entry straight from the definition of the 2:4 mask: keep the two largest of four
    i, j = 2, 4
    four = np.stack([S[:, 4 * i + m] for m in range(4) if m != sampled[i]] + [S[:, 4 * j + sampled[j]]], axis=1)
    assert cost[i, j] == (four.sum(axis=1) - np.sort(four, axis=1)[:, 2:].sum(axis=1)).sum()


@pytest.mark.parametrize("dtype,scored", [("f16", False), ("bf16", True)])
def test_search_never_increases_the_objective_and_matches_the_packing_oracle(dtype, scored):
    c = synth.small_case(32, 48, 8, 24, 4, dtype, 82)
    Wb = c.weights()
    rng = np.random.default_rng(83)
    rho = rng.integers(0, 50, size=(c.M, c.K)).astype(np.float32) if scored else None
    vec0 = orc.vector_index(Wb, dtype, c.V, c.Kv, rho)
    iters = 4
    samples = rng.integers(0, 4, size=(iters, c.T, c.Kv // 4))
    vec, obj = gyro.icp_search(Wb, dtype, rho, c.V, vec0, samples)
    for t in range(c.T):
        assert sorted(vec[t].tolist()) == vec0[t].tolist()               # the same columns, re-arranged
        start = gyro.pruned_saliency(gyro.kept_saliency(Wb, dtype, rho, c.V, vec0[t], t))
        trace = [start] + obj[:, t].tolist()
        assert all(b <= a + 1e-9 * max(1.0, abs(a)) for a, b in zip(trace, trace[1:]))
    # the final arrangement, handed to the packing oracle as a tile-wise order, prunes exactly the final objective
    sigma = np.stack([np.concatenate([vec[t], np.setdiff1d(np.arange(c.K), vec[t])]) for t in range(c.T)])
    vals, nm, pvec = orc.pack(Wb, dtype, c.V, c.Kv, sigma=sigma, rho=rho)
    assert np.array_equal(pvec, vec)
    kept = orc.mask(nm, pvec, c.M, c.K, c.V)
    sal = rho.astype(np.float64) if scored else np.abs(orc.decode(Wb, dtype))
    for t in range(c.T):
        rows = slice(t * c.V, (t + 1) * c.V)
        pruned = sal[rows][:, vec[t]].sum() - (sal[rows] * kept[rows]).sum()
        assert pruned == pytest.approx(obj[-1, t], rel=1e-12, abs=1e-12)


def test_fast_cost_is_the_plain_cost_bit_for_bit():
    rng = np.random.default_rng(84)
    S = (rng.standard_normal((7, 40)) ** 2).astype(np.float32).astype(np.float64)   # sums that do round
    sampled = rng.integers(0, 4, size=10)
    assert np.array_equal(gyro.icp_cost_fast(S, sampled), gyro.icp_cost(S, sampled))


# ---- output channels ------------------------------------------------------------------------------------

def test_hand_example_output_channels():
    ex = load_golden("hand_example_ocp.txt")
    S = ex["rho"].astype(np.float64)
    rows = ex["row_order"].reshape(2, 2)
    cost = gyro.ocp_cost(S, rows, ex["samples"], None, 2)
    assert cost.tolist() == ex["cost"].astype(np.float64).tolist()
    assign = gyro.icp_assign(cost)
    assert assign.tolist() == ex["assign"].reshape(-1).tolist()
    after = gyro.ocp_apply(rows, ex["samples"], None, assign)
    assert after.reshape(-1).tolist() == ex["row_order_after"].reshape(-1).tolist()
    Wb = synth.to_bits(ex["rho"].astype(np.float32), "bf16")
    order, obj = gyro.ocp_search(Wb, "bf16", None, 2, 2, ex["row_order"].reshape(-1), ex["samples"].reshape(1, 2, 1))
    assert order.tolist() == ex["row_order_after"].reshape(-1).tolist() and obj.tolist() == [16.0]


def _ocp_case(seed, T=4, V=6, K=10, n=2):
    rng = np.random.default_rng(seed)
    S = rng.integers(0, 9, size=(T * V, K)).astype(np.float64)
    rows = rng.permutation(T * V).reshape(T, V)
    sampled = np.stack([rng.permutation(V)[:n] for _ in range(T)])
    clusters = rng.permutation(T * n).reshape(T, n)
    return S, rows, sampled, clusters


def test_output_channel_cost_against_the_packing_oracle_and_brute_force():
    import itertools
    T, V, K, n, Kv = 4, 6, 10, 2, 8      # Kv % 8 == 0 so that the packing oracle accepts the shape
    S, rows, sampled, clusters = _ocp_case(85, T, V, K, n)
    for cl in (None, clusters):
        cost = gyro.ocp_cost(S, rows, sampled, cl, Kv)
        assign = gyro.icp_assign(cost)
        best = min(sum(cost[i, p[i]] for i in range(T)) for p in itertools.permutations(range(T)))
        assert gyro.assignment_cost(cost, assign) == best
        for perm in (np.arange(T), assign, np.array([3, 2, 1, 0])):
            after = gyro.ocp_apply(rows, sampled, cl, perm)
            assert sorted(after.reshape(-1).tolist()) == list(range(T * V))        # still a permutation of the channels
            # the vector scores of the packing oracle on the re-ordered saliency: what is not kept is the cost
            R = S[after.reshape(-1)].astype(np.float32)
            scores = orc.vector_scores_rho(R, V)
            kept = orc.vector_index(np.zeros((T * V, K), dtype=np.uint16), "f16", V, Kv, rho=R)
            pruned = sum(scores[t].sum() - scores[t][kept[t]].sum() for t in range(T))
            assert pruned == gyro.assignment_cost(cost, perm)
    # with every tile's own samples as its cluster nothing moves under the identity assignment
    assert np.array_equal(gyro.ocp_apply(rows, sampled, None, np.arange(T)), rows)


def test_output_channel_search_never_increases_the_objective():
    c = synth.small_case(48, 40, 8, 16, 4, "f16", 86)
    Wb = c.weights()
    rng = np.random.default_rng(87)
    iters, n = 4, 3
    samples = np.stack([np.stack([rng.permutation(c.V)[:n] for _ in range(c.T)]) for _ in range(iters)])
    order, obj = gyro.ocp_search(Wb, c.dtype, None, c.V, c.Kv, np.arange(c.M), samples)
    assert sorted(order.tolist()) == list(range(c.M))
    S = gyro.saliency_matrix(Wb, c.dtype, None)
    start = sum(gyro.vector_pruned_saliency(S[t * c.V:(t + 1) * c.V], c.Kv) for t in range(c.T))
    seq = [start] + obj.tolist()
    assert all(b <= a * (1 + 1e-12) for a, b in zip(seq, seq[1:]))
    end = sum(gyro.vector_pruned_saliency(S[order[t * c.V:(t + 1) * c.V]], c.Kv) for t in range(c.T))
    assert end == pytest.approx(obj[-1], rel=1e-12)


# ---- balanced K-means over the sampled channels (one reading of the clustering phase) -------------------

def test_balanced_assignment_is_the_brute_force_minimum():
    import itertools
    rng = np.random.default_rng(88)
    T, n = 3, 2
    d = rng.integers(0, 30, size=(T * n, T)).astype(np.float64)
    best = None
    for labels in set(itertools.permutations([0, 0, 1, 1, 2, 2])):
        tot = sum(d[q, labels[q]] for q in range(T * n))
        best = tot if best is None or tot < best else best
    cluster = gyro.kmeans_balanced_assignment(d, n)
    assert sorted(np.bincount(cluster, minlength=T).tolist()) == [n] * T
    assert gyro.kmeans_objective(d, cluster) == best


def test_kmeans_recovers_well_separated_groups_and_never_gets_worse():
    rng = np.random.default_rng(89)
    T, n, K = 4, 3, 6
    centres = rng.integers(0, 5, size=(T, K)).astype(np.float64) * 100.0
    truth = rng.permutation(np.repeat(np.arange(T), n))
    truth[0::n] = np.arange(T)                 # the first sample of every tile comes from a different group
    F = centres[truth] + rng.standard_normal((T * n, K))
    clusters, C, obj = gyro.balanced_kmeans(F, n, 3)
    for c in range(T):
        assert len(set(truth[clusters[c]].tolist())) == 1         # every cluster is one of the planted groups
    assert all(b <= a * (1 + 1e-12) for a, b in zip(obj, obj[1:]))
    # distances against the textbook expression, centroids against the mean
    d = gyro.kmeans_distances(F, C)
    assert np.allclose(d, ((F[:, None, :] - C[None, :, :]) ** 2).sum(axis=2), rtol=1e-12)
    lab = np.empty(T * n, dtype=np.int64)
    for c in range(T):
        lab[clusters[c]] = c
    assert np.allclose(gyro.kmeans_centroids(F, lab, T, n), np.stack([F[clusters[c]].mean(axis=0) for c in range(T)]))


def test_kmeans_with_one_sample_per_tile_keeps_every_point_alone():
    rng = np.random.default_rng(90)
    F = rng.standard_normal((5, 7))
    clusters, C, obj = gyro.balanced_kmeans(F, 1, 2)
    assert clusters.reshape(-1).tolist() == [0, 1, 2, 3, 4] and obj.tolist() == [0.0, 0.0]
    assert np.array_equal(C, F)
