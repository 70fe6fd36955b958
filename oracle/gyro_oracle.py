"""CPU oracle for the two permutation searches of gyro-permutation: tile-wise input channels
(icp_*) and output channels (ocp_*).

TEST INFRASTRUCTURE ONLY.  Slow, plain definition of what the HIP library's search computes; it
shares no code with the HIP path and must never be imported by it.

What it follows (arXiv 2407.20496):
  * Section 4.1, Eq. 3: after column-vector pruning, the kept column vectors of every tile are
    re-arranged so that the 2:4 step retains as much saliency as possible; every four consecutive
    kept vectors form one partition (one 2:4 group per row).
  * Section 4.2: one iteration = sampling (here exactly one column vector per partition, so the
    clustering phase is bypassed), the cost of placing sample j into partition i (Eq. 4: the
    saliency that the 2:4 step would prune in partition i's three remaining vectors plus sample j),
    and an assignment of samples to partitions that minimises the total cost (the paper names the
    Hungarian algorithm; any exact solver of the linear assignment problem reaches the same minimum).

  * Section 4.1, Eq. 2 and Section 4.2 for the output channels: the partitions are the tiles of V
    output channels; the same number of channels is sampled from every tile, the sampled channels are
    grouped into as many clusters as there are tiles (the paper uses balanced K-means; here the grouping
    is an input, by default every tile's own samples form a cluster; balanced_kmeans_* below is one
    reading of that step), cost[i][j] (Eq. 4) is the
    saliency column-vector pruning would remove from tile i's remaining channels plus cluster j, and
    the clusters are assigned to the tiles at minimal total cost.

Readings where the paper is silent (repeated in the design notes): which member of a partition is
sampled is an input (the caller draws it); a sample moves into the slot its destination partition
vacated; the cost is the plain sum of the pruned saliencies (not total minus retained), per row the
two smallest of the four values added exactly, rows accumulated in binary64 in ascending order;
saliency = caller-given rho (float32) or |w|; several assignments may reach the minimum, any of
them is a correct result, and the number of iterations is the caller's.  Output channels: the column
scores of a candidate tile are (sum over the remaining channels in position order) + (sum over the
cluster's channels in cluster order), each in binary64; the cost is the sum of the K - Kv smallest
scores (which of several equal scores is pruned does not change it), here added with exact rounding;
the channels of a cluster fill the slots the tile vacated in position order.  Balanced K-means
(the paper only names it): points = the sampled channels' saliency rows, T clusters of exactly n
points, squared Euclidean distance in binary64 (columns added in ascending order), a round = a
minimal-cost assignment of points to clusters under the size constraint followed by centroids =
mean of the members (added in ascending item order, then divided by n); initial centroids = the
first sample of every tile.  parity unpinned by the paper: it prints no detail of this step.

Pins: tests/test_oracle_gyro.py (brute force over all assignments, the hand-derived example in
tests/golden/hand_example_icp.txt, cost of the identity assignment = current pruned saliency,
total cost of an assignment = pruned saliency after the move, the objective never increases, and
the final arrangement fed to the packing oracle prunes exactly the final objective; for the output
channels a second hand-derived example, brute force over assignments, and the vector scores of the
packing oracle on the re-ordered matrix).
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np
from scipy.optimize import linear_sum_assignment

from oracle import hinm_oracle as orc


def kept_saliency(W_bits: np.ndarray, dtype: str, rho: Optional[np.ndarray], V: int, vec_idx_t: np.ndarray,
                  t: int) -> np.ndarray:
    """Saliency of tile t's entries in the columns vec_idx_t, float64 [V, len(vec_idx_t)]: the
    caller's rho, or |w|."""
    rows = slice(t * V, (t + 1) * V)
    if rho is not None:
        return np.asarray(rho)[rows][:, vec_idx_t].astype(np.float64)
    return np.abs(orc.decode(np.asarray(W_bits)[rows][:, vec_idx_t], dtype))


def pruned_saliency(S: np.ndarray) -> float:
    """S: float64 [V, Kv], columns in arrangement order.  What the 2:4 step prunes: per row and group of
    four the two smallest values; groups in ascending order, inside a group rows in ascending order."""
    V, Kv = S.shape
    total = 0.0
    for g in range(Kv // 4):
        acc = 0.0
        for r in range(V):
            four = np.sort(S[r, 4 * g:4 * g + 4])
            acc = acc + (four[0] + four[1])
        total = total + acc
    return total


def icp_cost(S: np.ndarray, sampled: np.ndarray) -> np.ndarray:
    """Eq. 4 for one tile.  S: float64 [V, Kv] in arrangement order; sampled[i] in 0..3 = the member of
    partition i that is taken out.  cost[i, j] = saliency pruned in partition i when its vacated slot
    holds sample j: float64 [P, P]."""
    V, Kv = S.shape
    P = Kv // 4
    cost = np.zeros((P, P), dtype=np.float64)
    for i in range(P):
        rem = [4 * i + m for m in range(4) if m != int(sampled[i])]
        for j in range(P):
            col = 4 * j + int(sampled[j])
            acc = 0.0
            for r in range(V):   # sequential on purpose: pins the rounding order
                four = np.sort(np.array([S[r, rem[0]], S[r, rem[1]], S[r, rem[2]], S[r, col]]))
                acc = acc + (four[0] + four[1])
            cost[i, j] = acc
    return cost


def icp_cost_fast(S: np.ndarray, sampled: np.ndarray) -> np.ndarray:
    """Same result as :func:`icp_cost` bit for bit (pinned in the tests), vectorised over the (i, j) pairs
    so that full-size tiles finish in seconds; the rows are still added one after the other."""
    V, Kv = S.shape
    P = Kv // 4
    sampled = np.asarray(sampled).astype(np.int64)
    members = S.reshape(V, P, 4)
    samp = np.take_along_axis(members, sampled[None, :, None], axis=2)[:, :, 0]            # [V, P]
    keep = np.array([[m for m in range(4) if m != int(sampled[i])] for i in range(P)])      # [P, 3]
    rem = np.take_along_axis(members, np.broadcast_to(keep[None], (V, P, 3)), axis=2)       # [V, P, 3]
    cost = np.zeros((P, P), dtype=np.float64)
    for r in range(V):
        four = np.concatenate([np.broadcast_to(rem[r][:, None, :], (P, P, 3)),
                               np.broadcast_to(samp[r][None, :, None], (P, P, 1))], axis=2)
        four = np.sort(four, axis=2)
        cost = cost + (four[:, :, 0] + four[:, :, 1])
    return cost


def icp_assign(cost: np.ndarray) -> np.ndarray:
    """assign[i] = the sample placed into partition i, minimising sum_i cost[i, assign[i]]."""
    rows, cols = linear_sum_assignment(cost)
    out = np.empty(cost.shape[0], dtype=np.int64)
    out[rows] = cols
    return out


def assignment_cost(cost: np.ndarray, assign: np.ndarray) -> float:
    """Total cost of an assignment, partitions added in ascending order."""
    total = 0.0
    for i in range(cost.shape[0]):
        total = total + cost[i, int(assign[i])]
    return total


def icp_apply(arrangement: np.ndarray, sampled: np.ndarray, assign: np.ndarray) -> np.ndarray:
    """Moves sample assign[i] into the slot partition i vacated.  arrangement: the tile's kept columns
    in order [Kv]; returns the new order."""
    out = np.array(arrangement, copy=True)
    for i in range(len(sampled)):
        j = int(assign[i])
        out[4 * i + int(sampled[i])] = arrangement[4 * j + int(sampled[j])]
    return out


def icp_search(W_bits: np.ndarray, dtype: str, rho: Optional[np.ndarray], V: int, vec_idx: np.ndarray,
               samples: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """samples: [iters, T, Kv/4] members 0..3.  Returns (vec_idx after all iterations [T, Kv],
    objective [iters, T] = saliency pruned by the 2:4 step after each iteration)."""
    vec = np.array(vec_idx, copy=True)
    iters, T, P = samples.shape
    objective = np.zeros((iters, T), dtype=np.float64)
    for it in range(iters):
        for t in range(T):
            S = kept_saliency(W_bits, dtype, rho, V, vec[t], t)
            cost = icp_cost(S, samples[it, t])
            assign = icp_assign(cost)
            objective[it, t] = assignment_cost(cost, assign)
            vec[t] = icp_apply(vec[t], samples[it, t], assign)
    return vec, objective


# --------------------------------------------------------------------------
# Section 4.1 Eq. 2 / Section 4.2: output-channel permutation
# --------------------------------------------------------------------------


def saliency_matrix(W_bits: np.ndarray, dtype: str, rho: Optional[np.ndarray]) -> np.ndarray:
    """float64 [M, K]: the caller's rho, or |w|."""
    if rho is not None:
        return np.asarray(rho).astype(np.float64)
    return np.abs(orc.decode(W_bits, dtype))


def vector_pruned_saliency(S_rows: np.ndarray, Kv: int) -> float:
    """S_rows: float64 [V, K], the channels of one tile in position order.  What column-vector pruning
    removes: the sum of the K - Kv smallest column sums (rows added in order, binary64)."""
    V, K = S_rows.shape
    col = np.zeros(K, dtype=np.float64)
    for r in range(V):
        col = col + S_rows[r]
    return math.fsum(np.sort(col)[:K - Kv].tolist())


def ocp_cost(S: np.ndarray, rows: np.ndarray, sampled: np.ndarray, clusters: Optional[np.ndarray], Kv: int) -> np.ndarray:
    """Eq. 4 for the output channels.  S: float64 [M, K] saliency; rows: int [T, V], rows[t, p] = the
    channel at position p of tile t; sampled: int [T, n] distinct positions taken out of every tile;
    clusters: int [T, n], a grouping of the T * n sampled channels (item q = sample q % n of tile
    q // n) into T clusters, None = every tile's own samples.  cost[i, j] = saliency that vector pruning
    removes from tile i's remaining channels plus cluster j: float64 [T, T]."""
    T, V = rows.shape
    n = sampled.shape[1]
    K = S.shape[1]
    if clusters is None:
        clusters = np.arange(T * n).reshape(T, n)
    pool = [int(rows[q // n, sampled[q // n, q % n]]) for q in range(T * n)]
    base = np.zeros((T, K), dtype=np.float64)
    clus = np.zeros((T, K), dtype=np.float64)
    for t in range(T):
        out = set(int(x) for x in sampled[t])
        assert len(out) == n
        for pos in range(V):
            if pos not in out:
                base[t] = base[t] + S[rows[t, pos]]
        for e in range(n):
            clus[t] = clus[t] + S[pool[int(clusters[t, e])]]
    cost = np.zeros((T, T), dtype=np.float64)
    for i in range(T):
        for j in range(T):
            col = base[i] + clus[j]
            cost[i, j] = math.fsum(np.sort(col)[:K - Kv].tolist())
    return cost


def ocp_apply(rows: np.ndarray, sampled: np.ndarray, clusters: Optional[np.ndarray], assign: np.ndarray) -> np.ndarray:
    """The channels of cluster assign[i] fill the positions tile i vacated, in order."""
    T, V = rows.shape
    n = sampled.shape[1]
    if clusters is None:
        clusters = np.arange(T * n).reshape(T, n)
    pool = [int(rows[q // n, sampled[q // n, q % n]]) for q in range(T * n)]
    out = np.array(rows, copy=True)
    for i in range(T):
        for e in range(n):
            out[i, sampled[i, e]] = pool[int(clusters[int(assign[i]), e])]
    return out


def ocp_search(W_bits: np.ndarray, dtype: str, rho: Optional[np.ndarray], V: int, Kv: int, row_order: np.ndarray,
               samples: np.ndarray, clusters: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """row_order: int [M], row_order[t * V + p] = the channel at position p of tile t.  samples:
    [iters, T, n]; clusters: [iters, T, n] or None.  Returns (row order after all iterations [M],
    objective [iters] = saliency removed by vector pruning over all tiles after each iteration)."""
    S = saliency_matrix(W_bits, dtype, rho)
    rows = np.array(row_order, copy=True).reshape(-1, V)
    iters = samples.shape[0]
    objective = np.zeros(iters, dtype=np.float64)
    for it in range(iters):
        cl = None if clusters is None else clusters[it]
        cost = ocp_cost(S, rows, samples[it], cl, Kv)
        assign = icp_assign(cost)
        objective[it] = assignment_cost(cost, assign)
        rows = ocp_apply(rows, samples[it], cl, assign)
    return rows.reshape(-1), objective


# --------------------------------------------------------------------------
# Section 4.2, clustering phase: balanced K-means over the sampled output channels
# --------------------------------------------------------------------------


def sampled_features(S: np.ndarray, rows: np.ndarray, sampled: np.ndarray) -> np.ndarray:
    """float64 [T * n, K]: the saliency row of every sampled channel, item q = sample q % n of tile q // n."""
    T, n = sampled.shape
    return np.stack([S[int(rows[q // n, sampled[q // n, q % n]])] for q in range(T * n)])


def kmeans_initial_centroids(F: np.ndarray, n: int) -> np.ndarray:
    """Centroid c starts as the first sample of tile c: float64 [T, K]."""
    return np.array(F[0::n], copy=True)


def kmeans_distances(F: np.ndarray, C: np.ndarray) -> np.ndarray:
    """d[q, c] = sum_k (F[q, k] - C[c, k])^2, binary64, columns added in ascending order."""
    Np, K = F.shape
    d = np.zeros((Np, C.shape[0]), dtype=np.float64)
    for k in range(K):   # sequential on purpose: pins the rounding order
        diff = F[:, k][:, None] - C[:, k][None, :]
        d = d + diff * diff
    return d


def kmeans_balanced_assignment(d: np.ndarray, n: int) -> np.ndarray:
    """cluster[q] minimising sum_q d[q, cluster[q]] with exactly n points per cluster: a linear assignment of
    the points to the T * n (cluster, slot) pairs."""
    rows, cols = linear_sum_assignment(np.repeat(d, n, axis=1))
    out = np.empty(d.shape[0], dtype=np.int64)
    out[rows] = cols // n
    return out


def kmeans_centroids(F: np.ndarray, cluster: np.ndarray, T: int, n: int) -> np.ndarray:
    """Mean of the members: added in ascending item order, then divided by n."""
    C = np.zeros((T, F.shape[1]), dtype=np.float64)
    for q in range(F.shape[0]):
        C[int(cluster[q])] = C[int(cluster[q])] + F[q]
    return C / float(n)


def kmeans_clusters(cluster: np.ndarray, T: int, n: int) -> np.ndarray:
    """int [T, n]: the items of every cluster in ascending order (the `clusters` input of ocp_cost)."""
    return np.stack([np.nonzero(np.asarray(cluster) == c)[0] for c in range(T)]).reshape(T, n)


def kmeans_objective(d: np.ndarray, cluster: np.ndarray) -> float:
    total = 0.0
    for q in range(d.shape[0]):
        total = total + d[q, int(cluster[q])]
    return total


def balanced_kmeans(F: np.ndarray, n: int, rounds: int, C: Optional[np.ndarray] = None):
    """Returns (clusters [T, n], centroids [T, K], objective per round)."""
    T = F.shape[0] // n
    C = kmeans_initial_centroids(F, n) if C is None else np.array(C, copy=True)
    cluster = np.arange(F.shape[0]) // n
    objective = []
    for _ in range(rounds):
        d = kmeans_distances(F, C)
        cluster = kmeans_balanced_assignment(d, n)
        objective.append(kmeans_objective(d, cluster))
        C = kmeans_centroids(F, cluster, T, n)
    return kmeans_clusters(cluster, T, n), C, np.array(objective)
