"""CPU oracle for hierarchical N:M (HiNM) sparsity: masks, packing, product.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
HIP library computes.  It shares no code with the HIP path and must never be
imported by it; only tests, the smoke check and the benchmark's CPU-baseline
leg may call it.

What it follows (arXiv 2407.20496):
  * Section 1 (Figure 1 and its walk-through): a dense weight matrix is first
    pruned by V x 1 column vectors inside every tile of V consecutive output
    channels (a *vector index* records the surviving columns), then every
    1 x 4 group of surviving entries in a row loses two elements (an *NM
    index* records the two kept positions); total sparsity is
    1 - (1 - s_v) * 0.5.
  * Section 3.1: the pruning order is vector pruning first, then 2:4.
  * Section 4.1, Eq. 2 and Eq. 3 (with identity orders): each mask maximises
    the retained saliency under its structural constraint.
  * Section 3.2 and Section 5.3: the run-time product reads input channels
    through the vector index composed with an input-channel order and writes
    output channels in the layer's own output-channel order, so the result is
    Y = P_out (W_HiNM (P_in X)).
  * Section 3.2 ("tile-wise input channel permutation") and Section 4.2: the
    kept column vectors of a tile may be arranged in a caller-given order before
    the 2:4 step (tile_order, pack's sigma argument); the search that finds a
    good order is not part of this file.
  * Section 4.1 (Eq. 1-3) and Section 5.1: both masks maximise a retained
    saliency rho that need not come from the weights themselves (magnitude or
    second-order scores); pack's rho argument takes such a score per weight.
  * Section 5.1.2: during gradual pruning a layer first carries the column-vector
    mask alone and receives the 2:4 mask later; pack_vectors / unpack_vectors
    hold that intermediate state (all Kv surviving entries of every row).

Readings where the paper is silent (all repeated in the design notes):
  saliency of a V x 1 vector = sum of squares (L2), accumulated in binary64 in
  ascending row order; ties -> lower column; the vector index is ascending;
  2:4 saliency = |w|, ties -> lower position, always exactly two kept; the
  packed pair is stored in position order and the NM nibble is p0 | p1 << 2,
  two groups per byte, low nibble first; P_in gathers (row k of P_in X is row
  pi_in[k] of X) and P_out scatters (row r of the product lands in row
  pi_out[r] of Y); the product is accumulated in float32 unless float64 is
  requested, and rounded to the storage type with round-to-nearest-even.
  With a caller-given rho (float32, one score per weight, no NaN): the saliency
  of a vector is the plain sum of its V scores, accumulated in binary64 in
  ascending row order starting from +0; larger sum wins, equal sums -> lower
  column; inside a group of four the two largest scores are kept, equal scores
  -> lower position (-0 and +0 are equal); the stored values are always W's.

16-bit tensors are uint16 bit patterns plus a dtype tag, "f16" or "bf16".

Pins: tests/test_oracle_*.py (brute-force enumeration of Eq. 2 / Eq. 3 on tiny
inputs, exact kept counts, the sparsity formula, pack/unpack round trip,
identity-permutation and dense-library reductions, the hand-derived examples in
tests/golden/, one with a tile-wise order and one with caller-given scores; for
rho also the reductions rho = w^2 and V = 1, and for the vector-only state its
2:4 completion).  The paper prints no numeric worked example for this path.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------
# storage types
# --------------------------------------------------------------------------


def decode(bits: np.ndarray, dtype: str) -> np.ndarray:
    """uint16 bit patterns -> exact float64 values."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def round_to_storage(y: np.ndarray, dtype: str) -> np.ndarray:
    """float32/float64 -> uint16 bit patterns, round-to-nearest-even."""
    if dtype == "f16":
        return np.asarray(y).astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        y32 = np.ascontiguousarray(y, dtype=np.float32)
        out = np.empty(y32.shape, dtype=np.uint16)
        flat_in = y32.reshape(-1).view(np.uint32)
        flat_out = out.reshape(-1)
        upper = (flat_in >> np.uint32(16)).astype(np.uint32)
        lower = flat_in & np.uint32(0xFFFF)
        round_up = (lower > np.uint32(0x8000)) | ((lower == np.uint32(0x8000)) & ((upper & np.uint32(1)) == 1))
        res = upper + round_up.astype(np.uint32)
        nan = np.isnan(y32.reshape(-1))
        res = np.where(nan, np.uint32(0x7FC0), res)
        flat_out[:] = res.astype(np.uint16)
        return out
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# Section 1 / Section 3.1 / Eq. 2: column-vector mask
# --------------------------------------------------------------------------


def vector_scores(W_bits: np.ndarray, dtype: str, V: int) -> np.ndarray:
    """score[t, k] = sum_{i<V} W[tV+i, k]^2, binary64, rows added in ascending
    order (the L2 saliency of the V x 1 vector of tile t at input channel k)."""
    W = decode(W_bits, dtype)
    M, K = W.shape
    assert M % V == 0
    T = M // V
    Wt = W.reshape(T, V, K)
    s = np.zeros((T, K), dtype=np.float64)
    for i in range(V):  # sequential on purpose: pins the rounding order
        s = s + Wt[:, i, :] * Wt[:, i, :]
    return s


def vector_scores_rho(rho: np.ndarray, V: int) -> np.ndarray:
    """score[t, k] = sum_{i<V} rho[tV+i, k] for caller-given per-weight saliency
    (Section 4.1, the rho of Eq. 1-3; Section 5.1 names magnitude and second-order
    scores): float32 inputs, binary64 sum from +0, rows added in ascending order."""
    rho = np.asarray(rho)
    assert rho.dtype == np.float32 and not np.isnan(rho).any()
    M, K = rho.shape
    assert M % V == 0
    Rt = rho.astype(np.float64).reshape(M // V, V, K)
    s = np.zeros((M // V, K), dtype=np.float64)
    for i in range(V):  # sequential on purpose: pins the rounding order
        s = s + Rt[:, i, :]
    return s


def vector_index(W_bits: np.ndarray, dtype: str, V: int, Kv: int, rho: Optional[np.ndarray] = None) -> np.ndarray:
    """Per tile, the Kv columns of largest score (ties: lower column first),
    returned in ascending column order: int32 [T, Kv].  The score is the L2
    saliency of W's vectors, or the summed caller-given rho."""
    s = vector_scores(W_bits, dtype, V) if rho is None else vector_scores_rho(rho, V)
    T, K = s.shape
    assert 0 < Kv <= K
    cols = np.arange(K)
    out = np.empty((T, Kv), dtype=np.int32)
    for t in range(T):
        order = np.lexsort((cols, -s[t]))  # primary: score descending; secondary: column ascending
        out[t] = np.sort(order[:Kv])
    return out


def tile_order(vec_idx: np.ndarray, sigma: Optional[np.ndarray], K: int) -> np.ndarray:
    """Tile-wise input-channel permutation (Section 3.2, "tile-wise input channel
    permutation"; Section 4.2, the sigma_i^t of Eq. 4): the kept column vectors of tile t are
    arranged in the order in which they appear in sigma[t], a permutation of all K input
    channels given by the caller, instead of ascending column order.  Which columns are kept
    does not change; which four of them form a 2:4 group does.  sigma None = ascending order."""
    if sigma is None:
        return vec_idx
    sigma = np.asarray(sigma)
    T, Kv = vec_idx.shape
    assert sigma.shape == (T, K)
    out = np.empty_like(vec_idx)
    for t in range(T):
        assert sorted(sigma[t].tolist()) == list(range(K)), "sigma[t] must be a permutation of the input channels"
        kept = set(vec_idx[t].tolist())
        out[t] = [c for c in sigma[t].tolist() if c in kept]
    return out


def order_from_arrangement(arrangement: np.ndarray, K: int) -> np.ndarray:
    """The other direction of tile_order (Section 3.2: any arrangement of a tile's kept vectors is a valid
    layer; Section 4.2 searches over them): an order of all K input channels per tile that reproduces a given
    arrangement of the kept ones -- those Kv channels as arranged, then the pruned channels ascending."""
    arrangement = np.asarray(arrangement)
    T, Kv = arrangement.shape
    out = np.empty((T, K), dtype=np.int32)
    for t in range(T):
        kept = arrangement[t].tolist()
        assert len(set(kept)) == Kv and all(0 <= c < K for c in kept), "a row must name Kv distinct channels"
        members = set(kept)
        out[t] = kept + [c for c in range(K) if c not in members]
    return out


# --------------------------------------------------------------------------
# Section 1 / Eq. 3 constraint: 2:4 selection on the surviving columns
# --------------------------------------------------------------------------


def nm_positions(C: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """C: float64 [..., G, 4].  For every group of four return the kept
    positions p0 < p1: the two largest |value|, ties -> lower position."""
    mag = np.abs(C)
    order = np.argsort(-mag, axis=-1, kind="stable")  # stable keeps lower position first among ties
    kept = np.sort(order[..., :2], axis=-1)
    return kept[..., 0], kept[..., 1]


def nm_positions_signed(R: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """R: float64 [..., G, 4] of caller-given scores.  Kept positions p0 < p1: the two
    largest scores as signed numbers, ties (including -0 against +0) -> lower position."""
    order = np.argsort(-(R + 0.0), axis=-1, kind="stable")  # adding +0 turns -0 into +0
    kept = np.sort(order[..., :2], axis=-1)
    return kept[..., 0], kept[..., 1]


def pack(W_bits: np.ndarray, dtype: str, V: int, Kv: int, sigma: Optional[np.ndarray] = None,
         rho: Optional[np.ndarray] = None):
    """Dense W (uint16 bits [M, K]) -> (vals uint16 [M, Kv/2], nm_idx uint8
    [M, Kv/8], vec_idx int32 [T, Kv]).  sigma (int [T, K], optional): per-tile order of the
    input channels, see tile_order.  rho (float32 [M, K], optional): per-weight saliency that
    replaces W's own magnitudes in both selections (Section 4.1); the stored values stay W's."""
    W_bits = np.ascontiguousarray(W_bits, dtype=np.uint16)
    M, K = W_bits.shape
    assert M % V == 0 and Kv % 8 == 0 and 0 < Kv <= K
    T = M // V
    vec_idx = tile_order(vector_index(W_bits, dtype, V, Kv, rho), sigma, K)
    G = Kv // 4
    vals = np.empty((M, Kv // 2), dtype=np.uint16)
    nm_idx = np.empty((M, Kv // 8), dtype=np.uint8)
    for t in range(T):
        Cb = W_bits[t * V:(t + 1) * V][:, vec_idx[t]]            # compressed tile, bits, [V, Kv]
        if rho is None:
            p0, p1 = nm_positions(decode(Cb, dtype).reshape(V, G, 4))     # saliency of an entry: its magnitude
        else:
            R = np.asarray(rho)[t * V:(t + 1) * V][:, vec_idx[t]].astype(np.float64)
            p0, p1 = nm_positions_signed(R.reshape(V, G, 4))
        Cb4 = Cb.reshape(V, G, 4)
        v0 = np.take_along_axis(Cb4, p0[..., None], axis=-1)[..., 0]
        v1 = np.take_along_axis(Cb4, p1[..., None], axis=-1)[..., 0]
        tile_vals = np.empty((V, G, 2), dtype=np.uint16)
        tile_vals[..., 0] = v0
        tile_vals[..., 1] = v1
        vals[t * V:(t + 1) * V] = tile_vals.reshape(V, G * 2)
        nib = (p0 | (p1 << 2)).astype(np.uint8)                   # [V, G]
        nm_idx[t * V:(t + 1) * V] = nib[:, 0::2] | (nib[:, 1::2] << 4)
    return vals, nm_idx, vec_idx


def pack_vectors(W_bits: np.ndarray, dtype: str, V: int, Kv: int, sigma: Optional[np.ndarray] = None,
                 rho: Optional[np.ndarray] = None):
    """The layer after column-vector pruning alone (Section 3.1, first step; Section 5.1.2, the
    state a layer is in until the target vector sparsity is reached): (vals_v uint16 [M, Kv],
    vec_idx int32 [T, Kv]) with vals_v[r, j] = W[r, vec_idx[r // V, j]]."""
    W_bits = np.ascontiguousarray(W_bits, dtype=np.uint16)
    M, K = W_bits.shape
    assert M % V == 0 and 0 < Kv <= K
    T = M // V
    vec_idx = tile_order(vector_index(W_bits, dtype, V, Kv, rho), sigma, K)
    vals_v = np.empty((M, Kv), dtype=np.uint16)
    for t in range(T):
        vals_v[t * V:(t + 1) * V] = W_bits[t * V:(t + 1) * V][:, vec_idx[t]]
    return vals_v, vec_idx


def unpack_vectors(vals_v: np.ndarray, vec_idx: np.ndarray, M: int, K: int, V: int) -> np.ndarray:
    """Inverse of pack_vectors into an all-zero matrix: uint16 bits [M, K] of M_v (.) W."""
    T, Kv = vec_idx.shape
    assert T * V == M
    W = np.zeros((M, K), dtype=np.uint16)
    for r in range(M):
        for j in range(Kv):
            W[r, vec_idx[r // V, j]] = vals_v[r, j]
    return W


def unpack(vals: np.ndarray, nm_idx: np.ndarray, vec_idx: np.ndarray, M: int, K: int, V: int) -> np.ndarray:
    """Inverse of pack into an all-zero matrix: uint16 bits [M, K] of W_HiNM."""
    T, Kv = vec_idx.shape
    assert T * V == M
    G = Kv // 4
    W = np.zeros((M, K), dtype=np.uint16)
    for r in range(M):
        t = r // V
        for g in range(G):
            byte = int(nm_idx[r, g >> 1])
            nib = (byte >> (4 * (g & 1))) & 0xF
            p0, p1 = nib & 3, (nib >> 2) & 3
            W[r, vec_idx[t, 4 * g + p0]] = vals[r, 2 * g]
            W[r, vec_idx[t, 4 * g + p1]] = vals[r, 2 * g + 1]
    return W


def mask(nm_idx: np.ndarray, vec_idx: np.ndarray, M: int, K: int, V: int) -> np.ndarray:
    """Boolean [M, K]: True where W_HiNM keeps an entry."""
    T, Kv = vec_idx.shape
    G = Kv // 4
    m = np.zeros((M, K), dtype=bool)
    for r in range(M):
        t = r // V
        for g in range(G):
            nib = (int(nm_idx[r, g >> 1]) >> (4 * (g & 1))) & 0xF
            m[r, vec_idx[t, 4 * g + (nib & 3)]] = True
            m[r, vec_idx[t, 4 * g + ((nib >> 2) & 3)]] = True
    return m


def unpack_fast(vals: np.ndarray, nm_idx: np.ndarray, vec_idx: np.ndarray, M: int, K: int, V: int) -> np.ndarray:
    """Same result as :func:`unpack`, vectorised per tile so that full-size
    layers finish in seconds (pinned against :func:`unpack` in the tests)."""
    T, Kv = vec_idx.shape
    G = Kv // 4
    W = np.zeros((M, K), dtype=np.uint16)
    g = np.arange(G)
    for t in range(T):
        rows = slice(t * V, (t + 1) * V)
        nib = (nm_idx[rows][:, g >> 1] >> (4 * (g & 1)).astype(np.uint8)) & np.uint8(0xF)   # [V, G]
        p0 = (nib & 3).astype(np.int64)
        p1 = ((nib >> 2) & 3).astype(np.int64)
        c0 = vec_idx[t][4 * g[None, :] + p0]                      # [V, G] destination columns
        c1 = vec_idx[t][4 * g[None, :] + p1]
        rr = np.arange(t * V, (t + 1) * V)[:, None]
        W[rr, c0] = vals[rows][:, 0::2]
        W[rr, c1] = vals[rows][:, 1::2]
    return W


# --------------------------------------------------------------------------
# Section 3.2 / Section 5.3: the product with channel orders
# --------------------------------------------------------------------------


def perm_matrix_in(pi_in: Optional[Sequence[int]], K: int, dt=np.float32) -> np.ndarray:
    """P_in with (P_in X)[k, :] = X[pi_in[k], :]."""
    P = np.zeros((K, K), dtype=dt)
    idx = np.arange(K) if pi_in is None else np.asarray(pi_in)
    P[np.arange(K), idx] = 1
    return P


def perm_matrix_out(pi_out: Optional[Sequence[int]], M: int, dt=np.float32) -> np.ndarray:
    """P_out with (P_out Z)[pi_out[r], :] = Z[r, :]."""
    P = np.zeros((M, M), dtype=dt)
    idx = np.arange(M) if pi_out is None else np.asarray(pi_out)
    P[idx, np.arange(M)] = 1
    return P


def matmul_naive(A: np.ndarray, B: np.ndarray, dt=np.float32) -> np.ndarray:
    """Textbook triple loop, accumulating in `dt` in ascending k.  Tiny sizes only."""
    A = np.asarray(A, dtype=dt)
    B = np.asarray(B, dtype=dt)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    C = np.zeros((m, n), dtype=dt)
    for i in range(m):
        for j in range(n):
            acc = dt(0)
            for p in range(k):
                acc = dt(acc + dt(A[i, p] * B[p, j]))
            C[i, j] = acc
    return C


def product(Wh_bits: np.ndarray, X_bits: np.ndarray, dtype: str,
            pi_in: Optional[Sequence[int]] = None, pi_out: Optional[Sequence[int]] = None,
            acc=np.float32, naive: bool = False, relu: bool = False) -> np.ndarray:
    """Y_acc = P_out (W_HiNM (P_in X)) with explicit 0/1 permutation matrices,
    accumulated in `acc` (float32 or float64); optional ReLU.  Returns the
    un-rounded accumulator-precision matrix [M, N]."""
    Wh = decode(Wh_bits, dtype).astype(acc)
    X = decode(X_bits, dtype).astype(acc)
    M, K = Wh.shape
    P_in = perm_matrix_in(pi_in, K, acc)
    P_out = perm_matrix_out(pi_out, M, acc)
    mm = (lambda a, b: matmul_naive(a, b, acc)) if naive else np.matmul
    Y = mm(P_out, mm(Wh, mm(P_in, X)))
    if relu:
        Y = np.maximum(Y, acc(0))
    return Y


def spmm(Wh_bits, X_bits, dtype, pi_in=None, pi_out=None, acc=np.float32, relu=False) -> np.ndarray:
    """Product rounded to the storage type: uint16 bits [M, N]."""
    return round_to_storage(product(Wh_bits, X_bits, dtype, pi_in, pi_out, acc, relu=relu), dtype)


def product_entries(Wh_bits: np.ndarray, X_bits: np.ndarray, dtype: str,
                    pi_in: Optional[Sequence[int]], pi_out: Optional[Sequence[int]],
                    rows: Sequence[int], cols: Sequence[int], relu: bool = False) -> np.ndarray:
    """The same product written out element by element, for sampled outputs of
    layers too large for the matrix form:
        Y[pi_out[r], n] = sum_k W_HiNM[r, k] * X[pi_in[k], n]
    which is entry (pi_out[r], n) of P_out (W_HiNM (P_in X)).  `rows` are rows
    r of W; returns float64 [len(rows), len(cols)] together with nothing else;
    the caller looks the value up at Y[pi_out[r], n]."""
    Wh_bits = np.asarray(Wh_bits)
    K = Wh_bits.shape[1]
    pin = np.arange(K) if pi_in is None else np.asarray(pi_in)
    cols = np.asarray(cols)
    out = np.empty((len(rows), len(cols)), dtype=np.float64)
    for a, r in enumerate(rows):
        w = decode(Wh_bits[r], dtype)                  # [K]
        nz = np.nonzero(w)[0]
        xr = decode(np.asarray(X_bits)[pin[nz]][:, cols], dtype)   # [nnz, len(cols)]
        y = (w[nz, None] * xr).sum(axis=0)
        out[a] = np.maximum(y, 0.0) if relu else y
    return out


def product_rows(Wh_rows_bits: np.ndarray, X_bits: np.ndarray, dtype: str,
                 pi_in: Optional[Sequence[int]], relu: bool = False) -> np.ndarray:
    """Whole rows of the same product for a subset of W's rows, in binary64, for layers too large
    for the matrix form with explicit permutation matrices:
        out[a, n] = sum_k W_HiNM[r_a, k] * X[pi_in[k], n]
    where Wh_rows_bits holds the rows r_a of W_HiNM.  Row k of (P_in X) is row pi_in[k] of X by
    the definition of P_in, so the 0/1 matrix product is written as that row selection; the
    contraction is one binary64 matrix product.  Entry (pi_out[r_a], n) of P_out (W_HiNM (P_in X))
    is out[a, n]: the caller looks the value up there."""
    Wr = decode(Wh_rows_bits, dtype)
    K = Wr.shape[1]
    pin = np.arange(K) if pi_in is None else np.asarray(pi_in)
    Xp = decode(np.asarray(X_bits)[pin], dtype)          # (P_in X)[k, :] = X[pi_in[k], :]
    Y = Wr @ Xp
    return np.maximum(Y, 0.0) if relu else Y


def chain(layers, X_bits: np.ndarray, dtype: str, acc=np.float32) -> np.ndarray:
    """Consecutive layers with independent channel orders (Section 3.2,
    "maintaining layer consistency"): every layer is (Wh_bits, pi_in, pi_out,
    relu).  Each layer's output is rounded to the storage type before the next
    layer reads it.  Returns uint16 bits of the last layer's output."""
    H = X_bits
    for (Wh_bits, pi_in, pi_out, relu) in layers:
        H = spmm(Wh_bits, H, dtype, pi_in, pi_out, acc, relu=relu)
    return H
