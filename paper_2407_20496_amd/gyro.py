"""Host-side driver of the permutation search (arXiv 2407.20496, Section 4.2) over the C-ABI entry points.

Everything the method computes runs in the library's kernels (hinm_ocp_cluster, hinm_ocp_search,
hinm_pack_vectors, hinm_icp_search, hinm_tile_order, hinm_pack_ordered / hinm_pack_scored).  This module only does what the
paper leaves to the caller: it draws the samples of every iteration from a seeded generator, decides how many
channels are sampled per iteration, and hands arrays from one call to the next.  PyTorch is used for device
memory only.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np
import torch

from . import binding as hb


def default_sample_schedule(V: int, iters: int) -> Sequence[int]:
    """Channels sampled per tile and iteration: from V/8 down to 1, halving at equal intervals (the paper
    compares this number to a learning rate and lowers it during the search; the schedule itself is ours)."""
    if iters <= 0:
        return []
    top = max(1, V // 8)
    levels = int(np.log2(top)) + 1
    return [max(1, top >> min(levels - 1, (i * levels) // iters)) for i in range(iters)]


def gyro_permute(W: torch.Tensor, V: int, Kv: int, dtype, rho: Optional[torch.Tensor] = None, ocp_iters: int = 8,
                 ocp_samples: Optional[Sequence[int]] = None, kmeans_rounds: int = 2, icp_iters: int = 8,
                 seed: int = 0) -> Dict[str, object]:
    """Output-channel search, column-vector pruning, tile-wise input-channel search, 2:4 packing of one layer.

    W: 16-bit [M][K] on the GPU (float16 / bfloat16, or int16 bit patterns with dtype "f16" / "bf16");
    rho: optional float32 [M][K] saliency (default |w|).  Returns the packed arrays of W's rows in the order
    found (`row_order`: row r of the packed layer is channel row_order[r] of W; use it as pi_out), and the
    saliency pruned after every iteration of both searches."""
    M, K = W.shape
    T, P = M // V, Kv // 4
    dev = W.device
    rng = np.random.default_rng(seed)
    Wb = W.contiguous().view(torch.int16)
    row_order = torch.arange(M, dtype=torch.int32, device=dev)
    ocp_trace = []
    schedule = list(ocp_samples) if ocp_samples is not None else list(default_sample_schedule(V, ocp_iters))
    for n in schedule:
        n = int(min(max(1, n), V))
        samples = torch.from_numpy(np.stack([rng.permutation(V)[:n] for _ in range(T)]).astype(np.int32)).to(dev)
        clusters = None
        if n > 1 and T * n <= 1024 and kmeans_rounds > 0:
            wsb = hb.hinm_ocp_cluster_sizes(M, K, V, Kv, dtype, n)
            ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
            centroids = torch.empty((T, K), dtype=torch.float64, device=dev)
            clusters = torch.empty((T, n), dtype=torch.int32, device=dev)
            hb.hinm_ocp_cluster(M, K, V, Kv, dtype, Wb, rho, row_order, samples, n, kmeans_rounds, centroids, True,
                                clusters, None, ws, wsb)
        wsb = hb.hinm_ocp_sizes(M, K, V, Kv, dtype, n)
        ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
        obj = torch.zeros(1, dtype=torch.float64, device=dev)
        hb.hinm_ocp_search(M, K, V, Kv, dtype, Wb, rho, row_order, samples, clusters, n, 1, obj, ws, wsb)
        ocp_trace.append(obj)
    # the layer with its rows in the order found
    Wp = torch.empty_like(Wb)
    hb.hinm_apply_row_order(Wb, Wp, row_order, M, K * 2)
    rho_p = None
    if rho is not None:
        rho_c = rho.contiguous()
        rho_p = torch.empty((M, K), dtype=rho.dtype, device=dev)
        hb.hinm_apply_row_order(rho_c, rho_p, row_order, M, K * 4)
    vb, nb, cb, wb = hb.hinm_pack_sizes(M, K, V, Kv, dtype)
    ws = torch.empty(wb // 8, dtype=torch.float64, device=dev)
    vals_v = torch.empty(M * Kv, dtype=torch.int16, device=dev)
    vec_idx = torch.empty((T, Kv), dtype=torch.int32, device=dev)
    hb.hinm_pack_vectors(M, K, V, Kv, dtype, Wp, rho_p, None, vals_v, vec_idx, ws, wb)
    del vals_v
    icp_trace = None
    if icp_iters > 0:
        samples = torch.from_numpy(rng.integers(0, 4, size=(icp_iters, T, P), dtype=np.uint8)).to(dev)
        wsb = hb.hinm_icp_sizes(M, K, V, Kv, dtype)
        ws2 = torch.empty(wsb, dtype=torch.uint8, device=dev)
        icp_trace = torch.zeros((icp_iters, T), dtype=torch.float64, device=dev)
        hb.hinm_icp_search(M, K, V, Kv, dtype, Wp, rho_p, vec_idx, samples, icp_iters, icp_trace, ws2, wsb)
    sigma = torch.empty((T, K), dtype=torch.int32, device=dev)
    hb.hinm_tile_order(M, K, V, Kv, dtype, vec_idx, sigma)
    vals = torch.empty(vb // 2, dtype=torch.int16, device=dev)
    nm_idx = torch.empty(nb, dtype=torch.uint8, device=dev)
    vec_out = torch.empty((T, Kv), dtype=torch.int32, device=dev)
    if rho_p is None:
        hb.hinm_pack_ordered(M, K, V, Kv, dtype, Wp, sigma, vals, nm_idx, vec_out, ws, wb)
    else:
        hb.hinm_pack_scored(M, K, V, Kv, dtype, Wp, rho_p, sigma, vals, nm_idx, vec_out, ws, wb)
    torch.cuda.synchronize()
    return {
        "row_order": row_order, "vals": vals.view(M, Kv // 2), "nm_idx": nm_idx.view(M, Kv // 8), "vec_idx": vec_out,
        "tile_order": sigma, "samples_per_iteration": schedule,
        "vector_pruned_saliency": [float(o.item()) for o in ocp_trace],
        "nm_pruned_saliency": None if icp_trace is None else icp_trace.sum(dim=1).cpu().tolist(),
    }
