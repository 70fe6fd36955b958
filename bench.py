#!/usr/bin/env python3
"""Benchmark of the HiNM sparse-GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5]

A step is one pass of the run-time path (gather through vector index o pi_in,
sparse-MFMA product, pi_out scatter epilogue: hinm_spmm, or hinm_chain for c4)
over one batch of synthetic input that is already resident in HBM.  Packing is
the offline compression step of the method; it is timed by `--workload pack-c5`.
Consecutive steps rotate over enough independent copies of (packed W, X, Y)
to exceed the 256 MB Infinity Cache, so the traffic really comes from HBM.

Other workloads: `pack-c5[-ordered|-scored|-vectors]` (the offline compression step and its variants),
`vectors-<case>` (the product of a layer that carries the column-vector mask alone), `sweep-bert` /
`sweep-resnet` (every layer of a model block at several vector sizes and vector sparsities, with and
without channel orders, beside the dense GEMM).

The default workload is the largest configuration, C5 (16384 x 16384 bf16, N = 8192); the same run then times
every other configuration (C1, C2, the twelve C3 cases, the C4 chain) briefly and reports them under
`per_config`.  `--workload calib` runs the calibration kernels (measured ceilings of the machine) alone.

Prints ONE JSON line: metric / value / unit (dense-equivalent TFLOP/s of the whole job), ms_per_step, the
workload in `config`, `roofline` (algorithmic bytes or stored-value flops per launch over the average launch
duration from HIP events over the timed region, against the nominal HBM or MFMA peak and against this run's
calibration), `per_config`, `calibration` and `cpu_baseline` (the CPU oracle timed on a bounded sample).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import hinm_synth as synth  # noqa: E402

HBM_PEAK_GBPS = 8000.0
MFMA_DENSE_PEAK_TFLOPS = 2500.0   # fp16 / bf16 dense; useful (stored-value) flops are priced against this


PACK_WORKLOADS = ("pack-c5", "pack-c5-ordered", "pack-c5-scored", "pack-c5-vectors")


SWEEP_WORKLOADS = ("sweep-bert", "sweep-resnet")
ICP_WORKLOADS = ("icp-c2", "icp-c4")
OCP_WORKLOADS = ("ocp-c2", "ocp-c5", "ocp-cluster-c2")
FP64_ADD_PEAK_TOPS = 39.3         # 256 compute units x 64 lanes x 2.4 GHz = half the fp64 FMA flop figure


def workloads():
    w = {"c1": synth.c1(), "c2": synth.c2(), "c4": synth.c4(), "c5": synth.c5()}
    for c in synth.c3_cases():
        keep = "50" if c.Kv * 2 == c.K else "75"
        w[f"c3-{c.M}x{c.K}-s{keep}-n{c.N}"] = c
    return w


def algorithmic_bytes(c, N, layers=1):
    """Compulsory HBM traffic of one step: packed values + NM nibbles + vector index (int32) +
    both permutations + X + Y, each moved once."""
    per_layer = (c.M * c.Kv // 2 * 2 + c.M * c.Kv // 8 + c.T * c.Kv * 4 + c.K * 4 + c.M * 4
                 + c.K * N * 2 + c.M * N * 2)
    return per_layer * layers


def graph_replay_ms(torch, launch, steps):
    """Captures `steps` calls of launch(i) into one HIP graph, replays it once untimed and once between two
    HIP events recorded on the stream the replay is launched on; returns (wall ms, event ms) of the timed replay."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(steps):
                launch(i)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    graph.replay()
    ev1.record()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3, ev0.elapsed_time(ev1)


def calibrate(torch, hinm, dev, dtype, quick=True):
    """Ceilings of this machine measured with the plain kernels of include/hinm_calib.h, each between two HIP
    events: streaming copy / fill / read over 1 GiB (beyond the 256 MB memory-side cache), the issue rate of the
    32x32x32 sparse matrix instruction from registers, the cost of an empty graph node."""
    out = {}
    nbytes = 1 << 30
    a = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    b = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    sink = torch.zeros(2048 * 256, dtype=torch.float32, device=dev)
    a.fill_(1)
    b.fill_(2)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    reps = 5 if quick else 20
    for nt in (False, True):
        tag = "_nt" if nt else ""
        ms = timed(lambda: hinm.hinm_calib_copy(a, b, nbytes, nt), reps)
        out["copy" + tag + "_gbps"] = round(2 * nbytes / ms / 1e6, 1)       # bytes read + bytes written
        ms = timed(lambda: hinm.hinm_calib_fill(b, nbytes, nt), reps)
        out["write" + tag + "_gbps"] = round(nbytes / ms / 1e6, 1)
        ms = timed(lambda: hinm.hinm_calib_read(a, nbytes, sink, nt), reps)
        out["read" + tag + "_gbps"] = round(nbytes / ms / 1e6, 1)
    iters = 4000
    flops = [0.0]

    def smf():
        flops[0] = hinm.hinm_calib_smfmac(dtype, iters, sink)
    ms = timed(smf, reps)
    out["smfmac_stored_tflops"] = round(flops[0] / ms / 1e9, 1)                # hardware rating counts twice this
    out["smfmac_kernel_ms"] = round(ms, 4)
    nodes = 1000
    _, ev_ms = graph_replay_ms(torch, lambda i: hinm.hinm_calib_empty(), nodes)
    out["graph_node_floor_us"] = round(ev_ms * 1e3 / nodes, 3)
    if not quick:
        # compute units drawing data into LDS: a 2 MB region every workgroup walks (stays in L2), and a 1 GiB region
        # split into disjoint parts (every line comes from HBM); all 256 units at once, and 32 workgroups only
        # (HBM far from saturated: what one unit's memory pipeline sustains at the miss latency)
        region, chunks = 2 << 20, 16384
        for wgs in (32, 256, 512):
            ms = timed(lambda: hinm.hinm_calib_lds_stream(a, region, 8192, chunks, wgs), reps)
            out[f"l2_to_lds_gbps_{wgs}_workgroups"] = round(wgs * chunks * 8192 / ms / 1e6, 1)
        for wgs in (8, 32, 256):
            per = (nbytes // wgs) // 8192
            ms = timed(lambda: hinm.hinm_calib_lds_stream(a, nbytes, per * 8192, per, wgs), 3)
            out[f"hbm_to_lds_gbps_{wgs}_workgroups"] = round(wgs * per * 8192 / ms / 1e6, 1)
        # the tile kernels' request pattern without their stages and barriers: 1 KB segments of rows 16 KB apart,
        # copied into LDS by 1, 2, 4 or 8 waves of each of 256 workgroups, 16 copies in flight per wave; from a
        # 4 MB set of rows (L2 hits) and from 16384 rows = 256 MB (beyond L2; the memory-side cache holds part of it)
        pitch, copies = 16384, 4096
        for label, rows in (("l2", 256), ("far", 16384)):
            for waves in (1, 2, 4, 8):
                per = copies // waves
                ms = timed(lambda: hinm.hinm_calib_gather_stream(a, nbytes, pitch, rows, waves, 16, per, 256), 3)
                out[f"gathered_rows_to_lds_gbps_{label}_{waves}_waves"] = round(256 * waves * per * 1024 / ms / 1e6, 1)
        # store-only passes shaped like the C2 output (3072 x 4096 fp16): natural and permuted rows, three piece sizes
        M, N = 3072, 4096
        Ys = [torch.empty((M, N), dtype=torch.int16, device=dev) for _ in range(24)]    # 600 MB rotated
        rows = torch.from_numpy(np.random.default_rng(20496).permutation(M).astype(np.int32)).to(dev)
        for piece in (64, 128, 256, 512):
            for label, r in (("natural", None), ("permuted", rows)):
                _, ev_ms = graph_replay_ms(
                    torch, lambda i: hinm.hinm_calib_scatter_rows(Ys[i % len(Ys)], M, N, N, r, piece), 240)
                out[f"c2_output_store_only_us_{piece}B_{label}"] = round(ev_ms * 1e3 / 240, 2)
        del Ys
    del a, b
    torch.cuda.empty_cache()
    return out


class CaseRun:
    """One workload resident in HBM: packed (and prepared) on the GPU, enough rotated copies to exceed the
    memory-side cache, and the launch closure that bench times."""

    def __init__(self, key, c, args, torch, hinm, dev, keep_dense=False, columns=0):
        self.key, self.torch, self.hinm = key, torch, hinm
        if columns:
            import dataclasses
            c = dataclasses.replace(c, N=columns, name=f"{c.name} at N = {columns}")
        self.c = c
        self.chain = key == "c4"
        N = self.N = c.N
        self.n_layers = 2 if self.chain else 1
        self.variant = args.variant
        self.use_prepared = (not args.canonical) and c.V % 32 == 0

        def dev_bits(a):
            return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev)

        vb, nb, cb, wb = hinm.hinm_pack_sizes(c.M, c.K, c.V, c.Kv, c.dtype)
        packed = []
        self.W_dense = None
        for l in range(self.n_layers):
            W = dev_bits(c.weights(l))
            vals = torch.empty(vb // 2, dtype=torch.int16, device=dev)
            nm = torch.empty(nb, dtype=torch.uint8, device=dev)
            vec = torch.empty(cb // 4, dtype=torch.int32, device=dev)
            ws = torch.empty(wb // 8, dtype=torch.float64, device=dev)
            hinm.hinm_pack(c.M, c.K, c.V, c.Kv, c.dtype, W, vals, nm, vec, ws, wb)
            torch.cuda.synchronize()
            del ws
            pin = None if args.identity else torch.from_numpy(c.pi_in(l)).to(dev)
            pout = None if args.identity else torch.from_numpy(c.pi_out(l)).to(dev)
            prep = None
            if self.use_prepared:
                pbytes = hinm.hinm_prepare_sizes(c.M, c.K, c.V, c.Kv, c.dtype)
                prep = torch.empty(pbytes, dtype=torch.uint8, device=dev)
                hinm.hinm_prepare(c.M, c.K, c.V, c.Kv, c.dtype, vals, nm, vec, pin, pout, prep, pbytes)
                torch.cuda.synchronize()
            if l == 0 and keep_dense:
                self.W_dense = W
            del W
            packed.append((vals, nm, vec, pin, pout, prep))
        ldn = self.ldn = N if N == 1 else (N + 7) // 8 * 8 + args.ld_pad
        Xh = np.zeros((c.K, ldn), dtype=np.uint16)
        Xh[:, :N] = c.activations()
        self.X0 = dev_bits(Xh)
        per_set = sum(t.numel() * t.element_size() for (v, n, ve, _, _, _) in packed for t in (v, n, ve)) \
            + (c.K + c.M) * ldn * 2 * self.n_layers
        self.n_sets = n_sets = args.sets if args.sets else max(2, min(64, int(np.ceil(600e6 / per_set))))
        self.sets = []
        for i in range(n_sets):
            layers = []
            for (vals, nm, vec, pin, pout, prep) in packed:
                if self.use_prepared:
                    layers.append((None, None, None, None, None, prep if i == 0 else prep.clone()))
                elif i == 0:
                    layers.append((vals, nm, vec, pin, pout, None))
                else:
                    layers.append((vals.clone(), nm.clone(), vec.clone(), pin, pout, None))
            X = self.X0 if i == 0 else self.X0.clone()
            Y = torch.zeros((c.M, ldn), dtype=torch.int16, device=dev)
            scratch = torch.empty(c.M * ldn * 2, dtype=torch.uint8, device=dev) if self.chain else None
            self.sets.append((layers, X, Y, scratch))
        self.ws_bytes = hinm.hinm_spmm_prepared_workspace(c.M, c.K, c.V, c.Kv, c.dtype, N) if self.use_prepared else 0
        self.ws = torch.zeros(self.ws_bytes, dtype=torch.uint8, device=dev) if self.ws_bytes else None
        self.bytes_step = algorithmic_bytes(c, N, self.n_layers)
        self.flops_dense_equiv = 2.0 * c.M * c.K * N * self.n_layers
        self.flops_stored = 2.0 * c.M * (c.Kv // 2) * N * self.n_layers
        # which kernels one step launches: asked of the library (a dry run of its dispatch), not re-derived here
        if self.use_prepared:
            text, n = hinm.hinm_spmm_prepared_plan(c.M, c.K, c.V, c.Kv, c.dtype, N, ldn, ldn, self.variant << 16)
            self.kernels, self.kernel_launches_per_step = text, n * self.n_layers
        else:
            self.kernels = "hinm_spmm on the canonical arrays (kernel chosen by the library)"
            self.kernel_launches_per_step = self.n_layers
        # a layer whose tiles are split over two kernel launches (whole rounds + remainder) is still one product:
        # bytes and flops are priced per layer, over the time of the layer's launches together
        self.launches_per_step = self.n_layers

    def step(self, i):
        hinm, c, N, ldn = self.hinm, self.c, self.N, self.ldn
        layers, X, Y, scratch = self.sets[i % self.n_sets]
        vflag = self.variant << 16
        if self.chain:
            ls = [hinm.Layer(c.M, c.K, c.V, c.Kv, c.dtype, v, n, ve, pi, po,
                             (hinm.EPI_RELU if l == 0 else 0) | (vflag if pr is not None else 0), pr)
                  for l, (v, n, ve, pi, po, pr) in enumerate(layers)]
            hinm.hinm_chain(ls, N, X, ldn, Y, ldn, scratch, scratch.numel())
        else:
            v, n, ve, pi, po, pr = layers[0]
            if pr is not None:
                hinm.hinm_spmm_prepared(c.M, c.K, c.V, c.Kv, c.dtype, N, pr, X, ldn, Y, ldn, vflag, self.ws, self.ws_bytes)
            else:
                hinm.hinm_spmm(c.M, c.K, c.V, c.Kv, c.dtype, N, v, n, ve, pi, po, X, ldn, Y, ldn, 0)

    def estimate_step_s(self):
        torch = self.torch
        self.step(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(3):
            self.step(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / 3

    def time_steps(self, steps, warmup, graph=True):
        """(wall ms per step, HIP-event ms per step) over exactly `steps` timed steps after `warmup` untimed ones."""
        torch = self.torch
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        if graph:
            wall, ev = graph_replay_ms(torch, self.step, steps)
        else:
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            ev0.record()
            for i in range(steps):
                self.step(i)
            ev1.record()
            torch.cuda.synchronize()
            wall, ev = (time.perf_counter() - t0) * 1e3, ev0.elapsed_time(ev1)
        return wall / steps, ev / steps

    def tile_parts(self, steps):
        """Where the layer's tile kernel spends its time: the same launch with only its copy stream, and with only
        its LDS reads and MFMAs (hinm_calib_tile_part), each graph-timed over the rotated buffer sets.  None for a
        workload that does not run on one tile-kernel launch per layer."""
        if not self.use_prepared or self.variant or "spmm_tile_prepared_kernel" not in self.kernels \
                or self.kernel_launches_per_step != self.n_layers:
            return None
        hinm, c, out = self.hinm, self.c, {}

        def part(p):
            def launch(i):
                layers, X, _, _ = self.sets[i % self.n_sets]
                hinm.hinm_calib_tile_part(c.M, c.K, c.V, c.Kv, c.dtype, self.N, layers[0][5], X, self.ldn, p)
            return launch
        try:
            for p, name in ((1, "copy_stream_only_us"), (2, "lds_reads_and_mfma_only_us")):
                part(p)(0)
                self.torch.cuda.synchronize()
                _, ev = graph_replay_ms(self.torch, part(p), steps)
                out[name] = round(ev * 1e3 / steps, 2)
        except RuntimeError:
            return None
        out["note"] = ("first layer's tile kernel launched with one side removed (nothing stored): which of the two "
                       "the whole kernel's time follows says what bounds it")
        return out

    def roofline(self, launch_ms, calib):
        """The dominant kernel against the roofline that bounds it: algorithmic bytes (or stored-value flops) of one
        launch over the average launch duration measured with HIP events over the timed region."""
        n = self.n_layers
        mem_bound = (self.bytes_step / HBM_PEAK_GBPS / 1e9) >= (self.flops_stored / MFMA_DENSE_PEAK_TFLOPS / 1e12)
        if mem_bound:
            ach = self.bytes_step / n / (launch_ms * 1e-3) / 1e9
            r = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                 "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None}
            if calib:
                r["peak_calibrated"] = calib["copy_gbps"]
                r["frac_calibrated"] = round(ach / calib["copy_gbps"], 4)
                r["peak_calibrated_is"] = "1 GiB device copy kernel, bytes read + written per second"
        else:
            ach = self.flops_stored / n / (launch_ms * 1e-3) / 1e12
            r = {"bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_DENSE_PEAK_TFLOPS, "unit": "TFLOP/s",
                 "frac": round(ach / MFMA_DENSE_PEAK_TFLOPS, 4), "traffic": None}
            if calib:
                r["peak_calibrated"] = calib["smfmac_stored_tflops"]
                r["frac_calibrated"] = round(ach / calib["smfmac_stored_tflops"], 4)
                r["peak_calibrated_is"] = "register-resident 32x32x32 sparse-MFMA loop, stored-value flops per second"
        r["kernel"] = self.kernels
        r["layers_per_step"] = self.n_layers
        r["kernel_launches_per_step"] = self.kernel_launches_per_step
        if calib and mem_bound:
            r["frac_of_read_stream"] = round(ach / calib["read_gbps"], 4)
        r["avg_layer_ms_hip_events_over_timed_region"] = round(launch_ms, 6)
        r["algorithmic_bytes_per_launch"] = self.bytes_step // n
        r["stored_value_flops_per_launch"] = self.flops_stored / n
        return r

    def free(self):
        self.sets = None
        self.X0 = self.W_dense = self.ws = None
        self.torch.cuda.empty_cache()


def stored_traffic(key, canonical):
    """HBM bytes per launch from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            tr = json.load(f).get(key if not canonical else key + "-canonical")
        if tr:
            return tr["fetch_bytes"] + tr["write_bytes"], "stored summary, not measured in this run: " + tr.get("source", "")
    except (OSError, ValueError):
        pass
    return None, None


def measure_traffic_live(key, extra_args):
    """HBM bytes per launch of the workload's SpMM kernels from two rocprofv3 --pmc runs (FETCH_SIZE, then
    WRITE_SIZE) of this script as child processes, each scaled by what the same counter reads for the 256 MiB
    bitwise_not probe of known size in the same run.  Must run before this process touches the GPU."""
    import csv
    import glob
    import subprocess
    import tempfile
    totals, factors = {}, {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        out = tempfile.mkdtemp(prefix="hinm_pmc_", dir="/tmp")
        cmd = ["rocprofv3", "--pmc", counter, "--output-format", "csv", "-d", out, "-o", "p", "--",
               "python3", os.path.abspath(__file__), "--workload", key, "--no-cpu", "--no-dense", "--no-graph",
               "--no-per-config", "--no-calib", "--steps", "4", "--warmup", "1", "--copy-probe"] + extra_args
        env = dict(os.environ, TMPDIR="/tmp")
        res = subprocess.run(cmd, cwd="/tmp", env=env, capture_output=True, text=True, timeout=300)
        files = glob.glob(os.path.join(out, "**", "*counter_collection.csv"), recursive=True)
        if res.returncode != 0 or not files:
            return None, f"rocprofv3 --pmc {counter} failed (rc {res.returncode})"
        spmm, probe = {}, []
        with open(files[0]) as f:
            for r in csv.DictReader(f):
                if r["Counter_Name"] != counter:
                    continue
                k, v = r["Kernel_Name"], float(r["Counter_Value"])
                if "spmm_" in k:
                    spmm.setdefault(k, []).append(v)
                elif "bitwise_not" in k:
                    probe.append(v)
        if not spmm or not probe:
            return None, "no SpMM or probe dispatches in the counter output"
        factors[counter] = 262144.0 / (sum(probe) / len(probe))
        # one launch of each kernel per step (a step of two different kernels adds them)
        totals[counter] = sum(sum(v) / len(v) for v in spmm.values()) * 1024.0 * factors[counter]
    return int(totals["FETCH_SIZE"] + totals["WRITE_SIZE"]), (
        f"measured in this run: rocprofv3 --pmc FETCH_SIZE (x{factors['FETCH_SIZE']:.2f}) and WRITE_SIZE "
        f"(x{factors['WRITE_SIZE']:.2f}) on child runs, read {totals['FETCH_SIZE'] / 1e6:.1f} MB + written "
        f"{totals['WRITE_SIZE'] / 1e6:.1f} MB per launch")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c5")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-dense", action="store_true", help="skip the same-shape dense GEMM reference")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the short runs of the other configurations that fill `per_config`")
    ap.add_argument("--no-calib", action="store_true", help="skip the calibration kernels (measured peaks)")
    ap.add_argument("--measure-traffic", action="store_true",
                    help="measure roofline.traffic in this run with two rocprofv3 --pmc child runs instead of "
                         "reading the committed summary")
    ap.add_argument("--identity", action="store_true", help="run with identity permutations")
    ap.add_argument("--canonical", action="store_true",
                    help="call hinm_spmm on the canonical arrays instead of hinm_spmm_prepared")
    ap.add_argument("--variant", type=int, default=0, help="pin a tile-kernel configuration (tuning aid)")
    ap.add_argument("--sets", type=int, default=None,
                    help="number of rotated buffer sets (default: enough to exceed the Infinity Cache)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (calibrates the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--kernel-us", type=float, default=None,
                    help="icp / ocp workloads: average duration of the cost kernel from a rocprofv3 summary, to price it")
    ap.add_argument("--columns", type=int, default=0,
                    help="run the workload's layer(s) at this many columns instead of its own N (not a BASELINE configuration)")
    ap.add_argument("--ld-pad", type=int, default=0,
                    help="add this many elements (a multiple of 8) to the leading dimensions of X and Y")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every step from the host instead of replaying one captured HIP graph of K steps")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    live_traffic = None
    if args.measure_traffic and args.workload in workloads():
        extra = (["--identity"] if args.identity else []) + (["--canonical"] if args.canonical else []) \
            + (["--variant", str(args.variant)] if args.variant else [])
        try:
            live_traffic = measure_traffic_live(args.workload, extra)
        except Exception as err:  # the headline run goes on without it
            live_traffic = (None, f"live traffic measurement failed: {err!r}")

    import torch
    import paper_2407_20496_amd as hinm
    hinm.load_library()  # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.workload == "calib":
        return bench_calib(args, torch, hinm, dev)
    if args.workload in PACK_WORKLOADS:
        return bench_pack(args, torch, hinm, dev)
    if args.workload in SWEEP_WORKLOADS:
        return bench_sweep(args, torch, hinm, dev)
    if args.workload in ICP_WORKLOADS:
        return bench_icp(args, torch, hinm, dev)
    if args.workload in OCP_WORKLOADS:
        return bench_ocp(args, torch, hinm, dev)
    wl = workloads()
    if args.workload.startswith("vectors-") and args.workload[8:] in wl:
        return bench_vectors(args, torch, hinm, dev, wl[args.workload[8:]])
    if args.workload not in wl:
        print("unknown workload; choose from: calib " + " ".join(PACK_WORKLOADS + SWEEP_WORKLOADS + ICP_WORKLOADS + OCP_WORKLOADS) + " "
              + " ".join(wl)
              + " vectors-<any of the latter>", file=sys.stderr)
        sys.exit(2)

    run = CaseRun(args.workload, wl[args.workload], args, torch, hinm, dev, keep_dense=not args.no_dense,
                  columns=args.columns)
    c, N, n_layers, chain = run.c, run.N, run.n_layers, run.chain
    calib = None if args.no_calib else calibrate(torch, hinm, dev, c.dtype)

    est = run.estimate_step_s()
    steps = args.steps if args.steps is not None else int(min(5000, max(20, 1.0 / max(est, 1e-6))))
    warmup = args.warmup if args.warmup is not None else max(3, steps // 10)
    # The K timed steps are captured once into a HIP graph and replayed: a step of the small configurations lasts
    # a few microseconds, less than a host-side launch through Python, so launching from the host would time the
    # interpreter.  The graph holds exactly K steps (kernel_launches_per_step kernel nodes each).
    ms_per_step, gpu_ms_per_step = run.time_steps(steps, warmup, graph=not args.no_graph)
    launch_ms = gpu_ms_per_step / run.launches_per_step

    roofline = run.roofline(launch_ms, calib)
    if not args.no_calib:
        parts = run.tile_parts(max(20, steps // 4))
        if parts:
            roofline["kernel_parts"] = parts
    if not args.columns:
        if live_traffic is not None:
            roofline["traffic"], roofline["traffic_source"] = live_traffic
        else:
            roofline["traffic"], roofline["traffic_source"] = stored_traffic(args.workload, args.canonical)
        if roofline["traffic"]:
            roofline["traffic_over_algorithmic"] = round(roofline["traffic"] / (run.bytes_step / n_layers), 2)

    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.bitwise_not(src, out=dst)   # an elementwise kernel of its own: reads and writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- same-shape dense GEMM (library) on the same tensors, same timing method ---------------
    dense = None
    if run.W_dense is not None:
        tdt = torch.float16 if c.dtype == "f16" else torch.bfloat16
        Wd = run.W_dense.view(tdt).reshape(c.M, c.K)
        Xd = run.X0.view(tdt).reshape(c.K, run.ldn)[:, :N].contiguous()
        for _ in range(3):
            torch.matmul(Wd, Xd)
        torch.cuda.synchronize()
        reps = max(5, min(200, steps // 10))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            torch.matmul(Wd, Xd)
        e1.record()
        torch.cuda.synchronize()
        dms = e0.elapsed_time(e1) / reps
        dense = {"ms": round(dms, 5), "tflops": round(2.0 * c.M * c.K * N / dms / 1e9, 2),
                 "note": "torch.matmul on the unpruned W, single buffer set (cache-warm)"}
        del Wd, Xd

    value = run.flops_dense_equiv / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": "hinm_spmm_dense_equiv_tflops", "value": round(value, 3), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": c.dtype, "data": "synthetic",
        "config": {"workload": c.name + (" (two-layer chain)" if chain else ""), "M": c.M, "K": c.K, "V": c.V,
                   "Kv": c.Kv, "N": N, "layers": n_layers,
                   "permutation": "identity" if args.identity else "seeded random pi_in/pi_out",
                   "buffer_sets_rotated": run.n_sets,
                   "entry_point": ("hinm_chain" if chain else "hinm_spmm")
                   + ("_prepared" if run.use_prepared and not chain else "") + (" (prepared layers)" if chain and run.use_prepared else ""),
                   "variant": args.variant,
                   "launch": "host loop" if args.no_graph else "one HIP graph of K steps"},
        "gpu_ms_per_step_events": round(gpu_ms_per_step, 6),
        "hbm_gbps_algorithmic": round(run.bytes_step / (gpu_ms_per_step * 1e-3) / 1e9, 1),
        "stored_value_tflops": round(run.flops_stored / (gpu_ms_per_step * 1e-3) / 1e12, 3),
        "roofline": roofline, "cpu_baseline": None, "dense_gemm": dense, "calibration": calib,
    }
    run.free()

    # ---- the other configurations, one short graph-timed run each -------------------------------
    if not args.no_per_config and not args.columns:
        per = {args.workload: {"us_per_step": round(gpu_ms_per_step * 1e3, 2), "bound": roofline["bound"],
                               "frac": roofline["frac"], "frac_calibrated": roofline.get("frac_calibrated"),
                               "kernel": roofline["kernel"], "layers_per_step": run.n_layers}}
        for key, cc in wl.items():
            if key == args.workload or key == "c5":
                continue
            try:
                r = CaseRun(key, cc, args, torch, hinm, dev)
                e = r.estimate_step_s()
                k = int(min(2000, max(20, 0.25 / max(e, 1e-6))))
                _, g_ms = r.time_steps(k, max(3, k // 10))
                rf = r.roofline(g_ms / r.launches_per_step, calib)
                per[key] = {"us_per_step": round(g_ms * 1e3, 2), "steps": k, "bound": rf["bound"],
                            "achieved": rf["achieved"], "unit": rf["unit"], "frac": rf["frac"],
                            "frac_calibrated": rf.get("frac_calibrated"), "kernel": rf["kernel"],
                            "layers_per_step": r.n_layers,
                            "dense_equiv_tflops": round(r.flops_dense_equiv / (g_ms * 1e-3) / 1e12, 1)}
                parts = None if args.no_calib else r.tile_parts(max(20, k // 4))
                if parts:
                    per[key]["kernel_parts"] = {a: b for a, b in parts.items() if a != "note"}
                r.free()
                del r
            except Exception as err:   # one configuration failing must not lose the headline
                per[key] = {"error": repr(err)}
        out["per_config"] = per
        out["per_config_note"] = ("every BASELINE configuration timed in this run: HIP-event time of one graph replay / "
                                  "steps; frac against the nominal peak of the bound (8 TB/s HBM or 2.5 PFLOP/s dense "
                                  "fp16/bf16 on stored-value flops), frac_calibrated against this run's calibration; C1 is "
                                  "launch-bound (no roofline claim)")

    # ---- CPU oracle baseline on the host cores ---------------------------------------------------
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(c, N, chain)
    print(json.dumps(out))


def bench_calib(args, torch, hinm, dev):
    """The calibration kernels alone, long form: one JSON line with the measured ceilings."""
    cal = calibrate(torch, hinm, dev, "bf16", quick=False)
    cal16 = calibrate(torch, hinm, dev, "f16", quick=True)
    cal["smfmac_stored_tflops_f16"] = cal16["smfmac_stored_tflops"]
    print(json.dumps({"metric": "calibration", "value": cal["copy_gbps"], "unit": "GB/s", "n_gpus": 1, "steps": 20,
                      "warmup": 1, "ms_per_step": None, "higher_is_better": True, "scaling": "weak",
                      "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "calibration kernels (include/hinm_calib.h)"},
                      "calibration": cal, "roofline": None, "cpu_baseline": None}))


def cpu_baseline(c, N, chain):
    """The oracle as it stands (explicit masks, explicit permutation matrices, float32 matmul), timed on this
    box's host cores on a bounded sample of the workload: two whole tiles plus rows spread over all tiles
    (at most 1280 rows of W in all), all K input channels, and as many columns of X as keep the work near
    2 TFLOP of float32 matmul."""
    from oracle import hinm_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    rng = np.random.default_rng(20496)
    whole = sorted(set([0, c.T // 2]))
    extra_per_tile = max(1, min(8, (1280 - len(whole) * c.V) // max(1, c.T)))
    Wb = c.weights()
    rows = []
    t0 = time.perf_counter()
    packed_tiles = {}
    for t in range(c.T):
        pick = np.arange(c.V) if t in whole else np.sort(rng.choice(c.V, min(c.V, extra_per_tile), replace=False))
        rows.extend(t * c.V + pick)
    rows = np.array(rows[:1280]) if len(rows) > 1280 else np.array(rows)
    tiles = sorted(set((rows // c.V).tolist()))
    Wh_rows = np.zeros((len(rows), c.K), dtype=np.uint16)
    for t in tiles:
        sl = slice(t * c.V, (t + 1) * c.V)
        ov, on, oc = orc.pack(Wb[sl], c.dtype, c.V, c.Kv)
        Wh_t = orc.unpack_fast(ov, on, oc, c.V, c.K, c.V)
        sel = (rows // c.V) == t
        Wh_rows[sel] = Wh_t[rows[sel] - t * c.V]
    t_pack = time.perf_counter() - t0
    del Wb
    # columns: the permutation product P_in X dominates (2 K^2 n flops); keep the whole sample near 2 TFLOP
    per_col = 2.0 * c.K * c.K + 2.0 * len(rows) * c.K + 2.0 * len(rows) * len(rows)
    n = int(max(1, min(N, 2e12 // per_col)))
    Xb = c.activations()[:, :n]
    pin = c.pi_in()
    pout = np.argsort(np.argsort(c.pi_out()[rows])).astype(np.int32)   # the sampled rows' own output order
    reps, t_prod = 0, 0.0
    while t_prod < 8.0 and reps < 20:
        t0 = time.perf_counter()
        orc.spmm(Wh_rows, Xb, c.dtype, pin, pout)
        t_prod += time.perf_counter() - t0
        reps += 1
    t_one = t_prod / reps
    layers = 2 if chain else 1
    return {"value": round(2.0 * len(rows) * c.K * n / t_one / 1e12, 5), "unit": "TFLOP/s", "cores": int(threads),
            "kind": "oracle",
            "sample": f"oracle product (explicit permutation matrices, float32 numpy matmul) on {len(rows)} rows of W "
                      f"(tiles {whole} whole, {extra_per_tile} rows of each other tile: {len(tiles)} of {c.T} tiles) x "
                      f"{n} of {N} columns, {reps} repetitions, {t_one * 1e3:.1f} ms each; dense-equivalent flops of "
                      f"the sample over that time; oracle pack of the {len(tiles)} tiles {t_pack * 1e3:.0f} ms; "
                      f"host cpu_count {os.cpu_count()}" + ("; one layer of the two" if layers == 2 else "")}


def bench_pack(args, torch, hinm, dev):
    """The offline compression step on the C5 layer: hinm_pack, or one of its variants (a tile-wise order of
    the kept vectors, caller-given saliency scores, column-vector pruning alone)."""
    c = synth.c5()
    W = torch.from_numpy(c.weights().view(np.int16)).to(dev)
    vb, nb, cb, wb = hinm.hinm_pack_sizes(c.M, c.K, c.V, c.Kv, c.dtype)
    kind = args.workload[len("pack-c5"):].lstrip("-") or "plain"
    vals = torch.empty(c.M * c.Kv if kind == "vectors" else vb // 2, dtype=torch.int16, device=dev)
    nm = torch.empty(nb, dtype=torch.uint8, device=dev)
    vec = torch.empty(cb // 4, dtype=torch.int32, device=dev)
    ws = torch.empty(wb // 8, dtype=torch.float64, device=dev)
    steps = args.steps or 10
    warmup = args.warmup or 2
    sigma = rho = None
    rng = np.random.default_rng(20496)
    if kind == "ordered":   # a seeded random order of the input channels per tile (stands in for a search result)
        sigma = torch.from_numpy(np.stack([rng.permutation(c.K) for _ in range(c.T)]).astype(np.int32)).to(dev)
    if kind == "scored":    # seeded non-negative scores with a wide range (stand in for second-order saliency)
        rho = torch.from_numpy(rng.standard_normal((c.M, c.K), dtype=np.float32) ** 2).to(dev)

    def pack_once():
        if kind == "ordered":
            hinm.hinm_pack_ordered(c.M, c.K, c.V, c.Kv, c.dtype, W, sigma, vals, nm, vec, ws, wb)
        elif kind == "scored":
            hinm.hinm_pack_scored(c.M, c.K, c.V, c.Kv, c.dtype, W, rho, None, vals, nm, vec, ws, wb)
        elif kind == "vectors":
            hinm.hinm_pack_vectors(c.M, c.K, c.V, c.Kv, c.dtype, W, None, None, vals, vec, ws, wb)
        else:
            hinm.hinm_pack(c.M, c.K, c.V, c.Kv, c.dtype, W, vals, nm, vec, ws, wb)
    for _ in range(warmup):
        pack_once()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        pack_once()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    ms = e0.elapsed_time(e1) / steps
    w_bytes = c.M * c.K * 2
    traffic = 2 * w_bytes + vb + nb + cb + 2 * wb          # W read twice, outputs, scores written + read
    if kind == "ordered":
        traffic += c.T * c.K * 4 + 2 * cb                  # the order read once, the vector index re-read and re-written
    if kind == "scored":
        traffic += 2 * c.M * c.K * 4 - w_bytes             # the scores read twice, W only once
    if kind == "vectors":
        traffic += c.M * c.Kv * 2 - vb - nb                # all surviving entries written, no NM index
    entry = {"plain": "hinm_pack", "ordered": "hinm_pack_ordered", "scored": "hinm_pack_scored",
             "vectors": "hinm_pack_vectors"}[kind]
    out = {"metric": "hinm_pack_gbps", "value": round(traffic / (ms * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1,
           "steps": steps, "warmup": warmup, "ms_per_step": round(wall * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": c.dtype, "data": "synthetic",
           "config": {"workload": entry + " of " + c.name},
           "roofline": {"bound": "hbm", "achieved": round(traffic / (ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS,
                        "unit": "GB/s", "frac": round(traffic / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                        "traffic": None, "algorithmic_bytes_per_launch": traffic},
           "cpu_baseline": None}
    print(json.dumps(out))


def bench_vectors(args, torch, hinm, dev, c):
    """The product of a layer that carries the column-vector mask alone (hinm_pack_vectors, then
    hinm_spmm_vectors per step): a dense contraction over the gathered input rows, priced against the dense
    MFMA peak on its stored values, or against HBM when the compulsory bytes take longer."""
    N = c.N
    ldn = N if N == 1 else (N + 7) // 8 * 8
    _, _, cb, wb = hinm.hinm_pack_sizes(c.M, c.K, c.V, c.Kv, c.dtype)
    W = torch.from_numpy(c.weights().view(np.int16)).to(dev)
    vals_v = torch.empty(c.M * c.Kv, dtype=torch.int16, device=dev)
    vec = torch.empty(cb // 4, dtype=torch.int32, device=dev)
    ws = torch.empty(wb // 8, dtype=torch.float64, device=dev)
    hinm.hinm_pack_vectors(c.M, c.K, c.V, c.Kv, c.dtype, W, None, None, vals_v, vec, ws, wb)
    torch.cuda.synchronize()
    del W, ws
    pin = None if args.identity else torch.from_numpy(c.pi_in()).to(dev)
    pout = None if args.identity else torch.from_numpy(c.pi_out()).to(dev)
    Xh = np.zeros((c.K, ldn), dtype=np.uint16)
    Xh[:, :N] = c.activations()
    X0 = torch.from_numpy(Xh.view(np.int16)).to(dev)
    per_set = c.M * c.Kv * 2 + cb + (c.K + c.M) * ldn * 2
    n_sets = args.sets if args.sets else max(2, min(64, int(np.ceil(600e6 / per_set))))
    sets = [(vals_v if i == 0 else vals_v.clone(), vec if i == 0 else vec.clone(), X0 if i == 0 else X0.clone(),
             torch.zeros((c.M, ldn), dtype=torch.int16, device=dev)) for i in range(n_sets)]

    def step(i):
        v, ve, X, Y = sets[i % n_sets]
        hinm.hinm_spmm_vectors(c.M, c.K, c.V, c.Kv, c.dtype, N, v, ve, pin, pout, X, ldn, Y, ldn, 0)

    step(0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(3):
        step(i)
    torch.cuda.synchronize()
    est = (time.perf_counter() - t0) / 3
    steps = args.steps if args.steps is not None else int(min(2000, max(10, 1.0 / max(est, 1e-6))))
    warmup = args.warmup if args.warmup is not None else max(2, steps // 10)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(steps):
                step(i)
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    graph.replay()
    ev1.record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    kernel_ms = ev0.elapsed_time(ev1) / steps
    flops = 2.0 * c.M * c.Kv * N
    bytes_step = c.M * c.Kv * 2 + cb + (c.K + c.M) * 4 + c.K * N * 2 + c.M * N * 2
    if bytes_step / HBM_PEAK_GBPS / 1e9 >= flops / MFMA_DENSE_PEAK_TFLOPS / 1e12:
        ach = bytes_step / (kernel_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None}
    else:
        ach = flops / (kernel_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_DENSE_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / MFMA_DENSE_PEAK_TFLOPS, 4), "traffic": None}
    roofline.update({"kernel": "spmm_vectors_kernel", "kernel_ms_avg": round(kernel_ms, 6),
                     "algorithmic_bytes_per_launch": bytes_step, "stored_value_flops_per_launch": flops})
    out = {"metric": "hinm_spmm_dense_equiv_tflops", "value": round(2.0 * c.M * c.K * N / (ms_per_step * 1e-3) / 1e12, 3),
           "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 6),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": c.dtype, "data": "synthetic",
           "config": {"workload": "vector-pruned only (no 2:4 step): " + c.name, "M": c.M, "K": c.K, "V": c.V,
                      "Kv": c.Kv, "N": N, "permutation": "identity" if args.identity else "seeded random pi_in/pi_out",
                      "buffer_sets_rotated": n_sets, "entry_point": "hinm_spmm_vectors",
                      "launch": "one HIP graph of K steps"},
           "stored_value_tflops": round(flops / (kernel_ms * 1e-3) / 1e12, 3), "roofline": roofline,
           "cpu_baseline": None}
    print(json.dumps(out))


def bench_icp(args, torch, hinm, dev):
    """Tile-wise input-channel permutation search (hinm_icp_search) on a packed layer: K iterations in one call,
    samples drawn on the host from a seeded generator.  `value` = iterations per second over all tiles; the
    roofline object prices the cost-matrix kernel (two binary64 additions per partition x sample x row) against
    the binary64 add rate of the vector units."""
    c = synth.c2() if args.workload == "icp-c2" else synth.c4()
    P = c.Kv // 4
    W = torch.from_numpy(c.weights().view(np.int16)).to(dev)
    vb, nb, cb, wb = hinm.hinm_pack_sizes(c.M, c.K, c.V, c.Kv, c.dtype)
    vals = torch.empty(vb // 2, dtype=torch.int16, device=dev)
    nm = torch.empty(nb, dtype=torch.uint8, device=dev)
    vec0 = torch.empty(cb // 4, dtype=torch.int32, device=dev)
    ws = torch.empty(wb // 8, dtype=torch.float64, device=dev)
    hinm.hinm_pack(c.M, c.K, c.V, c.Kv, c.dtype, W, vals, nm, vec0, ws, wb)
    del ws
    steps = args.steps or 20
    warmup = args.warmup or 2
    rng = np.random.default_rng(20496)
    samples = torch.from_numpy(rng.integers(0, 4, size=(steps, c.T, P), dtype=np.uint8)).to(dev)
    wsb = hinm.hinm_icp_sizes(c.M, c.K, c.V, c.Kv, c.dtype)
    work = torch.empty(wsb, dtype=torch.uint8, device=dev)
    obj = torch.zeros((steps, c.T), dtype=torch.float64, device=dev)
    vec = vec0.clone()
    hinm.hinm_icp_search(c.M, c.K, c.V, c.Kv, c.dtype, W, None, vec, samples, warmup, obj, work, wsb)
    torch.cuda.synchronize()
    vec.copy_(vec0)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    hinm.hinm_icp_search(c.M, c.K, c.V, c.Kv, c.dtype, W, None, vec, samples, steps, obj, work, wsb)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ms = e0.elapsed_time(e1) / steps
    o = obj.cpu().numpy()
    # per-kernel share from a short second run under events is not available here; the cost kernel's own time
    # is in the rocprofv3 summary.  Its work per iteration:
    adds = 2.0 * c.T * P * P * c.V
    out = {"metric": "hinm_icp_iterations_per_s", "value": round(1e3 / ms, 2), "unit": "iterations/s", "n_gpus": 1,
           "steps": steps, "warmup": warmup, "ms_per_step": round(wall_ms, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
           "config": {"workload": "tile-wise input-channel permutation search on " + c.name, "tiles": c.T,
                      "partitions_per_tile": P, "rows_per_tile": c.V,
                      "pruned_saliency_first_iteration": float(o[0].sum()),
                      "pruned_saliency_last_iteration": float(o[-1].sum())},
           "gpu_ms_per_iteration": round(ms, 4),
           "roofline": {"bound": "alu", "kernel": "icp_cost_kernel", "achieved": None, "peak": FP64_ADD_PEAK_TOPS,
                        "unit": "Tadd/s (binary64)", "frac": None, "traffic": None,
                        "adds_per_launch": adds,
                        "note": "achieved = adds_per_launch / the kernel's average duration in the rocprofv3 summary"},
           "cpu_baseline": None}
    if args.kernel_us:
        ach = adds / (args.kernel_us * 1e-6) / 1e12
        out["roofline"].update({"achieved": round(ach, 3), "frac": round(ach / FP64_ADD_PEAK_TOPS, 4),
                                "kernel_us_avg": args.kernel_us})
    print(json.dumps(out))


def bench_ocp(args, torch, hinm, dev):
    """Output-channel permutation search (hinm_ocp_search) on a dense layer: K iterations in one call, samples
    drawn on the host from a seeded generator, every tile's own samples as its cluster.  `value` = iterations
    per second; the roofline object prices the cost kernel (64 counting passes of 64-bit compares over the K
    column scores of every tile x cluster pair) against the 64-bit rate of the vector units."""
    c = synth.c5() if args.workload == "ocp-c5" else synth.c2()
    n = max(1, c.V // 8)
    W = torch.from_numpy(c.weights().view(np.int16)).to(dev)
    steps = args.steps or 10
    warmup = args.warmup or 2
    rng = np.random.default_rng(20496)
    samples = torch.from_numpy(np.stack([np.stack([rng.permutation(c.V)[:n] for _ in range(c.T)])
                                         for _ in range(steps)]).astype(np.int32)).to(dev)
    if args.workload == "ocp-cluster-c2":
        # the clustering phase alone: K rounds of balanced K-means over one iteration's samples
        wsb = hinm.hinm_ocp_cluster_sizes(c.M, c.K, c.V, c.Kv, c.dtype, n)
        work = torch.empty(wsb, dtype=torch.uint8, device=dev)
        order = torch.arange(c.M, dtype=torch.int32, device=dev)
        cen = torch.empty((c.T, c.K), dtype=torch.float64, device=dev)
        clusters = torch.empty((c.T, n), dtype=torch.int32, device=dev)
        obj = torch.zeros(steps, dtype=torch.float64, device=dev)
        hinm.hinm_ocp_cluster(c.M, c.K, c.V, c.Kv, c.dtype, W, None, order, samples[0], n, 1, cen, True, clusters, obj,
                              work, wsb)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        hinm.hinm_ocp_cluster(c.M, c.K, c.V, c.Kv, c.dtype, W, None, order, samples[0], n, steps, cen, True, clusters,
                              obj, work, wsb)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        ms = e0.elapsed_time(e1) / steps
        o = obj.cpu().numpy()
        print(json.dumps({
            "metric": "hinm_ocp_cluster_rounds_per_s", "value": round(1e3 / ms, 2), "unit": "rounds/s", "n_gpus": 1,
            "steps": steps, "warmup": 1, "ms_per_step": round(wall_ms, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f64", "data": "synthetic",
            "config": {"workload": "balanced K-means over the sampled channels of " + c.name, "points": c.T * n,
                       "clusters": c.T, "features": c.K, "distance_first_round": float(o[0]),
                       "distance_last_round": float(o[-1])},
            "gpu_ms_per_round": round(ms, 4), "roofline": None, "cpu_baseline": None}))
        return
    wsb = hinm.hinm_ocp_sizes(c.M, c.K, c.V, c.Kv, c.dtype, n)
    work = torch.empty(wsb, dtype=torch.uint8, device=dev)
    obj = torch.zeros(steps, dtype=torch.float64, device=dev)
    order = torch.arange(c.M, dtype=torch.int32, device=dev)
    hinm.hinm_ocp_search(c.M, c.K, c.V, c.Kv, c.dtype, W, None, order, samples, None, n, warmup, obj, work, wsb)
    torch.cuda.synchronize()
    order = torch.arange(c.M, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    hinm.hinm_ocp_search(c.M, c.K, c.V, c.Kv, c.dtype, W, None, order, samples, None, n, steps, obj, work, wsb)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ms = e0.elapsed_time(e1) / steps
    o = obj.cpu().numpy()
    compares = 64.0 * c.T * c.T * c.K
    out = {"metric": "hinm_ocp_iterations_per_s", "value": round(1e3 / ms, 2), "unit": "iterations/s", "n_gpus": 1,
           "steps": steps, "warmup": warmup, "ms_per_step": round(wall_ms, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
           "config": {"workload": "output-channel permutation search on " + c.name, "tiles": c.T,
                      "samples_per_tile": n, "clusters": "every tile's own samples",
                      "pruned_saliency_first_iteration": float(o[0]), "pruned_saliency_last_iteration": float(o[-1])},
           "gpu_ms_per_iteration": round(ms, 4),
           "roofline": {"bound": "alu", "kernel": "ocp_cost_kernel", "achieved": None, "peak": FP64_ADD_PEAK_TOPS,
                        "unit": "T 64-bit compares/s", "frac": None, "traffic": None, "compares_per_launch": compares,
                        "note": "achieved = compares_per_launch / the kernel's average duration in the rocprofv3 summary"},
           "cpu_baseline": None}
    if args.kernel_us:
        ach = compares / (args.kernel_us * 1e-6) / 1e12
        out["roofline"].update({"achieved": round(ach, 3), "frac": round(ach / FP64_ADD_PEAK_TOPS, 4),
                                "kernel_us_avg": args.kernel_us})
    print(json.dumps(out))


def bench_sweep(args, torch, hinm, dev):
    """Section 5.3 (latency figure): the same layers at several vector sizes and vector sparsities, with seeded
    random channel orders and with identity orders, beside the dense GEMM of the unpruned layer.  One JSON
    line; `value` is the dense-equivalent rate of the whole sweep with channel orders, `table` holds one row
    per (V, vector sparsity): microseconds summed over the layers."""
    layers = synth.sweep_layers(args.workload)
    bert = args.workload == "sweep-bert"
    v_list = (32, 64, 128) if bert else (32,)
    keep_list = ((2, "50"), (4, "75"), (8, "87.5"))         # Kv = K / keep -> total sparsity 75 / 87.5 / 93.75 %
    dtype = "f16"
    tdt = torch.float16
    steps = args.steps or 200

    def graph_time_us(launch, n_sets):
        for i in range(3):
            launch(i)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                for i in range(steps):
                    launch(i)
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / steps

    table, dense_us = [], {}
    flops_total, time_total = 0.0, 0.0
    for li, (name, M, K, N) in enumerate(layers):
        ldn = (N + 7) // 8 * 8
        Wb = synth.gaussian_bits((M, K), 0.02, dtype, synth.seed_for(5, 0) + 1000 * li)
        Xh = np.zeros((K, ldn), dtype=np.uint16)
        Xh[:, :N] = synth.gaussian_bits((K, N), 1.0, dtype, synth.seed_for(5, 1) + 1000 * li)
        Wd = torch.from_numpy(Wb.view(np.int16)).to(dev)
        n_sets = max(2, min(32, int(np.ceil(600e6 / ((K + M) * ldn * 2)))))
        Xs = [torch.from_numpy(Xh.view(np.int16)).to(dev) for _ in range(n_sets)]
        Ys = [torch.zeros((M, ldn), dtype=torch.int16, device=dev) for _ in range(n_sets)]
        Wt = Wd.view(tdt).reshape(M, K)
        Yd = [torch.empty((M, N), dtype=tdt, device=dev) for _ in range(n_sets)]
        Xt = [x.view(tdt).reshape(K, ldn)[:, :N] for x in Xs]
        dense_us[name] = graph_time_us(lambda i: torch.matmul(Wt, Xt[i % n_sets], out=Yd[i % n_sets]), n_sets)
        del Yd
        pin = torch.from_numpy(synth.permutation(K, synth.seed_for(5, 2) + 1000 * li)).to(dev)
        pout = torch.from_numpy(synth.permutation(M, synth.seed_for(5, 3) + 1000 * li)).to(dev)
        for V in v_list:
            if M % V:
                continue
            for keep, label in keep_list:
                Kv = K // keep
                vb, nb, cb, wb = hinm.hinm_pack_sizes(M, K, V, Kv, dtype)
                vals = torch.empty(vb // 2, dtype=torch.int16, device=dev)
                nm = torch.empty(nb, dtype=torch.uint8, device=dev)
                vec = torch.empty(cb // 4, dtype=torch.int32, device=dev)
                ws = torch.empty(wb // 8, dtype=torch.float64, device=dev)
                hinm.hinm_pack(M, K, V, Kv, dtype, Wd, vals, nm, vec, ws, wb)
                pbytes = hinm.hinm_prepare_sizes(M, K, V, Kv, dtype)
                wsb = hinm.hinm_spmm_prepared_workspace(M, K, V, Kv, dtype, N)
                wsp = torch.zeros(max(wsb, 1), dtype=torch.uint8, device=dev)
                us = {}
                for ident in (False, True):
                    preps = []
                    for _ in range(n_sets):
                        pr = torch.empty(pbytes, dtype=torch.uint8, device=dev)
                        hinm.hinm_prepare(M, K, V, Kv, dtype, vals, nm, vec, None if ident else pin,
                                          None if ident else pout, pr, pbytes)
                        preps.append(pr)
                    torch.cuda.synchronize()
                    us[ident] = graph_time_us(
                        lambda i: hinm.hinm_spmm_prepared(M, K, V, Kv, dtype, N, preps[i % n_sets], Xs[i % n_sets], ldn,
                                                          Ys[i % n_sets], ldn, 0, wsp if wsb else None, wsb), n_sets)
                    del preps
                table.append({"layer": name, "M": M, "K": K, "N": N, "V": V, "vector_sparsity": label, "Kv": Kv,
                              "us": round(us[False], 2), "us_identity": round(us[True], 2),
                              "us_dense_gemm": round(dense_us[name], 2)})
                flops_total += 2.0 * M * K * N
                time_total += us[False] * 1e-6
    # one row per (V, vector sparsity): all layers of the model block summed
    summary = []
    for V in v_list:
        for _, label in keep_list:
            rows = [r for r in table if r["V"] == V and r["vector_sparsity"] == label]
            if not rows:
                continue
            t, ti, td = (sum(r[k] for r in rows) for k in ("us", "us_identity", "us_dense_gemm"))
            summary.append({"V": V, "vector_sparsity": label, "layers": len(rows), "us": round(t, 1),
                            "us_identity": round(ti, 1), "permutation_overhead": round(t / ti - 1.0, 4),
                            "us_dense_gemm": round(td, 1), "speedup_vs_dense": round(td / t, 3)})
    out = {"metric": "hinm_spmm_dense_equiv_tflops", "value": round(flops_total / time_total / 1e12, 3),
           "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": 3, "ms_per_step": round(time_total * 1e3, 6),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
           "config": {"workload": ("BERT-base encoder layer, 8 x 512 tokens" if bert else
                                   "ResNet 3x3 convolutions as GEMMs, 8 images") + ": every layer x V x vector sparsity",
                      "entry_point": "hinm_spmm_prepared", "launch": "one HIP graph of K steps per case"},
           "summary": summary, "table": table, "roofline": None, "cpu_baseline": None}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
