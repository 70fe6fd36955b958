"""ctypes binding of libhinm.so; names mirror include/hinm.h."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

F16, BF16 = 0, 1
EPI_RELU, OUT_F32 = 1, 2
KERNEL_REFERENCE, KERNEL_SMFMAC, KERNEL_GEMV = 0x100, 0x200, 0x400

_HERE = os.path.dirname(os.path.abspath(__file__))
# HINM_LIBRARY names another build of the same library (the host-sanitized one of build.py --sanitize)
_LIB_PATH = os.environ.get("HINM_LIBRARY") or os.path.join(_HERE, "libhinm.so")
_lib = None


class HinmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({hinm_status_str(status)})")


class _Shape(C.Structure):
    _fields_ = [("M", C.c_int32), ("K", C.c_int32), ("V", C.c_int32), ("Kv", C.c_int32), ("dtype", C.c_int32)]


class _Layer(C.Structure):
    _fields_ = [("shape", _Shape), ("vals", C.c_void_p), ("nm_idx", C.c_void_p), ("vec_idx", C.c_void_p),
                ("pi_in", C.c_void_p), ("pi_out", C.c_void_p), ("flags", C.c_uint32), ("prepared", C.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def exported_symbols() -> Tuple[str, ...]:
    """Entry points include/hinm.h declares."""
    return ("hinm_pack_sizes", "hinm_pack", "hinm_pack_static", "hinm_pack_ordered", "hinm_tile_order", "hinm_apply_row_order", "hinm_pack_scored", "hinm_pack_vectors",
            "hinm_icp_sizes", "hinm_icp_search", "hinm_ocp_sizes", "hinm_ocp_search",
            "hinm_ocp_cluster_sizes", "hinm_ocp_cluster", "hinm_unpack", "hinm_spmm", "hinm_spmm_vectors", "hinm_prepare_sizes", "hinm_prepare",
            "hinm_spmm_prepared_workspace", "hinm_spmm_prepared", "hinm_spmm_prepared_plan", "hinm_chain_sizes",
            "hinm_chain", "hinm_status_str", "hinm_version") + calib_symbols()


def calib_symbols() -> Tuple[str, ...]:
    """Entry points include/hinm_calib.h declares (measurement aids)."""
    return ("hinm_calib_copy", "hinm_calib_fill", "hinm_calib_read", "hinm_calib_scatter_rows", "hinm_calib_smfmac",
            "hinm_calib_empty", "hinm_calib_lds_stream", "hinm_calib_gather_stream", "hinm_calib_tile_part")


def load_library():
    """Load libhinm.so (built in-tree by ``python -m paper_2407_20496_amd.build``).
    Raises if it is missing: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2407_20496_amd.build`; "
                           "this package has no CPU or PyTorch fallback")
    # PyTorch ships its own HIP runtime (same soname as the system one).  It must be in the process
    # before libhinm.so is opened so that both bind to ONE runtime: with two, streams, events and
    # device pointers of one are meaningless to the other.
    import torch  # noqa: F401
    lib = C.CDLL(_LIB_PATH)
    sp = C.POINTER(_Shape)
    szp = C.POINTER(C.c_size_t)
    lib.hinm_pack_sizes.argtypes = [sp, szp, szp, szp, szp]
    lib.hinm_pack.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.hinm_pack_static.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.hinm_tile_order.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.hinm_apply_row_order.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_size_t, C.c_void_p]
    lib.hinm_pack_ordered.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_size_t, C.c_void_p]
    lib.hinm_pack_scored.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    lib.hinm_pack_vectors.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_size_t, C.c_void_p]
    lib.hinm_spmm_vectors.argtypes = [sp, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_int64, C.c_void_p, C.c_int64, C.c_uint32, C.c_void_p]
    lib.hinm_icp_sizes.argtypes = [sp, szp]
    lib.hinm_icp_search.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
    lib.hinm_ocp_sizes.argtypes = [sp, C.c_int32, szp]
    lib.hinm_ocp_search.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                    C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.hinm_ocp_cluster_sizes.argtypes = [sp, C.c_int32, szp]
    lib.hinm_ocp_cluster.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.hinm_unpack.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.hinm_spmm.argtypes = [sp, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                              C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_uint32, C.c_void_p, C.c_size_t,
                              C.c_void_p]
    lib.hinm_chain_sizes.argtypes = [C.c_int32, C.POINTER(_Layer), C.c_int32, szp]
    lib.hinm_chain.argtypes = [C.c_int32, C.POINTER(_Layer), C.c_int32, C.c_void_p, C.c_int64, C.c_void_p,
                               C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.hinm_prepare_sizes.argtypes = [sp, szp]
    lib.hinm_prepare.argtypes = [sp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_size_t, C.c_void_p]
    lib.hinm_spmm_prepared_workspace.argtypes = [sp, C.c_int32, szp]
    lib.hinm_spmm_prepared.argtypes = [sp, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                       C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.hinm_spmm_prepared_plan.argtypes = [sp, C.c_int32, C.c_int64, C.c_int64, C.c_uint32, C.c_char_p, C.c_size_t,
                                            C.POINTER(C.c_int32)]
    lib.hinm_spmm_prepared_plan.restype = C.c_int
    for name in ("hinm_pack_sizes", "hinm_pack", "hinm_pack_static", "hinm_pack_ordered", "hinm_tile_order", "hinm_apply_row_order", "hinm_pack_scored", "hinm_pack_vectors",
                 "hinm_icp_sizes", "hinm_icp_search", "hinm_ocp_sizes", "hinm_ocp_search",
                 "hinm_ocp_cluster_sizes", "hinm_ocp_cluster", "hinm_unpack", "hinm_spmm", "hinm_spmm_vectors", "hinm_chain_sizes", "hinm_chain",
                 "hinm_prepare_sizes", "hinm_prepare", "hinm_spmm_prepared_workspace", "hinm_spmm_prepared"):
        getattr(lib, name).restype = C.c_int
    lib.hinm_calib_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p]
    lib.hinm_calib_fill.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p]
    lib.hinm_calib_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.c_void_p]
    lib.hinm_calib_scatter_rows.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_void_p, C.c_int32,
                                            C.c_void_p]
    lib.hinm_calib_smfmac.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
    lib.hinm_calib_empty.argtypes = [C.c_void_p]
    lib.hinm_calib_lds_stream.argtypes = [C.c_void_p, C.c_size_t, C.c_size_t, C.c_int64, C.c_int32, C.c_void_p]
    lib.hinm_calib_gather_stream.argtypes = [C.c_void_p, C.c_size_t, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_int32, C.c_void_p]
    lib.hinm_calib_tile_part.argtypes = [sp, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
    for name in calib_symbols():
        getattr(lib, name).restype = C.c_int
    lib.hinm_status_str.argtypes = [C.c_int]
    lib.hinm_status_str.restype = C.c_char_p
    lib.hinm_version.argtypes = []
    lib.hinm_version.restype = C.c_int32
    _lib = lib
    return lib


def hinm_status_str(status: int) -> str:
    return load_library().hinm_status_str(int(status)).decode()


def hinm_version() -> int:
    return int(load_library().hinm_version())


def _dtype_code(dtype) -> int:
    if dtype in (F16, "f16"):
        return F16
    if dtype in (BF16, "bf16"):
        return BF16
    try:
        import torch
        if dtype == torch.float16:
            return F16
        if dtype == torch.bfloat16:
            return BF16
    except ImportError:  # pragma: no cover
        pass
    raise ValueError(f"dtype must be f16 or bf16, got {dtype!r}")


def _shape(M, K, V, Kv, dtype) -> _Shape:
    return _Shape(int(M), int(K), int(V), int(Kv), _dtype_code(dtype))


def _ptr(t) -> Optional[int]:
    """Device (or raw integer) pointer of a tensor; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        if torch.cuda.is_available():
            return torch.cuda.current_stream().cuda_stream or None
        return None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(status: int, where: str):
    if status != 0:
        raise HinmError(status, where)


def hinm_pack_sizes(M, K, V, Kv, dtype) -> Tuple[int, int, int, int]:
    """(vals_bytes, nm_bytes, vec_bytes, workspace_bytes)."""
    lib = load_library()
    out = [C.c_size_t(0) for _ in range(4)]
    _check(lib.hinm_pack_sizes(C.byref(_shape(M, K, V, Kv, dtype)), *[C.byref(o) for o in out]), "hinm_pack_sizes")
    return tuple(int(o.value) for o in out)


def hinm_pack(M, K, V, Kv, dtype, W, vals, nm_idx, vec_idx, workspace, workspace_bytes, stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_pack(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(W), _ptr(vals), _ptr(nm_idx), _ptr(vec_idx),
                         _ptr(workspace), int(workspace_bytes), _stream(stream)), "hinm_pack")


PACK_STATIC_MAX_SCORES = 524288


def hinm_pack_static(M, K, V, Kv, dtype, W, vals, nm_idx, vec_idx, stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_pack_static(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(W), _ptr(vals), _ptr(nm_idx), _ptr(vec_idx),
                                _stream(stream)), "hinm_pack_static")


def hinm_apply_row_order(src, dst, row_order, rows, row_bytes, stream=None) -> None:
    _check(load_library().hinm_apply_row_order(_ptr(src), _ptr(dst), _ptr(row_order), int(rows), int(row_bytes),
                                               _stream(stream)), "hinm_apply_row_order")


def hinm_tile_order(M, K, V, Kv, dtype, vec_idx, tile_order, stream=None) -> None:
    _check(load_library().hinm_tile_order(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(vec_idx), _ptr(tile_order),
                                          _stream(stream)), "hinm_tile_order")


def hinm_pack_ordered(M, K, V, Kv, dtype, W, tile_order, vals, nm_idx, vec_idx, workspace, workspace_bytes,
                      stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_pack_ordered(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(W), _ptr(tile_order), _ptr(vals),
                                 _ptr(nm_idx), _ptr(vec_idx), _ptr(workspace), int(workspace_bytes),
                                 _stream(stream)), "hinm_pack_ordered")


def hinm_pack_scored(M, K, V, Kv, dtype, W, rho, tile_order, vals, nm_idx, vec_idx, workspace, workspace_bytes,
                     stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_pack_scored(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(W), _ptr(rho), _ptr(tile_order), _ptr(vals),
                                _ptr(nm_idx), _ptr(vec_idx), _ptr(workspace), int(workspace_bytes),
                                _stream(stream)), "hinm_pack_scored")


def hinm_pack_vectors(M, K, V, Kv, dtype, W, rho, tile_order, vals_v, vec_idx, workspace, workspace_bytes,
                      stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_pack_vectors(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(W), _ptr(rho), _ptr(tile_order),
                                 _ptr(vals_v), _ptr(vec_idx), _ptr(workspace), int(workspace_bytes),
                                 _stream(stream)), "hinm_pack_vectors")


def hinm_spmm_vectors(M, K, V, Kv, dtype, N, vals_v, vec_idx, pi_in, pi_out, X, ldx, Y, ldy, flags=0,
                      stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_spmm_vectors(C.byref(_shape(M, K, V, Kv, dtype)), int(N), _ptr(vals_v), _ptr(vec_idx),
                                 _ptr(pi_in), _ptr(pi_out), _ptr(X), int(ldx), _ptr(Y), int(ldy), int(flags),
                                 _stream(stream)), "hinm_spmm_vectors")


def hinm_icp_sizes(M, K, V, Kv, dtype) -> int:
    """Workspace bytes of hinm_icp_search."""
    lib = load_library()
    out = C.c_size_t(0)
    _check(lib.hinm_icp_sizes(C.byref(_shape(M, K, V, Kv, dtype)), C.byref(out)), "hinm_icp_sizes")
    return int(out.value)


def hinm_icp_search(M, K, V, Kv, dtype, W, rho, vec_idx, samples, iters, objective, workspace, workspace_bytes,
                    stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_icp_search(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(W), _ptr(rho), _ptr(vec_idx), _ptr(samples),
                               int(iters), _ptr(objective), _ptr(workspace), int(workspace_bytes), _stream(stream)),
           "hinm_icp_search")


def hinm_ocp_sizes(M, K, V, Kv, dtype, n_samples) -> int:
    """Workspace bytes of hinm_ocp_search."""
    lib = load_library()
    out = C.c_size_t(0)
    _check(lib.hinm_ocp_sizes(C.byref(_shape(M, K, V, Kv, dtype)), int(n_samples), C.byref(out)), "hinm_ocp_sizes")
    return int(out.value)


def hinm_ocp_search(M, K, V, Kv, dtype, W, rho, row_order, samples, clusters, n_samples, iters, objective, workspace,
                    workspace_bytes, stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_ocp_search(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(W), _ptr(rho), _ptr(row_order), _ptr(samples),
                               _ptr(clusters), int(n_samples), int(iters), _ptr(objective), _ptr(workspace),
                               int(workspace_bytes), _stream(stream)), "hinm_ocp_search")


def hinm_ocp_cluster_sizes(M, K, V, Kv, dtype, n_samples) -> int:
    """Workspace bytes of hinm_ocp_cluster."""
    lib = load_library()
    out = C.c_size_t(0)
    _check(lib.hinm_ocp_cluster_sizes(C.byref(_shape(M, K, V, Kv, dtype)), int(n_samples), C.byref(out)),
           "hinm_ocp_cluster_sizes")
    return int(out.value)


def hinm_ocp_cluster(M, K, V, Kv, dtype, W, rho, row_order, samples, n_samples, rounds, centroids, init_centroids,
                     clusters, objective, workspace, workspace_bytes, stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_ocp_cluster(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(W), _ptr(rho), _ptr(row_order), _ptr(samples),
                                int(n_samples), int(rounds), _ptr(centroids), int(bool(init_centroids)), _ptr(clusters),
                                _ptr(objective), _ptr(workspace), int(workspace_bytes), _stream(stream)),
           "hinm_ocp_cluster")


def hinm_unpack(M, K, V, Kv, dtype, vals, nm_idx, vec_idx, W_out, stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_unpack(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(vals), _ptr(nm_idx), _ptr(vec_idx),
                           _ptr(W_out), _stream(stream)), "hinm_unpack")


def hinm_spmm(M, K, V, Kv, dtype, N, vals, nm_idx, vec_idx, pi_in, pi_out, X, ldx, Y, ldy, flags=0,
              workspace=None, workspace_bytes=0, stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_spmm(C.byref(_shape(M, K, V, Kv, dtype)), int(N), _ptr(vals), _ptr(nm_idx), _ptr(vec_idx),
                         _ptr(pi_in), _ptr(pi_out), _ptr(X), int(ldx), _ptr(Y), int(ldy), int(flags),
                         _ptr(workspace), int(workspace_bytes), _stream(stream)), "hinm_spmm")


def hinm_prepare_sizes(M, K, V, Kv, dtype) -> int:
    lib = load_library()
    out = C.c_size_t(0)
    _check(lib.hinm_prepare_sizes(C.byref(_shape(M, K, V, Kv, dtype)), C.byref(out)), "hinm_prepare_sizes")
    return int(out.value)


def hinm_prepare(M, K, V, Kv, dtype, vals, nm_idx, vec_idx, pi_in, pi_out, prepared, prepared_bytes,
                 stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_prepare(C.byref(_shape(M, K, V, Kv, dtype)), _ptr(vals), _ptr(nm_idx), _ptr(vec_idx),
                            _ptr(pi_in), _ptr(pi_out), _ptr(prepared), int(prepared_bytes), _stream(stream)),
           "hinm_prepare")


def hinm_spmm_prepared_workspace(M, K, V, Kv, dtype, N) -> int:
    lib = load_library()
    out = C.c_size_t(0)
    _check(lib.hinm_spmm_prepared_workspace(C.byref(_shape(M, K, V, Kv, dtype)), int(N), C.byref(out)),
           "hinm_spmm_prepared_workspace")
    return int(out.value)


def hinm_spmm_prepared(M, K, V, Kv, dtype, N, prepared, X, ldx, Y, ldy, flags=0, workspace=None,
                       workspace_bytes=0, stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_spmm_prepared(C.byref(_shape(M, K, V, Kv, dtype)), int(N), _ptr(prepared), _ptr(X), int(ldx),
                                  _ptr(Y), int(ldy), int(flags), _ptr(workspace), int(workspace_bytes),
                                  _stream(stream)), "hinm_spmm_prepared")


def hinm_spmm_prepared_plan(M, K, V, Kv, dtype, N, ldx, ldy, flags=0) -> Tuple[str, int]:
    """(description of the kernel launches hinm_spmm_prepared would make, their number)."""
    lib = load_library()
    buf = C.create_string_buffer(1024)
    n = C.c_int32(0)
    _check(lib.hinm_spmm_prepared_plan(C.byref(_shape(M, K, V, Kv, dtype)), int(N), int(ldx), int(ldy), int(flags),
                                       buf, len(buf), C.byref(n)), "hinm_spmm_prepared_plan")
    return buf.value.decode(), int(n.value)


# ---- measurement aids (include/hinm_calib.h) -------------------------------------------------------

def hinm_calib_copy(src, dst, nbytes, nontemporal=False, stream=None) -> None:
    _check(load_library().hinm_calib_copy(_ptr(src), _ptr(dst), int(nbytes), int(bool(nontemporal)), _stream(stream)),
           "hinm_calib_copy")


def hinm_calib_fill(dst, nbytes, nontemporal=False, stream=None) -> None:
    _check(load_library().hinm_calib_fill(_ptr(dst), int(nbytes), int(bool(nontemporal)), _stream(stream)),
           "hinm_calib_fill")


def hinm_calib_read(src, nbytes, sink, nontemporal=False, stream=None) -> None:
    _check(load_library().hinm_calib_read(_ptr(src), int(nbytes), int(bool(nontemporal)), _ptr(sink), _stream(stream)),
           "hinm_calib_read")


def hinm_calib_scatter_rows(dst, M, N, ld, rows, piece_bytes, stream=None) -> None:
    _check(load_library().hinm_calib_scatter_rows(_ptr(dst), int(M), int(N), int(ld), _ptr(rows), int(piece_bytes),
                                                  _stream(stream)), "hinm_calib_scatter_rows")


def hinm_calib_smfmac(dtype, iterations, sink, stream=None) -> float:
    """Enqueues the loop; returns the launch's flops counted on stored values."""
    flops = C.c_double(0.0)
    _check(load_library().hinm_calib_smfmac(_dtype_code(dtype), int(iterations), _ptr(sink), C.byref(flops),
                                            _stream(stream)), "hinm_calib_smfmac")
    return float(flops.value)


def hinm_calib_empty(stream=None) -> None:
    _check(load_library().hinm_calib_empty(_stream(stream)), "hinm_calib_empty")


def hinm_calib_lds_stream(region, region_bytes, start_stride_bytes, chunks_per_workgroup, workgroups,
                          stream=None) -> None:
    _check(load_library().hinm_calib_lds_stream(_ptr(region), int(region_bytes), int(start_stride_bytes),
                                                int(chunks_per_workgroup), int(workgroups), _stream(stream)),
           "hinm_calib_lds_stream")


def hinm_calib_gather_stream(region, region_bytes, row_pitch_bytes, rows, waves, outstanding, copies_per_wave, workgroups,
                             stream=None) -> None:
    _check(load_library().hinm_calib_gather_stream(_ptr(region), int(region_bytes), int(row_pitch_bytes), int(rows), int(waves),
                                                   int(outstanding), int(copies_per_wave), int(workgroups), _stream(stream)),
           "hinm_calib_gather_stream")


def hinm_calib_tile_part(M, K, V, Kv, dtype, N, prepared, X, ldx, part, stream=None) -> None:
    _check(load_library().hinm_calib_tile_part(C.byref(_shape(M, K, V, Kv, dtype)), int(N), _ptr(prepared), _ptr(X),
                                               int(ldx), int(part), _stream(stream)), "hinm_calib_tile_part")


@dataclass
class Layer:
    M: int
    K: int
    V: int
    Kv: int
    dtype: object
    vals: object
    nm_idx: object
    vec_idx: object
    pi_in: object = None
    pi_out: object = None
    flags: int = 0
    prepared: object = None


def _layers(layers: Sequence[Layer]):
    arr = (_Layer * len(layers))()
    for i, l in enumerate(layers):
        arr[i] = _Layer(_shape(l.M, l.K, l.V, l.Kv, l.dtype), _ptr(l.vals), _ptr(l.nm_idx), _ptr(l.vec_idx),
                        _ptr(l.pi_in), _ptr(l.pi_out), int(l.flags), _ptr(l.prepared))
    return arr


def hinm_chain_sizes(layers: Sequence[Layer], N: int) -> int:
    lib = load_library()
    out = C.c_size_t(0)
    _check(lib.hinm_chain_sizes(len(layers), _layers(layers), int(N), C.byref(out)), "hinm_chain_sizes")
    return int(out.value)


def hinm_chain(layers: Sequence[Layer], N, X, ldx, Y, ldy, scratch, scratch_bytes, stream=None) -> None:
    lib = load_library()
    _check(lib.hinm_chain(len(layers), _layers(layers), int(N), _ptr(X), int(ldx), _ptr(Y), int(ldy),
                          _ptr(scratch), int(scratch_bytes), _stream(stream)), "hinm_chain")
