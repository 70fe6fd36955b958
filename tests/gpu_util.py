"""Helpers for the GPU parity tests: move bit-pattern arrays to the device, call
the library through its C ABI binding, bring results back.  No arithmetic of
the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2407_20496_amd as hinm

DEV = "cuda:0"


def dev_bits(a: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> int16 device tensor (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV)


def dev_i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


class Packed:
    def __init__(self, M, K, V, Kv, dtype, vals, nm_idx, vec_idx):
        self.M, self.K, self.V, self.Kv, self.dtype = M, K, V, Kv, dtype
        self.vals, self.nm_idx, self.vec_idx = vals, nm_idx, vec_idx

    def host(self):
        return (host_bits(self.vals).reshape(self.M, self.Kv // 2),
                self.nm_idx.cpu().numpy().reshape(self.M, self.Kv // 8),
                self.vec_idx.cpu().numpy().reshape(self.M // self.V, self.Kv))


def dev_f32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def gpu_pack(W_bits: np.ndarray, dtype: str, V: int, Kv: int, W_dev=None, sigma=None, rho=None) -> Packed:
    """hinm_pack; hinm_pack_ordered when sigma (int [T, K], per-tile channel order) is given;
    hinm_pack_scored when rho (float32 [M, K], per-weight saliency) is given (sigma optional)."""
    M, K = W_bits.shape
    vb, nb, cb, wb = hinm.hinm_pack_sizes(M, K, V, Kv, dtype)
    Wd = dev_bits(W_bits) if W_dev is None else W_dev
    vals = torch.empty(vb // 2, dtype=torch.int16, device=DEV)
    nm = torch.empty(nb, dtype=torch.uint8, device=DEV)
    vec = torch.empty(cb // 4, dtype=torch.int32, device=DEV)
    ws = torch.empty(wb // 8, dtype=torch.float64, device=DEV)
    sig = None if sigma is None else dev_i32(sigma)
    if rho is not None:
        hinm.hinm_pack_scored(M, K, V, Kv, dtype, Wd, dev_f32(rho), sig, vals, nm, vec, ws, wb)
    elif sigma is None:
        hinm.hinm_pack(M, K, V, Kv, dtype, Wd, vals, nm, vec, ws, wb)
    else:
        hinm.hinm_pack_ordered(M, K, V, Kv, dtype, Wd, sig, vals, nm, vec, ws, wb)
    torch.cuda.synchronize()
    return Packed(M, K, V, Kv, dtype, vals, nm, vec)


class VectorPacked:
    """A layer with the column-vector mask alone: vals_v [M][Kv], vec_idx [T][Kv]."""

    def __init__(self, M, K, V, Kv, dtype, vals_v, vec_idx):
        self.M, self.K, self.V, self.Kv, self.dtype = M, K, V, Kv, dtype
        self.vals_v, self.vec_idx = vals_v, vec_idx

    def host(self):
        return (host_bits(self.vals_v).reshape(self.M, self.Kv),
                self.vec_idx.cpu().numpy().reshape(self.M // self.V, self.Kv))


def gpu_pack_vectors(W_bits: np.ndarray, dtype: str, V: int, Kv: int, sigma=None, rho=None) -> VectorPacked:
    M, K = W_bits.shape
    _, _, cb, wb = hinm.hinm_pack_sizes(M, K, V, Kv, dtype)
    vals_v = torch.full((M * Kv,), 0x7B7B, dtype=torch.int16, device=DEV)
    vec = torch.empty(cb // 4, dtype=torch.int32, device=DEV)
    ws = torch.empty(wb // 8, dtype=torch.float64, device=DEV)
    hinm.hinm_pack_vectors(M, K, V, Kv, dtype, dev_bits(W_bits), None if rho is None else dev_f32(rho),
                           None if sigma is None else dev_i32(sigma), vals_v, vec, ws, wb)
    torch.cuda.synchronize()
    return VectorPacked(M, K, V, Kv, dtype, vals_v, vec)


def gpu_spmm_vectors(p: VectorPacked, X_bits: np.ndarray, pi_in, pi_out, flags=0, ldx=None, ldy=None):
    """Returns uint16 bits [M, N], or float32 [M, N] with OUT_F32."""
    K, N = X_bits.shape
    ldx = ldx or (N if N == 1 else (N + 7) // 8 * 8)
    ldy = ldy or (N if N == 1 else (N + 7) // 8 * 8)
    Xp = np.zeros((K, ldx), dtype=np.uint16)
    Xp[:, :N] = X_bits
    X_dev = dev_bits(Xp)
    f32 = bool(flags & hinm.OUT_F32)
    Y = (torch.full((p.M, ldy), float("nan"), dtype=torch.float32, device=DEV) if f32
         else torch.full((p.M, ldy), 0x7B7B, dtype=torch.int16, device=DEV))
    hinm.hinm_spmm_vectors(p.M, p.K, p.V, p.Kv, p.dtype, N, p.vals_v, p.vec_idx,
                           None if pi_in is None else dev_i32(pi_in), None if pi_out is None else dev_i32(pi_out),
                           X_dev, ldx, Y, ldy, flags)
    torch.cuda.synchronize()
    if f32:
        out = Y.cpu().numpy()
        assert np.all(np.isnan(out[:, N:])), "columns beyond N were written"
        return out[:, :N].copy()
    out = host_bits(Y)
    assert np.all(out[:, N:] == 0x7B7B), "columns beyond N were written"
    return out[:, :N].copy()


def upload_packed(M, K, V, Kv, dtype, vals, nm_idx, vec_idx) -> Packed:
    return Packed(M, K, V, Kv, dtype, dev_bits(vals), torch.from_numpy(np.ascontiguousarray(nm_idx)).to(DEV),
                  dev_i32(vec_idx))


def gpu_unpack(p: Packed) -> np.ndarray:
    W = torch.full((p.M, p.K), 0x7B7B, dtype=torch.int16, device=DEV)   # poison: must be overwritten
    hinm.hinm_unpack(p.M, p.K, p.V, p.Kv, p.dtype, p.vals, p.nm_idx, p.vec_idx, W)
    torch.cuda.synchronize()
    return host_bits(W)


def gpu_spmm(p: Packed, X_bits: np.ndarray, pi_in, pi_out, flags=0, ldx=None, ldy=None, X_dev=None):
    """Returns uint16 bits [M, N], or float32 [M, N] with OUT_F32."""
    K, N = X_bits.shape
    ldx = ldx or (N if N == 1 else (N + 7) // 8 * 8)
    ldy = ldy or (N if N == 1 else (N + 7) // 8 * 8)
    if X_dev is None:
        Xp = np.zeros((K, ldx), dtype=np.uint16)
        Xp[:, :N] = X_bits
        X_dev = dev_bits(Xp)
    f32 = bool(flags & hinm.OUT_F32)
    if f32:
        Y = torch.full((p.M, ldy), float("nan"), dtype=torch.float32, device=DEV)
    else:
        Y = torch.full((p.M, ldy), 0x7B7B, dtype=torch.int16, device=DEV)
    hinm.hinm_spmm(p.M, p.K, p.V, p.Kv, p.dtype, N, p.vals, p.nm_idx, p.vec_idx,
                   None if pi_in is None else dev_i32(pi_in), None if pi_out is None else dev_i32(pi_out),
                   X_dev, ldx, Y, ldy, flags)
    torch.cuda.synchronize()
    if f32:
        out = Y.cpu().numpy()
        pad = out[:, N:]
        assert np.all(np.isnan(pad)), "columns beyond N were written"
        return out[:, :N].copy()
    out = host_bits(Y)
    assert np.all(out[:, N:] == 0x7B7B), "columns beyond N were written"
    return out[:, :N].copy()


def check_close(got_f64: np.ndarray, want_f64: np.ndarray, rel_fro=1e-3, max_abs=1e-2, what=""):
    """The tolerance the benchmark spec states: relative Frobenius error and max abs error."""
    diff = got_f64 - want_f64
    fro = np.linalg.norm(diff) / max(np.linalg.norm(want_f64), 1e-30)
    mx = np.abs(diff).max() if diff.size else 0.0
    assert fro <= rel_fro and mx <= max_abs, f"{what}: rel-Fro {fro:.3e} (<= {rel_fro}), max-abs {mx:.3e} (<= {max_abs})"
    return fro, mx


class Prepared:
    def __init__(self, p: Packed, buf, nbytes, pi_in, pi_out):
        self.p, self.buf, self.nbytes, self.pi_in, self.pi_out = p, buf, nbytes, pi_in, pi_out


def gpu_prepare(p: Packed, pi_in, pi_out) -> Prepared:
    nbytes = hinm.hinm_prepare_sizes(p.M, p.K, p.V, p.Kv, p.dtype)
    buf = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device=DEV)
    hinm.hinm_prepare(p.M, p.K, p.V, p.Kv, p.dtype, p.vals, p.nm_idx, p.vec_idx,
                      None if pi_in is None else dev_i32(pi_in), None if pi_out is None else dev_i32(pi_out),
                      buf, nbytes)
    torch.cuda.synchronize()
    return Prepared(p, buf, nbytes, pi_in, pi_out)


def gpu_spmm_prepared(pr: Prepared, X_bits: np.ndarray, flags=0, variant=0, ldx=None, ldy=None, X_dev=None):
    p = pr.p
    K, N = X_bits.shape
    ldx = ldx or (1 if N == 1 else (N + 7) // 8 * 8)
    ldy = ldy or (1 if N == 1 else (N + 7) // 8 * 8)
    if X_dev is None:
        Xp = np.zeros((K, ldx), dtype=np.uint16)
        Xp[:, :N] = X_bits
        X_dev = dev_bits(Xp)
    f32 = bool(flags & hinm.OUT_F32)
    Y = (torch.full((p.M, ldy), float("nan"), dtype=torch.float32, device=DEV) if f32
         else torch.full((p.M, ldy), 0x7B7B, dtype=torch.int16, device=DEV))
    wsb = hinm.hinm_spmm_prepared_workspace(p.M, p.K, p.V, p.Kv, p.dtype, N)
    ws = torch.zeros(max(wsb, 1), dtype=torch.uint8, device=DEV)
    hinm.hinm_spmm_prepared(p.M, p.K, p.V, p.Kv, p.dtype, N, pr.buf, X_dev, ldx, Y, ldy, flags | (variant << 16),
                            ws if wsb else None, wsb)
    torch.cuda.synchronize()
    if wsb:
        pr.last_workspace = ws
    if f32:
        out = Y.cpu().numpy()
        assert np.all(np.isnan(out[:, N:])), "columns beyond N were written"
        return out[:, :N].copy()
    out = host_bits(Y)
    assert np.all(out[:, N:] == 0x7B7B), "columns beyond N were written"
    return out[:, :N].copy()
