"""fp64 CPU oracle for T = (I + A)^{-1} on delta-rule chunk matrices.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The HIP library never imports or links anything from this package, and
this package imports nothing from the HIP package.

`tri_inv`, `build_A`, `gdn_chunk_tri_inv` call the plain-C implementation
(oracle/triinv_oracle.c: exact widening to fp64, difference-form gate, row-oriented forward
substitution; paper Sec. 1 Eq. 3, Table 1).  `oracle.methods` holds fp64 / rounding-emulated
numpy statements of the paper's Algorithms 2-6 and `oracle.metrics` the paper's three
forward-error measures plus the residual.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence

import numpy as np

from . import build as _build

F32, F16, BF16 = 0, 1, 2
GATE_SCALAR, GATE_PER_CHANNEL, GATE_NONE = 0, 1, 2

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(_build.build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        L.oracle_hw_threads.restype = i32
        L.oracle_tri_inv_f64.argtypes = [vp, vp, i64, i32, i32]
        L.oracle_tri_inv.argtypes = [vp, i32, vp, i64, i32, i32]
        L.oracle_build_A.argtypes = [vp, i32, vp, vp, i32, vp, i32, i64, i32, i32, i32, vp, i64, i32]
        L.oracle_gdn_chunk_tri_inv.argtypes = [vp, i32, vp, vp, i32, vp, i32, i64, i32, i32, i32, vp, i64, i32]
        _lib = L
    return _lib


def hw_threads() -> int:
    return int(lib().oracle_hw_threads())


def _raw(x):
    """(pointer, dtype code, keep-alive) for a torch tensor or numpy array of stored values."""
    import torch

    if isinstance(x, torch.Tensor):
        x = x.detach().cpu().contiguous()
        if x.dtype == torch.float32:
            return x.data_ptr(), F32, x
        if x.dtype == torch.float16:
            return x.data_ptr(), F16, x
        if x.dtype == torch.bfloat16:
            return x.data_ptr(), BF16, x
        raise TypeError(f"unsupported stored dtype {x.dtype}")
    x = np.ascontiguousarray(x)
    if x.dtype == np.float32:
        return x.ctypes.data, F32, x
    if x.dtype == np.float16:
        return x.ctypes.data, F16, x
    raise TypeError(f"unsupported stored dtype {x.dtype}")


def _f32ptr(x):
    import torch

    if x is None:
        return None, None
    if isinstance(x, torch.Tensor):
        x = x.detach().cpu().contiguous().to(torch.float32)
        return x.data_ptr(), x
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x.ctypes.data, x


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def tri_inv(A, n_threads: int = 0) -> np.ndarray:
    """T = (I + strict_lower(A))^{-1} in fp64.  A: [n_mat, C, C] stored fp32/fp16/bf16 (torch or
    numpy) or a numpy float64 array; entries on or above the diagonal are ignored."""
    if isinstance(A, np.ndarray) and A.dtype == np.float64:
        A = np.ascontiguousarray(A)
        n_mat, C, C2 = A.shape
        assert C == C2
        T = np.empty_like(A)
        _check(lib().oracle_tri_inv_f64(A.ctypes.data, T.ctypes.data, n_mat, C, n_threads), "tri_inv_f64")
        return T
    ptr, code, keep = _raw(A)
    n_mat, C, C2 = keep.shape
    assert C == C2
    T = np.empty((n_mat, C, C), dtype=np.float64)
    _check(lib().oracle_tri_inv(ptr, code, T.ctypes.data, n_mat, C, n_threads), "tri_inv")
    return T


def _sel(sel: Optional[Sequence[int]]):
    if sel is None:
        return None, 0, None
    arr = np.ascontiguousarray(np.asarray(sel, dtype=np.int64))
    return arr.ctypes.data, arr.size, arr


def build_A(K, beta, g, gate_kind: int, C: int, sel: Optional[Sequence[int]] = None, n_threads: int = 0) -> np.ndarray:
    """fp64 chunk matrices A [n_mat or len(sel), C, C] from stored K [B,Tlen,H,d_k], beta, g."""
    kp, kcode, kkeep = _raw(K)
    B, Tlen, H, d_k = kkeep.shape
    bp, bkeep = _f32ptr(beta)
    gp, gkeep = _f32ptr(g)
    sp, ns, skeep = _sel(sel)
    n_out = ns if sel is not None else B * (Tlen // C) * H
    A = np.empty((n_out, C, C), dtype=np.float64)
    _check(lib().oracle_build_A(kp, kcode, bp, gp, gate_kind, A.ctypes.data, B, Tlen, H, d_k, C, sp, ns, n_threads),
           "build_A")
    return A


def gdn_chunk_tri_inv(K, beta, g, gate_kind: int, C: int, sel: Optional[Sequence[int]] = None,
                      n_threads: int = 0) -> np.ndarray:
    """Fused flavour: build A from the stored inputs in fp64, then invert."""
    kp, kcode, kkeep = _raw(K)
    B, Tlen, H, d_k = kkeep.shape
    bp, bkeep = _f32ptr(beta)
    gp, gkeep = _f32ptr(g)
    sp, ns, skeep = _sel(sel)
    n_out = ns if sel is not None else B * (Tlen // C) * H
    T = np.empty((n_out, C, C), dtype=np.float64)
    _check(lib().oracle_gdn_chunk_tri_inv(kp, kcode, bp, gp, gate_kind, T.ctypes.data, B, Tlen, H, d_k, C,
                                          sp, ns, n_threads), "gdn_chunk_tri_inv")
    return T


def _pad_to_chunks(K, beta, g, C: int):
    """[B, Tlen, ...] stored tensors padded along the token axis to a multiple of C with tokens whose key
    and beta are zero (g = 0 there): the padded rows and columns of A vanish (paper Sec. 1: chunks of at
    most C tokens; a short last chunk is the leading block of a C x C matrix that is the identity elsewhere)."""
    import torch

    K = torch.as_tensor(K)
    Tlen = K.shape[1]
    pad = (-Tlen) % C
    if pad == 0:
        return K, beta, g

    def grow(x):
        if x is None:
            return None
        x = torch.as_tensor(x)
        z = torch.zeros((x.shape[0], pad) + tuple(x.shape[2:]), dtype=x.dtype)
        return torch.cat([x.cpu(), z], dim=1)

    return grow(K), grow(beta), grow(g)


def gdn_chunk_tri_inv_ragged(K, beta, g, gate_kind: int, C: int, n_threads: int = 0) -> np.ndarray:
    """Fused flavour for any Tlen: ceil(Tlen / C) chunks per sequence, the last one zero-padded."""
    Kp, bp, gp = _pad_to_chunks(K, beta, g, C)
    return gdn_chunk_tri_inv(Kp, bp, gp, gate_kind, C, n_threads=n_threads)


def build_A_ragged(K, beta, g, gate_kind: int, C: int, n_threads: int = 0) -> np.ndarray:
    Kp, bp, gp = _pad_to_chunks(K, beta, g, C)
    return build_A(Kp, bp, gp, gate_kind, C, n_threads=n_threads)


def gdn_chunk_tri_inv_varlen(K, beta, g, seqlens, gate_kind: int, C: int, n_threads: int = 0) -> np.ndarray:
    """Packed variable-length sequences (K [total, H, d_k], beta [total, H], g [total, H(, d_k)]): every
    sequence is chunked on its own; results concatenated in sequence order, chunk-major, head-minor."""
    import torch

    K = torch.as_tensor(K)
    out, t0 = [], 0
    for n in seqlens:
        n = int(n)
        if n > 0:
            sl = slice(t0, t0 + n)
            out.append(gdn_chunk_tri_inv_ragged(K[sl][None], torch.as_tensor(beta)[sl][None],
                                                None if g is None else torch.as_tensor(g)[sl][None], gate_kind, C,
                                                n_threads=n_threads))
        t0 += n
    H = K.shape[1]
    return np.concatenate(out, axis=0) if out else np.empty((0, C, C), dtype=np.float64)


def gdn_chunk_tri_solve(K, beta, g, X, row_scale, gate_kind: int, C: int, n_threads: int = 0) -> np.ndarray:
    """W = (I + A)^{-1} diag(s) X chunk by chunk, in fp64 (the chunk-local solve in which the layer uses the
    inverse, paper Sec. 1 Eq. 3 and Sec. 5.2): X [B, Tlen, H, d_x] stored values widened exactly, s = row_scale
    [B, Tlen, H] or None (all ones).  Row-oriented forward substitution on the right-hand sides themselves,
        W_i = s_i X_i - sum_{j < i} A_ij W_j     within each chunk,
    so the inverse is never formed.  Any Tlen: a short last chunk is the leading block (see _pad_to_chunks).
    Returns W [B, Tlen, H, d_x]."""
    import torch

    A = build_A_ragged(K, beta, g, gate_kind, C, n_threads=n_threads)          # [B * n_chunk * H, C, C]
    Xf = torch.as_tensor(X).cpu().to(torch.float64).numpy()
    B, Tlen, H, d_x = Xf.shape
    if row_scale is not None:
        Xf = Xf * torch.as_tensor(row_scale).cpu().to(torch.float64).numpy()[..., None]
    n_chunk = -(-Tlen // C)
    A = A.reshape(B, n_chunk, H, C, C)
    # all chunks side by side: rows beyond Tlen are padding (zero right-hand side, identity rows of I + A), cut off below
    R = np.zeros((B, n_chunk * C, H, d_x), dtype=np.float64)
    R[:, :Tlen] = Xf
    R = R.reshape(B, n_chunk, C, H, d_x)
    W = np.zeros_like(R)
    for i in range(C):
        acc = R[:, :, i].copy()                                                 # [B, n_chunk, H, d_x]
        for j in range(i):
            acc -= A[:, :, :, i, j][..., None] * W[:, :, j]
        W[:, :, i] = acc
    return W.reshape(B, n_chunk * C, H, d_x)[:, :Tlen].copy()


def gdn_chunk_tri_solve_varlen(K, beta, g, X, row_scale, seqlens, gate_kind: int, C: int, n_threads: int = 0) -> np.ndarray:
    """gdn_chunk_tri_solve on packed sequences (K [total, H, d_k], X [total, H, d_x], ...): every sequence is chunked on
    its own.  Returns W [total, H, d_x]."""
    import torch

    X = torch.as_tensor(X)
    W = np.zeros(tuple(X.shape), dtype=np.float64)
    t0 = 0
    for n in seqlens:
        n = int(n)
        if n > 0:
            sl = slice(t0, t0 + n)
            W[sl] = gdn_chunk_tri_solve(torch.as_tensor(K)[sl][None], torch.as_tensor(beta)[sl][None],
                                        None if g is None else torch.as_tensor(g)[sl][None], X[sl][None],
                                        None if row_scale is None else torch.as_tensor(row_scale)[sl][None], gate_kind, C,
                                        n_threads=n_threads)[0]
        t0 += n
    return W
