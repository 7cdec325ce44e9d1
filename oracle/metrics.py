"""Error measures for an approximate inverse (paper Sec. 4.1: max-abs, max-rel over j <= i,
relative Frobenius) and the residual of (I + A) T = I.  Test infrastructure only; fp64 numpy."""
from __future__ import annotations

import numpy as np


def forward_errors(T_ref: np.ndarray, T_hat: np.ndarray) -> dict:
    """Per-matrix errors of T_hat against the fp64 reference T_ref; both [n, C, C]."""
    T_ref = np.asarray(T_ref, dtype=np.float64)
    T_hat = np.asarray(T_hat, dtype=np.float64)
    diff = T_hat - T_ref
    with np.errstate(invalid="ignore", divide="ignore"):
        fro = np.sqrt((diff ** 2).sum(axis=(1, 2))) / np.sqrt((T_ref ** 2).sum(axis=(1, 2)))
        max_abs = np.abs(diff).max(axis=(1, 2))
        C = T_ref.shape[-1]
        low = np.tril(np.ones((C, C), dtype=bool))
        guard = low[None] & (np.abs(T_ref) >= 1e-30)
        rel = np.where(guard, np.abs(diff) / np.where(guard, np.abs(T_ref), 1.0), 0.0)
        max_rel = rel.max(axis=(1, 2))
    return {"rel_fro": fro, "max_abs": max_abs, "max_rel": max_rel}


def residual(A: np.ndarray, T_hat: np.ndarray) -> dict:
    """||(I + A) T_hat - I||_F per matrix, absolute and normalised by ||I + A||_F ||T_hat||_F."""
    A = np.asarray(A, dtype=np.float64)
    T_hat = np.asarray(T_hat, dtype=np.float64)
    C = A.shape[-1]
    M = np.eye(C)[None] + np.tril(A, -1)
    with np.errstate(invalid="ignore", over="ignore"):
        R = M @ T_hat - np.eye(C)[None]
        r = np.sqrt((R ** 2).sum(axis=(1, 2)))
        nrm = np.sqrt((M ** 2).sum(axis=(1, 2))) * np.sqrt((T_hat ** 2).sum(axis=(1, 2)))
    return {"abs": r, "normalised": r / nrm}


def structure_ok(T_hat: np.ndarray) -> bool:
    """Exact zeros above the diagonal and exact ones on it."""
    T_hat = np.asarray(T_hat)
    C = T_hat.shape[-1]
    up = np.triu(np.ones((C, C), dtype=bool), 1)
    return bool((T_hat[:, up] == 0).all() and (T_hat[:, np.arange(C), np.arange(C)] == 1).all())


def summarise(per_matrix: np.ndarray) -> dict:
    x = np.asarray(per_matrix, dtype=np.float64)
    bad = ~np.isfinite(x)
    return {"max": float(np.nanmax(np.where(bad, np.inf, x))) if x.size else 0.0,
            "median": float(np.median(np.where(bad, np.inf, x))) if x.size else 0.0,
            "non_finite": int(bad.sum())}
