"""Numpy statements of the paper's matrix-product inversion algorithms.

TEST INFRASTRUCTURE ONLY.  Each function follows the corresponding algorithm of the paper in
its own order and notation, on one C x C strictly-lower matrix `L` (the chunk matrix A), for
the convention  result = (I + L)^{-1}.  They exist (i) to pin the exact intermediate
invariants the HIP kernels rely on and (ii) to predict, by emulating operand rounding, which
method/precision combinations can meet a tolerance on a given workload.

Precision emulation (`op`): every matrix product rounds both operands to the operand type
(round-to-nearest-even), multiplies and sums in fp64, then rounds the product matrix to fp32
-- a model of "low-precision operands, fp32 accumulate" (paper Sec. 4.1).  Sums outside
products are rounded to fp32 as well.  op=None keeps everything in fp64 (exact algebra).
"""
from __future__ import annotations

from typing import Optional

import numpy as np


# ----------------------------------------------------------------------------- rounding
def round_bf16(x: np.ndarray) -> np.ndarray:
    f = np.asarray(x, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    out = rounded.astype(np.uint32).view(np.float32)
    out = np.where(np.isnan(f), np.float32(np.nan), out)
    return out.astype(np.float64)


def round_f16(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)


def round_f32(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


_ROUNDERS = {None: lambda x: x, "f64": lambda x: x, "f32": round_f32, "f16": round_f16, "bf16": round_bf16}


class Arith:
    """Product / sum with the emulated precision."""

    def __init__(self, op: Optional[str]):
        self.op = op
        self.rnd = _ROUNDERS[op]
        self.acc = (lambda x: x) if op in (None, "f64") else round_f32

    def mm(self, X, Y):
        with np.errstate(over="ignore", invalid="ignore"):
            return self.acc(self.rnd(X) @ self.rnd(Y))

    def add(self, X, Y):
        with np.errstate(over="ignore", invalid="ignore"):
            return self.acc(X + Y)


def _strict_lower(L):
    return np.tril(np.asarray(L, dtype=np.float64), -1)


# ----------------------------------------------------------------------------- Alg. 5 (MCH)
def mch(L, op: Optional[str] = None, iters: Optional[int] = None, return_Y: bool = False):
    """Repeated-squaring Neumann product (paper Alg. 5, Sec. 3.2):
    X <- I - L, Y <- L; then log2(n/2) times: Y <- Y Y ; X <- X + X Y.
    After k iterations X = sum_{i < 2^(k+1)} (-L)^i, complete once 2^(k+1) >= n."""
    L = _strict_lower(L)
    n = L.shape[0]
    ar = Arith(op)
    if iters is None:
        iters = max(int(np.ceil(np.log2(n / 2))), 0) if n > 1 else 0
    X = ar.acc(np.eye(n) - L)
    Y = ar.acc(L.copy())
    for _ in range(iters):
        Y = ar.mm(Y, Y)
        X = ar.add(X, ar.mm(X, Y))
    return (X, Y) if return_Y else X


# ----------------------------------------------------------------------------- Alg. 4 (MBH)
def _even_odd_blocks(X, b):
    """D_e, D_o: the 0-indexed even / odd b x b diagonal blocks of X (paper App. C, Lemma C.1)."""
    n = X.shape[0]
    De = np.zeros_like(X)
    Do = np.zeros_like(X)
    for t in range(n // b):
        s = slice(t * b, (t + 1) * b)
        (De if t % 2 == 0 else Do)[s, s] = X[s, s]
    return De, Do


def mbh(L, X0=None, b0: int = 1, op: Optional[str] = None, levels_out: Optional[list] = None):
    """Unrolled blocked 2x2 recursion (paper Alg. 4, Sec. 3.3, Lemma C.1), lower-triangular
    reading:  X <- X0; for b = b0, 2 b0, ..., n/2:  X <- D_e + D_o - D_o L D_e.
    X0 must hold the inverses of the b0 x b0 diagonal blocks of I + L (identity when b0 = 1).
    If `levels_out` is a list, the X after every level is appended (for the block invariant)."""
    L = _strict_lower(L)
    n = L.shape[0]
    ar = Arith(op)
    X = np.eye(n) if X0 is None else np.asarray(X0, dtype=np.float64).copy()
    b = b0
    while b < n:
        De, Do = _even_odd_blocks(X, b)
        X = ar.add(De + Do, -ar.mm(Do, ar.mm(L, De)))
        if levels_out is not None:
            levels_out.append((b, X.copy()))
        b *= 2
    return X


# ----------------------------------------------------------------------------- Alg. 6 (IR)
def ir(Y, L, op: Optional[str] = None):
    """One step of iterative refinement (paper Alg. 6, Eq. 9) for the matrix I + L:
    R <- I - Y (I + L);  X <- Y + R Y."""
    L = _strict_lower(L)
    n = L.shape[0]
    ar = Arith(op)
    R = ar.add(np.eye(n), -ar.mm(Y, np.eye(n) + L))
    return ar.add(Y, ar.mm(R, Y))


# ----------------------------------------------------------------------------- Alg. 2 (MXR)
def mxr(L, b0: int = 16, r: int = 0, op: Optional[str] = None):
    """Mixed recursion (paper Alg. 2, Sec. 3.4): MCH on the b0 x b0 diagonal blocks, r
    refinement steps on that block-diagonal start, then MBH from block size b0."""
    L = _strict_lower(L)
    n = L.shape[0]
    D = np.zeros_like(L)
    for t in range(n // b0):
        s = slice(t * b0, (t + 1) * b0)
        D[s, s] = L[s, s]
    Y = np.zeros_like(L)
    for t in range(n // b0):
        s = slice(t * b0, (t + 1) * b0)
        Y[s, s] = mch(D[s, s], op=op)
    for _ in range(r):
        Y = ir(Y, D, op=op)
    return mbh(L, X0=Y, b0=b0, op=op)


# ----------------------------------------------------------------------------- Alg. 3 (NS)
def ns(L, m: int, X0=None, op: Optional[str] = None):
    """Newton-Schulz (paper Alg. 3, Eq. 8): A <- I + L; X <- X0; m times: Y <- A X; X <- 2X - X Y."""
    L = _strict_lower(L)
    n = L.shape[0]
    ar = Arith(op)
    A = np.eye(n) + L
    X = np.eye(n) / n if X0 is None else np.asarray(X0, dtype=np.float64).copy()
    for _ in range(m):
        Y = ar.mm(A, X)
        X = ar.add(2.0 * X, -ar.mm(X, Y))
    return X


# ----------------------------------------------------------------------------- direct forms
def neumann_sum(L):
    """sum_{i=0}^{n-1} (-L)^i in fp64 -- exact inverse because L is nilpotent (paper Sec. 3.2)."""
    L = _strict_lower(L)
    n = L.shape[0]
    acc = np.eye(n)
    P = np.eye(n)
    for _ in range(1, n):
        P = P @ (-L)
        acc = acc + P
    return acc


def forward_substitution(L, op: Optional[str] = None):
    """Row-wise forward substitution with emulated fp32 arithmetic (the direct baseline)."""
    L = _strict_lower(L)
    n = L.shape[0]
    acc = (lambda x: x) if op in (None, "f64") else round_f32
    Lr = acc(L)
    T = np.eye(n)
    for i in range(1, n):
        row = np.zeros(n)
        for j in range(i):
            row = acc(row - acc(Lr[i, j] * T[j, :]))
        row[i] = 1.0
        T[i, :] = row
    return T


# ----------------------------------------------------------------------------- closed forms of the same methods
# What each iteration above must equal in exact arithmetic, written from the closed form rather than from the
# iteration: the pins hold the algorithm statements above against these.
def neumann_factor_product(L, k_max: Optional[int] = None):
    """prod_{k=0}^{k_max} (I + (-L)^(2^k)), the product form of the truncated Neumann series (paper Sec. 3.2):
    equals sum_{i < 2^(k_max+1)} (-L)^i, i.e. (I + L)^{-1} once 2^(k_max+1) >= n.  Powers by explicit repeated
    multiplication from -L (no squaring of an intermediate that the product also uses)."""
    L = _strict_lower(L)
    n = L.shape[0]
    if k_max is None:
        k_max = max(int(np.ceil(np.log2(n))) - 1, 0)
    out = np.eye(n)
    for k in range(k_max + 1):
        out = out @ (np.eye(n) + np.linalg.matrix_power(-L, 2 ** k))
    return out


def newton_schulz_closed_form(L, m: int, X0=None):
    """The m-th Newton-Schulz iterate from its residual recurrence E_{k+1} = E_k^2 (paper Eq. 8):
    with A = I + L and E_0 = I - A X0,  X_m = A^{-1} (I - E_0^(2^m))."""
    L = _strict_lower(L)
    n = L.shape[0]
    A = np.eye(n) + L
    X0 = np.eye(n) / n if X0 is None else np.asarray(X0, dtype=np.float64)
    E = np.eye(n) - A @ X0
    return np.linalg.solve(A, np.eye(n) - np.linalg.matrix_power(E, 2 ** m))


def block_inverse_2x2(L):
    """(I + L)^{-1} by the 2 x 2 block formula applied recursively (paper Eq. 7 read for a lower-triangular matrix):
    [[A11, 0], [A21, A22]]^{-1} = [[T11, 0], [-T22 A21 T11, T22]]."""
    L = _strict_lower(L)
    n = L.shape[0]
    if n == 1:
        return np.ones((1, 1))
    h = n // 2
    T11 = block_inverse_2x2(L[:h, :h])
    T22 = block_inverse_2x2(L[h:, h:])
    out = np.zeros((n, n))
    out[:h, :h] = T11
    out[h:, h:] = T22
    out[h:, :h] = -T22 @ L[h:, :h] @ T11
    return out
