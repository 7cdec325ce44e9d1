"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only *draws* inputs (keys, beta, log-decay) with the shapes and value
distributions of the five workload configurations.  It holds none of the method's
arithmetic: it neither forms the chunk matrix A nor inverts anything, so the CPU
oracle and the HIP path can both consume its tensors without sharing any code.

All tensors are produced on the host with a ``torch.Generator('cpu')`` seeded with
``SEED_BASE + config_index``; the draw order is fixed (K, beta, gate rate, extras).
"Stored in bf16" means: generate in fp32, L2-normalise in fp32, round to nearest
even to bf16.  Both consumers see the rounded values.

Layouts (token-major, heads interleaved):
  K    [B, Tlen, H, d_k]   fp32 or bf16
  beta [B, Tlen, H]        fp32
  g    [B, Tlen, H]        fp32 (scalar gate)  |  [B, Tlen, H, d_k] fp32 (per-channel gate)  |  None
g is the *chunk-local inclusive cumulative* log-decay (the cumulative sum restarts at
every chunk boundary).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import torch

SEED_BASE = 260521325

# E[softplus(z)], z ~ N(0,1); used to scale the config-2 decay rate to a mean of 0.05.
_MEAN_SOFTPLUS_STD_NORMAL = 0.80603

GATE_SCALAR = 0
GATE_PER_CHANNEL = 1
GATE_NONE = 2


@dataclass(frozen=True)
class Workload:
    index: int
    name: str
    B: int
    Tlen: int
    H: int
    d_k: int
    C: int
    k_dtype: str          # "f32" | "bf16"
    gate_kind: int        # GATE_*
    rate_scale: float     # multiplies softplus(N(0,1)) to give the per-token decay rate
    keys: str             # "gaussian" | "rank4"
    beta: str             # "sigmoid" | "uniform_0.9_1.0"

    @property
    def n_mat(self) -> int:
        return self.B * ((self.Tlen + self.C - 1) // self.C) * self.H


WORKLOADS = (
    Workload(0, "gdn_tiny", 1, 256, 2, 64, 64, "f32", GATE_SCALAR, 0.1, "gaussian", "sigmoid"),
    Workload(1, "gdn_prefill_1x4096", 1, 4096, 16, 128, 64, "bf16", GATE_SCALAR, 0.1, "gaussian", "sigmoid"),
    Workload(2, "gdn_batched_8x8192", 8, 8192, 16, 128, 64, "bf16", GATE_SCALAR,
             0.05 / _MEAN_SOFTPLUS_STD_NORMAL, "gaussian", "sigmoid"),
    Workload(3, "kda_4x16384", 4, 16384, 32, 128, 64, "bf16", GATE_PER_CHANNEL, 0.05, "gaussian", "sigmoid"),
    Workload(4, "stress_c128", 1, 32768, 32, 128, 128, "bf16", GATE_NONE, 0.0, "rank4", "uniform_0.9_1.0"),
)


def workload(index: int, **overrides) -> Workload:
    """Config `index`, optionally shrunk (e.g. B=1, Tlen=512) while keeping its recipe and seed."""
    return replace(WORKLOADS[index], **overrides)


def _l2_normalise(x: torch.Tensor) -> torch.Tensor:
    return x / x.norm(dim=-1, keepdim=True).clamp_min(1e-12)


def make_inputs(w: Workload, seed_offset: int = 0) -> dict:
    """Draw K, beta, g for workload `w`.  Returns a dict of CPU tensors (g may be None)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(SEED_BASE + w.index + 1000003 * seed_offset)
    B, Tlen, H, d_k, C = w.B, w.Tlen, w.H, w.d_k, w.C

    # --- keys -----------------------------------------------------------------------------
    if w.keys == "gaussian":
        K = torch.randn(B, Tlen, H, d_k, generator=gen, dtype=torch.float32)
    elif w.keys == "rank4":
        # k_t = c_t . U + 0.05 * eps_t ; U is one 4 x d_k Gaussian basis per head, shared by
        # every token and batch; c_t ~ N(0,1)^4 per (batch, token, head).
        U = torch.randn(H, 4, d_k, generator=gen, dtype=torch.float32)
        c = torch.randn(B, Tlen, H, 4, generator=gen, dtype=torch.float32)
        eps = torch.randn(B, Tlen, H, d_k, generator=gen, dtype=torch.float32)
        K = torch.einsum("bthr,hrd->bthd", c, U) + 0.05 * eps
    else:
        raise ValueError(w.keys)
    K = _l2_normalise(K)
    if w.k_dtype == "bf16":
        K = K.to(torch.bfloat16)
    elif w.k_dtype != "f32":
        raise ValueError(w.k_dtype)

    # --- beta -----------------------------------------------------------------------------
    if w.beta == "sigmoid":
        beta = torch.sigmoid(torch.randn(B, Tlen, H, generator=gen, dtype=torch.float32))
    elif w.beta == "uniform_0.9_1.0":
        beta = 0.9 + 0.1 * torch.rand(B, Tlen, H, generator=gen, dtype=torch.float32)
    else:
        raise ValueError(w.beta)

    # --- gate -----------------------------------------------------------------------------
    g: Optional[torch.Tensor]
    if w.gate_kind == GATE_NONE:
        g = None
    else:
        shape = (B, Tlen, H) if w.gate_kind == GATE_SCALAR else (B, Tlen, H, d_k)
        rate = -torch.nn.functional.softplus(torch.randn(*shape, generator=gen, dtype=torch.float32))
        rate = rate * w.rate_scale
        # inclusive cumulative sum over the tokens of each chunk, restarted per chunk
        # (a last chunk with fewer than C tokens is padded for the reshape and cut again)
        pad = (-Tlen) % C
        if pad:
            rate = torch.cat([rate, torch.zeros(B, pad, *shape[2:])], dim=1)
        g = rate.reshape(B, (Tlen + pad) // C, C, *shape[2:]).cumsum(dim=2).reshape(B, Tlen + pad, *shape[2:])
        g = g[:, :Tlen].contiguous()

    return {"K": K.contiguous(), "beta": beta.contiguous(), "g": g, "workload": w}


def random_strict_lower(n_mat: int, C: int, scale: float, seed: int, garbage_upper: bool = True) -> torch.Tensor:
    """n_mat dense C x C fp32 matrices: N(0, scale^2) below the diagonal; on and above the
    diagonal either zeros or garbage (large values and NaNs) that a correct consumer ignores."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(SEED_BASE + 7919 * seed + C)
    A = torch.randn(n_mat, C, C, generator=gen, dtype=torch.float32) * scale
    lower = torch.tril(torch.ones(C, C, dtype=torch.bool), diagonal=-1)
    if garbage_upper:
        junk = torch.randn(n_mat, C, C, generator=gen, dtype=torch.float32) * 1e6
        junk[:, 0::7, 0::5] = float("nan")
        A = torch.where(lower, A, junk)
    else:
        A = torch.where(lower, A, torch.zeros(()))
    return A.contiguous()


def make_rhs(w: Workload, d_x: int, dtype: torch.dtype = torch.bfloat16, seed_offset: int = 0) -> dict:
    """Right-hand sides for the chunk-local solve on workload `w`: X [B, Tlen, H, d_x] ~ N(0, 1) (the layer's
    value / key rows), stored in `dtype`, and a positive per-token row scale [B, Tlen, H] in (0, 1) (a beta-like
    factor), from a generator of their own so that make_inputs' draws are unchanged."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(SEED_BASE + 100 + w.index + 1000003 * seed_offset)
    X = torch.randn(w.B, w.Tlen, w.H, d_x, generator=gen, dtype=torch.float32).to(dtype)
    s = torch.sigmoid(torch.randn(w.B, w.Tlen, w.H, generator=gen, dtype=torch.float32))
    return {"X": X.contiguous(), "row_scale": s.contiguous()}
