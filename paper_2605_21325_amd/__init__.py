"""Batched triangular inversion T = (I + A)^{-1} for delta-rule linear attention on MI355X.

Thin binding over the hand-written HIP library `libtriinv.so` (C-ABI in include/triinv.h).
"""
from .binding import (  # noqa: F401
    BF16, BLOCK_DIRECT, BLOCK_RECURSIVE, F16, F32, FWD_SUBST, GATE_NONE, GATE_PER_CHANNEL, GATE_SCALAR, MIXED, MIXED_B32, NEUMANN, NEWTON_SCHULZ, FLAG_REFINE1, FLAG_OUT_F16, FLAG_OUT_BF16, FLAG_FWD_SHUFFLE, flag_iters, flag_mxr_r,
    DTYPE_NAMES, EXPORTS, METHOD_NAMES, TriInvError,
    gdn_chunk_tri_inv, gdn_chunk_tri_inv_ex, gdn_chunk_tri_inv_varlen, gdn_chunk_build_A, gdn_chunk_tri_solve, gdn_chunk_tri_solve_multi, gdn_chunk_tri_solve_varlen, varlen_chunk_offsets, lib, status_string, tri_inv, tri_inv_ex, version,
)
