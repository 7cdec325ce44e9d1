"""ctypes binding of libtriinv.so -- argument marshalling only.

Every step of the path (Gram products, gating, masking, inversion, store) runs in the HIP
kernels behind the C-ABI declared in include/triinv.h; PyTorch is used here for device memory
and for the current stream, nothing else.  There is no CPU fallback: if the shared library is
missing or cannot be loaded, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # imported before the library is opened so that its HIP runtime is the one in use

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtriinv.so")

# enums of include/triinv.h
F32, F16, BF16 = 0, 1, 2
FWD_SUBST, BLOCK_RECURSIVE, NEUMANN, MIXED, BLOCK_DIRECT, NEWTON_SCHULZ, MIXED_B32 = 0, 1, 2, 3, 4, 5, 6
FLAG_REFINE1 = 0x1
FLAG_OUT_F16 = 0x2
FLAG_OUT_BF16 = 0x4
FLAG_FWD_SHUFFLE = 0x8


def flag_mxr_r(r: int) -> int:
    """flags bits carrying the number of refinement steps inside the mixed recursion (default 1)."""
    return ((int(r) + 1) & 7) << 16


def flag_iters(n: int) -> int:
    """flags bits carrying the Newton-Schulz iteration count."""
    return (int(n) & 0xFF) << 8

GATE_SCALAR, GATE_PER_CHANNEL, GATE_NONE = 0, 1, 2
OK = 0

METHOD_NAMES = {FWD_SUBST: "fwd_subst", BLOCK_RECURSIVE: "block_recursive", NEUMANN: "neumann", MIXED: "mixed",
                BLOCK_DIRECT: "block_direct", NEWTON_SCHULZ: "newton_schulz", MIXED_B32: "mixed_b32"}
DTYPE_NAMES = {F32: "f32", F16: "f16", BF16: "bf16"}

EXPORTS = ("tri_inv", "tri_inv_ex", "gdn_chunk_tri_inv", "gdn_chunk_tri_inv_ex", "gdn_chunk_tri_inv_varlen", "gdn_chunk_build_A",
           "gdn_chunk_tri_solve", "gdn_chunk_tri_solve_multi", "gdn_chunk_tri_solve_varlen", "triinv_status_string", "triinv_version")

_lib: Optional[ctypes.CDLL] = None


class TriInvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library (raw ctypes handle).  Built by `paper_2605_21325_amd.build`."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2605_21325_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u32 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint32
        L.tri_inv.argtypes = [vp, vp, i64, i32, i32, i32]
        L.tri_inv.restype = i32
        L.tri_inv_ex.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, u32]
        L.tri_inv_ex.restype = i32
        L.gdn_chunk_tri_inv.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32]
        L.gdn_chunk_tri_inv.restype = i32
        L.gdn_chunk_tri_inv_ex.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, i32, i32, vp, u32]
        L.gdn_chunk_tri_inv_ex.restype = i32
        L.gdn_chunk_tri_inv_varlen.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i64, i32, i32, i32, i32, i32, i32, i32, vp, u32]
        L.gdn_chunk_tri_inv_varlen.restype = i32
        L.gdn_chunk_build_A.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, i32, vp, u32]
        L.gdn_chunk_build_A.restype = i32
        L.gdn_chunk_tri_solve.argtypes = [vp, vp, vp, vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, i32, i32, i32, vp, u32]
        L.gdn_chunk_tri_solve.restype = i32
        L.gdn_chunk_tri_solve_multi.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, i32, i32, vp, u32]
        L.gdn_chunk_tri_solve_multi.restype = i32
        L.gdn_chunk_tri_solve_varlen.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i64, i64, i32, i32, i32, i32, i32, i32, i32, i32, vp, u32]
        L.gdn_chunk_tri_solve_varlen.restype = i32
        L.triinv_status_string.argtypes = [i32]
        L.triinv_status_string.restype = ctypes.c_char_p
        L.triinv_version.argtypes = []
        L.triinv_version.restype = i32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().triinv_status_string(int(status)).decode()


def version() -> int:
    return int(lib().triinv_version())


def dtype_code(dt: torch.dtype) -> int:
    try:
        return {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}[dt]
    except KeyError:
        raise TypeError(f"unsupported element type {dt}") from None


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) or None


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def tri_inv(A: torch.Tensor, T: Optional[torch.Tensor] = None, method: int = BLOCK_RECURSIVE) -> torch.Tensor:
    """T = (I + strict_lower(A))^{-1};  A [n_mat, C, C] fp32/fp16/bf16 on the GPU.  Short form of
    the C-ABI: operands in A's own type, default stream."""
    n_mat, C, _ = A.shape
    if T is None:
        T = torch.empty((n_mat, C, C), dtype=torch.float32, device=A.device)
    st = lib().tri_inv(_dev(A, "A"), _dev(T, "T"), n_mat, C, dtype_code(A.dtype), method)
    if st != OK:
        raise TriInvError(st, "tri_inv")
    return T


_OUT_FLAG = {torch.float32: 0, torch.float16: FLAG_OUT_F16, torch.bfloat16: FLAG_OUT_BF16}


def _out(T: Optional[torch.Tensor], out_dtype: Optional[torch.dtype], shape, device, flags: int):
    """The output tensor (allocated if not given) and flags with the TRIINV_FLAG_OUT_* bit of its element type."""
    if T is None:
        T = torch.empty(shape, dtype=out_dtype or torch.float32, device=device)
    elif out_dtype is not None and T.dtype != out_dtype:
        raise TypeError(f"T is {T.dtype}, out_dtype asks for {out_dtype}")
    if T.dtype not in _OUT_FLAG:
        raise TypeError(f"unsupported output dtype {T.dtype}")
    return T, (flags & ~(FLAG_OUT_F16 | FLAG_OUT_BF16)) | _OUT_FLAG[T.dtype]


def tri_inv_ex(A: torch.Tensor, T: Optional[torch.Tensor] = None, method: int = BLOCK_RECURSIVE,
               op_dtype: Optional[int] = None, stream=None, flags: int = 0,
               out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    n_mat, C, _ = A.shape
    T, flags = _out(T, out_dtype, (n_mat, C, C), A.device, flags)
    in_dt = dtype_code(A.dtype)
    st = lib().tri_inv_ex(_dev(A, "A"), _dev(T, "T"), n_mat, C, in_dt, method,
                          in_dt if op_dtype is None else op_dtype, _stream_ptr(stream), flags)
    if st != OK:
        raise TriInvError(st, "tri_inv_ex")
    return T


def _n_mat(K: torch.Tensor, C: int) -> int:
    B, Tlen, H, _ = K.shape
    return B * ((Tlen + C - 1) // C) * H


def gdn_chunk_tri_inv(K: torch.Tensor, beta: torch.Tensor, g: torch.Tensor, C: int,
                      T: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Fused build + invert, short form: bf16 keys [B, Tlen, H, d_k], scalar gate, blocked
    recursion with bf16 operands, default stream."""
    B, Tlen, H, d_k = K.shape
    if K.dtype != torch.bfloat16:
        raise TypeError("the short form takes bf16 keys; use gdn_chunk_tri_inv_ex")
    if T is None:
        T = torch.empty((_n_mat(K, C), C, C), dtype=torch.float32, device=K.device)
    st = lib().gdn_chunk_tri_inv(_dev(K, "K"), _dev(beta, "beta"), _dev(g, "g"), _dev(T, "T"), B, Tlen, H, d_k, C)
    if st != OK:
        raise TriInvError(st, "gdn_chunk_tri_inv")
    return T


def gdn_chunk_tri_inv_ex(K: torch.Tensor, beta: torch.Tensor, g: Optional[torch.Tensor], C: int,
                         T: Optional[torch.Tensor] = None, gate_kind: int = GATE_SCALAR,
                         method: int = BLOCK_RECURSIVE, op_dtype: int = BF16, stream=None, flags: int = 0,
                         out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    B, Tlen, H, d_k = K.shape
    T, flags = _out(T, out_dtype, (_n_mat(K, C), C, C), K.device, flags)
    gp = None if g is None else _dev(g, "g")
    st = lib().gdn_chunk_tri_inv_ex(_dev(K, "K"), _dev(beta, "beta"), gp, _dev(T, "T"), B, Tlen, H, d_k, C,
                                    dtype_code(K.dtype), gate_kind, method, op_dtype, _stream_ptr(stream), flags)
    if st != OK:
        raise TriInvError(st, "gdn_chunk_tri_inv_ex")
    return T


def varlen_chunk_offsets(seqlens, C: int):
    """Host lists (cu_seqlens, cu_chunks) for sequences of the given lengths: argument preparation
    for gdn_chunk_tri_inv_varlen (sequence s owns ceil(len_s / C) consecutive chunk ids)."""
    cu_s, cu_c = [0], [0]
    for n in seqlens:
        n = int(n)
        cu_s.append(cu_s[-1] + n)
        cu_c.append(cu_c[-1] + (n + C - 1) // C)
    return cu_s, cu_c


def gdn_chunk_tri_inv_varlen(K: torch.Tensor, beta: torch.Tensor, g: Optional[torch.Tensor], seqlens, C: int,
                             T: Optional[torch.Tensor] = None, gate_kind: int = GATE_SCALAR,
                             method: int = BLOCK_RECURSIVE, op_dtype: int = BF16, stream=None, flags: int = 0,
                             out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """Fused build + invert on packed variable-length sequences: K [total_tokens, H, d_k], beta
    [total_tokens, H], g [total_tokens, H] (or [total_tokens, H, d_k]); seqlens = host sequence of lengths."""
    total, H, d_k = K.shape
    cu_s, cu_c = varlen_chunk_offsets(seqlens, C)
    if cu_s[-1] != total:
        raise ValueError(f"sequence lengths sum to {cu_s[-1]}, K holds {total} tokens")
    cu_seqlens = torch.tensor(cu_s, dtype=torch.int64, device=K.device)
    cu_chunks = torch.tensor(cu_c, dtype=torch.int64, device=K.device)
    T, flags = _out(T, out_dtype, (cu_c[-1] * H, C, C), K.device, flags)
    gp = None if g is None else _dev(g, "g")
    st = lib().gdn_chunk_tri_inv_varlen(_dev(K, "K"), _dev(beta, "beta"), gp, _dev(T, "T") if T.numel() else None,
                                        cu_seqlens.data_ptr(), cu_chunks.data_ptr(), len(cu_s) - 1, total, cu_c[-1], H, d_k, C,
                                        dtype_code(K.dtype), gate_kind, method, op_dtype, _stream_ptr(stream), flags)
    if st != OK:
        raise TriInvError(st, "gdn_chunk_tri_inv_varlen")
    T._triinv_keepalive = (cu_seqlens, cu_chunks)  # the launch is asynchronous: the offsets live as long as the result
    return T


def gdn_chunk_build_A(K: torch.Tensor, beta: torch.Tensor, g: Optional[torch.Tensor], C: int,
                      A: Optional[torch.Tensor] = None, gate_kind: int = GATE_SCALAR, op_dtype: int = BF16, stream=None,
                      out_dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """The chunk matrices A alone ([n_mat, C, C], strictly lower triangular), from K [B, Tlen, H, d_k], beta, g."""
    B, Tlen, H, d_k = K.shape
    A, flags = _out(A, out_dtype, (_n_mat(K, C), C, C), K.device, 0)
    gp = None if g is None else _dev(g, "g")
    st = lib().gdn_chunk_build_A(_dev(K, "K"), _dev(beta, "beta"), gp, _dev(A, "A") if A.numel() else None, B, Tlen, H, d_k, C,
                                 dtype_code(K.dtype), gate_kind, op_dtype, _stream_ptr(stream), flags)
    if st != OK:
        raise TriInvError(st, "gdn_chunk_build_A")
    return A


def gdn_chunk_tri_solve(K: torch.Tensor, beta: torch.Tensor, g: Optional[torch.Tensor], X: torch.Tensor, C: int,
                        row_scale: Optional[torch.Tensor] = None, W: Optional[torch.Tensor] = None,
                        gate_kind: int = GATE_SCALAR, method: int = BLOCK_RECURSIVE, stream=None, flags: int = 0) -> torch.Tensor:
    """W = (I + A)^{-1} diag(row_scale) X chunk by chunk: K [B, Tlen, H, d_k], X and W [B, Tlen, H, d_x]; the element type
    of X is the operand type of every product."""
    B, Tlen, H, d_k = K.shape
    d_x = X.shape[-1]
    if tuple(X.shape[:3]) != (B, Tlen, H):
        raise ValueError("X must be [B, Tlen, H, d_x]")
    if W is None:
        W = torch.empty_like(X)
    elif W.shape != X.shape or W.dtype != X.dtype:
        raise ValueError("W must have the shape and element type of X")
    gp = None if g is None else _dev(g, "g")
    sp = None if row_scale is None else _dev(row_scale, "row_scale")
    st = lib().gdn_chunk_tri_solve(_dev(K, "K"), _dev(beta, "beta"), gp, _dev(X, "X") if X.numel() else None, sp,
                                   _dev(W, "W") if W.numel() else None, B, Tlen, H, d_k, d_x, C, dtype_code(K.dtype), gate_kind,
                                   method, dtype_code(X.dtype), _stream_ptr(stream), flags)
    if st != OK:
        raise TriInvError(st, "gdn_chunk_tri_solve")
    return W


def gdn_chunk_tri_solve_varlen(K: torch.Tensor, beta: torch.Tensor, g: Optional[torch.Tensor], X: torch.Tensor, seqlens, C: int,
                               row_scale: Optional[torch.Tensor] = None, W: Optional[torch.Tensor] = None,
                               gate_kind: int = GATE_SCALAR, method: int = BLOCK_RECURSIVE, stream=None, flags: int = 0) -> torch.Tensor:
    """gdn_chunk_tri_solve on packed sequences: K [total, H, d_k], X and W [total, H, d_x]; seqlens = host sequence of lengths."""
    total, H, d_k = K.shape
    d_x = X.shape[-1]
    if tuple(X.shape[:2]) != (total, H):
        raise ValueError("X must be [total_tokens, H, d_x]")
    cu_s, cu_c = varlen_chunk_offsets(seqlens, C)
    if cu_s[-1] != total:
        raise ValueError(f"sequence lengths sum to {cu_s[-1]}, K holds {total} tokens")
    cu_seqlens = torch.tensor(cu_s, dtype=torch.int64, device=K.device)
    cu_chunks = torch.tensor(cu_c, dtype=torch.int64, device=K.device)
    if W is None:
        W = torch.empty_like(X)
    elif W.shape != X.shape or W.dtype != X.dtype:
        raise ValueError("W must have the shape and element type of X")
    gp = None if g is None else _dev(g, "g")
    sp = None if row_scale is None else _dev(row_scale, "row_scale")
    st = lib().gdn_chunk_tri_solve_varlen(_dev(K, "K"), _dev(beta, "beta"), gp, _dev(X, "X") if X.numel() else None, sp,
                                          _dev(W, "W") if W.numel() else None, cu_seqlens.data_ptr(), cu_chunks.data_ptr(),
                                          len(cu_s) - 1, total, cu_c[-1], H, d_k, d_x, C, dtype_code(K.dtype), gate_kind, method,
                                          dtype_code(X.dtype), _stream_ptr(stream), flags)
    if st != OK:
        raise TriInvError(st, "gdn_chunk_tri_solve_varlen")
    W._triinv_keepalive = (cu_seqlens, cu_chunks)  # the launch is asynchronous: the offsets live as long as the result
    return W


def gdn_chunk_tri_solve_multi(K: torch.Tensor, beta: torch.Tensor, g: Optional[torch.Tensor], Xs, C: int, row_scales=None, Ws=None,
                              gate_kind: int = GATE_SCALAR, method: int = BLOCK_RECURSIVE, stream=None, flags: int = 0):
    """W_k = (I + A)^{-1} diag(row_scales[k]) Xs[k] for one or two right-hand sides sharing one inversion per chunk.
    Xs: sequence of [B, Tlen, H, d_x_k] tensors of one element type; row_scales: sequence of [B, Tlen, H] tensors or None."""
    B, Tlen, H, d_k = K.shape
    n = len(Xs)
    if row_scales is None:
        row_scales = [None] * n
    if Ws is None:
        Ws = [torch.empty_like(x) for x in Xs]
    if len(row_scales) != n or len(Ws) != n:
        raise ValueError("Xs, row_scales and Ws must have the same length")
    for x, w in zip(Xs, Ws):
        if tuple(x.shape[:3]) != (B, Tlen, H) or x.dtype != Xs[0].dtype or w.shape != x.shape or w.dtype != x.dtype:
            raise ValueError("every X must be [B, Tlen, H, d_x] of one element type, every W like its X")
    vp_arr = ctypes.c_void_p * n
    xp = vp_arr(*[_dev(x, "X") if x.numel() else None for x in Xs])
    sp = vp_arr(*[None if s is None else _dev(s, "row_scale") for s in row_scales])
    wp = vp_arr(*[_dev(w, "W") if w.numel() else None for w in Ws])
    dx = (ctypes.c_int32 * n)(*[int(x.shape[-1]) for x in Xs])
    gp = None if g is None else _dev(g, "g")
    st = lib().gdn_chunk_tri_solve_multi(_dev(K, "K"), _dev(beta, "beta"), gp, n, ctypes.cast(xp, ctypes.c_void_p),
                                         ctypes.cast(sp, ctypes.c_void_p), ctypes.cast(wp, ctypes.c_void_p),
                                         ctypes.cast(dx, ctypes.c_void_p), B, Tlen, H, d_k, C, dtype_code(K.dtype), gate_kind, method,
                                         dtype_code(Xs[0].dtype), _stream_ptr(stream), flags)
    if st != OK:
        raise TriInvError(st, "gdn_chunk_tri_solve_multi")
    return Ws
