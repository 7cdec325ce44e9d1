"""The C-ABI boundary without a GPU: the library loads, exports everything include/triinv.h
declares, and every argument error is reported by the host-side checks before any launch."""
import ctypes
import os
import re

import pytest

import paper_2605_21325_amd as tri
from paper_2605_21325_amd import build as tri_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "triinv.h")


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(tri.binding.LIB_PATH):
        tri_build.build()
    return tri.lib()


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return re.findall(r"^\s*(?:const\s+char\s*\*|int)\s+(\w+)\s*\(", src, flags=re.M)


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert set(names) == set(tri.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_header_enums_match_binding():
    src = open(HEADER).read()
    for name, val in [("TRIINV_F32", tri.F32), ("TRIINV_F16", tri.F16), ("TRIINV_BF16", tri.BF16),
                      ("TRIINV_FWD_SUBST", tri.FWD_SUBST), ("TRIINV_BLOCK_RECURSIVE", tri.BLOCK_RECURSIVE),
                      ("TRIINV_NEUMANN", tri.NEUMANN), ("TRIINV_MIXED", tri.MIXED), ("TRIINV_BLOCK_DIRECT", tri.BLOCK_DIRECT), ("TRIINV_NEWTON_SCHULZ", tri.NEWTON_SCHULZ), ("TRIINV_MIXED_B32", tri.MIXED_B32),
                      ("TRIINV_GATE_SCALAR", tri.GATE_SCALAR), ("TRIINV_GATE_PER_CHANNEL", tri.GATE_PER_CHANNEL),
                      ("TRIINV_GATE_NONE", tri.GATE_NONE)]:
        assert re.search(rf"\b{name}\s*=\s*{val}\b", src), name


def test_version_and_status_strings(L):
    assert tri.version() >= 100
    seen = set()
    for code in range(0, -10, -1):
        s = tri.status_string(code)
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 10
    assert tri.status_string(-99) == "unknown status"


# fake, never dereferenced device addresses (all checks below fail before any launch)
P = 0x7F0000000000
Q = 0x7F1000000000


def test_tri_inv_argument_errors(L):
    ex = L.tri_inv_ex
    ok_args = dict(A=P, T=Q, n=4, C=64, dt=0, m=1, op=0)

    def call(**kw):
        a = {**ok_args, **kw}
        return ex(a["A"], a["T"], a["n"], a["C"], a["dt"], a["m"], a["op"], None, 0)

    assert call(n=0) == 0                       # empty batch: success, nothing launched
    assert call(n=0, A=None, T=None) == 0
    assert call(C=48) == -2 and call(C=96) == -2 and call(C=0) == -2 and call(C=256) == -2
    assert call(dt=3) == -3 and call(op=-1) == -3
    assert call(m=7) == -4 and call(m=-1) == -4
    assert call(n=-1) == -5
    assert call(A=None) == -1 and call(T=None) == -1
    assert call(A=P + 4) == -6 and call(T=Q + 8) == -6
    assert call(T=P) == -7                                  # same buffer
    assert call(T=P + 64 * 64 * 4 * 4 - 16) == -7           # tail overlap
    assert L.tri_inv(None, None, 0, 64, 0, 1) == 0
    assert L.tri_inv(P, Q, 1, 64, 7, 1) == -3


def test_adjacent_buffers_do_not_alias(L):
    # checked through a failing later argument so that nothing is launched: flags != 0 is
    # rejected after the alias test
    n = 4
    assert L.tri_inv_ex(P, P + n * 64 * 64 * 4, n, 64, 0, 1, 0, None, 0x80) == -9
    assert L.tri_inv_ex(P, P + n * 64 * 64 * 4 - 16, n, 64, 0, 1, 0, None, 0x80) == -7
    assert L.tri_inv_ex(P, P + n * 64 * 64 * 2, n, 64, 2, 1, 0, None, 0x80) == -9   # bf16 input is half the size


def test_gdn_argument_errors(L):
    ex = L.gdn_chunk_tri_inv_ex
    base = dict(K=P, beta=Q, g=Q + (1 << 30), T=Q + (2 << 30), B=1, Tlen=128, H=2, d_k=128, C=64, kd=2, gate=0, m=1, op=2)

    def call(**kw):
        a = {**base, **kw}
        return ex(a["K"], a["beta"], a["g"], a["T"], a["B"], a["Tlen"], a["H"], a["d_k"], a["C"], a["kd"], a["gate"],
                  a["m"], a["op"], None, 0)

    assert call(Tlen=0) == 0
    assert call(C=100) == -2
    assert call(kd=5) == -3 and call(op=9) == -3
    assert call(m=17) == -4 and call(gate=3) == -4
    assert call(B=0) == -5 and call(H=-1) == -5 and call(d_k=0) == -5
    assert call(Tlen=-64) == -5
    assert call(B=1 << 20, Tlen=1 << 40) == -5      # more than 2^31 - 1 matrices
    assert call(d_k=48) == -5 and call(d_k=512) == -5
    assert call(K=None) == -1 and call(beta=None) == -1 and call(T=None) == -1 and call(g=None) == -1
    assert call(K=P + 2) == -6 and call(g=Q + (1 << 30) + 4) == -6
    assert call(T=P) == -7 and call(T=Q) == -7 and call(T=Q + (1 << 30)) == -7
    assert L.gdn_chunk_tri_inv(P, Q, None, Q + (2 << 30), 1, 128, 2, 128, 64) == -1


def test_varlen_argument_errors(L):
    vl = L.gdn_chunk_tri_inv_varlen
    R = Q + (3 << 30)
    base = dict(K=P, beta=Q, g=Q + (1 << 30), T=Q + (2 << 30), cs=R, cc=R + 4096, n_seq=3, tok=200, chunks=5, H=2, d_k=128,
                C=64, kd=2, gate=0, m=1, op=2)

    def call(**kw):
        a = {**base, **kw}
        return vl(a["K"], a["beta"], a["g"], a["T"], a["cs"], a["cc"], a["n_seq"], a["tok"], a["chunks"], a["H"], a["d_k"],
                  a["C"], a["kd"], a["gate"], a["m"], a["op"], None, 0)

    assert call(tok=0, chunks=0) == 0               # nothing to do
    assert call(C=48) == -2 and call(kd=7) == -3 and call(m=9) == -4 and call(gate=-1) == -4
    assert call(n_seq=0) == -5 and call(H=0) == -5 and call(d_k=40) == -5 and call(tok=-1) == -5
    assert call(chunks=3) == -5                     # 3 chunks of 64 cannot hold 200 tokens
    assert call(chunks=201) == -5                   # more chunks than tokens
    assert call(chunks=8) == -5                     # more than one partly filled chunk per sequence
    assert call(cs=None) == -1 and call(cc=None) == -1 and call(K=None) == -1
    assert call(cs=R + 4) == -6 and call(T=Q + (2 << 30) + 8) == -6
    assert call(T=R) == -7 and call(T=P) == -7


def test_solve_argument_errors(L):
    sv, vl = L.gdn_chunk_tri_solve, L.gdn_chunk_tri_solve_varlen
    G = 1 << 30
    base = dict(K=P, beta=Q, g=Q + G, X=Q + 2 * G, s=Q + 3 * G, W=Q + 4 * G, B=1, Tlen=128, H=2, d_k=128, d_x=128, C=64, kd=2,
                gate=0, m=1, op=2, flags=0)

    def call(**kw):
        a = {**base, **kw}
        return sv(a["K"], a["beta"], a["g"], a["X"], a["s"], a["W"], a["B"], a["Tlen"], a["H"], a["d_k"], a["d_x"], a["C"], a["kd"],
                  a["gate"], a["m"], a["op"], None, a["flags"])

    assert call(Tlen=0) == 0                                   # nothing to do
    assert call(C=48) == -2 and call(kd=4) == -3 and call(op=3) == -3 and call(m=9) == -4 and call(gate=3) == -4
    assert call(B=0) == -5 and call(H=0) == -5 and call(d_k=40) == -5 and call(Tlen=-1) == -5
    assert call(d_x=0) == -5 and call(d_x=4) == -5 and call(d_x=60) == -5 and call(d_x=520) == -5
    assert call(K=None) == -1 and call(X=None) == -1 and call(W=None) == -1 and call(g=None) == -1
    assert call(X=Q + 2 * G + 8) == -6 and call(W=Q + 4 * G + 2) == -6 and call(s=Q + 3 * G + 2) == -6
    assert call(W=P) == -7 and call(W=Q + 2 * G) == -7 and call(W=Q + 3 * G) == -7 and call(W=Q + G) == -7
    # valid arguments, combination not built: other methods, refinement and output-type flags (checked before any launch)
    assert call(m=0) == -9 and call(m=2) == -9 and call(m=4) == -9 and call(m=5) == -9 and call(m=6) == -9
    assert call(flags=0x1) == -9 and call(flags=0x4) == -9

    R = Q + 5 * G
    vbase = dict(base, cs=R, cc=R + 4096, n_seq=3, tok=200, chunks=5)

    def vcall(**kw):
        a = {**vbase, **kw}
        return vl(a["K"], a["beta"], a["g"], a["X"], a["s"], a["W"], a["cs"], a["cc"], a["n_seq"], a["tok"], a["chunks"], a["H"],
                  a["d_k"], a["d_x"], a["C"], a["kd"], a["gate"], a["m"], a["op"], None, a["flags"])

    assert vcall(tok=0, chunks=0) == 0
    assert vcall(C=100) == -2 and vcall(n_seq=0) == -5 and vcall(chunks=3) == -5 and vcall(chunks=8) == -5 and vcall(d_x=12) == -5
    assert vcall(cs=None) == -1 and vcall(cc=None) == -1 and vcall(W=None) == -1
    assert vcall(cs=R + 4) == -6
    assert vcall(W=R) == -7 and vcall(W=Q + 2 * G) == -7
    assert vcall(m=2) == -9


def test_solve_multi_argument_errors(L):
    import ctypes

    G = 1 << 30
    mv = L.gdn_chunk_tri_solve_multi

    def call(n=2, X=(Q + 2 * G, Q + 3 * G), S=(None, Q + 4 * G), W=(Q + 5 * G, Q + 6 * G), dx=(128, 64), C=64, m=1, K=P):
        arr = ctypes.c_void_p * len(X)
        xs, ss, ws = arr(*X), arr(*S), arr(*W)
        ds = (ctypes.c_int32 * len(dx))(*dx)
        cast = lambda a: ctypes.cast(a, ctypes.c_void_p)
        return mv(K, Q, Q + G, n, cast(xs), cast(ss), cast(ws), cast(ds), 1, 128, 2, 128, C, 2, 0, m, 2, None, 0)

    assert call(n=0) == -5 and call(n=3, X=(P,) * 3, S=(None,) * 3, W=(Q,) * 3, dx=(8,) * 3) == -5
    assert call(dx=(128, 12)) == -5
    assert call(X=(Q + 2 * G, None)) == -1 and call(W=(None, Q + 6 * G)) == -1 and call(K=None) == -1
    assert call(W=(Q + 5 * G, Q + 6 * G + 4)) == -6 and call(S=(None, Q + 4 * G + 1)) == -6
    assert call(W=(Q + 5 * G, Q + 5 * G)) == -7              # the two results in one buffer
    assert call(W=(Q + 3 * G, Q + 6 * G)) == -7              # result 0 on top of right-hand side 1
    assert call(W=(Q + 5 * G, Q + 4 * G)) == -7              # result 1 on top of scale 1
    assert call(m=2) == -9


def test_binding_refuses_host_tensors_and_missing_library(monkeypatch, L):
    import torch

    A = torch.zeros(1, 64, 64)
    with pytest.raises(ValueError):
        tri.tri_inv(A)
    with pytest.raises(TypeError):
        tri.binding.dtype_code(torch.float64)
    # no fallback: a missing shared library is an error, not a silent CPU path
    monkeypatch.setattr(tri.binding, "_lib", None)
    monkeypatch.setattr(tri.binding, "LIB_PATH", "/nonexistent/libtriinv.so")
    with pytest.raises(FileNotFoundError):
        tri.lib()


def test_no_kernel_uses_scratch_memory_or_spills():
    """Every kernel in the library keeps its whole state in registers and LDS: no per-lane scratch memory (a stack array
    the compiler could not keep in registers, or spilled registers) and no spilled vector registers.  A build whose
    Neumann kernel for C = 128 spilled at the full 512-register budget aborted on the GPU; combinations that do not fit
    are routed to another kernel or report 'combination not built' instead.  The report is written by the build from the
    compiler's resource remarks."""
    import json

    path = os.path.join(os.path.dirname(tri.binding.LIB_PATH), "kernel_resources.json")
    if not os.path.exists(path):
        pytest.skip("no compiler resource report beside the library")
    res = json.load(open(path))
    assert len(res) > 50
    bad = {k: v for k, v in res.items() if v.get("scratch", 0) > 0 or v.get("vgpr_spill", 0) > 0}
    assert not bad, bad
