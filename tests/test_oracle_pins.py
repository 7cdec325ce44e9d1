"""Pins for the fp64 CPU oracle: each test checks it against something other than itself --
closed forms, library routines, brute force, algebraic identities the paper states.  A dropped
term, a wrong sign or index, or a transposed operand in the oracle fails at least one of them.
"""
import math

import numpy as np
import pytest
import scipy.linalg
import torch

import oracle
from oracle import methods, metrics
import synth_inputs as si


def ones_strict(C):
    return np.tril(np.ones((C, C)), -1)


# ---------------------------------------------------------------- closed forms (P1-P3)
@pytest.mark.parametrize("C", [2, 4, 16, 64, 128])
def test_difference_operator(C):
    # inverse of the cumulative-sum matrix is the first-difference matrix
    T = oracle.tri_inv(ones_strict(C)[None])[0]
    expect = np.eye(C) - np.eye(C, k=-1)
    assert np.array_equal(T, expect)


@pytest.mark.parametrize("C,beta", [(8, 0.25), (64, 0.7), (128, 0.95)])
def test_geometric_rows(C, beta):
    # A = beta * ones_strict  =>  T_ij = -beta (1 - beta)^(i-j-1) for i > j
    T = oracle.tri_inv((beta * ones_strict(C))[None])[0]
    i, j = np.indices((C, C))
    expect = np.where(i > j, -beta * (1.0 - beta) ** np.clip(i - j - 1, 0, None), (i == j).astype(float))
    assert np.allclose(T, expect, rtol=1e-13, atol=1e-300)


@pytest.mark.parametrize("C", [4, 64, 128])
def test_powers_of_two(C):
    # A = -ones_strict  =>  T_ij = 2^(i-j-1), exact in fp64 up to 2^126
    T = oracle.tri_inv((-ones_strict(C))[None])[0]
    i, j = np.indices((C, C))
    expect = np.where(i > j, np.ldexp(1.0, np.clip(i - j - 1, 0, None)), (i == j).astype(float))
    assert np.array_equal(T, expect)


# ---------------------------------------------------------------- P4 binomial powers (Sec. 3.2)
@pytest.mark.parametrize("C", [16, 64])
def test_binomial_powers_pin_neumann_helper(C):
    # (ones_strict^k)_ij = binom(i-j-1, k-1): pins the repeated-squaring Y of Alg. 5
    L = ones_strict(C)
    for iters in range(0, int(math.log2(C // 2)) + 1):
        _, Y = methods.mch(L, iters=iters, return_Y=True)
        k = 2 ** iters
        for (i, j) in [(C - 1, 0), (C // 2, 0), (C - 1, C // 4), (k, 0), (k - 1, 0)]:
            want = math.comb(i - j - 1, k - 1) if i - j >= k else 0
            assert Y[i, j] == pytest.approx(want, rel=1e-12), (iters, i, j)
    # corner of L^(n/2) grows like 2^n / sqrt(n): overflows fp16 long before n = 64
    assert math.comb(C - 2, C // 2 - 1) > (65504 if C >= 32 else 0)


# ---------------------------------------------------------------- library routines (P11), brute force (P12)
def _cofactor_inverse(M):
    n = M.shape[0]

    def det(X):
        if X.shape[0] == 1:
            return X[0, 0]
        return sum((-1) ** c * X[0, c] * det(np.delete(np.delete(X, 0, 0), c, 1)) for c in range(X.shape[0]))

    d = det(M)
    inv = np.empty_like(M)
    for r in range(n):
        for c in range(n):
            minor = np.delete(np.delete(M, r, 0), c, 1)
            inv[c, r] = (-1) ** (r + c) * (det(minor) if n > 1 else 1.0) / d
    return inv


@pytest.mark.parametrize("C", [2, 4, 6])
def test_brute_force_cofactor(C):
    rng = np.random.default_rng(C)
    A = np.tril(rng.normal(size=(3, C, C)), -1)
    T = oracle.tri_inv(A)
    for m in range(3):
        assert np.allclose(T[m], _cofactor_inverse(np.eye(C) + A[m]), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("C", [8, 64, 128])
def test_library_inverse_and_triangular_solve(C):
    rng = np.random.default_rng(100 + C)
    A = np.tril(rng.normal(size=(4, C, C)) * (0.5 / math.sqrt(C)), -1)
    T = oracle.tri_inv(A)
    for m in range(4):
        M = np.eye(C) + A[m]
        assert np.allclose(T[m], np.linalg.inv(M), rtol=1e-10, atol=1e-12)
        ts = scipy.linalg.solve_triangular(M, np.eye(C), lower=True, unit_diagonal=True)
        assert np.allclose(T[m], ts, rtol=1e-12, atol=1e-14)


def test_upper_triangle_and_diagonal_are_ignored():
    A = si.random_strict_lower(3, 64, 0.1, seed=1, garbage_upper=True)
    clean = torch.tril(torch.nan_to_num(A, nan=0.0), -1)
    assert np.array_equal(oracle.tri_inv(A), oracle.tri_inv(clean))


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
def test_stored_values_are_widened_exactly(dtype):
    A = si.random_strict_lower(2, 64, 0.1, seed=2, garbage_upper=False).to(dtype)
    ref = oracle.tri_inv(A.to(torch.float64).numpy())
    assert np.array_equal(oracle.tri_inv(A), ref)
    if dtype == torch.float16:  # subnormal fp16 values survive the widening
        tiny = torch.zeros(1, 4, 4, dtype=torch.float16)
        tiny[0, 1, 0] = 6e-8
        assert oracle.tri_inv(tiny)[0, 1, 0] == -float(tiny[0, 1, 0])


# ---------------------------------------------------------------- P5-P8 on the workload generators
def _small(idx, **kw):
    return si.make_inputs(si.workload(idx, **kw))


@pytest.mark.parametrize("idx,kw", [(0, {}), (1, dict(Tlen=256, H=2)), (2, dict(B=1, Tlen=256, H=2)),
                                    (3, dict(B=1, Tlen=128, H=2)), (4, dict(Tlen=512, H=2))])
def test_structure_residual_nilpotency_entry_bound(idx, kw):
    inp = _small(idx, **kw)
    w = inp["workload"]
    A = oracle.build_A(inp["K"], inp["beta"], inp["g"], w.gate_kind, w.C)
    T = oracle.gdn_chunk_tri_inv(inp["K"], inp["beta"], inp["g"], w.gate_kind, w.C)
    assert A.shape == (w.n_mat, w.C, w.C)
    assert metrics.structure_ok(T)                                        # unit lower triangular
    assert np.array_equal(A, np.tril(A, -1))
    assert np.array_equal(T, oracle.tri_inv(A))                           # fused == build then invert
    res = metrics.residual(A, T)
    assert res["normalised"].max() < w.C * 2.0 ** -52                     # (I + A) T = I
    assert np.abs(T).max() <= 1.0 + 1e-12                                 # entries of the inverse in [-1, 1]
    M = np.eye(w.C)[None] + A
    cond = np.linalg.cond(M[: min(8, w.n_mat)])
    assert cond.max() <= w.C ** 2                                         # Cor. 2.1
    # nilpotency: A^C = 0 and the finite Neumann sum is the inverse (benign inputs only)
    if idx != 4:
        for m in range(min(4, w.n_mat)):
            assert np.array_equal(np.linalg.matrix_power(A[m], w.C), np.zeros((w.C, w.C)))
            assert np.allclose(methods.neumann_sum(A[m]), T[m], rtol=0, atol=1e-13)


# ---------------------------------------------------------------- build_A: independent einsum, P9, P13
def test_build_A_matches_independent_einsum_scalar_gate():
    inp = _small(1, Tlen=128, H=3)
    w = inp["workload"]
    K = inp["K"].to(torch.float64)
    B, Tlen, H, d = K.shape
    Kc = K.reshape(B, Tlen // w.C, w.C, H, d)
    S = torch.einsum("bnihd,bnjhd->bnhij", Kc, Kc)
    g = inp["g"].to(torch.float64).reshape(B, Tlen // w.C, w.C, H).permute(0, 1, 3, 2)
    beta = inp["beta"].to(torch.float64).reshape(B, Tlen // w.C, w.C, H).permute(0, 1, 3, 2)
    A = beta[..., :, None] * torch.exp(g[..., :, None] - g[..., None, :]) * S
    A = torch.tril(A, -1).reshape(-1, w.C, w.C).numpy()
    got = oracle.build_A(inp["K"], inp["beta"], inp["g"], w.gate_kind, w.C)
    assert np.allclose(got, A, rtol=1e-12, atol=1e-15)


def test_build_A_per_channel_matches_factored_form():
    # (K * Gamma)(K / Gamma)^T with Gamma = exp(g) -- the KDA row of Table 1 -- equals the
    # difference form the oracle evaluates
    inp = _small(3, B=1, Tlen=128, H=2)
    w = inp["workload"]
    K = inp["K"].to(torch.float64)
    g = inp["g"].to(torch.float64)
    B, Tlen, H, d = K.shape
    Kp = (K * torch.exp(g)).reshape(B, Tlen // w.C, w.C, H, d)
    Km = (K * torch.exp(-g)).reshape(B, Tlen // w.C, w.C, H, d)
    S = torch.einsum("bnihd,bnjhd->bnhij", Kp, Km)
    beta = inp["beta"].to(torch.float64).reshape(B, Tlen // w.C, w.C, H).permute(0, 1, 3, 2)
    A = torch.tril(beta[..., :, None] * S, -1).reshape(-1, w.C, w.C).numpy()
    got = oracle.build_A(inp["K"], inp["beta"], inp["g"], w.gate_kind, w.C)
    assert np.allclose(got, A, rtol=1e-11, atol=1e-15)


def test_matrix_index_order_and_selection():
    inp = _small(1, B=2, Tlen=192, H=3)
    w = inp["workload"]
    A = oracle.build_A(inp["K"], inp["beta"], inp["g"], w.gate_kind, w.C)
    # m = (b * n_chunk + chunk) * H + h
    b, chunk, h = 1, 2, 1
    m = (b * (w.Tlen // w.C) + chunk) * w.H + h
    Kc = inp["K"][b, chunk * w.C:(chunk + 1) * w.C, h].to(torch.float64).numpy()
    gc = inp["g"][b, chunk * w.C:(chunk + 1) * w.C, h].to(torch.float64).numpy()
    bc = inp["beta"][b, chunk * w.C:(chunk + 1) * w.C, h].to(torch.float64).numpy()
    want = np.tril(bc[:, None] * np.exp(gc[:, None] - gc[None, :]) * (Kc @ Kc.T), -1)
    assert np.allclose(A[m], want, rtol=1e-12, atol=1e-15)
    sel = [m, 0, 5]
    assert np.array_equal(oracle.build_A(inp["K"], inp["beta"], inp["g"], w.gate_kind, w.C, sel=sel), A[sel])
    T = oracle.gdn_chunk_tri_inv(inp["K"], inp["beta"], inp["g"], w.gate_kind, w.C)
    assert np.array_equal(oracle.gdn_chunk_tri_inv(inp["K"], inp["beta"], inp["g"], w.gate_kind, w.C, sel=sel), T[sel])


def test_scalar_gate_similarity():
    # A_gated = Gamma A Gamma^-1  =>  T_gated[i,j] = T_ungated[i,j] * exp(g_i - g_j)
    inp = _small(2, B=1, Tlen=128, H=2)
    w = inp["workload"]
    T_g = oracle.gdn_chunk_tri_inv(inp["K"], inp["beta"], inp["g"], si.GATE_SCALAR, w.C)
    T_0 = oracle.gdn_chunk_tri_inv(inp["K"], inp["beta"], None, si.GATE_NONE, w.C)
    g = inp["g"].to(torch.float64).reshape(w.B, w.Tlen // w.C, w.C, w.H).permute(0, 1, 3, 2).reshape(-1, w.C).numpy()
    scale = np.exp(g[:, :, None] - g[:, None, :])
    assert np.allclose(T_g, T_0 * scale, rtol=1e-12, atol=1e-15)


def test_per_channel_gate_reduces_to_scalar_gate_and_to_deltanet():
    inp = _small(2, B=1, Tlen=128, H=2)
    w = inp["workload"]
    g_bcast = inp["g"][..., None].expand(-1, -1, -1, w.d_k).contiguous()
    A_s = oracle.build_A(inp["K"], inp["beta"], inp["g"], si.GATE_SCALAR, w.C)
    A_c = oracle.build_A(inp["K"], inp["beta"], g_bcast, si.GATE_PER_CHANNEL, w.C)
    assert np.allclose(A_s, A_c, rtol=1e-12, atol=1e-16)
    A_0 = oracle.build_A(inp["K"], inp["beta"], None, si.GATE_NONE, w.C)
    A_z = oracle.build_A(inp["K"], inp["beta"], torch.zeros_like(inp["g"]), si.GATE_SCALAR, w.C)
    assert np.array_equal(A_0, A_z)


# ---------------------------------------------------------------- paper algorithms in exact arithmetic
@pytest.mark.parametrize("C", [16, 64, 128])
def test_paper_algorithms_reach_the_oracle_in_fp64(C):
    rng = np.random.default_rng(C)
    Kn = rng.normal(size=(C, 32))
    Kn /= np.linalg.norm(Kn, axis=1, keepdims=True)
    L = np.tril(Kn @ Kn.T * rng.uniform(0.2, 1.0, size=(C, 1)), -1)
    T = oracle.tri_inv(L[None])[0]
    assert np.allclose(methods.mch(L), T, atol=1e-11)
    assert np.allclose(methods.mbh(L), T, atol=1e-12)
    assert np.allclose(methods.mxr(L, b0=16), T, atol=1e-12)
    assert np.allclose(methods.mxr(L, b0=16, r=1), T, atol=1e-12)
    assert np.allclose(methods.ir(T + 1e-4 * np.tril(rng.normal(size=(C, C))), L), T, atol=1e-6)
    assert np.allclose(methods.ns(L, m=4 * int(math.log2(C))), T, atol=1e-10)
    assert np.allclose(methods.forward_substitution(L), T, atol=1e-13)


@pytest.mark.parametrize("C", [4, 16, 64])
def test_algorithm_statements_agree_with_their_closed_forms(C):
    # each iteration, step by step, against the closed form of what it must have reached: the factor product for
    # Alg. 5 after every iteration, the residual recurrence of Eq. 8 for Alg. 3 after every iteration (also where it
    # has not converged), the recursive 2 x 2 block formula of Eq. 7 for Alg. 4
    rng = np.random.default_rng(100 + C)
    L = np.tril(rng.normal(size=(C, C)) * 0.25, -1)
    for k in range(int(math.log2(C))):
        assert np.allclose(methods.mch(L, iters=k), methods.neumann_factor_product(L, k_max=k), atol=1e-11), k
    assert np.allclose(methods.neumann_factor_product(L), oracle.tri_inv(L[None])[0], atol=1e-11)
    X0 = np.eye(C) / C + 1e-3 * rng.normal(size=(C, C))
    for m in range(0, 7):
        assert np.allclose(methods.ns(L, m=m, X0=X0), methods.newton_schulz_closed_form(L, m, X0=X0), atol=1e-9), m
    assert np.allclose(methods.mbh(L), methods.block_inverse_2x2(L), atol=1e-12)
    assert np.allclose(methods.block_inverse_2x2(L), np.linalg.inv(np.eye(C) + L), atol=1e-11)


def test_mch_partial_sums():
    # after k iterations of Alg. 5, X = sum_{i < 2^(k+1)} (-L)^i
    rng = np.random.default_rng(5)
    L = np.tril(rng.normal(size=(32, 32)) * 0.2, -1)
    for k in range(0, 5):
        want = sum(np.linalg.matrix_power(-L, i) for i in range(2 ** (k + 1)))
        assert np.allclose(methods.mch(L, iters=k), want, atol=1e-12)


@pytest.mark.parametrize("C", [16, 64])
def test_mbh_block_invariant(C):
    # after the level with block size b, every 2b x 2b diagonal block of X is the inverse of the
    # same block of I + L (Lemma C.1 induction)
    rng = np.random.default_rng(C + 1)
    L = np.tril(rng.normal(size=(C, C)) * 0.3, -1)
    levels = []
    methods.mbh(L, levels_out=levels)
    assert [b for b, _ in levels] == [2 ** k for k in range(int(math.log2(C)))]
    for b, X in levels:
        for t in range(C // (2 * b)):
            s = slice(2 * b * t, 2 * b * (t + 1))
            want = oracle.tri_inv(L[s, s][None])[0]
            assert np.allclose(X[s, s], want, atol=1e-10), (b, t)


def test_matmul_counts_table2(monkeypatch):
    """The numpy statements of Alg. 3-6 execute exactly the number of matrix products the paper's Table 2
    gives (fixture tests/golden/table2_matmul_counts.txt)."""
    import os

    want = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table2_matmul_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, n, cnt = line.split()
                want[(name, int(n))] = int(cnt)
    calls = []
    real_mm = methods.Arith.mm
    monkeypatch.setattr(methods.Arith, "mm", lambda self, X, Y: (calls.append(1), real_mm(self, X, Y))[1])

    def count(fn):
        calls.clear()
        fn()
        return len(calls)

    rng = np.random.default_rng(0)
    for n in (64, 128):
        L = np.tril(rng.standard_normal((n, n)) * 0.05, -1)
        assert count(lambda: methods.mch(L)) == want[("MCH", n)] == 2 * math.ceil(math.log2(n / 2))
        assert count(lambda: methods.mbh(L)) == want[("MBH", n)] == 2 * int(math.log2(n))
        Y = np.eye(n) - L
        assert count(lambda: methods.ir(Y, L)) == want[("IR1", n)]
        assert want[("MCS", n)] == n - 1
    L = np.tril(rng.standard_normal((64, 64)) * 0.05, -1)
    assert count(lambda: methods.ns(L, m=12)) == want[("NS12", 64)]


# ---------------------------------------------------------------- short last chunk, packed sequences
def _direct_A(k, b, g, gate_kind):
    """A of one chunk from fp64 arrays, written with an explicit double loop (independent of oracle/)."""
    n = k.shape[0]
    A = np.zeros((n, n))
    for i in range(n):
        for j in range(i):
            if gate_kind == 0:
                A[i, j] = b[i] * math.exp(g[i] - g[j]) * float(k[i] @ k[j])
            elif gate_kind == 1:
                A[i, j] = b[i] * float(np.sum(k[i] * k[j] * np.exp(g[i] - g[j])))
            else:
                A[i, j] = b[i] * float(k[i] @ k[j])
    return A


@pytest.mark.parametrize("gate_kind", [0, 1, 2])
@pytest.mark.parametrize("Tlen", [1, 37, 64, 100])
def test_short_last_chunk_is_the_leading_block_of_an_identity_padded_matrix(gate_kind, Tlen):
    C, H = 64, 2
    idx = {0: 1, 1: 3, 2: 4}[gate_kind]
    inp = _small(idx, B=1, Tlen=Tlen, H=H, C=C, d_k=32)
    T = oracle.gdn_chunk_tri_inv_ragged(inp["K"], inp["beta"], inp["g"], gate_kind, C)
    n_chunk = (Tlen + C - 1) // C
    assert T.shape == (n_chunk * H, C, C)
    for chunk in range(n_chunk):
        v = min(C, Tlen - chunk * C)
        for h in range(H):
            sl = slice(chunk * C, chunk * C + v)
            k = inp["K"][0, sl, h].double().numpy()
            b = inp["beta"][0, sl, h].double().numpy()
            g = None if inp["g"] is None else inp["g"][0, sl, h].double().numpy()
            ref = np.linalg.inv(np.eye(v) + _direct_A(k, b, g, gate_kind))
            Tm = T[chunk * H + h]
            assert np.allclose(Tm[:v, :v], ref, rtol=0, atol=1e-12)
            assert np.array_equal(Tm[v:, :v], np.zeros((C - v, v)))       # padded rows: identity
            assert np.array_equal(Tm[v:, v:], np.eye(C - v))
            assert np.array_equal(Tm[:v, v:], np.zeros((v, C - v)))


def test_packed_sequences_are_chunked_one_by_one():
    C, H, d = 64, 3, 32
    seqlens = [64, 1, 0, 133, 63]
    inp = _small(1, B=1, Tlen=sum(seqlens), H=H, C=C, d_k=d)
    K, beta = inp["K"][0], inp["beta"][0]
    # chunk-local cumulative gate per sequence
    gen = torch.Generator().manual_seed(5)
    g = torch.zeros(sum(seqlens), H)
    t0 = 0
    for n in seqlens:
        for c0 in range(0, n, C):
            m = min(C, n - c0)
            g[t0 + c0:t0 + c0 + m] = torch.cumsum(-0.1 * torch.rand(m, H, generator=gen), 0)
        t0 += n
    T = oracle.gdn_chunk_tri_inv_varlen(K, beta, g, seqlens, 0, C)
    assert T.shape == ((1 + 1 + 0 + 3 + 1) * H, C, C)
    # sequence 3 (133 tokens) starts at token 65 and at chunk id 2; its last chunk has 5 tokens
    t0, c0, h = 65 + 128, 2 + 2, 1
    k, b, gg = K[t0:t0 + 5, h].double().numpy(), beta[t0:t0 + 5, h].double().numpy(), g[t0:t0 + 5, h].double().numpy()
    ref = np.linalg.inv(np.eye(5) + _direct_A(k, b, gg, 0))
    assert np.allclose(T[c0 * H + h][:5, :5], ref, rtol=0, atol=1e-13)
    assert np.array_equal(T[c0 * H + h][5:, 5:], np.eye(C - 5))
    # the one-token sequence: A = 0, T = I
    assert np.array_equal(T[1 * H + 0], np.eye(C))


# ---------------------------------------------------------------- residual identities of the iterations
def test_refinement_step_squares_the_left_residual():
    # Eq. 9: with R = I - Y (I + L), the refined X = Y + R Y has I - X (I + L) = R^2 exactly;
    # the mirrored update Y + Y R does not (Y is a generic lower-triangular matrix here, so it
    # does not commute with I + L)
    rng = np.random.default_rng(11)
    C = 24
    L = np.tril(rng.normal(size=(C, C)) * 0.3, -1)
    M = np.eye(C) + L
    Y = np.linalg.inv(M) + 0.05 * np.tril(rng.normal(size=(C, C)))
    R = np.eye(C) - Y @ M
    X = methods.ir(Y, L)
    assert np.allclose(np.eye(C) - X @ M, R @ R, atol=1e-12)
    assert not np.allclose(np.eye(C) - (Y + Y @ R) @ M, R @ R, atol=1e-6)


@pytest.mark.parametrize("m", [1, 2, 3, 5])
def test_newton_schulz_squares_the_right_residual(m):
    # Eq. 8: X <- X (2 I - A X) gives I - A X_m = (I - A X_0)^(2^m) for any start X_0
    rng = np.random.default_rng(12 + m)
    C = 16
    L = np.tril(rng.normal(size=(C, C)) * 0.3, -1)
    A = np.eye(C) + L
    X0 = np.linalg.inv(A) + 0.02 * rng.normal(size=(C, C))
    want = np.linalg.matrix_power(np.eye(C) - A @ X0, 2 ** m)
    assert np.allclose(np.eye(C) - A @ methods.ns(L, m=m, X0=X0), want, atol=1e-12)


def test_newton_schulz_default_start_is_identity_over_n():
    # Alg. 3 starts from X_0 = I / n: one iteration from it is (2 I - A / n) / n
    C = 8
    L = np.tril(np.arange(C * C, dtype=np.float64).reshape(C, C) / 50.0, -1)
    A = np.eye(C) + L
    assert np.allclose(methods.ns(L, m=1), (2 * np.eye(C) - A / C) / C, atol=1e-15)


# ---------------------------------------------------------------- error measures on hand-computed cases
def test_error_measures_by_hand():
    # T_ref = [[1,0],[2,1]], T_hat = [[1,0],[2.5,1]]: diff has the single entry 0.5
    T_ref = np.array([[[1.0, 0.0], [2.0, 1.0]]])
    T_hat = np.array([[[1.0, 0.0], [2.5, 1.0]]])
    e = metrics.forward_errors(T_ref, T_hat)
    assert e["rel_fro"][0] == pytest.approx(0.5 / math.sqrt(6.0), rel=1e-15)
    assert e["max_abs"][0] == 0.5
    assert e["max_rel"][0] == 0.25
    # (I + A) T_hat - I with A = [[0,0],[-2,0]] is [[0,0],[0.5,0]]
    A = np.array([[[0.0, 7.0], [-2.0, 9.0]]])          # diagonal and upper part are not read
    r = metrics.residual(A, T_hat)
    assert r["abs"][0] == pytest.approx(0.5, rel=1e-15)
    assert r["normalised"][0] == pytest.approx(0.5 / (math.sqrt(6.0) * math.sqrt(8.25)), rel=1e-15)
    assert metrics.structure_ok(T_hat)
    assert not metrics.structure_ok(np.array([[[1.0, 1e-30], [2.0, 1.0]]]))
    assert not metrics.structure_ok(np.array([[[1.0, 0.0], [2.0, 1.0 + 2.0 ** -40]]]))
    s = metrics.summarise(np.array([1.0, 3.0, np.nan]))
    assert s["non_finite"] == 1 and s["max"] == np.inf


def test_max_rel_looks_at_the_lower_triangle_only():
    T_ref = np.array([[[1.0, 0.0], [4.0, 1.0]]])
    T_hat = np.array([[[1.0, 3.0], [5.0, 1.0]]])
    assert metrics.forward_errors(T_ref, T_hat)["max_rel"][0] == 0.25


# ---------------------------------------------------------------- operand rounding of the emulated precisions
def test_operand_rounding_is_to_nearest_even():
    # bf16 keeps 8 significant bits (spacing 2^-7 in [1, 2)), fp16 keeps 11 (spacing 2^-10)
    u = 2.0 ** -7
    x = np.array([1.0, 1 + u / 2, 1 + 3 * u / 2, 1 + u / 2 + 2.0 ** -20, 1 + 0.49 * u, -1 - 3 * u / 2, 3.0e38])
    want = np.array([1.0, 1.0, 1 + 2 * u, 1 + u, 1.0, -1 - 2 * u, 2.0 ** 127 * (1 + 98 / 128)])
    assert np.array_equal(methods.round_bf16(x), want)
    assert np.array_equal(methods.round_bf16(x), torch.tensor(x, dtype=torch.float32).bfloat16().double().numpy())
    h = 2.0 ** -10
    xh = np.array([1.0, 1 + h / 2, 1 + 3 * h / 2, 1 + 0.51 * h, 65520.0])
    assert np.array_equal(methods.round_f16(xh), np.array([1.0, 1.0, 1 + 2 * h, 1 + h, np.inf]))
    assert methods.round_f32(np.array([1 + 2.0 ** -24]))[0] == 1.0
    assert methods.round_f32(np.array([1 + 3 * 2.0 ** -24]))[0] == 1 + 2.0 ** -22


def test_emulated_product_rounds_operands_then_accumulates_exactly():
    # bf16 operands: 1 + 2^-8 becomes 1 before the product; the fp32 accumulator keeps 2^-20
    ar = methods.Arith("bf16")
    X = np.array([[1 + 2.0 ** -8, 2.0 ** -10]])
    Y = np.array([[1.0], [2.0 ** -10]])
    assert ar.mm(X, Y)[0, 0] == 1.0 + 2.0 ** -20
    assert methods.Arith(None).mm(X, Y)[0, 0] == (1 + 2.0 ** -8) + 2.0 ** -20


# ---------------------------------------------------------------- chunk-local solve W = (I + A)^{-1} diag(s) X
def _solve_case(seed, B=2, Tlen=96, H=3, d_k=32, d_x=24, gate_kind=0):
    rng = np.random.default_rng(seed)
    K = rng.normal(size=(B, Tlen, H, d_k)).astype(np.float32)
    K /= np.linalg.norm(K, axis=-1, keepdims=True)
    beta = rng.uniform(0.1, 1.0, size=(B, Tlen, H)).astype(np.float32)
    shape = (B, Tlen, H, d_k) if gate_kind == 1 else (B, Tlen, H)
    g = None if gate_kind == 2 else np.cumsum(-rng.uniform(0.0, 0.1, size=shape), axis=1).astype(np.float32)
    X = rng.normal(size=(B, Tlen, H, d_x)).astype(np.float32)
    s = rng.uniform(0.5, 1.5, size=(B, Tlen, H)).astype(np.float32)
    return K, beta, g, X, s


@pytest.mark.parametrize("gate_kind,Tlen,C", [(0, 96, 32), (1, 64, 16), (2, 100, 32), (0, 37, 64)])
def test_chunk_solve_against_library_triangular_solve(gate_kind, Tlen, C):
    K, beta, g, X, s = _solve_case(21 + gate_kind, Tlen=Tlen, gate_kind=gate_kind)
    W = oracle.gdn_chunk_tri_solve(K, beta, g, X, s, gate_kind, C)
    B, _, H, d_x = X.shape
    for b in range(B):
        for h in range(H):
            for t0 in range(0, Tlen, C):
                t1 = min(Tlen, t0 + C)
                # the short block's own matrix from an explicit double loop
                n = t1 - t0
                A = np.zeros((n, n))
                for i in range(n):
                    for j in range(i):
                        k_i, k_j = K[b, t0 + i, h].astype(np.float64), K[b, t0 + j, h].astype(np.float64)
                        if gate_kind == 0:
                            w = math.exp(float(g[b, t0 + i, h]) - float(g[b, t0 + j, h])) * (k_i @ k_j)
                        elif gate_kind == 1:
                            w = float(np.sum(k_i * k_j * np.exp(g[b, t0 + i, h].astype(np.float64) - g[b, t0 + j, h].astype(np.float64))))
                        else:
                            w = k_i @ k_j
                        A[i, j] = float(beta[b, t0 + i, h]) * w
                rhs = s[b, t0:t1, h, None].astype(np.float64) * X[b, t0:t1, h].astype(np.float64)
                want = scipy.linalg.solve_triangular(np.eye(n) + A, rhs, lower=True, unit_diagonal=True)
                assert np.allclose(W[b, t0:t1, h], want, rtol=1e-11, atol=1e-12), (b, h, t0)


def test_chunk_solve_is_the_inverse_applied():
    K, beta, g, X, s = _solve_case(31, Tlen=128)
    C = 64
    W = oracle.gdn_chunk_tri_solve(K, beta, g, X, s, 0, C)
    T = oracle.gdn_chunk_tri_inv(K, beta, g, 0, C).reshape(2, 2, 3, C, C)        # [B, chunk, H, C, C]
    sX = (s[..., None].astype(np.float64) * X).reshape(2, 2, C, 3, -1)           # [B, chunk, C, H, d_x]
    want = np.einsum("bchij,bcjhx->bcihx", T, sX).reshape(W.shape)
    assert np.allclose(W, want, rtol=1e-11, atol=1e-12)
    # no scale = scale of ones
    assert np.array_equal(oracle.gdn_chunk_tri_solve(K, beta, g, X, None, 0, C),
                          oracle.gdn_chunk_tri_solve(K, beta, g, X, np.ones_like(s), 0, C))


def test_chunk_solve_closed_form_differences():
    # all keys equal and of unit length, beta = 1, no gate: I + A is the lower-triangular all-ones matrix,
    # whose inverse takes first differences within each chunk: W_0 = X_0, W_i = X_i - X_{i-1}
    B, Tlen, H, d_k, d_x, C = 1, 48, 2, 8, 5, 16
    K = np.zeros((B, Tlen, H, d_k), dtype=np.float32)
    K[..., 3] = 1.0
    beta = np.ones((B, Tlen, H), dtype=np.float32)
    X = np.random.default_rng(7).normal(size=(B, Tlen, H, d_x)).astype(np.float32)
    W = oracle.gdn_chunk_tri_solve(K, beta, None, X, None, 2, C)
    want = X.astype(np.float64).copy()
    want[:, 1:] -= X[:, :-1]
    want[:, ::C] = X[:, ::C]
    assert np.allclose(W, want, atol=1e-13)


def test_chunk_solve_packed_sequences_are_solved_one_by_one():
    # packed [total, H, ...] tensors: each sequence's result equals the fixed-layout result of that sequence alone,
    # and a chunk never reaches across a sequence boundary (first differences restart at every sequence and chunk)
    H, d_k, d_x, C = 2, 8, 3, 16
    seqlens = [20, 0, 5, 33]
    total = sum(seqlens)
    K = np.zeros((total, H, d_k), dtype=np.float32)
    K[..., 0] = 1.0
    beta = np.ones((total, H), dtype=np.float32)
    X = np.random.default_rng(3).normal(size=(total, H, d_x)).astype(np.float32)
    W = oracle.gdn_chunk_tri_solve_varlen(K, beta, None, X, None, seqlens, 2, C)
    want = X.astype(np.float64).copy()
    want[1:] -= X[:-1]
    t0 = 0
    for n in seqlens:
        for c0 in range(0, n, C):
            want[t0 + c0] = X[t0 + c0]
        t0 += n
    assert np.allclose(W, want, atol=1e-13)
