// Inversion cores on register tiles: one 64-lane wavefront inverts one C x C matrix, C = 16 * NB.
//
// All functions take the strictly-lower chunk matrix A through a "tile source" object
//     template <bool TR> v4f get(int i, int j) const;      // 16x16 tile (i, j), i >= j
// returning the tile in N orientation (TR = false: registers hold A_ij) or in T orientation
// (TR = true: registers hold A_ij^T).  Diagonal tiles come back already masked to their
// strictly-lower part.  See tile_ops.hpp for the register layout and the tn primitive.
#pragma once
#include "tile_ops.hpp"

namespace triinv {

// ---------------------------------------------------------------------------------------------
// 16 x 16 leaves.  Both return the leaf inverse in both orientations (XN = X, XT = X^T).
// ---------------------------------------------------------------------------------------------

// Blocked recursion inside the leaf (paper Alg. 4 with b0 = 1, Lemma C.1): block sizes 1, 2, 4, 8.
// The level b = 1 starts from X = I, so D_o A D_e only picks the entries A[i][i-1], i odd.
// Each later level applies X <- X - D_o A_b D_e with A_b = A restricted to its 2b x 2b diagonal
// blocks; the restriction drops the entries the unrolled product would create outside those
// blocks, which the paper's next level discards when it re-selects diagonal blocks.
template <int OP>
__device__ __forceinline__ void leaf_block_recursive(v4f LN, v4f LT, v4f& XN, v4f& XT, Lane ln)
{
    const Opnd<OP> LNo = negated<OP>(pack<OP>(LN)), LTo = negated<OP>(pack<OP>(LT));  // -A: every level subtracts D_o A D_e
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int a = 4 * ln.q + r, b = ln.n;  // XN[r] = X[a][b], XT[r] = X[b][a]
        XN[r] = (a == b) ? 1.f : (((a & 1) && b == a - 1) ? -LN[r] : 0.f);
        XT[r] = (a == b) ? 1.f : (((b & 1) && a == b - 1) ? -LT[r] : 0.f);
    }
#pragma unroll
    for (int lb = 1; lb < 4; ++lb) {  // block size b = 2^lb
        bool ke[4], ko[4], ks[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int a = 4 * ln.q + r, b = ln.n;
            const bool same_b = (a >> lb) == (b >> lb);
            const bool even = ((a >> lb) & 1) == 0;
            ke[r] = same_b && even;                        // D_e (the same predicate serves D_o^T: it is symmetric)
            ko[r] = same_b && !even;                       // D_o
            ks[r] = (a >> (lb + 1)) == (b >> (lb + 1));    // inside one 2b x 2b diagonal block
        }
        const Mask<OP> Me = make_mask<OP>(ke[0], ke[1], ke[2], ke[3]);
        const Mask<OP> Mo = make_mask<OP>(ko[0], ko[1], ko[2], ko[3]);
        const Mask<OP> Ms = make_mask<OP>(ks[0], ks[1], ks[2], ks[3]);
        const Opnd<OP> eNo = masked<OP>(pack<OP>(XN), Me);     // D_e        (N)
        const Opnd<OP> oTo = masked<OP>(pack<OP>(XT), Mo);     // D_o^T      (T)
        // A restricted to the 2b-block diagonal: D_o A D_e then has no entry outside those blocks
        const v4f P1 = tn<OP>(masked<OP>(LTo, Ms), eNo, zero4());   // -A D_e
        const v4f P2 = tn<OP>(masked<OP>(LNo, Ms), oTo, zero4());   // -A^T D_o^T = -(D_o A)^T
        XN = tn<OP>(oTo, pack<OP>(P1), XN);                         // X - D_o A D_e
        XT = tn<OP>(eNo, pack<OP>(P2), XT);                         // (X - D_o A D_e)^T
    }
}

// Neumann product on the leaf (paper Alg. 5 with n = 16: three squarings), both orientations, followed
// by r steps of iterative refinement on the leaf (paper Alg. 2: the refinement of the mixed recursion
// acts on the b0 x b0 diagonal blocks, before the merges; Alg. 6 / Eq. 9 read for I + L):
//   R <- I - Y (I + L) = I - Y - Y L;   Y <- Y + R Y.
template <int OP>
__device__ __forceinline__ void leaf_neumann(v4f LN, v4f LT, v4f& XN, v4f& XT, Lane ln, int r = 0)
{
    v4f YN = LN, YT = LT;
    v4f id;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        id[e] = (4 * ln.q + e == ln.n) ? 1.f : 0.f;
        XN[e] = id[e] - LN[e];
        XT[e] = id[e] - LT[e];
    }
#pragma unroll
    for (int it = 0; it < 3; ++it) {
        const Opnd<OP> YNo = pack<OP>(YN), YTo = pack<OP>(YT);
        YN = tn<OP>(YTo, YNo, zero4());                        // Y <- Y Y
        if (it < 2) YT = tn<OP>(YNo, YTo, zero4());            // (Y Y)^T
        const Opnd<OP> Yn = pack<OP>(YN), XTo = pack<OP>(XT);
        const v4f XNn = tn<OP>(XTo, Yn, XN);                   // X + X Y
        XT = tn<OP>(Yn, XTo, XT);                              // (X + X Y)^T
        XN = XNn;
    }
    const Opnd<OP> LNo = pack<OP>(LN);
#pragma unroll 1
    for (int s = 0; s < r; ++s) {
        const Opnd<OP> Xn = pack<OP>(XN), Xt = pack<OP>(XT);
        const v4f RT = id - XT - tn<OP>(LNo, Xt, zero4());     // R^T = I - X^T - L^T X^T
        const Opnd<OP> Rt = pack<OP>(RT);
        const v4f XNn = tn<OP>(Rt, Xn, XN);                    // X + R X
        XT = tn<OP>(Xn, Rt, XT);                               // (X + R X)^T = X^T + X^T R^T
        XN = XNn;
    }
}

// ---------------------------------------------------------------------------------------------
// Leaves by forward substitution in fp32 vector arithmetic (the direct method of paper Sec. 3.1
// as the start X0 of Alg. 4 at b0 = 16).  Four leaves at a time: lane group q solves leaf q, lane
// n its column n; the leaf's rows are read back from LDS with one address per lane group (LDS
// broadcast).  lds: LEAF_FWD_FLOATS floats, wave-private.
// ---------------------------------------------------------------------------------------------
constexpr int LEAF_LD = 20;                       // row stride inside a staged leaf
constexpr int LEAF_STRIDE = 16 * LEAF_LD + 8;     // leaf stride: the four groups' rows fall into different banks
constexpr int LEAF_FWD_FLOATS = 4 * LEAF_STRIDE;

__device__ __forceinline__ void leaf_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int NB, class ASrc>
__device__ __forceinline__ void leaves_forward_substitution(const ASrc& A, v4f (&leafN)[NB], v4f (&leafT)[NB], float* lds, Lane ln)
{
    constexpr int PER = NB < 4 ? NB : 4;
#pragma unroll
    for (int pass = 0; pass < (NB + 3) / 4; ++pass) {
#pragma unroll
        for (int d = 0; d < PER; ++d) {  // T orientation = row-major pieces: v[r] = A[16 leaf + n][16 leaf + 4q + r]
            const v4f v = A.template get<true>(4 * pass + d, 4 * pass + d);
            *reinterpret_cast<v4f*>(&lds[d * LEAF_STRIDE + ln.n * LEAF_LD + 4 * ln.q]) = v;
        }
        leaf_lds_sync();
        const float* Al = lds + ln.q * LEAF_STRIDE;  // this lane group's leaf
        const int c = ln.n;
        float t[16];
        t[0] = (c == 0) ? 1.f : 0.f;
#pragma unroll
        for (int i = 1; i < 16; ++i) {
            float acc = 0.f;
#pragma unroll
            for (int j4 = 0; j4 < i; j4 += 4) {
                const v4f a = *reinterpret_cast<const v4f*>(&Al[i * LEAF_LD + j4]);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (j4 + r < i) acc += a[r] * t[j4 + r];
            }
            t[i] = (c < i) ? -acc : ((c == i) ? 1.f : 0.f);
        }
        leaf_lds_sync();
#pragma unroll
        for (int i = 0; i < 16; ++i) lds[ln.q * LEAF_STRIDE + i * LEAF_LD + c] = t[i];
        leaf_lds_sync();
#pragma unroll
        for (int d = 0; d < PER; ++d) {
#pragma unroll
            for (int r = 0; r < 4; ++r) leafN[4 * pass + d][r] = lds[d * LEAF_STRIDE + (4 * ln.q + r) * LEAF_LD + ln.n];
            leafT[4 * pass + d] = *reinterpret_cast<const v4f*>(&lds[d * LEAF_STRIDE + ln.n * LEAF_LD + 4 * ln.q]);
        }
        leaf_lds_sync();
    }
}

// ---------------------------------------------------------------------------------------------
// Tile transpose through a wave-private LDS patch of 16 x 20 floats.
// ---------------------------------------------------------------------------------------------
constexpr int XPOSE_LD = 20;
constexpr int XPOSE_FLOATS = 16 * XPOSE_LD;

__device__ __forceinline__ v4f transpose_tile(v4f t, float* patch, Lane ln)
{
#pragma unroll
    for (int r = 0; r < 4; ++r) patch[(4 * ln.q + r) * XPOSE_LD + ln.n] = t[r];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    v4f o = *reinterpret_cast<const v4f*>(&patch[ln.n * XPOSE_LD + 4 * ln.q]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    return o;
}

// ---------------------------------------------------------------------------------------------
// Blocked 2x2 recursion above the leaves (paper Sec. 3.3, Eq. 7, lower-triangular reading):
//   inv [[A11, 0], [A21, A22]] = [[T11, 0], [-T22 A21 T11, T22]].
// Levels are unrolled over tile-block sizes h = 1, 2, ..., NB/2; at each level the pairs are
// independent.  A pair's left factor T22 is held in T orientation and its right factor T11 in
// N orientation, so both products are tn() calls on registers.  A block that will be the odd
// (left-factor) child of its parent is produced in T orientation, an even child in N.
//
// Result: Tt[tix(i, j)] for the lower tiles; final orientation given by result_is_T().
// ---------------------------------------------------------------------------------------------
template <int NB, bool ROOT_T>
__host__ __device__ constexpr bool result_is_T(int i, int j)
{
    return (NB == 1) ? false : ((j >= NB / 2) ? true : ((i < NB / 2) ? false : ROOT_T));
}

enum : int { LEAF_BLOCK_RECURSIVE = 0, LEAF_NEUMANN = 1, LEAF_FORWARD = 2, LEAF_NEUMANN32 = 3 };

template <int OP, int NB, class ASrc> __device__ __forceinline__ void neumann(const ASrc& A, v4f (&Xt)[NB * (NB + 1) / 2], Lane ln);
template <int OP, int NB, class ASrc, class IsT>
__device__ __forceinline__ void refine_once(const ASrc& A, v4f (&Tt)[NB * (NB + 1) / 2], IsT is_t, float* patch, Lane ln);

// The 32 x 32 diagonal block that starts at tile P, as a tile source of its own.
template <class ASrc> struct PairView {
    const ASrc& a;
    int P;
    template <bool TR> __device__ __forceinline__ v4f get(int i, int j) const { return a.template get<TR>(P + i, P + j); }
};

// A tile of A as a packed matrix-core operand.  Sources that already hold packed tiles say so by specialising
// PackedSource and providing operand<TR>(i, j); every other source has its fp32 tile packed here.
template <class ASrc> struct PackedSource {
    static constexpr bool value = false;
};
template <int OP, bool TR, class ASrc> __device__ __forceinline__ Opnd<OP> tile_operand(const ASrc& A, int i, int j)
{
    if constexpr (PackedSource<ASrc>::value)
        return A.template operand<TR>(i, j);
    else
        return pack<OP>(A.template get<TR>(i, j));
}

struct NoHook {
    __device__ __forceinline__ void operator()() const {}
};

// after_last_fetch: called in the last merge once its tiles of A have been fetched, i.e. when A is no longer needed
// (a source that builds its tiles from keys held in registers has those registers free from here on).
// leaves_out: if not null, receives the 16 x 16 diagonal blocks of the result in both orientations ([2 d] = N, [2 d + 1] = T).
template <int OP, int NB, bool ROOT_T, int LEAF, class ASrc, class Hook = NoHook>
__device__ __forceinline__ void block_recursive(const ASrc& A, v4f (&Tt)[NB * (NB + 1) / 2], float* patch, Lane ln, int leaf_r = 0,
                                                Hook after_last_fetch = Hook(), v4f* leaves_out = nullptr)
{
    v4f leafN[NB], leafT[NB];
    if constexpr (LEAF == LEAF_FORWARD) {
        leaves_forward_substitution<NB>(A, leafN, leafT, patch, ln);
    } else if constexpr (LEAF == LEAF_NEUMANN32) {
        // paper Alg. 2 with b0 = 32: Neumann product (four squarings) on every 32 x 32 diagonal block, leaf_r
        // refinement steps on it, and the merges below start at block size 32.  The product comes out in T
        // orientation; the block is brought to the orientation its parent expects (diagonal tiles to both).
        static_assert(NB >= 2, "b0 = 32 needs C >= 32");
#pragma unroll
        for (int p = 0; p < NB / 2; ++p) {
            const PairView<ASrc> pv{A, 2 * p};
            v4f X[3];
            neumann<OP, 2>(pv, X, ln);
#pragma unroll 1
            for (int s = 0; s < leaf_r; ++s) refine_once<OP, 2>(pv, X, [](int, int) { return true; }, patch, ln);
            const bool blockT = (2 == NB) ? ROOT_T : ((p & 1) != 0);
            leafT[2 * p] = X[tix(0, 0)];
            leafT[2 * p + 1] = X[tix(1, 1)];
            leafN[2 * p] = transpose_tile(X[tix(0, 0)], patch, ln);
            leafN[2 * p + 1] = transpose_tile(X[tix(1, 1)], patch, ln);
            Tt[tix(2 * p + 1, 2 * p)] = blockT ? X[tix(1, 0)] : transpose_tile(X[tix(1, 0)], patch, ln);
        }
    } else {
#pragma unroll
        for (int d = 0; d < NB; ++d) {
            const v4f LN = A.template get<false>(d, d), LT = A.template get<true>(d, d);
            if (LEAF == LEAF_BLOCK_RECURSIVE)
                leaf_block_recursive<OP>(LN, LT, leafN[d], leafT[d], ln);
            else
                leaf_neumann<OP>(LN, LT, leafN[d], leafT[d], ln, leaf_r);
        }
    }

#pragma unroll
    for (int h = (LEAF == LEAF_NEUMANN32 ? 2 : 1); h < NB; h *= 2) {
#pragma unroll
        for (int p = 0; p < NB / (2 * h); ++p) {
            const int lo = 2 * h * p, mid = lo + h, hi = lo + 2 * h;
            const bool blockT = (2 * h == NB) ? ROOT_T : ((p & 1) != 0);
            // packed operands of the two children
            constexpr int NH = (NB / 2) * (NB / 2 + 1) / 2 > 0 ? (NB / 2) * (NB / 2 + 1) / 2 : 1;
            Opnd<OP> t11[NH], t22[NH];
#pragma unroll
            for (int d = 0; d < h; ++d)
#pragma unroll
                for (int c = 0; c <= d; ++c) {
                    t11[tix(d, c)] = pack<OP>(d == c ? leafN[lo + d] : Tt[tix(lo + d, lo + c)]);
                    t22[tix(d, c)] = pack<OP>(d == c ? leafT[mid + d] : Tt[tix(mid + d, mid + c)]);
                }
            // off-diagonal tiles of A, fetched once: T orientation for an N block, N for a T block
            Opnd<OP> a21[(NB / 2) * (NB / 2) > 0 ? (NB / 2) * (NB / 2) : 1];
#pragma unroll
            for (int b = 0; b < h; ++b)
#pragma unroll
                for (int d = 0; d < h; ++d)
                    a21[b * h + d] = blockT ? tile_operand<OP, false>(A, mid + b, lo + d) : tile_operand<OP, true>(A, mid + b, lo + d);
            if (2 * h == NB) after_last_fetch();
            if (!blockT) {
                // W = -T22 (A21 T11), N orientation
#pragma unroll
                for (int c = 0; c < h; ++c) {
                    Opnd<OP> P[NB / 2 > 0 ? NB / 2 : 1];
#pragma unroll
                    for (int b = 0; b < h; ++b) {
                        v4f acc = zero4();
#pragma unroll
                        for (int d = c; d < h; ++d) acc = tn<OP>(a21[b * h + d], t11[tix(d, c)], acc);
                        P[b] = negated<OP>(pack<OP>(acc));  // the sign of -T22 (A21 T11)
                    }
#pragma unroll
                    for (int a = 0; a < h; ++a) {
                        v4f acc = zero4();
#pragma unroll
                        for (int b = 0; b <= a; ++b) acc = tn<OP>(t22[tix(a, b)], P[b], acc);
                        Tt[tix(mid + a, lo + c)] = acc;
                    }
                }
            } else {
                // W^T = -T11^T (A21^T T22^T), T orientation
#pragma unroll
                for (int a = 0; a < h; ++a) {
                    Opnd<OP> Q[NB / 2 > 0 ? NB / 2 : 1];
#pragma unroll
                    for (int d = 0; d < h; ++d) {
                        v4f acc = zero4();
#pragma unroll
                        for (int b = 0; b <= a; ++b) acc = tn<OP>(a21[b * h + d], t22[tix(a, b)], acc);
                        Q[d] = negated<OP>(pack<OP>(acc));
                    }
#pragma unroll
                    for (int c = 0; c < h; ++c) {
                        v4f acc = zero4();
#pragma unroll
                        for (int d = c; d < h; ++d) acc = tn<OP>(t11[tix(d, c)], Q[d], acc);
                        Tt[tix(mid + a, lo + c)] = acc;
                    }
                }
            }
            // bring the children to this block's orientation (leaves have both already)
            if (2 * h != NB) {
                const int clo = blockT ? lo : mid;  // child to convert: even child if T, odd child if N
#pragma unroll
                for (int d = 1; d < h; ++d)
#pragma unroll
                    for (int c = 0; c < d; ++c)
                        Tt[tix(clo + d, clo + c)] = transpose_tile(Tt[tix(clo + d, clo + c)], patch, ln);
            }
        }
    }
#pragma unroll
    for (int d = 0; d < NB; ++d) Tt[tix(d, d)] = result_is_T<NB, ROOT_T>(d, d) ? leafT[d] : leafN[d];
    if (leaves_out != nullptr) {
#pragma unroll
        for (int d = 0; d < NB; ++d) {
            leaves_out[2 * d] = leafN[d];
            leaves_out[2 * d + 1] = leafT[d];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Neumann product on the whole matrix (paper Alg. 5, Sec. 3.2):
//   X <- I - A, Y <- A;  log2(C/2) times:  Y <- Y Y;  X <- X + X Y.
// State: Y in both orientations, X in T orientation (X^T <- X^T + Y^T X^T is the literal update
// transposed).  The running power Y = A^p is structurally zero in tiles with 16 (i-j) + 15 < p;
// those tiles and the products through them are skipped.
// Result: Xt[tix(i, j)], every tile in T orientation.
// ---------------------------------------------------------------------------------------------
__host__ __device__ constexpr bool power_tile_nonzero(int d, int p) { return 16 * d + 15 >= p; }
__host__ __device__ constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

template <int OP, int NB, class ASrc>
__device__ __forceinline__ void neumann(const ASrc& A, v4f (&Xt)[NB * (NB + 1) / 2], Lane ln)
{
    constexpr int NT = NB * (NB + 1) / 2;
    Opnd<OP> Yn[NT], Yt[NT];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            const v4f an = A.template get<false>(i, j), at = A.template get<true>(i, j);
            Yn[tix(i, j)] = pack<OP>(an);
            Yt[tix(i, j)] = pack<OP>(at);
            v4f x;
#pragma unroll
            for (int r = 0; r < 4; ++r) x[r] = ((i == j && 4 * ln.q + r == ln.n) ? 1.f : 0.f) - at[r];
            Xt[tix(i, j)] = x;
        }
    constexpr int iters = ilog2(16 * NB / 2);  // log2(C / 2)
#pragma unroll
    for (int it = 0; it < iters; ++it) {
        const int p = 1 << it, pn = 2 << it;  // Y = A^p becomes A^pn
        const bool last = (it == iters - 1);
        v4f Nn[NT], Nt[NT];
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = 0; j <= i; ++j) {
                v4f accn = zero4(), acct = zero4();
                if (power_tile_nonzero(i - j, pn)) {
#pragma unroll
                    for (int k = j; k <= i; ++k)
                        if (power_tile_nonzero(i - k, p) && power_tile_nonzero(k - j, p)) {
                            accn = tn<OP>(Yt[tix(i, k)], Yn[tix(k, j)], accn);
                            if (!last) acct = tn<OP>(Yn[tix(k, j)], Yt[tix(i, k)], acct);
                        }
                }
                Nn[tix(i, j)] = accn;
                Nt[tix(i, j)] = acct;
            }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            Yn[t] = pack<OP>(Nn[t]);
            Yt[t] = pack<OP>(Nt[t]);
        }
        // X^T(i,j) += sum_k Y(k,j)^T X(i,k)^T ; ascending j keeps the old X(i,k), k >= j, intact
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            Opnd<OP> xo[NB];
#pragma unroll
            for (int k = 0; k <= i; ++k) xo[k] = pack<OP>(Xt[tix(i, k)]);
#pragma unroll
            for (int j = 0; j <= i; ++j) {
                v4f acc = Xt[tix(i, j)];
#pragma unroll
                for (int k = j; k <= i; ++k)
                    if (power_tile_nonzero(k - j, pn)) acc = tn<OP>(Yn[tix(k, j)], xo[k], acc);
                Xt[tix(i, j)] = acc;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Newton-Schulz iteration (paper Alg. 3, Eq. 8) for the matrix I + A:
//   X <- X0 = I / C;   n_iter times:  Y <- (I + A) X;   X <- 2 X - X Y.
// Every iterate is a polynomial in A, hence lower triangular: the same tile structure as above.
// State: X in both orientations (X Y needs X as a left factor, (I + A) X as a right factor).
// Result: Xt, every tile in T orientation.
// ---------------------------------------------------------------------------------------------
template <int OP, int NB, class ASrc>
__device__ __forceinline__ void newton_schulz(const ASrc& A, v4f (&Xt)[NB * (NB + 1) / 2], int n_iter, Lane ln)
{
    constexpr int NT = NB * (NB + 1) / 2;
    Opnd<OP> Lt[NT];
    v4f Xn[NT];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            Lt[tix(i, j)] = pack<OP>(A.template get<true>(i, j));
            v4f x;
#pragma unroll
            for (int r = 0; r < 4; ++r) x[r] = (i == j && 4 * ln.q + r == ln.n) ? 1.f / (16 * NB) : 0.f;
            Xn[tix(i, j)] = x;
            Xt[tix(i, j)] = x;
        }
#pragma unroll 1
    for (int it = 0; it < n_iter; ++it) {
        Opnd<OP> xn[NT], xt[NT], yn[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            xn[t] = pack<OP>(Xn[t]);
            xt[t] = pack<OP>(Xt[t]);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = 0; j <= i; ++j) {  // Y = X + A X
                v4f acc = Xn[tix(i, j)];
#pragma unroll
                for (int k = j; k <= i; ++k) acc = tn<OP>(Lt[tix(i, k)], xn[tix(k, j)], acc);
                yn[tix(i, j)] = pack<OP>(acc);
            }
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = 0; j <= i; ++j) {  // X <- 2 X - X Y, in both orientations
                v4f pn = zero4(), pt = zero4();
#pragma unroll
                for (int k = j; k <= i; ++k) {
                    pn = tn<OP>(xt[tix(i, k)], yn[tix(k, j)], pn);
                    pt = tn<OP>(yn[tix(k, j)], xt[tix(i, k)], pt);
                }
                Xn[tix(i, j)] = 2.f * Xn[tix(i, j)] - pn;
                Xt[tix(i, j)] = 2.f * Xt[tix(i, j)] - pt;
            }
    }
}

// ---------------------------------------------------------------------------------------------
// One step of iterative refinement (paper Alg. 6, Eq. 9, for the matrix I + A):
//   R <- I - Y (I + A);   X <- Y + R Y.
// Y comes in as the tiles Tt in the orientations is_t() reports; each tile is brought to both
// orientations (transpose through the LDS patch), then
//   R^T(i,j) = [i==j] I - Y^T(i,j) - sum_k A(k,j)^T Y(i,k)^T,     X^T(i,j) = Y^T(i,j) + sum_k Y(k,j)^T R(i,k)^T.
// Result: X in Tt, every tile in T orientation.  Operands are rounded to OP at each product; R and
// all sums stay fp32.
// ---------------------------------------------------------------------------------------------
template <int OP, int NB, class ASrc, class IsT>
__device__ __forceinline__ void refine_once(const ASrc& A, v4f (&Tt)[NB * (NB + 1) / 2], IsT is_t, float* patch, Lane ln)
{
    constexpr int NT = NB * (NB + 1) / 2;
    v4f Yt[NT];
    Opnd<OP> Yn[NT], Yto[NT];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            const v4f other = transpose_tile(Tt[tix(i, j)], patch, ln);
            const v4f n = is_t(i, j) ? other : Tt[tix(i, j)];
            Yt[tix(i, j)] = is_t(i, j) ? Tt[tix(i, j)] : other;
            Yn[tix(i, j)] = pack<OP>(n);
            Yto[tix(i, j)] = pack<OP>(Yt[tix(i, j)]);
        }
    Opnd<OP> An[NT], Rt[NT];
#pragma unroll
    for (int k = 0; k < NB; ++k)
#pragma unroll
        for (int j = 0; j <= k; ++j) An[tix(k, j)] = pack<OP>(A.template get<false>(k, j));
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            v4f acc = zero4();
#pragma unroll
            for (int k = j; k <= i; ++k) acc = tn<OP>(An[tix(k, j)], Yto[tix(i, k)], acc);
            v4f r;
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = ((i == j && 4 * ln.q + e == ln.n) ? 1.f : 0.f) - Yt[tix(i, j)][e] - acc[e];
            Rt[tix(i, j)] = pack<OP>(r);
        }
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            v4f acc = Yt[tix(i, j)];
#pragma unroll
            for (int k = j; k <= i; ++k) acc = tn<OP>(Yn[tix(k, j)], Rt[tix(i, k)], acc);
            Tt[tix(i, j)] = acc;
        }
}

}  // namespace triinv
