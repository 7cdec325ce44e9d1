// Instantiations of the apply-instead-of-store kernels (solve.hpp) for one (C = 16 * TRIINV_INST_NB,
// operand type TRIINV_INST_OP) pair: blocked and mixed recursion.
#include "dispatch.hpp"
#include "solve.hpp"
#if TRIINV_INST_NB == 8
#include "c128_kda_solve.hpp"
#endif

#ifndef TRIINV_INST_NB
#error "compile with -DTRIINV_INST_NB=1|2|4|8 -DTRIINV_INST_OP=0|1|2"
#endif

namespace triinv {

#define CAT_(a, b, c, d) a##b##c##d
#define CAT(a, b, c, d) CAT_(a, b, c, d)

constexpr int NB = TRIINV_INST_NB;
constexpr int OP = TRIINV_INST_OP;
constexpr int WPB = NB <= 4 ? 4 : 1;  // four adjacent heads per workgroup at C <= 64, as in the storing kernels

// X's first loads.  C <= 64: every tile of A is formed first and kept packed, which frees the keys' registers, then all of X
// is requested before the recursion starts.  C = 128: the loads are split around the recursion (forming all of A first and
// requesting X before the recursion measured 10 % slower there: 181 against 165 us on the stress workload).
constexpr int XPOS = NB <= 4 ? 1 : 3;

static RhsList rhs_of(const SolveArgs& a)
{
    RhsList l{};
    for (int k = 0; k < a.n_rhs && k < MAX_RHS; ++k) l.r[k] = RhsArgs{a.X[k], a.scale[k], a.W[k], a.d_x[k]};
    return l;
}

// The two-wavefront kernels at C = 128 and every kernel at C <= 64 address a right-hand side with 32-bit row offsets: C
// rows of H * d_x elements.
[[maybe_unused]] static bool rows_fit_32_bits(const SolveArgs& a)
{
    for (int k = 0; k < a.n_rhs; ++k)
        if ((int64_t)a.f.H * a.d_x[k] * (OP == OP_F32 ? 4 : 2) * (16 * NB) >= (1LL << 31)) return false;
    return true;
}

// Two right-hand sides per launch are built at C <= 64.
constexpr bool HAS_PAIR = NB <= 4;

template <int KD, int METHOD, int DKS> static int go_gdn(const SolveArgs& a)
{
    const GdnArgs& f = a.f;
#if TRIINV_INST_NB == 8
    // C = 128 on two wavefronts per chunk (c128_solve.hpp).  Two right-hand sides: split by columns, the inverse's tiles
    // published once per side.  One right-hand side: split by rows (whole 256-byte row pieces on both waves, four
    // workgroups per compute unit) with 16-bit operands (154 against 170 us on the stress workload for the one-wavefront
    // kernel below, 156 against 164 us with the mixed recursion, 249 against 255 us at d_x = 256), and where it is the
    // only kernel: 16-bit keys of d_k = 64 (the one-wavefront build of that case does not fit the register file without
    // spilling) and fp32 keys of d_k = 128 (one wavefront cannot hold a chunk's 256 registers of keys).  fp32 operands
    // keep the one-wavefront kernel otherwise (363 against 444 us).
    constexpr bool SINGLE_ON_TWO_WAVES = (KD != OP_F32 && DKS == 2) || (KD == OP_F32 && DKS == 8);
    constexpr bool SINGLE_BY_ROWS = SINGLE_ON_TWO_WAVES || OP != OP_F32;
    if (a.n_rhs == 2 || SINGLE_ON_TWO_WAVES) {
        if (!rows_fit_32_bits(a)) return 1;
    }
    if constexpr (SINGLE_BY_ROWS)
        if (a.n_rhs == 1 && rows_fit_32_bits(a))
            return f.g ? launch_kernel(f.dry, k_gdn_tri_solve_c128_rows<KD, OP, METHOD, DKS, false>, dim3((unsigned)f.n_mat), dim3(128), 0,
                                       f.stream, f.K, f.beta, f.g, rhs_of(a), f.n_chunk, f.map, f.H, f.d_k, f.iters)
                       : launch_kernel(f.dry, k_gdn_tri_solve_c128_rows<KD, OP, METHOD, DKS, true>, dim3((unsigned)f.n_mat), dim3(128), 0,
                                       f.stream, f.K, f.beta, f.g, rhs_of(a), f.n_chunk, f.map, f.H, f.d_k, f.iters);
    // (fp32 operands: the two sets of fp32 tiles take 93 KB of LDS, one workgroup per compute unit)
    if (a.n_rhs == 2)
        return f.g ? launch_kernel(f.dry, k_gdn_tri_solve_c128<KD, OP, METHOD, DKS, 2, false>, dim3((unsigned)f.n_mat), dim3(128), 0, f.stream,
                                   f.K, f.beta, f.g, rhs_of(a), f.n_chunk, f.map, f.H, f.d_k, f.iters)
                   : launch_kernel(f.dry, k_gdn_tri_solve_c128<KD, OP, METHOD, DKS, 2, true>, dim3((unsigned)f.n_mat), dim3(128), 0, f.stream,
                                   f.K, f.beta, f.g, rhs_of(a), f.n_chunk, f.map, f.H, f.d_k, f.iters);
    if constexpr (!SINGLE_ON_TWO_WAVES)
#endif
    {
    const dim3 grid((unsigned)((f.n_mat + WPB - 1) / WPB)), block(64 * WPB);
    if (a.n_rhs == 1) {
        return launch_kernel(f.dry, k_gdn_tri_solve<KD, OP, NB, METHOD, DKS, WPB, XPOS, 1>, grid, block, 0, f.stream, f.K, f.beta, f.g,
                           rhs_of(a), f.n_chunk, f.map, f.H, f.d_k, f.iters, WPB > 1 ? head_spread(f.H) : 0);
    }
    if constexpr (HAS_PAIR) {
        return launch_kernel(f.dry, k_gdn_tri_solve<KD, OP, NB, METHOD, DKS, WPB, XPOS, 2>, grid, block, 0, f.stream, f.K, f.beta, f.g,
                           rhs_of(a), f.n_chunk, f.map, f.H, f.d_k, f.iters, WPB > 1 ? head_spread(f.H) : 0);
    }
    return 1;
    }
    return 1;
}

template <int KD, int DKS> static int gdn_method(const SolveArgs& a)
{
    if (a.f.method == M_BLOCK) return go_gdn<KD, M_BLOCK, DKS>(a);
    if (a.f.method == M_MIXED) return go_gdn<KD, M_MIXED, DKS>(a);
    return 1;
}

template <int METHOD> static int go_kda(const SolveArgs& a)
{
    const GdnArgs& f = a.f;
#if TRIINV_INST_NB == 8
    // C = 128: one chunk per workgroup of two wavefronts (c128_kda_solve.hpp)
    if (!rows_fit_32_bits(a)) return 1;
    if (a.n_rhs == 1)
        return launch_kernel(f.dry, k_kda_tri_solve_c128<OP, METHOD, 1>, dim3((unsigned)f.n_mat), dim3(128), 0, f.stream, f.K, f.beta, f.g,
                             rhs_of(a), f.n_chunk, f.map, f.H, f.d_k, f.k_dt, f.iters);
    return launch_kernel(f.dry, k_kda_tri_solve_c128<OP, METHOD, 2>, dim3((unsigned)f.n_mat), dim3(128), 0, f.stream, f.K, f.beta, f.g,
                         rhs_of(a), f.n_chunk, f.map, f.H, f.d_k, f.k_dt, f.iters);
#else
    const dim3 grid((unsigned)((f.n_mat + WPB - 1) / WPB)), block(64 * WPB);
    if (a.n_rhs == 1) {
        return launch_kernel(f.dry, k_kda_tri_solve<OP, NB, METHOD, WPB, 1>, grid, block, 0, f.stream, f.K, f.beta, f.g, rhs_of(a), f.n_chunk,
                           f.map, f.H, f.d_k, f.k_dt, f.iters, WPB > 1 ? head_spread(f.H) : 0);
    }
    if constexpr (HAS_PAIR) {
        return launch_kernel(f.dry, k_kda_tri_solve<OP, NB, METHOD, WPB, 2>, grid, block, 0, f.stream, f.K, f.beta, f.g, rhs_of(a), f.n_chunk,
                           f.map, f.H, f.d_k, f.k_dt, f.iters, WPB > 1 ? head_spread(f.H) : 0);
    }
    return 1;
#endif
}

#if TRIINV_INST_NB <= 4
// Head dimensions other than 64 / 128 (scalar / no-gate kinds), C <= 64.
template <int KD, int METHOD> static int go_any_dk(const SolveArgs& a)
{
    const GdnArgs& f = a.f;
    const dim3 grid((unsigned)f.n_mat), block(64);
    if (a.n_rhs == 1)
        return launch_kernel(f.dry, k_gdn_any_dk_tri_solve<KD, OP, NB, METHOD, 1>, grid, block, 0, f.stream, f.K, f.beta, f.g, rhs_of(a), f.n_chunk,
                           f.map, f.H, f.d_k, f.iters);
    else
        return launch_kernel(f.dry, k_gdn_any_dk_tri_solve<KD, OP, NB, METHOD, 2>, grid, block, 0, f.stream, f.K, f.beta, f.g, rhs_of(a), f.n_chunk,
                             f.map, f.H, f.d_k, f.iters);
}

template <int KD> static int any_dk_method(const SolveArgs& a)
{
    if (a.f.method == M_BLOCK) return go_any_dk<KD, M_BLOCK>(a);
    if (a.f.method == M_MIXED) return go_any_dk<KD, M_MIXED>(a);
    return 1;
}
#endif

int CAT(launch_solve_nb, TRIINV_INST_NB, _op, TRIINV_INST_OP)(const SolveArgs& a)
{
    const GdnArgs& f = a.f;
    if (f.refine) return 1;
    if (a.n_rhs < 1 || a.n_rhs > MAX_RHS) return 1;
    if (NB <= 4 && !rows_fit_32_bits(a)) return 1;  // (H * d_x beyond 8 million elements)
    if (f.gate == G_CHANNEL) {
        if (f.method == M_BLOCK) return go_kda<M_BLOCK>(a);
        if (f.method == M_MIXED) return go_kda<M_MIXED>(a);
        return 1;
    }
    if (f.k_dt == OP_F32) {
        if (f.d_k == 64) return gdn_method<OP_F32, 4>(a);
#if TRIINV_INST_NB <= 4
        if (f.d_k == 128) return gdn_method<OP_F32, 8>(a);
#else
        if (f.d_k == 128) return gdn_method<OP_F32, 8>(a);  // (two wavefronts per chunk, see go_gdn)
#endif
    } else if (f.k_dt == OP_BF16) {
        if (f.d_k == 64) return gdn_method<OP_BF16, 2>(a);
        if (f.d_k == 128) return gdn_method<OP_BF16, 4>(a);
    } else {
        if (f.d_k == 64) return gdn_method<OP_F16, 2>(a);
        if (f.d_k == 128) return gdn_method<OP_F16, 4>(a);
    }
#if TRIINV_INST_NB <= 4
    return f.k_dt == OP_F32 ? any_dk_method<OP_F32>(a) : f.k_dt == OP_BF16 ? any_dk_method<OP_BF16>(a) : any_dk_method<OP_F16>(a);
#else
    return 1;
#endif
}

}  // namespace triinv
