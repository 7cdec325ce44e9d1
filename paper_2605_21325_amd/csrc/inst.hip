// Kernel instantiations for one (C = 16 * TRIINV_INST_NB, operand type TRIINV_INST_OP) pair: the
// matrix-core methods, or -- with TRIINV_INST_FWD=1 -- forward substitution alone (its fully
// unrolled code is the slowest to compile, so it gets translation units of its own; the gated
// keys of the per-channel kernel still use TRIINV_INST_OP as their operand type).
#include "dispatch.hpp"
#include "kernels.hpp"
#if TRIINV_INST_NB == 8 && !TRIINV_INST_FWD
#include "c128.hpp"
#include "c128_kda.hpp"
#include "kda128.hpp"
#endif

#ifndef TRIINV_INST_NB
#error "compile with -DTRIINV_INST_NB=1|2|4|8 -DTRIINV_INST_OP=0|1|2 [-DTRIINV_INST_FWD=1]"
#endif
#ifndef TRIINV_INST_FWD
#define TRIINV_INST_FWD 0
#endif

namespace triinv {

#define CAT_(a, b, c, d, e) a##b##c##d##e
#define CAT(a, b, c, d, e) CAT_(a, b, c, d, e)
#if TRIINV_INST_FWD
#define SUFFIX _fwd
#else
#define SUFFIX
#endif

constexpr int NB = TRIINV_INST_NB;
constexpr int OP = TRIINV_INST_OP;

template <int METHOD, bool REFINE = false> static int go_tri(const TriInvArgs& a)
{
    return launch_kernel(a.dry, k_tri_inv<OP, NB, METHOD, REFINE>, dim3((unsigned)a.n_mat), dim3(64), 0, a.stream, a.A, a.T, a.n_mat,
                       a.in_dt, a.iters, a.out_dt);
}

// Fused matrix-core kernels at C <= 64 run four matrices (adjacent heads) per workgroup.
constexpr int WPB = (TRIINV_INST_NB <= 4 && !TRIINV_INST_FWD) ? 4 : 1;

// The refinement step is built for the blocked and the mixed recursion at C <= 64.
constexpr bool HAS_REFINE = (TRIINV_INST_NB <= 4) && !TRIINV_INST_FWD;

#if !(TRIINV_INST_FWD && TRIINV_INST_OP != 0)
int CAT(launch_tri_inv_nb, TRIINV_INST_NB, _op, TRIINV_INST_OP, SUFFIX)(const TriInvArgs& a)
{
    if (a.refine) {
        if constexpr (HAS_REFINE) {
            switch (a.method) {
            case M_BLOCK: return go_tri<M_BLOCK, true>(a);
            case M_MIXED: return go_tri<M_MIXED, true>(a);
            case M_BLOCK_DIRECT: return go_tri<M_BLOCK_DIRECT, true>(a);
            case M_NEUMANN: return go_tri<M_NEUMANN, true>(a);
            case M_NEWTON_SCHULZ: return go_tri<M_NEWTON_SCHULZ, true>(a);
#if TRIINV_INST_NB >= 2 && TRIINV_INST_NB <= 4
            case M_MIXED32: return go_tri<M_MIXED32, true>(a);
#endif
            default: return 1;
            }
        }
#if TRIINV_INST_NB == 8 && !TRIINV_INST_FWD
        // C = 128: the method as usual, then the refinement step as a second pass over T, in place (fp32 result only)
        if (a.out_dt == OP_F32) {
            TriInvArgs first = a;
            first.refine = false;
            if (const int rc = CAT(launch_tri_inv_nb, TRIINV_INST_NB, _op, TRIINV_INST_OP, SUFFIX)(first)) return rc;
            return launch_kernel(a.dry, k_tri_inv_refine128<OP>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.A, a.T, a.n_mat, a.in_dt);
        }
#endif
        return 1;
    }
    switch (a.method) {
#if TRIINV_INST_FWD
    case M_FWD:
        if (a.shuffle) {
#if TRIINV_INST_NB == 4
            return launch_kernel(a.dry, k_tri_inv_fwd_shuffle64<0>, dim3((unsigned)a.n_mat), dim3(64), 0, a.stream, a.A, a.T, a.n_mat, a.in_dt);
#else
            return 1;  // the shuffle variant is built at C = 64
#endif
        }
        return go_tri<M_FWD>(a);
#else
    case M_BLOCK: return go_tri<M_BLOCK>(a);
    case M_MIXED: return go_tri<M_MIXED>(a);
#if TRIINV_INST_NB >= 2
    case M_MIXED32: return go_tri<M_MIXED32>(a);
#endif
    case M_BLOCK_DIRECT: return go_tri<M_BLOCK_DIRECT>(a);
    case M_NEWTON_SCHULZ:
#if TRIINV_INST_NB <= 4
        return go_tri<M_NEWTON_SCHULZ>(a);
#else   // X in both orientations does not fit one wave's registers at C = 128: four waves, X and Y in LDS
        return launch_kernel(a.dry, k_tri_inv_ns128<OP>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.A, a.T, a.n_mat, a.in_dt, a.iters, a.out_dt);
#endif
    case M_NEUMANN:
#if TRIINV_INST_NB <= 4
        return go_tri<M_NEUMANN>(a);
#else   // C = 128: the one-wave register version would spill; a workgroup of four waves shares Y in LDS
        return launch_kernel(a.dry, k_tri_inv_neumann128<OP>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.A, a.T, a.n_mat, a.in_dt, a.out_dt);
#endif
#endif
    default: return 1;
    }
}

#endif

// Unused dynamic LDS that keeps a compute unit (160 KB of LDS) at two workgroups = two wavefronts per
// SIMD for the 16-bit-operand recursions at C = 64.  Those kernels are bound by the memory system,
// not by latency: with more wavefronts resident they measured 2-4 % slower (more requests queued at
// the memory controllers, none served sooner).
template <int METHOD> constexpr unsigned occupancy_pad_bytes()
{
    return (NB == 4 && WPB == 4 && OP != OP_F32 && (METHOD == M_BLOCK || METHOD == M_MIXED || METHOD == M_MIXED32 || METHOD == M_BLOCK_DIRECT)) ? 24576u : 0u;
}

template <int KD, int METHOD, int DKS, bool REFINE = false> static int go_gdn(const GdnArgs& a)
{
#if TRIINV_INST_NB == 8 && !TRIINV_INST_FWD
    // C = 128, the recursions with 16-bit operands: one matrix per workgroup of two wavefronts (c128.hpp).  fp32 operands
    // keep one wavefront per matrix: their four-instruction tile products make the kernel matrix-core bound, and the
    // exchange of fp32 tiles through LDS costs more than the second wavefront returns (250 against 226 us on the stress workload).
    if constexpr (!REFINE && OP != OP_F32 && (METHOD == M_BLOCK || METHOD == M_MIXED || METHOD == M_MIXED32 || METHOD == M_BLOCK_DIRECT))
        return a.g ? launch_kernel(a.dry, k_gdn_tri_inv_c128<KD, OP, METHOD, DKS, false>, dim3((unsigned)a.n_mat), dim3(128), 0, a.stream, a.K,
                                   a.beta, a.g, a.T, a.n_chunk, a.map, a.H, a.d_k, a.iters, a.out_dt)
                   : launch_kernel(a.dry, k_gdn_tri_inv_c128<KD, OP, METHOD, DKS, true>, dim3((unsigned)a.n_mat), dim3(128), 0, a.stream, a.K,
                                   a.beta, a.g, a.T, a.n_chunk, a.map, a.H, a.d_k, a.iters, a.out_dt);
    else
#endif
        return launch_kernel(a.dry, k_gdn_tri_inv<KD, OP, NB, METHOD, DKS, REFINE, WPB>, dim3((unsigned)((a.n_mat + WPB - 1) / WPB)),
                             dim3(64 * WPB), occupancy_pad_bytes<METHOD>(), a.stream, a.K, a.beta, a.g, a.T, a.n_chunk, a.map, a.H, a.d_k,
                             a.iters, a.out_dt, WPB > 1 ? head_spread(a.H) : 0);
}

template <int KD, int DKS> static int gdn_method(const GdnArgs& a)
{
    if (a.refine) {
        if constexpr (HAS_REFINE) {
            switch (a.method) {
            case M_BLOCK: return go_gdn<KD, M_BLOCK, DKS, true>(a);
            case M_MIXED: return go_gdn<KD, M_MIXED, DKS, true>(a);
            case M_BLOCK_DIRECT: return go_gdn<KD, M_BLOCK_DIRECT, DKS, true>(a);
            case M_NEUMANN: return go_gdn<KD, M_NEUMANN, DKS, true>(a);
            case M_NEWTON_SCHULZ: return go_gdn<KD, M_NEWTON_SCHULZ, DKS, true>(a);
#if TRIINV_INST_NB >= 2 && TRIINV_INST_NB <= 4
            case M_MIXED32: return go_gdn<KD, M_MIXED32, DKS, true>(a);
#endif
            default: return 1;
            }
        }
#if TRIINV_INST_NB == 8 && !TRIINV_INST_FWD
        if (a.out_dt == OP_F32) {
            GdnArgs first = a;
            first.refine = false;
            if (const int rc = gdn_method<KD, DKS>(first)) return rc;
            return launch_kernel(a.dry, k_gdn_tri_inv_refine128<KD, OP, DKS>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.K,
                               a.beta, a.g, a.T, a.n_chunk, a.map, a.H, a.d_k);
        }
#endif
        return 1;
    }
    switch (a.method) {
#if TRIINV_INST_FWD
    case M_FWD: return go_gdn<KD, M_FWD, DKS>(a);
#else
    case M_BUILD_A: return go_gdn<KD, M_BUILD_A, DKS>(a);
    case M_BLOCK: return go_gdn<KD, M_BLOCK, DKS>(a);
    case M_MIXED: return go_gdn<KD, M_MIXED, DKS>(a);
#if TRIINV_INST_NB >= 2
    case M_MIXED32: return go_gdn<KD, M_MIXED32, DKS>(a);
#endif
    case M_BLOCK_DIRECT: return go_gdn<KD, M_BLOCK_DIRECT, DKS>(a);
    case M_NEWTON_SCHULZ:
#if TRIINV_INST_NB <= 4
        return go_gdn<KD, M_NEWTON_SCHULZ, DKS>(a);
#else
        return launch_kernel(a.dry, k_gdn_tri_inv_ns128<KD, OP, DKS>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.K, a.beta,
                           a.g, a.T, a.n_chunk, a.map, a.H, a.d_k, a.iters, a.out_dt);
#endif
    case M_NEUMANN:
#if TRIINV_INST_NB <= 4
        return go_gdn<KD, M_NEUMANN, DKS>(a);
#else
        return launch_kernel(a.dry, k_gdn_tri_inv_neumann128<KD, OP, DKS>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.K,
                           a.beta, a.g, a.T, a.n_chunk, a.map, a.H, a.d_k, a.out_dt);
#endif
#endif
    default: return 1;
    }
}

template <int METHOD, bool REFINE = false> static int go_kda(const GdnArgs& a)
{
#if TRIINV_INST_NB == 8 && !TRIINV_INST_FWD
    // C = 128, the recursions: one matrix per workgroup of two wavefronts (c128_kda.hpp)
    if constexpr (!REFINE && (METHOD == M_BLOCK || METHOD == M_MIXED || METHOD == M_MIXED32 || METHOD == M_BLOCK_DIRECT))
        return launch_kernel(a.dry, k_kda_tri_inv_c128<OP, METHOD>, dim3((unsigned)a.n_mat), dim3(128), 0, a.stream, a.K, a.beta, a.g, a.T,
                             a.n_chunk, a.map, a.H, a.d_k, a.k_dt, a.iters, a.out_dt);
    else
#endif
        return launch_kernel(a.dry, k_kda_tri_inv<OP, NB, METHOD, WPB, REFINE>, dim3((unsigned)((a.n_mat + WPB - 1) / WPB)), dim3(64 * WPB), 0,
                             a.stream, a.K, a.beta, a.g, a.T, a.n_chunk, a.map, a.H, a.d_k, a.k_dt, a.iters, a.out_dt,
                             WPB > 1 ? head_spread(a.H) : 0);
}

static int kda_method(const GdnArgs& a)
{
    if (a.refine) {
        if constexpr (HAS_REFINE) {
            switch (a.method) {
            case M_BLOCK: return go_kda<M_BLOCK, true>(a);
            case M_MIXED: return go_kda<M_MIXED, true>(a);
            case M_BLOCK_DIRECT: return go_kda<M_BLOCK_DIRECT, true>(a);
            case M_NEUMANN: return go_kda<M_NEUMANN, true>(a);
            case M_NEWTON_SCHULZ: return go_kda<M_NEWTON_SCHULZ, true>(a);
#if TRIINV_INST_NB >= 2 && TRIINV_INST_NB <= 4
            case M_MIXED32: return go_kda<M_MIXED32, true>(a);
#endif
            default: return 1;
            }
        }
#if TRIINV_INST_NB == 8 && !TRIINV_INST_FWD
        // C = 128: the method as usual, then the refinement step as a second pass over T, in place (fp32 result only)
        if (a.out_dt == OP_F32) {
            GdnArgs first = a;
            first.refine = false;
            if (const int rc = kda_method(first)) return rc;
            return launch_kernel(a.dry, k_kda_tri_inv_refine128<OP>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.K, a.beta, a.g, a.T,
                                 a.n_chunk, a.map, a.H, a.d_k, a.k_dt);
        }
#endif
        return 1;
    }
    switch (a.method) {
#if TRIINV_INST_FWD
    case M_FWD: return go_kda<M_FWD>(a);
#else
    case M_BUILD_A: return go_kda<M_BUILD_A>(a);
    case M_BLOCK: return go_kda<M_BLOCK>(a);
    case M_MIXED: return go_kda<M_MIXED>(a);
#if TRIINV_INST_NB >= 2
    case M_MIXED32: return go_kda<M_MIXED32>(a);
#endif
    case M_BLOCK_DIRECT: return go_kda<M_BLOCK_DIRECT>(a);
#if TRIINV_INST_NB <= 4
    case M_NEWTON_SCHULZ: return go_kda<M_NEWTON_SCHULZ>(a);
    case M_NEUMANN: return go_kda<M_NEUMANN>(a);
#else
    // C = 128: one matrix per workgroup of four wavefronts that build A together (kda128.hpp)
    case M_NEWTON_SCHULZ:
        return launch_kernel(a.dry, k_kda_tri_inv_ns128<OP>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.K, a.beta, a.g, a.T, a.n_chunk,
                             a.map, a.H, a.d_k, a.k_dt, a.iters, a.out_dt);
    case M_NEUMANN:
        return launch_kernel(a.dry, k_kda_tri_inv_neumann128<OP>, dim3((unsigned)a.n_mat), dim3(256), 0, a.stream, a.K, a.beta, a.g, a.T,
                             a.n_chunk, a.map, a.H, a.d_k, a.k_dt, a.out_dt);
#endif
#endif
    default: return 1;
    }
}

// Head dimensions other than 64 / 128: every method at C <= 64; forward substitution, blocked recursion and blocked
// recursion from directly solved blocks at C = 128.
template <int KD, int METHOD> static int go_any_dk(const GdnArgs& a)
{
    return launch_kernel(a.dry, k_gdn_any_dk_tri_inv<KD, OP, NB, METHOD>, dim3((unsigned)a.n_mat), dim3(64), 0, a.stream, a.K, a.beta,
                       a.g, a.T, a.n_chunk, a.map, a.H, a.d_k, a.iters, a.out_dt);
}

template <int KD> static int any_dk_method(const GdnArgs& a)
{
    if (a.refine) return 1;
    switch (a.method) {
#if TRIINV_INST_FWD
    case M_FWD: return go_any_dk<KD, M_FWD>(a);
#else
    case M_BUILD_A: return go_any_dk<KD, M_BUILD_A>(a);
    case M_BLOCK: return go_any_dk<KD, M_BLOCK>(a);
    case M_BLOCK_DIRECT: return go_any_dk<KD, M_BLOCK_DIRECT>(a);
#if TRIINV_INST_NB <= 4
    // every tile of A in registers: the whole-matrix methods fit up to C = 64 (C = 128 takes the two-launch path)
    case M_MIXED: return go_any_dk<KD, M_MIXED>(a);
#if TRIINV_INST_NB >= 2
    case M_MIXED32: return go_any_dk<KD, M_MIXED32>(a);
#endif
    case M_NEUMANN: return go_any_dk<KD, M_NEUMANN>(a);
    case M_NEWTON_SCHULZ: return go_any_dk<KD, M_NEWTON_SCHULZ>(a);
#endif
#endif
    default: return 1;
    }
}

int CAT(launch_gdn_nb, TRIINV_INST_NB, _op, TRIINV_INST_OP, SUFFIX)(const GdnArgs& a)
{
    if (a.gate == G_CHANNEL) return kda_method(a);
#if TRIINV_INST_FWD && TRIINV_INST_OP != 0
    return 1;
#else
    if (a.k_dt == OP_F32) {
        if (a.d_k == 64) return gdn_method<OP_F32, 4>(a);
#if TRIINV_INST_NB <= 4
        if (a.d_k == 128) return gdn_method<OP_F32, 8>(a);
#elif !TRIINV_INST_FWD
        // C = 128 with 128 fp32 channels: on one wavefront the chunk's keys alone would take 256 registers per lane.  The
        // two-wavefront recursions (16-bit operands) hold half of them each; everything else runs the channel loop below
        // (keys consumed 32 channels at a time) like the other head dimensions
        if constexpr (OP != OP_F32) {
            if (a.d_k == 128 && !a.refine) {
                switch (a.method) {
                case M_BLOCK: return go_gdn<OP_F32, M_BLOCK, 8>(a);
                case M_MIXED: return go_gdn<OP_F32, M_MIXED, 8>(a);
                case M_MIXED32: return go_gdn<OP_F32, M_MIXED32, 8>(a);
                case M_BLOCK_DIRECT: return go_gdn<OP_F32, M_BLOCK_DIRECT, 8>(a);
                default: break;
                }
            }
        }
#endif
    } else if (a.k_dt == OP_BF16) {
        if (a.d_k == 64) return gdn_method<OP_BF16, 2>(a);
        if (a.d_k == 128) return gdn_method<OP_BF16, 4>(a);
    } else {
        if (a.d_k == 64) return gdn_method<OP_F16, 2>(a);
        if (a.d_k == 128) return gdn_method<OP_F16, 4>(a);
    }
    return a.k_dt == OP_F32 ? any_dk_method<OP_F32>(a) : a.k_dt == OP_BF16 ? any_dk_method<OP_BF16>(a) : any_dk_method<OP_F16>(a);
#endif
}

}  // namespace triinv
