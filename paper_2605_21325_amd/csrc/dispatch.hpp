// Host-side launch table: one launcher per (C, operand type) pair, each compiled in its own
// translation unit (inst.hip with TRIINV_INST_NB / TRIINV_INST_OP set) so the build parallelises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "chunk_map.hpp"

namespace triinv {

struct TriInvArgs {
    const void* A;
    float* T;
    int64_t n_mat;
    int in_dt;
    int method;
    hipStream_t stream;
    bool refine;  // one iterative-refinement step after the method
    int iters;    // Newton-Schulz iteration count; for the mixed recursion: refinement steps on the 16 x 16 blocks
    int out_dt;   // element type of T: 0 fp32, 1 fp16, 2 bf16
    bool shuffle; // forward substitution: broadcast A by wavefront shuffles (C = 64)
};

struct GdnArgs {
    const void* K;
    const float* beta;
    const float* g;  // null for the no-gate kind
    float* T;
    int64_t n_mat;
    int64_t n_chunk;  // total number of chunks
    ChunkMap map;     // where each chunk's tokens are
    int H;
    int d_k;
    int k_dt;
    int gate;
    int method;
    hipStream_t stream;
    bool refine;
    int iters;
    int out_dt;
};

// gdn_chunk_tri_solve: the fused arguments (T unused) plus the right-hand sides.
struct SolveArgs {
    GdnArgs f;
    int n_rhs;             // 1 or 2 right-hand sides sharing the inverse
    const void* X[2];      // [tokens][H][d_x], element type = operand type
    const float* scale[2]; // [tokens][H] or null
    void* W[2];            // [tokens][H][d_x]
    int d_x[2];
};

// The chunk stride of the few-heads workgroup map of the fused kernels (0 = the many-heads map): see fused_matrix_index.
inline int head_spread(int H) { return H >= 8 ? 0 : (H >= 4 ? 1 : 4 / H); }

// Return 0, or 1 when the combination is not instantiated; launch errors are left in hipGetLastError.
#define TRIINV_DECL(NB, OP)                                  \
    int launch_tri_inv_nb##NB##_op##OP(const TriInvArgs& a); \
    int launch_gdn_nb##NB##_op##OP(const GdnArgs& a);        \
    int launch_gdn_nb##NB##_op##OP##_fwd(const GdnArgs& a);
TRIINV_DECL(1, 0)
TRIINV_DECL(1, 1)
TRIINV_DECL(1, 2)
TRIINV_DECL(2, 0)
TRIINV_DECL(2, 1)
TRIINV_DECL(2, 2)
TRIINV_DECL(4, 0)
TRIINV_DECL(4, 1)
TRIINV_DECL(4, 2)
TRIINV_DECL(8, 0)
TRIINV_DECL(8, 1)
TRIINV_DECL(8, 2)
#undef TRIINV_DECL
#define TRIINV_DECL_SOLVE(NB) \
    int launch_solve_nb##NB##_op0(const SolveArgs& a); \
    int launch_solve_nb##NB##_op1(const SolveArgs& a); \
    int launch_solve_nb##NB##_op2(const SolveArgs& a);
TRIINV_DECL_SOLVE(1)
TRIINV_DECL_SOLVE(2)
TRIINV_DECL_SOLVE(4)
TRIINV_DECL_SOLVE(8)
#undef TRIINV_DECL_SOLVE
int launch_tri_inv_nb1_op0_fwd(const TriInvArgs& a);
int launch_tri_inv_nb2_op0_fwd(const TriInvArgs& a);
int launch_tri_inv_nb4_op0_fwd(const TriInvArgs& a);
int launch_tri_inv_nb8_op0_fwd(const TriInvArgs& a);

}  // namespace triinv
