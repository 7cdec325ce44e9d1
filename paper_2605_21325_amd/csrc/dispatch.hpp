// Host-side launch table: one launcher per (C, operand type) pair, each compiled in its own
// translation unit (inst.hip with TRIINV_INST_NB / TRIINV_INST_OP set) so the build parallelises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <tuple>
#include <utility>
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
    bool dry = false;  // only report whether the combination is built; launch nothing
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
    bool dry = false;  // only report whether the combination is built; launch nothing
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

// Launcher return codes.
enum : int { LAUNCHED = 0, NOT_BUILT = 1, LAUNCH_FAILED = 2 };

// One kernel launch whose own status is returned (the runtime's sticky per-thread error state, which may hold an
// unrelated earlier error of the caller, is neither read nor cleared).  The arguments are converted to the kernel's
// exact parameter types first.  dry: report LAUNCHED without launching.
template <class... KArgs, class... Args, size_t... I>
inline int launch_kernel_impl(void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t stream,
                              std::index_sequence<I...>, Args&&... args)
{
    std::tuple<KArgs...> vals{static_cast<KArgs>(std::forward<Args>(args))...};
    void* ptrs[sizeof...(KArgs)] = {(void*)&std::get<I>(vals)...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, stream) == hipSuccess ? LAUNCHED : LAUNCH_FAILED;
}
template <class... KArgs, class... Args>
inline int launch_kernel(bool dry, void (*kernel)(KArgs...), dim3 grid, dim3 block, unsigned lds_bytes, hipStream_t stream, Args&&... args)
{
    static_assert(sizeof...(KArgs) == sizeof...(Args), "one argument per kernel parameter");
    if (dry) return LAUNCHED;
    return launch_kernel_impl(kernel, grid, block, lds_bytes, stream, std::index_sequence_for<KArgs...>{}, std::forward<Args>(args)...);
}

// Every launcher returns one of the codes above.
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
