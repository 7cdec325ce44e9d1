// C-ABI of the library (see include/triinv.h): argument validation on the host, then dispatch
// to the kernel instantiation for (C, operand type, method).  No allocation, no synchronisation.
#include "../../include/triinv.h"
#include "dispatch.hpp"

namespace {

using namespace triinv;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool overlap(const void* a, uint64_t na, const void* b, uint64_t nb)
{
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

bool dtype_ok(int d) { return d == TRIINV_F32 || d == TRIINV_F16 || d == TRIINV_BF16; }
bool chunk_size_ok(int C) { return C == 16 || C == 32 || C == 64 || C == 128; }
bool method_ok(int m) { return m >= TRIINV_FWD_SUBST && m <= TRIINV_MIXED_B32; }

constexpr uint32_t KNOWN_FLAGS = TRIINV_FLAG_REFINE1 | TRIINV_FLAG_OUT_F16 | TRIINV_FLAG_OUT_BF16 | TRIINV_FLAG_FWD_SHUFFLE | 0xff00u | 0x70000u;

int ns_iterations(uint32_t flags, int C)
{
    const int n = (int)((flags >> 8) & 0xffu);
    return n ? n : (C == 16 ? 8 : C == 32 ? 10 : C == 64 ? 12 : 14);  // 2 log2 C (paper Sec. 3.5; 12 at C = 64, Sec. 4.2)
}
// The run-time count a method takes: Newton-Schulz iterations, or the refinement steps the mixed
// recursion applies to its 16 x 16 blocks (paper Alg. 2's r; default 1, the step the paper finds
// necessary and sufficient for the mixed recursion to reach the accuracy of the stable methods, Sec. 4.1).
int method_count(int method, uint32_t flags, int C)
{
    if (method == TRIINV_MIXED || method == TRIINV_MIXED_B32) {
        const int code = (int)((flags >> 16) & 7u);
        return code ? code - 1 : 1;
    }
    return ns_iterations(flags, C);
}
uint64_t esize(int d) { return d == TRIINV_F32 ? 4 : 2; }

// Element type of T asked for in flags; -1 when both 16-bit types are asked for at once.
int out_dtype(uint32_t flags)
{
    const bool h = (flags & TRIINV_FLAG_OUT_F16) != 0, b = (flags & TRIINV_FLAG_OUT_BF16) != 0;
    return (h && b) ? -1 : h ? TRIINV_F16 : b ? TRIINV_BF16 : TRIINV_F32;
}

// Launcher code -> status.  The launch's own return value is used; the runtime's sticky error state is left alone.
int finish(int launcher_code)
{
    return launcher_code == LAUNCHED ? TRIINV_OK : launcher_code == NOT_BUILT ? TRIINV_ERR_UNSUPPORTED : TRIINV_ERR_LAUNCH;
}

int pick_fused(const GdnArgs& a, int C, int op_dtype)
{
#define TRIINV_PICK_OP(NBV, SUFFIX) \
    (op_dtype == TRIINV_F32 ? launch_gdn_nb##NBV##_op0##SUFFIX(a) : op_dtype == TRIINV_F16 ? launch_gdn_nb##NBV##_op1##SUFFIX(a) : launch_gdn_nb##NBV##_op2##SUFFIX(a))
    if (a.method == TRIINV_FWD_SUBST && a.refine) return 1;
    if (a.method == TRIINV_FWD_SUBST)
        return C == 16 ? TRIINV_PICK_OP(1, _fwd) : C == 32 ? TRIINV_PICK_OP(2, _fwd) : C == 64 ? TRIINV_PICK_OP(4, _fwd) : TRIINV_PICK_OP(8, _fwd);
    return C == 16 ? TRIINV_PICK_OP(1, ) : C == 32 ? TRIINV_PICK_OP(2, ) : C == 64 ? TRIINV_PICK_OP(4, ) : TRIINV_PICK_OP(8, );
#undef TRIINV_PICK_OP
}

int pick_tri_inv(const TriInvArgs& a, int C, int op_dtype)
{
#define TRIINV_PICK_OP(NBV) \
    (op_dtype == TRIINV_F32 ? launch_tri_inv_nb##NBV##_op0(a) : op_dtype == TRIINV_F16 ? launch_tri_inv_nb##NBV##_op1(a) : launch_tri_inv_nb##NBV##_op2(a))
    if (a.method == TRIINV_FWD_SUBST)
        return a.refine ? 1
               : C == 16 ? launch_tri_inv_nb1_op0_fwd(a)
               : C == 32 ? launch_tri_inv_nb2_op0_fwd(a)
               : C == 64 ? launch_tri_inv_nb4_op0_fwd(a)
                         : launch_tri_inv_nb8_op0_fwd(a);
    return C == 16 ? TRIINV_PICK_OP(1) : C == 32 ? TRIINV_PICK_OP(2) : C == 64 ? TRIINV_PICK_OP(4) : TRIINV_PICK_OP(8);
#undef TRIINV_PICK_OP
}

// Shared tail of the fused entry points: everything but the token layout has been validated.
// A matrix-product method that has no fused kernel for this gate kind / head dimension / chunk size runs as two
// launches instead: the chunk matrices are written into T as fp32 (the build kernel every combination has), then the
// standalone kernel of the method inverts them in place.  In place is safe for those kernels: a wavefront stores rows of
// T only after it has fetched every tile of A in those rows (each stored row depends on all of them), and in the
// four-wavefront C = 128 kernels a wavefront fetches, before the first barrier, exactly the tile rows it later stores.
// The values of A are the fp32 tiles a fused kernel would hold in registers, so the result is the same.  Forward
// substitution (always fused), the refinement flag (needs A and T side by side) and a 16-bit result (T must hold an
// fp32 A) are not composed.
int launch_fused(const GdnArgs& a, int C, int op_dtype)
{
    int nb = pick_fused(a, C, op_dtype);
    if (nb == NOT_BUILT && !a.refine && a.out_dt == TRIINV_F32 && a.method != TRIINV_FWD_SUBST && a.method != 100 /* M_BUILD_A */) {
        GdnArgs b = a;
        b.method = 100;
        const int b_op = a.gate == TRIINV_GATE_PER_CHANNEL ? op_dtype : TRIINV_F32;
        TriInvArgs t{a.T, a.T, a.n_mat, TRIINV_F32, a.method, a.stream, false, a.iters, TRIINV_F32, false};
        // both halves must be built before the first one is launched: a failing call does no GPU work
        b.dry = t.dry = true;
        if (pick_fused(b, C, b_op) != LAUNCHED || pick_tri_inv(t, C, op_dtype) != LAUNCHED) return TRIINV_ERR_UNSUPPORTED;
        b.dry = t.dry = false;
        nb = pick_fused(b, C, b_op);
        if (nb == LAUNCHED) nb = pick_tri_inv(t, C, op_dtype);
    }
    return finish(nb);
}

// Checks common to both token layouts.  n_tok = number of (token, head) pairs, n_mat = matrices to write.
int check_fused(const void* K, const float* beta, const float* g, float* T, uint64_t n_tok, int64_t n_mat, int H, int d_k,
                       int C, int k_dtype, int gate_kind, int method, uint32_t flags)
{
    const int out_dt = out_dtype(flags);
    if (out_dt < 0) return TRIINV_ERR_BAD_DTYPE;
    const bool need_g = gate_kind != TRIINV_GATE_NONE;
    if (!K || !beta || !T || (need_g && !g)) return TRIINV_ERR_NULL;
    if (!aligned16(K) || !aligned16(beta) || !aligned16(T) || (need_g && !aligned16(g))) return TRIINV_ERR_ALIGN;
    const uint64_t t_bytes = (uint64_t)n_mat * C * C * esize(out_dt);
    if (overlap(K, n_tok * d_k * esize(k_dtype), T, t_bytes) || overlap(beta, n_tok * 4, T, t_bytes)) return TRIINV_ERR_ALIAS;
    if (need_g && overlap(g, n_tok * 4 * (gate_kind == TRIINV_GATE_PER_CHANNEL ? d_k : 1), T, t_bytes)) return TRIINV_ERR_ALIAS;
    if (flags & ~KNOWN_FLAGS) return TRIINV_ERR_UNSUPPORTED;
    if (flags & TRIINV_FLAG_FWD_SHUFFLE) return TRIINV_ERR_UNSUPPORTED;  // a variant of the standalone entry point
    (void)H;
    return TRIINV_OK;
}

// Shared tail of the applied-inverse entry points.  n_token: tokens in K / X / W; n_rhs right-hand sides (host arrays).
int solve_common(const void* K, const float* beta, const float* g, int n_rhs, const void* const* X, const float* const* row_scale,
                 void* const* W, const int* d_x, uint64_t n_token, int64_t n_chunk, const ChunkMap& map, int H, int d_k, int C,
                 int k_dtype, int gate_kind, int method, int op_dtype, void* hip_stream, uint32_t flags)
{
    if (!dtype_ok(k_dtype) || !dtype_ok(op_dtype)) return TRIINV_ERR_BAD_DTYPE;
    if (!method_ok(method)) return TRIINV_ERR_BAD_METHOD;
    if (gate_kind < TRIINV_GATE_SCALAR || gate_kind > TRIINV_GATE_NONE) return TRIINV_ERR_BAD_METHOD;
    if (H <= 0 || d_k <= 0 || d_k % 32 != 0 || d_k > 256) return TRIINV_ERR_BAD_SHAPE;
    if (n_rhs < 1 || n_rhs > 2) return TRIINV_ERR_BAD_SHAPE;
    if (!X || !row_scale || !W || !d_x) return TRIINV_ERR_NULL;
    for (int k = 0; k < n_rhs; ++k)
        if (d_x[k] < 8 || d_x[k] > 512 || d_x[k] % 8 != 0) return TRIINV_ERR_BAD_SHAPE;
    if (n_chunk > 0x7fffffffLL / H) return TRIINV_ERR_BAD_SHAPE;
    const int64_t n_mat = n_chunk * H;
    if (n_mat == 0) return TRIINV_OK;
    const bool need_g = gate_kind != TRIINV_GATE_NONE;
    if (!K || !beta || (need_g && !g)) return TRIINV_ERR_NULL;
    for (int k = 0; k < n_rhs; ++k)
        if (!X[k] || !W[k]) return TRIINV_ERR_NULL;
    if (!aligned16(K) || !aligned16(beta) || (need_g && !aligned16(g))) return TRIINV_ERR_ALIGN;
    for (int k = 0; k < n_rhs; ++k)
        if (!aligned16(X[k]) || !aligned16(W[k]) || (reinterpret_cast<uintptr_t>(row_scale[k]) & 3u)) return TRIINV_ERR_ALIGN;
    const uint64_t n_tok = n_token * H;
    for (int k = 0; k < n_rhs; ++k) {
        const uint64_t w_bytes = n_tok * d_x[k] * esize(op_dtype);
        if (overlap(K, n_tok * d_k * esize(k_dtype), W[k], w_bytes) || overlap(beta, n_tok * 4, W[k], w_bytes) ||
            (need_g && overlap(g, n_tok * 4 * (gate_kind == TRIINV_GATE_PER_CHANNEL ? d_k : 1), W[k], w_bytes)))
            return TRIINV_ERR_ALIAS;
        for (int j = 0; j < n_rhs; ++j) {  // no result may overlap any right-hand side, scale or other result
            const uint64_t x_bytes = n_tok * d_x[j] * esize(op_dtype);
            if (overlap(X[j], x_bytes, W[k], w_bytes) || (row_scale[j] && overlap(row_scale[j], n_tok * 4, W[k], w_bytes)) ||
                (j != k && overlap(W[j], x_bytes, W[k], w_bytes)))
                return TRIINV_ERR_ALIAS;
        }
    }
    if (flags & ~0x70000u) return TRIINV_ERR_UNSUPPORTED;  // TRIINV_FLAG_MXR_R only
    if (method != TRIINV_BLOCK_RECURSIVE && method != TRIINV_MIXED) return TRIINV_ERR_UNSUPPORTED;

    SolveArgs a{GdnArgs{K, beta, need_g ? g : nullptr, nullptr, n_mat, n_chunk, map, H, d_k, k_dtype, gate_kind, method,
                        static_cast<hipStream_t>(hip_stream), false, method_count(method, flags, C), TRIINV_F32},
                n_rhs, {}, {}, {}, {}};
    for (int k = 0; k < n_rhs; ++k) {
        a.X[k] = X[k];
        a.scale[k] = row_scale[k];
        a.W[k] = W[k];
        a.d_x[k] = d_x[k];
    }
    int nb = 1;
#define TRIINV_PICK_OP(NBV) \
    (op_dtype == TRIINV_F32 ? launch_solve_nb##NBV##_op0(a) : op_dtype == TRIINV_F16 ? launch_solve_nb##NBV##_op1(a) : launch_solve_nb##NBV##_op2(a))
    nb = C == 16 ? TRIINV_PICK_OP(1) : C == 32 ? TRIINV_PICK_OP(2) : C == 64 ? TRIINV_PICK_OP(4) : TRIINV_PICK_OP(8);
#undef TRIINV_PICK_OP
    return finish(nb);
}

}  // namespace

extern "C" {

int tri_inv_ex(const void* A, float* T, int64_t n_mat, int C, int in_dtype, int method, int op_dtype, void* hip_stream,
               uint32_t flags)
{
    if (!chunk_size_ok(C)) return TRIINV_ERR_BAD_C;
    if (!dtype_ok(in_dtype) || !dtype_ok(op_dtype)) return TRIINV_ERR_BAD_DTYPE;
    if (!method_ok(method)) return TRIINV_ERR_BAD_METHOD;
    if (n_mat < 0 || n_mat > 0x7fffffffLL) return TRIINV_ERR_BAD_SHAPE;
    if (n_mat == 0) return TRIINV_OK;
    if (!A || !T) return TRIINV_ERR_NULL;
    if (!aligned16(A) || !aligned16(T)) return TRIINV_ERR_ALIGN;
    const int out_dt = out_dtype(flags);
    if (out_dt < 0) return TRIINV_ERR_BAD_DTYPE;
    const uint64_t n_el = (uint64_t)n_mat * C * C;
    if (overlap(A, n_el * esize(in_dtype), T, n_el * esize(out_dt))) return TRIINV_ERR_ALIAS;
    if (flags & ~KNOWN_FLAGS) return TRIINV_ERR_UNSUPPORTED;
    if (method == TRIINV_FWD_SUBST && (flags & TRIINV_FLAG_FWD_SHUFFLE) && out_dt != TRIINV_F32) return TRIINV_ERR_UNSUPPORTED;
    if (method == TRIINV_FWD_SUBST) op_dtype = TRIINV_F32;

    TriInvArgs a{A, T, n_mat, in_dtype, method, static_cast<hipStream_t>(hip_stream), (flags & TRIINV_FLAG_REFINE1) != 0,
                 method_count(method, flags, C), out_dt, (flags & TRIINV_FLAG_FWD_SHUFFLE) != 0};
    if (a.shuffle && method != TRIINV_FWD_SUBST) return TRIINV_ERR_UNSUPPORTED;
    const int nb = pick_tri_inv(a, C, op_dtype);
    return finish(nb);
}

int tri_inv(const void* A, float* T, int64_t n_mat, int C, int in_dtype, int method)
{
    return tri_inv_ex(A, T, n_mat, C, in_dtype, method, in_dtype, nullptr, 0);
}

int gdn_chunk_tri_inv_ex(const void* K, const float* beta, const float* g, float* T, int B, int64_t Tlen, int H, int d_k,
                         int C, int k_dtype, int gate_kind, int method, int op_dtype, void* hip_stream, uint32_t flags)
{
    if (!chunk_size_ok(C)) return TRIINV_ERR_BAD_C;
    if (!dtype_ok(k_dtype) || !dtype_ok(op_dtype)) return TRIINV_ERR_BAD_DTYPE;
    if (!method_ok(method)) return TRIINV_ERR_BAD_METHOD;
    if (gate_kind < TRIINV_GATE_SCALAR || gate_kind > TRIINV_GATE_NONE) return TRIINV_ERR_BAD_METHOD;
    if (B <= 0 || H <= 0 || d_k <= 0 || Tlen < 0 || d_k % 32 != 0 || d_k > 256) return TRIINV_ERR_BAD_SHAPE;
    const int64_t cps = (Tlen + C - 1) / C;  // chunks per sequence; the last one may hold fewer than C tokens
    if (cps > 0x7fffffffLL / B) return TRIINV_ERR_BAD_SHAPE;
    const int64_t n_chunk = (int64_t)B * cps;
    if (n_chunk > 0x7fffffffLL / H) return TRIINV_ERR_BAD_SHAPE;
    const int64_t n_mat = n_chunk * H;
    if (n_mat == 0) return TRIINV_OK;
    const int st = check_fused(K, beta, g, T, (uint64_t)B * Tlen * H, n_mat, H, d_k, C, k_dtype, gate_kind, method, flags);
    if (st != TRIINV_OK) return st;
    if (method == TRIINV_FWD_SUBST && gate_kind != TRIINV_GATE_PER_CHANNEL) op_dtype = TRIINV_F32;

    const ChunkMap map{Tlen, (uint32_t)cps, 0u, nullptr, nullptr};
    GdnArgs a{K, beta, gate_kind != TRIINV_GATE_NONE ? g : nullptr, T, n_mat, n_chunk, map, H, d_k, k_dtype, gate_kind, method,
              static_cast<hipStream_t>(hip_stream), (flags & TRIINV_FLAG_REFINE1) != 0, method_count(method, flags, C), out_dtype(flags)};
    return launch_fused(a, C, op_dtype);
}

int gdn_chunk_build_A(const void* K, const float* beta, const float* g, float* A, int B, int64_t Tlen, int H, int d_k, int C,
                      int k_dtype, int gate_kind, int op_dtype, void* hip_stream, uint32_t flags)
{
    if (!chunk_size_ok(C)) return TRIINV_ERR_BAD_C;
    if (!dtype_ok(k_dtype) || !dtype_ok(op_dtype)) return TRIINV_ERR_BAD_DTYPE;
    if (gate_kind < TRIINV_GATE_SCALAR || gate_kind > TRIINV_GATE_NONE) return TRIINV_ERR_BAD_METHOD;
    if (B <= 0 || H <= 0 || d_k <= 0 || Tlen < 0 || d_k % 32 != 0 || d_k > 256) return TRIINV_ERR_BAD_SHAPE;
    const int64_t cps = (Tlen + C - 1) / C;
    if (cps > 0x7fffffffLL / B) return TRIINV_ERR_BAD_SHAPE;
    const int64_t n_chunk = (int64_t)B * cps;
    if (n_chunk > 0x7fffffffLL / H) return TRIINV_ERR_BAD_SHAPE;
    const int64_t n_mat = n_chunk * H;
    if (n_mat == 0) return TRIINV_OK;
    if (flags & ~(uint32_t)(TRIINV_FLAG_OUT_F16 | TRIINV_FLAG_OUT_BF16)) return TRIINV_ERR_UNSUPPORTED;
    const int st = check_fused(K, beta, g, A, (uint64_t)B * Tlen * H, n_mat, H, d_k, C, k_dtype, gate_kind, TRIINV_BLOCK_RECURSIVE, flags);
    if (st != TRIINV_OK) return st;
    const ChunkMap map{Tlen, (uint32_t)cps, 0u, nullptr, nullptr};
    GdnArgs a{K, beta, gate_kind != TRIINV_GATE_NONE ? g : nullptr, A, n_mat, n_chunk, map, H, d_k, k_dtype, gate_kind, 100 /* M_BUILD_A */,
              static_cast<hipStream_t>(hip_stream), false, 0, out_dtype(flags)};
    // only the per-channel gate rounds anything to op_dtype (its gated keys); otherwise the keys' own values are the operands
    return launch_fused(a, C, gate_kind == TRIINV_GATE_PER_CHANNEL ? op_dtype : TRIINV_F32);
}

int gdn_chunk_tri_inv_varlen(const void* K, const float* beta, const float* g, float* T, const int64_t* cu_seqlens,
                             const int64_t* cu_chunks, int n_seq, int64_t total_tokens, int64_t total_chunks, int H, int d_k,
                             int C, int k_dtype, int gate_kind, int method, int op_dtype, void* hip_stream, uint32_t flags)
{
    if (!chunk_size_ok(C)) return TRIINV_ERR_BAD_C;
    if (!dtype_ok(k_dtype) || !dtype_ok(op_dtype)) return TRIINV_ERR_BAD_DTYPE;
    if (!method_ok(method)) return TRIINV_ERR_BAD_METHOD;
    if (gate_kind < TRIINV_GATE_SCALAR || gate_kind > TRIINV_GATE_NONE) return TRIINV_ERR_BAD_METHOD;
    if (n_seq <= 0 || H <= 0 || d_k <= 0 || total_tokens < 0 || total_chunks < 0 || d_k % 32 != 0 || d_k > 256)
        return TRIINV_ERR_BAD_SHAPE;
    // every chunk holds between 1 and C tokens, and a sequence wastes at most one partly filled chunk
    if (total_chunks > total_tokens || total_chunks * C < total_tokens || total_chunks > (total_tokens + C - 1) / C + n_seq)
        return TRIINV_ERR_BAD_SHAPE;
    if (total_chunks > 0x7fffffffLL / H) return TRIINV_ERR_BAD_SHAPE;
    const int64_t n_mat = total_chunks * H;
    if (n_mat == 0) return TRIINV_OK;
    if (!cu_seqlens || !cu_chunks) return TRIINV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(cu_seqlens) & 7u) || (reinterpret_cast<uintptr_t>(cu_chunks) & 7u)) return TRIINV_ERR_ALIGN;
    const int st = check_fused(K, beta, g, T, (uint64_t)total_tokens * H, n_mat, H, d_k, C, k_dtype, gate_kind, method, flags);
    if (st != TRIINV_OK) return st;
    const uint64_t t_bytes = (uint64_t)n_mat * C * C * esize(out_dtype(flags)), cu_bytes = (uint64_t)(n_seq + 1) * 8;
    if (overlap(cu_seqlens, cu_bytes, T, t_bytes) || overlap(cu_chunks, cu_bytes, T, t_bytes)) return TRIINV_ERR_ALIAS;
    if (method == TRIINV_FWD_SUBST && gate_kind != TRIINV_GATE_PER_CHANNEL) op_dtype = TRIINV_F32;

    const ChunkMap map{total_tokens, 0u, (uint32_t)n_seq, cu_seqlens, cu_chunks};
    GdnArgs a{K, beta, gate_kind != TRIINV_GATE_NONE ? g : nullptr, T, n_mat, total_chunks, map, H, d_k, k_dtype, gate_kind, method,
              static_cast<hipStream_t>(hip_stream), (flags & TRIINV_FLAG_REFINE1) != 0, method_count(method, flags, C), out_dtype(flags)};
    return launch_fused(a, C, op_dtype);
}

int gdn_chunk_tri_solve(const void* K, const float* beta, const float* g, const void* X, const float* row_scale, void* W, int B,
                        int64_t Tlen, int H, int d_k, int d_x, int C, int k_dtype, int gate_kind, int method, int op_dtype,
                        void* hip_stream, uint32_t flags)
{
    if (!chunk_size_ok(C)) return TRIINV_ERR_BAD_C;
    if (B <= 0 || Tlen < 0) return TRIINV_ERR_BAD_SHAPE;
    const int64_t cps = (Tlen + C - 1) / C;
    if (cps > 0x7fffffffLL / B) return TRIINV_ERR_BAD_SHAPE;
    const ChunkMap map{Tlen, (uint32_t)cps, 0u, nullptr, nullptr};
    return solve_common(K, beta, g, 1, &X, &row_scale, &W, &d_x, (uint64_t)B * Tlen, (int64_t)B * cps, map, H, d_k, C, k_dtype,
                        gate_kind, method, op_dtype, hip_stream, flags);
}

int gdn_chunk_tri_solve_multi(const void* K, const float* beta, const float* g, int n_rhs, const void* const* X,
                              const float* const* row_scale, void* const* W, const int* d_x, int B, int64_t Tlen, int H, int d_k,
                              int C, int k_dtype, int gate_kind, int method, int op_dtype, void* hip_stream, uint32_t flags)
{
    if (!chunk_size_ok(C)) return TRIINV_ERR_BAD_C;
    if (B <= 0 || Tlen < 0) return TRIINV_ERR_BAD_SHAPE;
    const int64_t cps = (Tlen + C - 1) / C;
    if (cps > 0x7fffffffLL / B) return TRIINV_ERR_BAD_SHAPE;
    const ChunkMap map{Tlen, (uint32_t)cps, 0u, nullptr, nullptr};
    return solve_common(K, beta, g, n_rhs, X, row_scale, W, d_x, (uint64_t)B * Tlen, (int64_t)B * cps, map, H, d_k, C, k_dtype,
                        gate_kind, method, op_dtype, hip_stream, flags);
}

int gdn_chunk_tri_solve_varlen(const void* K, const float* beta, const float* g, const void* X, const float* row_scale, void* W,
                               const int64_t* cu_seqlens, const int64_t* cu_chunks, int n_seq, int64_t total_tokens,
                               int64_t total_chunks, int H, int d_k, int d_x, int C, int k_dtype, int gate_kind, int method,
                               int op_dtype, void* hip_stream, uint32_t flags)
{
    if (!chunk_size_ok(C)) return TRIINV_ERR_BAD_C;
    if (n_seq <= 0 || total_tokens < 0 || total_chunks < 0) return TRIINV_ERR_BAD_SHAPE;
    if (total_chunks > total_tokens || total_chunks * C < total_tokens || total_chunks > (total_tokens + C - 1) / C + n_seq)
        return TRIINV_ERR_BAD_SHAPE;
    if (total_chunks > 0 && (!cu_seqlens || !cu_chunks)) return TRIINV_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(cu_seqlens) & 7u) || (reinterpret_cast<uintptr_t>(cu_chunks) & 7u)) return TRIINV_ERR_ALIGN;
    if (W && total_chunks > 0 && H > 0 && d_x > 0) {
        const uint64_t w_bytes = (uint64_t)total_tokens * H * d_x * esize(op_dtype), cu_bytes = (uint64_t)(n_seq + 1) * 8;
        if (overlap(cu_seqlens, cu_bytes, W, w_bytes) || overlap(cu_chunks, cu_bytes, W, w_bytes)) return TRIINV_ERR_ALIAS;
    }
    const ChunkMap map{total_tokens, 0u, (uint32_t)n_seq, cu_seqlens, cu_chunks};
    return solve_common(K, beta, g, 1, &X, &row_scale, &W, &d_x, (uint64_t)total_tokens, total_chunks, map, H, d_k, C, k_dtype,
                        gate_kind, method, op_dtype, hip_stream, flags);
}

int gdn_chunk_tri_inv(const void* K, const float* beta, const float* g, float* T, int B, int64_t Tlen, int H, int d_k, int C)
{
    return gdn_chunk_tri_inv_ex(K, beta, g, T, B, Tlen, H, d_k, C, TRIINV_BF16, TRIINV_GATE_SCALAR, TRIINV_BLOCK_RECURSIVE,
                                TRIINV_BF16, nullptr, 0);
}

const char* triinv_status_string(int status)
{
    switch (status) {
    case TRIINV_OK: return "ok";
    case TRIINV_ERR_NULL: return "null pointer";
    case TRIINV_ERR_BAD_C: return "C must be 16, 32, 64 or 128";
    case TRIINV_ERR_BAD_DTYPE: return "unknown element type";
    case TRIINV_ERR_BAD_METHOD: return "unknown method or gate kind";
    case TRIINV_ERR_BAD_SHAPE: return "bad shape";
    case TRIINV_ERR_ALIGN: return "pointer not 16-byte aligned";
    case TRIINV_ERR_ALIAS: return "output overlaps an input";
    case TRIINV_ERR_LAUNCH: return "kernel launch failed";
    case TRIINV_ERR_UNSUPPORTED: return "combination not built";
    default: return "unknown status";
    }
}

int triinv_version(void) { return 200; }

}  // extern "C"
