/*
 * triinv -- batched inversion T = (I + A)^{-1} of small strictly-lower-triangular chunk
 * matrices for delta-rule linear attention, on one AMD MI355X (gfx950).
 *
 * The operation (paper Sec. 1, Eq. 3 and Table 1): a sequence of Tlen tokens is cut into
 * chunks of C tokens; for every (batch, chunk, head) the C x C matrix
 *      A_ij = beta_i * exp(g_i - g_j) * <k_i, k_j>              (scalar gate, GDN)
 *      A_ij = beta_i * sum_c k_ic k_jc exp(g_ic - g_jc)         (per-channel gate, KDA)
 *      A_ij = beta_i * <k_i, k_j>                               (no gate, DeltaNet)
 * for i > j, and 0 for i <= j, is strictly lower triangular, and the layer needs the
 * unit-lower-triangular inverse T = (I + A)^{-1}.  The matrices are independent.
 *
 * Conventions shared by every entry point
 *   - every pointer is a DEVICE pointer (hipMalloc / torch .data_ptr()), 16-byte aligned;
 *     the caller owns all buffers; nothing is allocated, freed or synchronised here;
 *   - work is enqueued on the given HIP stream (NULL = the default stream) and the call
 *     returns at once; the return value reports argument / launch errors only;
 *   - the return value is TRIINV_OK (0) or a negative triinv_status; argument errors are
 *     detected on the host before anything is launched, so a failing call does no GPU work;
 *   - T is dense row-major [n_mat][C][C], fp32 unless a TRIINV_FLAG_OUT_* bit asks for a 16-bit
 *     result, completely overwritten: exact 0 above the diagonal and exact 1 on it;
 *   - non-finite input values are not errors; they propagate inside their own matrix only.
 */
#ifndef TRIINV_H
#define TRIINV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element types: of a stored input (in_dtype, k_dtype) or of the matrix-core operands
 * (op_dtype; products always accumulate in fp32, paper Sec. 4.1). */
typedef enum { TRIINV_F32 = 0, TRIINV_F16 = 1, TRIINV_BF16 = 2 } triinv_dtype;

/* Inversion methods. */
typedef enum {
    /* Row-wise forward substitution in fp32 vector arithmetic; the direct, matmul-free, stable
     * baseline (the role of the vectorised column sweep, paper Sec. 3.1).  Ignores op_dtype. */
    TRIINV_FWD_SUBST = 0,
    /* Blocked 2x2 recursion (paper Alg. 4, Sec. 3.3, Eq. 7 in its lower-triangular reading):
     * X <- D_e + D_o - D_o A D_e for block sizes 1, 2, ..., C/2.  Log-stable. */
    TRIINV_BLOCK_RECURSIVE = 1,
    /* Neumann product prod_k (I + (-A)^(2^k)) by repeated squaring (paper Alg. 5, Sec. 3.2):
     * X <- I - A, Y <- A, then log2(C/2) times Y <- Y Y, X <- X + X Y.  Unstable: intermediate
     * powers may overflow / cancel; the result is returned as computed. */
    TRIINV_NEUMANN = 2,
    /* Mixed recursion (paper Alg. 2, Sec. 3.4): Neumann product on the 16 x 16 diagonal blocks, r steps
     * of iterative refinement on those blocks (r = TRIINV_FLAG_MXR_R(r) in flags, default 1), then the
     * blocked recursion from block size 16.  Log-stable. */
    TRIINV_MIXED = 3,
    /* Blocked recursion started at block size 16 (paper Alg. 4 with b0 = 16) from 16 x 16 diagonal
     * blocks inverted directly by forward substitution in fp32 (the stable direct method of
     * Sec. 3.1); only the merges -T22 A21 T11 use op_dtype operands. */
    TRIINV_BLOCK_DIRECT = 4,
    /* Newton-Schulz iteration (paper Alg. 3, Eq. 8): X <- I / C, then n times Y <- (I + A) X,
     * X <- 2X - XY.  n = TRIINV_FLAG_ITERS(n) in flags, default 12 (the count the paper finds
     * sufficient at C = 64; 2 log2 C elsewhere).  At C = 128 with the per-channel gate or with fp32 keys of
     * d_k = 128 it runs as the two-launch path described at gdn_chunk_tri_inv (fp32 T only). */
    TRIINV_NEWTON_SCHULZ = 5,
    /* Mixed recursion with b0 = 32 (the other block size the paper proposes, Sec. 3.4): Neumann product
     * (four squarings) and r refinement steps on the 32 x 32 diagonal blocks, blocked recursion from block
     * size 32.  C >= 32. */
    TRIINV_MIXED_B32 = 6
} triinv_method;

/* Gate kinds of the fused entry point. */
typedef enum {
    TRIINV_GATE_SCALAR = 0,      /* g is [B, Tlen, H]      */
    TRIINV_GATE_PER_CHANNEL = 1, /* g is [B, Tlen, H, d_k] */
    TRIINV_GATE_NONE = 2         /* g is ignored (may be NULL) */
} triinv_gate;

typedef enum {
    TRIINV_OK = 0,
    TRIINV_ERR_NULL = -1,        /* a required pointer is NULL while there is work to do */
    TRIINV_ERR_BAD_C = -2,       /* C is not 16, 32, 64 or 128 */
    TRIINV_ERR_BAD_DTYPE = -3,   /* unknown in_dtype / k_dtype / op_dtype */
    TRIINV_ERR_BAD_METHOD = -4,  /* unknown method or gate kind */
    TRIINV_ERR_BAD_SHAPE = -5,   /* n_mat < 0; B, H, d_k <= 0; Tlen < 0; d_k % 32 != 0; d_k > 256; more than 2^31 - 1 matrices;
                                    inconsistent varlen totals; d_x not a multiple of 8 in [8, 512] */
    TRIINV_ERR_ALIGN = -6,       /* a pointer is not 16-byte aligned */
    TRIINV_ERR_ALIAS = -7,       /* T (or W) overlaps an input buffer */
    TRIINV_ERR_LAUNCH = -8,      /* the HIP runtime refused the launch */
    TRIINV_ERR_UNSUPPORTED = -9  /* valid arguments, but this combination is not built */
} triinv_status;

/* Bits of `flags` (0 = none). */
#define TRIINV_FLAG_REFINE1 0x1u /* one iterative-refinement step X <- X + (I - X(I+A))X on the whole matrix after the
                                    method (paper Alg. 6, Eq. 9).  Built for every matrix-product method (all but
                                    TRIINV_FWD_SUBST): inside the method's kernel at C <= 64 (tri_inv and every fused
                                    gate kind); at C = 128 as a second kernel over T, in place, for an fp32 result
                                    (head dimensions 64 and 128 for the scalar / no-gate kinds, any supported one for
                                    the per-channel gate).  Anything else returns TRIINV_ERR_UNSUPPORTED */
#define TRIINV_FLAG_OUT_F16 0x2u  /* T holds fp16 elements: [n_mat][C][C], 2 bytes each (pass the buffer as float*) */
#define TRIINV_FLAG_OUT_BF16 0x4u /* T holds bf16 elements.  The fp32 result is rounded to nearest even on the way
                                     out; the diagonal is still exactly 1, the upper triangle exactly 0.  Every
                                     method (not with TRIINV_FLAG_FWD_SHUFFLE); both flags at once:
                                     TRIINV_ERR_BAD_DTYPE */

#define TRIINV_FLAG_FWD_SHUFFLE 0x8u /* tri_inv_ex, TRIINV_FWD_SUBST, C = 64: broadcast the entries of A with wavefront
                                       shuffles instead of through LDS (the plain shuffle baseline; slower) */

#define TRIINV_FLAG_MXR_R(r) ((((uint32_t)(r) + 1u) & 7u) << 16) /* refinement steps r = 0..6 inside TRIINV_MIXED
                                                                 (paper Alg. 2); flags without it: r = 1 */

#define TRIINV_FLAG_ITERS(n) (((uint32_t)(n) & 0xffu) << 8) /* iteration count of TRIINV_NEWTON_SCHULZ (0 = default) */

/*
 * tri_inv: invert n_mat precomputed matrices (paper Sec. 1 Eq. 3 with A given; App. D.1: the
 * input is a tensor of many small independent chunks).
 *   A        device, [n_mat][C][C] row-major, elements of type in_dtype.  Only entries with
 *            i > j are read into the arithmetic; entries with i <= j are ignored, so garbage or
 *            NaN there does not change the result (the mask of Eq. 3 is applied on load).
 *   T        device, [n_mat][C][C] fp32, output; must not overlap A.
 *   n_mat    number of matrices, >= 0; 0 is a successful no-op (pointers may then be NULL).
 *   C        16, 32, 64 or 128 (the chunk sizes used in practice, paper Sec. 1).
 *   in_dtype triinv_dtype of A.
 *   method   triinv_method.
 * Short form: op_dtype = in_dtype, default stream, flags 0.
 */
int tri_inv(const void* A, float* T, int64_t n_mat, int C, int in_dtype, int method);

/*
 * tri_inv_ex: as tri_inv, with
 *   op_dtype   type the matrix-core operands are rounded to (round-to-nearest-even) at every
 *              product; accumulators and all additions stay fp32.  Ignored by TRIINV_FWD_SUBST.
 *   hip_stream a hipStream_t (e.g. torch.cuda.current_stream().cuda_stream), or NULL.
 *   flags      TRIINV_FLAG_* bits.
 */
int tri_inv_ex(const void* A, float* T, int64_t n_mat, int C, int in_dtype, int method,
               int op_dtype, void* hip_stream, uint32_t flags);

/*
 * gdn_chunk_tri_inv: fused "build A from the keys, then invert" (paper Sec. 1 Eq. 3 with the
 * GDN row of Table 1), never writing A to memory.
 *   K     device, [B][Tlen][H][d_k] contiguous (token-major, heads interleaved), bf16.
 *   beta  device, [B][Tlen][H] fp32.
 *   g     device, [B][Tlen][H] fp32: the chunk-local cumulative log-decay (the running sum
 *         restarts at every chunk boundary).
 *   T     device, [n_mat][C][C] fp32 with n_mat = B * ceil(Tlen / C) * H and matrix index
 *         m = (b * ceil(Tlen / C) + chunk) * H + h; must not overlap an input.
 *   Tlen need not be a multiple of C: the last chunk of a sequence then has fewer than C tokens
 *   (paper Sec. 1: chunks of "at most" C tokens) and is treated as padded with tokens whose key and
 *   beta are zero, so its matrix still is C x C, with identity rows and columns for the padding;
 *   nothing is read beyond token Tlen - 1 of a sequence.  d_k: a multiple of 32, <= 256.
 *   d_k = 64 and 128 have specialised kernels for every method; other values run a channel loop
 *   with fused kernels for every method at C <= 64 and for TRIINV_FWD_SUBST, TRIINV_BLOCK_RECURSIVE and
 *   TRIINV_BLOCK_DIRECT at C = 128 (and for every method with the per-channel gate at C <= 64).  A matrix-product method without a fused kernel for the
 *   gate kind / d_k / C asked for runs as two launches on the same stream -- the chunk matrices written
 *   into T as fp32, then inverted in place by the method's tri_inv kernel -- with the same result;
 *   that path needs an fp32 T and does not take TRIINV_FLAG_REFINE1 (TRIINV_ERR_UNSUPPORTED).
 * Short form: k_dtype = BF16, scalar gate, method = TRIINV_BLOCK_RECURSIVE, op_dtype = BF16,
 * default stream, flags 0.
 */
int gdn_chunk_tri_inv(const void* K, const float* beta, const float* g, float* T,
                      int B, int64_t Tlen, int H, int d_k, int C);

/*
 * gdn_chunk_tri_inv_ex: as gdn_chunk_tri_inv, with
 *   k_dtype    triinv_dtype of K.  The Gram products <k_i, k_j> use the stored key values as
 *              matrix-core operands (exact products, fp32 accumulation) for the scalar and
 *              no-gate kinds.  For the per-channel gate the gated keys k*exp(+-(g - a)) are rounded
 *              to op_dtype, a = an anchor row of g.  C <= 64: one anchor per 16 rows, so only the
 *              fall of g within any 16 consecutive tokens must stay below ~80 (fp32, bf16 operands)
 *              or ~10 (fp16 operands), however strong the decay over the whole chunk is (g is taken
 *              to fall along the chunk, as a cumulative log-decay does).  C = 128: the recursions
 *              (TRIINV_BLOCK_RECURSIVE, _MIXED, _MIXED_B32, _BLOCK_DIRECT) use one anchor per 16 rows inside
 *              the two 64 x 64 diagonal blocks and row 64 for the block below them, so the bound applies to
 *              the fall of g over 64 tokens; the other methods use one anchor, the chunk's middle row, and
 *              the bound applies to the fall of g over the whole chunk.
 *   gate_kind  triinv_gate (KDA row of Table 1 for TRIINV_GATE_PER_CHANNEL).
 *   method, op_dtype, hip_stream, flags: as in tri_inv_ex.
 */
int gdn_chunk_tri_inv_ex(const void* K, const float* beta, const float* g, float* T,
                         int B, int64_t Tlen, int H, int d_k, int C,
                         int k_dtype, int gate_kind, int method, int op_dtype,
                         void* hip_stream, uint32_t flags);

/*
 * gdn_chunk_build_A: the first half of the fused operation alone -- the chunk matrices A of paper Sec. 1
 * Eq. 3 / Table 1 written out, for callers that keep the two steps apart (A then goes to tri_inv).
 *   A   device, [n_mat][C][C], fp32 (or fp16 / bf16 with TRIINV_FLAG_OUT_F16 / OUT_BF16): the entries
 *       with i > j, exact zeros on and above the diagonal; n_mat and the matrix order as in
 *       gdn_chunk_tri_inv; a short last chunk has zero rows and columns for its padding.
 *   K, beta, g, B, Tlen, H, d_k, C, k_dtype, gate_kind, hip_stream: as in gdn_chunk_tri_inv_ex.
 *   op_dtype  only used by the per-channel gate (type its gated keys are rounded to); otherwise the Gram
 *             products use the stored key values exactly and accumulate in fp32.
 *   flags     TRIINV_FLAG_OUT_* only.
 */
int gdn_chunk_build_A(const void* K, const float* beta, const float* g, float* A,
                      int B, int64_t Tlen, int H, int d_k, int C,
                      int k_dtype, int gate_kind, int op_dtype, void* hip_stream, uint32_t flags);

/*
 * gdn_chunk_tri_inv_varlen: the fused operation on sequences of different lengths packed back to
 * back (the layout serving frameworks use for batched prefill; paper Sec. 1 chunking applied to each
 * sequence on its own).
 *   K, beta, g     device, [total_tokens][H][d_k], [total_tokens][H], [total_tokens][H] (or
 *                  [total_tokens][H][d_k] for the per-channel gate); g restarts at every chunk.
 *   cu_seqlens     device, int64 [n_seq + 1]: row of the first token of each sequence, then
 *                  total_tokens.  Non-decreasing; an empty sequence has no chunk.
 *   cu_chunks      device, int64 [n_seq + 1]: id of the first chunk of each sequence, then
 *                  total_chunks; sequence s owns ceil(len_s / C) consecutive ids.
 *   total_tokens, total_chunks: the last entries of the two arrays, passed by value because the
 *                  host cannot read device memory without a synchronisation.
 *   T              device, [total_chunks * H][C][C] fp32, matrix index chunk_id * H + h; a last chunk
 *                  with fewer than C tokens is padded as in gdn_chunk_tri_inv.
 * The two arrays are trusted: the host only checks that the totals are consistent with each other
 * (TRIINV_ERR_BAD_SHAPE), the kernels clamp every row index into [first token of the chunk, last
 * token of the sequence].  8-byte alignment is required of cu_seqlens and cu_chunks.
 * Other arguments as in gdn_chunk_tri_inv_ex.
 */
int gdn_chunk_tri_inv_varlen(const void* K, const float* beta, const float* g, float* T,
                             const int64_t* cu_seqlens, const int64_t* cu_chunks, int n_seq,
                             int64_t total_tokens, int64_t total_chunks, int H, int d_k, int C,
                             int k_dtype, int gate_kind, int method, int op_dtype,
                             void* hip_stream, uint32_t flags);

/*
 * gdn_chunk_tri_solve: the fused operation with the inverse applied instead of stored,
 *     W = (I + A)^{-1} diag(s) X      chunk by chunk,
 * the form in which the layer consumes the inverse (paper Sec. 1 Eq. 3; direction of the fused layer
 * kernel of Sec. 5.2): A is built from K, beta, g and inverted in registers exactly as in
 * gdn_chunk_tri_inv_ex, the columns of the inverse are scaled by s in fp32, rounded to op_dtype and
 * multiplied into the chunk's rows of X on the matrix cores (fp32 accumulation).  Neither A nor the
 * inverse goes to memory.
 *   X          device, [B][Tlen][H][d_x], stored in op_dtype (fp32, fp16 or bf16), 16-byte aligned;
 *              d_x a multiple of 8, 8 <= d_x <= 512.  Read only.
 *   row_scale  device, fp32 [B][Tlen][H], or NULL for s = 1 (e.g. beta itself, or beta * exp(g)).
 *   W          device, [B][Tlen][H][d_x], same element type as X, 16-byte aligned; written by the
 *              call (rows of a short last chunk's padding do not exist and are not written).  Must
 *              not overlap X.  Caller-owned.
 *   K, beta, g, B, Tlen, H, d_k, C, k_dtype, gate_kind, hip_stream: as in gdn_chunk_tri_inv_ex.
 *   method     TRIINV_BLOCK_RECURSIVE or TRIINV_MIXED (with TRIINV_FLAG_MXR_R).  C <= 64 takes every gate kind
 *              and every supported d_k.  C = 128 takes the scalar / no-gate kinds with d_k = 64 or 128 and the
 *              per-channel gate with any supported d_k.  The rows of X one chunk covers (H * d_x * C elements)
 *              must stay below 2^31 bytes: the kernels address them with 32-bit offsets.
 *              Anything else returns TRIINV_ERR_UNSUPPORTED.
 *   flags      TRIINV_FLAG_MXR_R only.
 * Accuracy: that of the method's inverse (see tri_inv_ex) plus one rounding of the scaled inverse
 * and of W to op_dtype.
 */
int gdn_chunk_tri_solve(const void* K, const float* beta, const float* g,
                        const void* X, const float* row_scale, void* W,
                        int B, int64_t Tlen, int H, int d_k, int d_x, int C,
                        int k_dtype, int gate_kind, int method, int op_dtype,
                        void* hip_stream, uint32_t flags);

/*
 * gdn_chunk_tri_solve_multi: gdn_chunk_tri_solve for one or two right-hand sides that share the inverse,
 *     W_k = (I + A)^{-1} diag(s_k) X_k,   k = 0 .. n_rhs - 1,
 * with A built and inverted once per chunk (e.g. the key-side and the value-side product of a layer in one pass).
 *   n_rhs       1 or 2 (TRIINV_ERR_BAD_SHAPE otherwise).
 *   X, row_scale, W, d_x   HOST arrays of n_rhs entries: device pointers (row_scale[k] may be NULL) and column
 *               counts, each as in gdn_chunk_tri_solve; read during the call only.  No W_k may overlap any
 *               input, scale or other result.
 * Everything else as in gdn_chunk_tri_solve.
 */
int gdn_chunk_tri_solve_multi(const void* K, const float* beta, const float* g,
                              int n_rhs, const void* const* X, const float* const* row_scale,
                              void* const* W, const int* d_x,
                              int B, int64_t Tlen, int H, int d_k, int C,
                              int k_dtype, int gate_kind, int method, int op_dtype,
                              void* hip_stream, uint32_t flags);

/*
 * gdn_chunk_tri_solve_varlen: gdn_chunk_tri_solve on sequences of different lengths packed back to back
 * (paper Sec. 1 chunking applied to each sequence on its own).  K, beta, g as in
 * gdn_chunk_tri_inv_varlen; X, W device, [total_tokens][H][d_x]; row_scale device fp32 [total_tokens][H]
 * or NULL; cu_seqlens, cu_chunks, n_seq, total_tokens, total_chunks as in gdn_chunk_tri_inv_varlen
 * (trusted in the same way; must not overlap W).  Everything else as in gdn_chunk_tri_solve.
 */
int gdn_chunk_tri_solve_varlen(const void* K, const float* beta, const float* g,
                               const void* X, const float* row_scale, void* W,
                               const int64_t* cu_seqlens, const int64_t* cu_chunks, int n_seq,
                               int64_t total_tokens, int64_t total_chunks, int H, int d_k, int d_x, int C,
                               int k_dtype, int gate_kind, int method, int op_dtype,
                               void* hip_stream, uint32_t flags);

/* Human-readable name of a status code (static storage, never NULL). */
const char* triinv_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int triinv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TRIINV_H */
