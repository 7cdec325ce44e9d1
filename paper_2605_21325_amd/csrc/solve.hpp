// The inverse applied instead of stored:  W = (I + A)^{-1} diag(s) X  for one chunk (paper Sec. 1 Eq. 3;
// direction of the fused layer kernel of Sec. 5.2).  After the blocked / mixed recursion the tiles of the
// inverse sit in one wavefront's registers; they are brought to T orientation (the left-factor form of
// tn()), their columns scaled by s, rounded to the operand type, and multiplied into the chunk's rows of
// X on the matrix cores.  Neither A nor the inverse goes to memory.
//
// Column map of X and W.  The matrix-core column index n of a tile is free to stand for any memory
// column as long as the result is stored under the same map, so lane (q, n) owns the VEC CONSECUTIVE
// memory columns that fill 16 bytes (VEC = 8 for 16-bit elements, 4 for fp32): columns GW gi + VEC n ..
// + VEC - 1 of column group gi (GW = 16 VEC columns wide), and column tile c of the group takes column
// VEC n + c from every lane.  One 16-byte load per (row, lane) then feeds VEC tiles, one 16-byte store
// per (row, lane) takes one result from each of VEC accumulator tiles, every memory instruction moves
// whole 256-byte row segments (16 lanes x 16 B, four rows per instruction), and neither X nor W passes
// through LDS.  Lanes whose columns lie beyond d_x compute on a clamped address and store nothing.
#pragma once
#include "kernels.hpp"

namespace triinv {

struct RhsArgs {
    const void* X;       // [tokens][H][d_x], element type = operand type
    const float* scale;  // [tokens][H] or null
    void* W;             // [tokens][H][d_x]
    int d_x;
};

// Tile source for the recursion with every tile of A formed up front in the form the recursion consumes it: the
// off-diagonal tiles as packed operands in the orientation their merge asks for (half or a quarter of the registers of
// fp32 tiles in both orientations), the diagonal tiles in fp32 in both orientations (the leaves use them first).  Filling
// it from a source that builds tiles out of keys held in registers frees the keys before the recursion starts.
template <int OP, int NB> struct PackedA {
    static constexpr bool kFromMemory = false;
    Opnd<OP> off[NB * (NB + 1) / 2];
    v4f dn[NB], dt[NB];
    template <bool TR> __device__ __forceinline__ v4f get(int i, int) const { return TR ? dt[i] : dn[i]; }  // diagonal tiles only
    template <bool TR> __device__ __forceinline__ Opnd<OP> operand(int i, int j) const { return off[tix(i, j)]; }
    template <class Src> __device__ __forceinline__ void fill(const Src& s)
    {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
#pragma unroll
            for (int j = 0; j < i; ++j)
                off[tix(i, j)] = merge_block_is_T<NB>(i, j) ? pack<OP>(s.template get<false>(i, j)) : pack<OP>(s.template get<true>(i, j));
            dn[i] = s.template get<false>(i, i);
            dt[i] = s.template get<true>(i, i);
        }
    }
};
template <int OP, int NB> struct PackedSource<PackedA<OP, NB>> {
    static constexpr bool value = true;
};

// NRHS right-hand sides sharing one inverse: W_k = T diag(s_k) X_k.  NRHS is a compile-time count (1 or 2) so that
// every access to the list is a plain kernel-argument read.
constexpr int MAX_RHS = 2;
struct RhsList {
    RhsArgs r[MAX_RHS];
};

// Sixteen bytes of one row of X as stored: VEC consecutive columns.
template <int OP> struct XRow;
template <> struct XRow<OP_F32> { v4f f; };
template <> struct XRow<OP_F16> { v4u u; };
template <> struct XRow<OP_BF16> { v4u u; };

template <int OP> __device__ __forceinline__ XRow<OP> load_x(const char* p)
{
    if constexpr (OP == OP_F32) {
        return {*reinterpret_cast<const v4f*>(p)};
    } else {
        return {*reinterpret_cast<const v4u*>(p)};
    }
}

// Column tile c of a 16-row tile row of X as a matrix-core operand: rows 4q + r (r = 0..3) of this lane's column VEC n + c.
template <int OP> __device__ __forceinline__ Opnd<OP> x_operand(const XRow<OP> (&row)[4], int c)
{
    if constexpr (OP == OP_F32) {
        return {v4f{row[0].f[c], row[1].f[c], row[2].f[c], row[3].f[c]}};
    } else {
        const int d = c >> 1;
        uint32_t lo, hi;
        if (c & 1) {  // upper halves of the dwords
            lo = (row[0].u[d] >> 16) | (row[1].u[d] & 0xffff0000u);
            hi = (row[2].u[d] >> 16) | (row[3].u[d] & 0xffff0000u);
        } else {
            lo = (row[0].u[d] & 0xffffu) | (row[1].u[d] << 16);
            hi = (row[2].u[d] & 0xffffu) | (row[3].u[d] << 16);
        }
        Opnd<OP> o;
        o.x = __builtin_bit_cast(decltype(o.x), v2u{lo, hi});
        return o;
    }
}

// The right-hand sides of one chunk and head.
template <int OP, int NB> struct RhsX {
    static constexpr int ESZ = OP == OP_F32 ? 4 : 2;
    static constexpr int VEC = 16 / ESZ;  // columns per lane
    static constexpr int GW = 16 * VEC;   // columns per group
    // C <= 64: X and W are addressed through buffer descriptors based at the chunk's first row of this head, with one 32-bit
    // byte offset per row that loads and stores share (64 rows of H * d_x elements stay below 2^31 bytes; the launcher
    // checks).  With 64-bit pointers every row's load address and store address is a register pair of its own: 64
    // registers at C = 64, which cost the kernels with two right-hand sides their second wavefront per SIMD (299
    // registers against 236).
    // C = 128 (one wavefront per chunk: the fallback for tensors too wide for 32-bit offsets) keeps the pointers.
    static constexpr bool BUF = NB <= 4;
    static constexpr int CACHE_NT = 2;
    __amdgpu_buffer_rsrc_t xb, wb;
    const char* xc;      // element (chunk row 0, this head, column 0) of X
    char* wc;            // the same element of W
    int64_t row_bytes;   // H * d_x * ESZ
    int d_x, valid;
    Lane ln;
    v4f s_q[NB];         // s of rows 16 j + 4 q + r
    XRow<OP> raw[NB][4];

    // first token of the chunk tok0, head h; starts the loads of s
    __device__ __forceinline__ void init(const RhsArgs& a, int64_t tok0, int h, int H, int valid_, Lane ln_)
    {
        ln = ln_;
        d_x = a.d_x;
        valid = valid_;
        row_bytes = (int64_t)H * d_x * ESZ;
        const int64_t e0 = (tok0 * H + h) * (int64_t)d_x * ESZ;
        xc = static_cast<const char*>(a.X) + e0;
        wc = static_cast<char*>(a.W) + e0;
        if constexpr (BUF) {
            const int span = (valid - 1) * (int)row_bytes + d_x * ESZ;  // the chunk's real rows: nothing beyond is read or written
            xb = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(xc), 0, span, 0x00020000);
            wb = __builtin_amdgcn_make_buffer_rsrc(wc, 0, span, 0x00020000);
        }
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 16 * j + 4 * ln.q + r;
                const int rc = row < valid ? row : valid - 1;
                s_q[j][r] = a.scale ? a.scale[(tok0 + rc) * H + h] : 1.f;
            }
    }

    __device__ __forceinline__ bool active(int gi) const { return GW * gi + VEC * ln.n < d_x; }
    __device__ __forceinline__ int n_group() const { return (d_x + GW - 1) / GW; }

    // loads of column group gi: rows beyond the chunk's last token read that token (they only meet zero columns of the inverse)
    // (tile rows j0 .. j1 - 1 only: the caller may split the loads around other work)
    __device__ __forceinline__ void issue(int gi, int j0 = 0, int j1 = NB)
    {
        const int col = active(gi) ? GW * gi + VEC * ln.n : 0;
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (j < j0 || j >= j1) continue;
                const int row = 16 * j + 4 * ln.q + r;
                const int rc = row < valid ? row : valid - 1;
                if constexpr (BUF)
                    raw[j][r] = __builtin_bit_cast(XRow<OP>, __builtin_amdgcn_raw_buffer_load_b128(xb, rc * (int)row_bytes + col * ESZ, 0, 0));
                else
                    raw[j][r] = load_x<OP>(xc + rc * row_bytes + col * ESZ);
            }
    }

    // rows 16 i + 4 q + r of the result, VEC columns per lane: acc[c][r]
    __device__ __forceinline__ void store(int gi, int i, const v4f (&acc)[VEC])
    {
        if (!active(gi)) return;
        const int col = GW * gi + VEC * ln.n;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 16 * i + 4 * ln.q + r;
            if (row >= valid) continue;
            if constexpr (BUF) {
                // (the whole offset in the per-lane part of the address: a 16-byte buffer store with a register as its
                // uniform offset is not followed by the wait state its data registers need before they are written again)
                v4u v;
                if constexpr (OP == OP_F32)
                    v = __builtin_bit_cast(v4u, v4f{acc[0][r], acc[1][r], acc[2][r], acc[3][r]});
                else if constexpr (OP == OP_F16)
                    v = v4u{pack2_f16(acc[0][r], acc[1][r]), pack2_f16(acc[2][r], acc[3][r]), pack2_f16(acc[4][r], acc[5][r]),
                            pack2_f16(acc[6][r], acc[7][r])};
                else
                    v = v4u{pack2_bf16(acc[0][r], acc[1][r]), pack2_bf16(acc[2][r], acc[3][r]), pack2_bf16(acc[4][r], acc[5][r]),
                            pack2_bf16(acc[6][r], acc[7][r])};
                __builtin_amdgcn_raw_buffer_store_b128(v, wb, row * (int)row_bytes + col * ESZ, 0, CACHE_NT);
                continue;
            }
            char* p = wc + row * row_bytes + col * ESZ;
            if constexpr (OP == OP_F32) {
                __builtin_nontemporal_store(v4f{acc[0][r], acc[1][r], acc[2][r], acc[3][r]}, reinterpret_cast<v4f*>(p));
            } else if constexpr (OP == OP_F16) {
                __builtin_nontemporal_store(v4u{pack2_f16(acc[0][r], acc[1][r]), pack2_f16(acc[2][r], acc[3][r]),
                                                pack2_f16(acc[4][r], acc[5][r]), pack2_f16(acc[6][r], acc[7][r])},
                                            reinterpret_cast<v4u*>(p));
            } else {
                __builtin_nontemporal_store(v4u{pack2_bf16(acc[0][r], acc[1][r]), pack2_bf16(acc[2][r], acc[3][r]),
                                                pack2_bf16(acc[4][r], acc[5][r]), pack2_bf16(acc[6][r], acc[7][r])},
                                            reinterpret_cast<v4u*>(p));
            }
        }
    }
};

// Recursion (blocked, or mixed with aux refinement steps on the leaves), then W_k = T diag(s_k) X_k for the NRHS
// right-hand sides in turn; x holds the first one, next_rhs(k) re-initialises x for right-hand side k and starts the
// loads of its first column group.  Two right-hand sides are built at C <= 64 only, where the 10 fp32 tiles of T stay
// in registers beside everything else.
// ISSUE_FROM: the caller has started the loads of tile rows 0 .. ISSUE_FROM - 1 of X's first column group; the rest
// (none when ISSUE_FROM = NB) start here.  IN_MERGE says where: inside the recursion's last merge, as soon as its tiles
// of A exist (a source that holds keys in registers has them free from there on, and the merge's products run while
// the loads are in flight), or after the recursion.  lds: the transpose patch (XPOSE_FLOATS floats, wave-private).
template <int OP, int NB, int METHOD, int ISSUE_FROM, bool IN_MERGE, int NRHS, class ASrc, class NextRhs>
__device__ __forceinline__ void invert_and_apply(const ASrc& src, RhsX<OP, NB>& x, float* lds, Lane ln, int aux, NextRhs next_rhs)
{
    static_assert(METHOD == M_BLOCK || METHOD == M_MIXED, "built for the blocked and the mixed recursion");
    constexpr int NT = NB * (NB + 1) / 2;
    static_assert(NRHS == 1 || NB <= 4, "two right-hand sides: C <= 64");
    v4f Tm[NT];  // T orientation: Tm[tix(i, j)][r] = T[16 i + n][16 j + 4 q + r], exact unit diagonal, zeros above it
    {
        constexpr int LEAF = METHOD == M_MIXED ? LEAF_NEUMANN : LEAF_BLOCK_RECURSIVE;
        block_recursive<OP, NB, ROOT_T, LEAF>(src, Tm, lds, ln, aux, [&]() {
            if constexpr (ISSUE_FROM < NB && IN_MERGE) x.issue(0, ISSUE_FROM, NB);
        });
        if constexpr (ISSUE_FROM < NB && !IN_MERGE) x.issue(0, ISSUE_FROM, NB);
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = 0; j <= i; ++j) {
                v4f t = Tm[tix(i, j)];
                if (!result_is_T<NB, ROOT_T>(i, j)) t = transpose_tile(t, lds, ln);
                if (i == j) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int rr = ln.n, cc = 4 * ln.q + r;
                        t[r] = (rr == cc) ? 1.f : ((rr > cc) ? t[r] : 0.f);
                    }
                }
                Tm[tix(i, j)] = t;
            }
    }
    constexpr int VEC = RhsX<OP, NB>::VEC;
#pragma unroll
    for (int k = 0; k < NRHS; ++k) {
        if (k > 0) next_rhs(k);
        Opnd<OP> Top[NT];  // columns scaled by s in fp32, then rounded to the operand type
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int j = 0; j <= i; ++j) Top[tix(i, j)] = pack<OP>(Tm[tix(i, j)] * x.s_q[j]);
        const int n_group = x.n_group();
#pragma unroll 1
        for (int gi = 0;;) {
            Opnd<OP> xo[NB][VEC];
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int c = 0; c < VEC; ++c) xo[j][c] = x_operand<OP>(x.raw[j], c);
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                v4f acc[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = zero4();
#pragma unroll
                for (int j = 0; j <= i; ++j)
#pragma unroll
                    for (int c = 0; c < VEC; ++c) acc[c] = tn<OP>(Top[tix(i, j)], xo[j][c], acc[c]);
                x.store(gi, i, acc);
            }
            if (++gi >= n_group) break;
            x.issue(gi);
        }
    }
}

// XPOS: where the loads of X's first column group are issued -- 1: between the Gram products and the recursion (every
// tile of A is formed first, so the keys' registers are free); 2: after the recursion; 3: as many tile rows as fit beside
// the keys before the recursion, the rest inside its last merge or after it (see invert_and_apply).
// spread: see fused_matrix_index.
// (C = 64: at most two wavefronts per SIMD -- like the storing kernels, these run slower with more resident: 146 against
// 138 us at three on the batched workload, 122 against 120 us with d_k = 64, whose build would otherwise fit three)
template <int KD, int OP, int NB, int METHOD, int DKS, int WPB, int XPOS, int NRHS>
__global__ __launch_bounds__(64 * WPB) __attribute__((amdgpu_waves_per_eu(1, NB == 4 ? 2 : 8))) void k_gdn_tri_solve(const void* __restrict__ K, const float* __restrict__ beta,
                                                            const float* __restrict__ g, RhsList rhs, int64_t n_chunk, ChunkMap map,
                                                            int H, int d_k, int aux, int spread)
{
    constexpr int C = 16 * NB;
    constexpr int CORE = core_lds_floats<NB, METHOD, true>();
    constexpr int GATE = gate_lds_floats<NB>();
    constexpr int PER_WAVE = CORE > GATE ? CORE : GATE;
    __shared__ __attribute__((aligned(16))) float lds_all[WPB * PER_WAVE];
    float* lds = lds_all + ((WPB == 1) ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))) * PER_WAVE;
    const int64_t m = fused_matrix_index<WPB>(n_chunk, H, n_chunk * H, spread);  // chunk id * H + h
    if (m < 0) return;
    const uint32_t bc = (uint32_t)m / (uint32_t)H;
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const Lane ln = lane_id();
    GramA<KD, NB, DKS> src;
    src.ln = ln;
    const int64_t esz = (KD == OP_F32) ? 4 : 2;
    src.issue_gate(beta + tok0 * H + h, g ? g + tok0 * H + h : nullptr, H, pos.valid);
    src.load_keys(static_cast<const char*>(K) + (tok0 * H + h) * (int64_t)d_k * esz, (int64_t)H * d_k, pos.valid);
    RhsX<OP, NB> x;
    x.init(rhs.r[0], tok0, h, H, pos.valid, ln);
    auto next_rhs = [&](int k) {
        x.init(rhs.r[k < MAX_RHS ? k : 0], tok0, h, H, pos.valid, ln);
        x.issue(0);
    };
    src.stage_gate(lds);
    if constexpr (XPOS == 1) {
        // every tile of A first, packed (the key registers are free afterwards), then X's loads, then the recursion
        PackedA<OP, NB> pre;
        pre.fill(src);
        x.issue(0);
        invert_and_apply<OP, NB, METHOD, NB, false, NRHS>(pre, x, lds, ln, aux, next_rhs);
    } else if constexpr (XPOS == 2) {
        invert_and_apply<OP, NB, METHOD, 0, false, NRHS>(src, x, lds, ln, aux, next_rhs);
    } else {
        // the first tile rows of X before the recursion (as many as the registers beside the keys allow), the rest
        // after it: the first strips are multiplied and stored while the later rows' loads are still in flight
        constexpr int KEY_REGS = NB * DKS * 4;
        constexpr int EARLY = KEY_REGS <= 64 ? NB / 2 : KEY_REGS <= 128 ? NB / 4 : 0;
        constexpr bool IN_MERGE = KEY_REGS <= 128 && KD != OP_F32 && OP != OP_F32;  // elsewhere the registers do not allow it
        x.issue(0, 0, EARLY);
        invert_and_apply<OP, NB, METHOD, EARLY, IN_MERGE, NRHS>(src, x, lds, ln, aux, next_rhs);
    }
}

template <int OP, int NB, int METHOD, int WPB, int NRHS>
__global__ __launch_bounds__(64 * WPB) void k_kda_tri_solve(const void* __restrict__ K, const float* __restrict__ beta,
                                                            const float* __restrict__ g, RhsList rhs, int64_t n_chunk, ChunkMap map,
                                                            int H, int d_k, int k_dt, int aux, int spread)
{
    constexpr int C = 16 * NB;
    constexpr int CORE = core_lds_floats<NB, METHOD, true>();
    constexpr int PER_WAVE = CORE > C ? CORE : C;
    __shared__ __attribute__((aligned(16))) float lds_all[WPB * PER_WAVE];
    float* lds = lds_all + ((WPB == 1) ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))) * PER_WAVE;
    const int64_t m = fused_matrix_index<WPB>(n_chunk, H, n_chunk * H, spread);
    if (m < 0) return;
    const uint32_t bc = (uint32_t)m / (uint32_t)H;
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const Lane ln = lane_id();
    const int64_t esz = (k_dt == OP_F32) ? 4 : 2;
    const int64_t e0 = (tok0 * H + h) * (int64_t)d_k;
    PreA<NB> src;
    build_A_per_channel<OP, NB, METHOD>(src, static_cast<const char*>(K) + e0 * esz, k_dt, g + e0, (int64_t)H * d_k,
                                        beta + tok0 * H + h, H, d_k, lds, ln, pos.valid);
    RhsX<OP, NB> x;  // after the Gram passes, which need the registers
    x.init(rhs.r[0], tok0, h, H, pos.valid, ln);
    auto next_rhs = [&](int k) {
        x.init(rhs.r[k < MAX_RHS ? k : 0], tok0, h, H, pos.valid, ln);
        x.issue(0);
    };
    x.issue(0);
    invert_and_apply<OP, NB, METHOD, NB, false, NRHS>(src, x, lds, ln, aux, next_rhs);
}

// Scalar / no-gate kinds for head dimensions without a specialised build (any multiple of 32): the channel-loop Gram of
// the storing kernel, then the same recursion and products.  One wavefront per workgroup.
template <int KD, int OP, int NB, int METHOD, int NRHS>
__global__ __launch_bounds__(64) void k_gdn_any_dk_tri_solve(const void* __restrict__ K, const float* __restrict__ beta,
                                                             const float* __restrict__ g, RhsList rhs, int64_t n_chunk, ChunkMap map,
                                                             int H, int d_k, int aux)
{
    constexpr int C = 16 * NB;
    constexpr int CORE = core_lds_floats<NB, METHOD, true>();
    constexpr int GATE = gate_lds_floats<NB>();
    __shared__ __attribute__((aligned(16))) float lds[CORE > GATE ? CORE : GATE];
    const int64_t m = head_group_swizzle(blockIdx.x, n_chunk, H);
    const uint32_t bc = (uint32_t)m / (uint32_t)H;
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const Lane ln = lane_id();
    const int64_t esz = (KD == OP_F32) ? 4 : 2;
    PreA<NB> src;
    build_A_scalar_any_dk<KD, NB, METHOD>(src, static_cast<const char*>(K) + (tok0 * H + h) * (int64_t)d_k * esz, (int64_t)H * d_k,
                                          beta + tok0 * H + h, g ? g + tok0 * H + h : nullptr, H, d_k, lds, ln, pos.valid);
    RhsX<OP, NB> x;
    x.init(rhs.r[0], tok0, h, H, pos.valid, ln);
    auto next_rhs = [&](int k) {
        x.init(rhs.r[k < MAX_RHS ? k : 0], tok0, h, H, pos.valid, ln);
        x.issue(0);
    };
    x.issue(0);
    invert_and_apply<OP, NB, METHOD, NB, false, NRHS>(src, x, lds, ln, aux, next_rhs);
}

}  // namespace triinv
