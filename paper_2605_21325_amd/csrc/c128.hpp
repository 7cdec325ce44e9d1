// C = 128: one chunk matrix per workgroup of TWO wavefronts (blocked 2 x 2 recursion, paper Sec. 3.3, Eq. 7 in its
// lower-triangular reading, taken literally at the top level):
//     inv [[A11, 0], [A21, A22]] = [[T11, 0], [-T22 A21 T11, T22]].
// Wave 0 owns the top 64 rows of the chunk (keys, A11, T11), wave 1 the bottom 64 (keys, A22, T22); each inverts its
// 64 x 64 diagonal block in registers exactly as the one-wavefront C = 64 kernels do.  The keys the other wave needs and
// the packed tiles of T11 / T22 are exchanged through LDS, and the off-diagonal block W = -T22 (A21 T11) is split by tile
// COLUMNS: wave 0 forms columns {0, 3}, wave 1 columns {1, 2} (20 + 20 tile products each; a wave forms the tiles of A21
// it needs itself, from its own keys and the other half's keys in LDS).  Wave 0 stores rows 0..63, wave 1 rows 64..127
// (wave 0's tiles of W reach it through LDS), so each wave reads 64 key rows and writes 32 KB: half a matrix per
// wavefront streams measurably faster than a whole one (a data mover with this access pattern: 130 against 138 us on
// the 8192 matrices of the stress workload), and the two halves of the recursion run side by side.
#pragma once
#include "kernels.hpp"

namespace triinv {

// The 64 key rows of one half of the chunk in matrix-core operand layout (as GramA holds a whole chunk's).
template <int KD, int DKS> struct HalfKeys {
    typedef typename KeyVec<KD>::type kvec;
    static constexpr int KSTEP = (KD == OP_F32) ? 16 : 32;
    kvec k[4][DKS];

    // Kc: first key element of (chunk row 0, this head); rows row0 .. row0 + 63 of the chunk; rows >= valid read the
    // chunk's last real token (a valid address) and become zero keys.
    __device__ __forceinline__ void load(const void* Kc, int64_t row_stride, int valid, int row0, Lane ln)
    {
        constexpr int per_lane = (KD == OP_F32) ? 4 : 8;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int s = 0; s < DKS; ++s) {
                const int row = row0 + 16 * i + ln.n;
                const int64_t off = (int64_t)(row < valid ? row : valid - 1) * row_stride + KSTEP * s + per_lane * ln.q;
                if (KD == OP_F32)
                    k[i][s] = *reinterpret_cast<const kvec*>(static_cast<const float*>(Kc) + off);
                else
                    k[i][s] = *reinterpret_cast<const kvec*>(static_cast<const uint16_t*>(Kc) + off);
            }
        if (row0 + 64 > valid) {  // wave-uniform: only a sequence's last chunk comes here
            const kvec zero = __builtin_bit_cast(kvec, v4u{0u, 0u, 0u, 0u});
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int s = 0; s < DKS; ++s)
                    if (row0 + 16 * i + ln.n >= valid) k[i][s] = zero;
        }
    }
};

// LDS of one workgroup: the bottom half's keys and tile rows 1..3 of the top half's (operand layout:
// [tile row][k-step][lane], 16 bytes each), the packed tiles of T22 (all ten, T orientation: left factors) and of T11
// that the other wave needs (N orientation: right factors), wave 0's private area (gate staging, tile transposes, leaf
// staging) and wave 1's.  The two store strips take the place of the keys, which are dead by then.
// WITH_MAIL (the storing kernel): wave 0's private area is 8 KB and later carries its tiles of W to wave 1.  With 16-bit
// keys of d_k = 128 that makes 45 KB, three workgroups = six wavefronts per compute unit, which the storing kernel
// measured best at (140.5 us on the stress workload against 142.6 us at four: the kernel alternates between memory
// phases and arithmetic, and other resident wavefronts keep the memory system busy meanwhile).  Without the mail (the
// applied-inverse kernels, which publish their tiles elsewhere) the same case takes 38 KB and four workgroups fit,
// which those kernels measured best at (154 against 163 us).
template <int KD, int OP, int DKS, int METHOD, bool WITH_MAIL = true> struct C128Lds {
    static constexpr int KEY_TILE_ROW = DKS * 64 * 16;                     // bytes of one 16-row tile row of keys
    static constexpr int KEYS_BOT = 0;                                     // 4 tile rows
    static constexpr int KEYS_TOP = KEYS_BOT + 4 * KEY_TILE_ROW;           // tile rows 1..3
    static constexpr int STRIPS = 0;                                       // one store strip per wave (alias the keys)
    static constexpr int KEYS_END = (KEYS_TOP + 3 * KEY_TILE_ROW) > 2 * STORE_LDS_FLOATS * 4 || !WITH_MAIL ? (KEYS_TOP + 3 * KEY_TILE_ROW) : 2 * STORE_LDS_FLOATS * 4;
    static constexpr int OPND = (int)sizeof(Opnd<OP>);
    static constexpr int T22 = KEYS_END;                                   // 10 tiles
    static constexpr int T11 = T22 + 10 * 64 * OPND;                       // tiles (1,1) (2,1) (3,1) (2,2) (3,2)
    static constexpr int PRIVATE_FLOATS = METHOD == M_BLOCK_DIRECT ? LEAF_FWD_FLOATS : XPOSE_FLOATS;
    static constexpr int PRIVATE0 = T11 + 5 * 64 * OPND;                   // wave 0's private area
    static constexpr int MAIL = PRIVATE0;                                  // (WITH_MAIL) 8 fp32 tiles, after wave 0's private use of the same bytes
    static constexpr int PRIVATE1 = PRIVATE0 + (WITH_MAIL ? 8 * 1024 : PRIVATE_FLOATS * 4);  // wave 1's private area
    static constexpr int BYTES = PRIVATE1 + PRIVATE_FLOATS * 4;
    static_assert(XPOSE_FLOATS >= 2 * 128 && 2048 >= LEAF_FWD_FLOATS, "the private areas fit their users");
    static_assert(PRIVATE0 % 16 == 0 && PRIVATE1 % 16 == 0, "16-byte accesses");
};

// Slot of tile (d, c) of T11 in the LDS copy (only the five tiles wave 1 reads are there).
__host__ __device__ constexpr int c128_t11_slot(int d, int c) { return c == 1 ? d - 1 : (d - 2) + 3; }

// Tile source of a wave's own 64 x 64 diagonal block: Gram products of its own keys, the scalar gate of the whole
// chunk (tile rows / columns 4 W .. 4 W + 3).
template <int KD, int DKS, int W, bool NOGATE> struct DiagA {
    static constexpr bool kFromMemory = false;
    const HalfKeys<KD, DKS>& hk;
    const GateVec<8, NOGATE>& gate;
    Lane ln;
    template <bool TR> __device__ __forceinline__ v4f get(int i, int j) const
    {
        v4f s = zero4();
#pragma unroll
        for (int t = 0; t < DKS; ++t) s = TR ? gram_step<KD>(hk.k[j][t], hk.k[i][t], s) : gram_step<KD>(hk.k[i][t], hk.k[j][t], s);
        return gate.template apply<TR>(4 * W + i, 4 * W + j, s, ln);
    }
};

template <int METHOD> constexpr int c128_leaf()
{
    return METHOD == M_MIXED ? LEAF_NEUMANN : METHOD == M_MIXED32 ? LEAF_NEUMANN32 : METHOD == M_BLOCK_DIRECT ? LEAF_FORWARD : LEAF_BLOCK_RECURSIVE;
}

// The inverse of one chunk matrix, distributed over the two waves: wave W holds its diagonal block D (10 lower tiles,
// fp32; wave 0: T11 in N orientation, wave 1: T22 in T orientation; diagonal tiles not yet masked to unit form) and
// the tiles Wc[k][a] of W = -T22 A21 T11 (N orientation) in tile rows a = 0..3 of its two columns: wave 0 columns
// {0, 3}, wave 1 columns {1, 2} (k = 0, 1 in that order).
template <int W> __host__ __device__ constexpr int c128_col(int k) { return W == 0 ? (k == 0 ? 0 : 3) : (k == 0 ? 1 : 2); }

template <int OP, int W>
__device__ __forceinline__ void c128_merge(const Opnd<OP> (&a21)[4][4], const v4f (&D)[10], v4f (&Wc)[2][4], const Opnd<OP>* t11_lds,
                                           const Opnd<OP>* t22_lds, Lane ln);

// A wave's own 64 x 64 diagonal block: the C = 64 recursion on the tile source `diag`; wave 0 produces an N block (the
// right factor of the merge), wave 1 a T block (the left factor); the packed tiles the other wave needs go to LDS (no
// barrier here).  small: the wave's private LDS area.
template <int OP, int METHOD, int W, class DiagSrc>
__device__ __forceinline__ void c128_diagonal_block(const DiagSrc& diag, v4f (&D)[10], float* small, Opnd<OP>* t11_lds, Opnd<OP>* t22_lds,
                                                    int aux, Lane ln)
{
    const int lane = 16 * ln.q + ln.n;
    v4f leaves[8];
    block_recursive<OP, 4, W == 1, c128_leaf<METHOD>()>(diag, D, small, ln, aux, NoHook(), leaves);
    if (W == 0) {
        D[tix(3, 2)] = transpose_tile(D[tix(3, 2)], small, ln);  // the odd child of the block came out in T orientation
#pragma unroll
        for (int d = 0; d < 4; ++d) D[tix(d, d)] = leaves[2 * d];
#pragma unroll
        for (int c = 1; c <= 2; ++c)
#pragma unroll
            for (int d = c; d < 4; ++d) t11_lds[c128_t11_slot(d, c) * 64 + lane] = pack<OP>(D[tix(d, c)]);
    } else {
        D[tix(1, 0)] = transpose_tile(D[tix(1, 0)], small, ln);  // the even child came out in N orientation
#pragma unroll
        for (int d = 0; d < 4; ++d) D[tix(d, d)] = leaves[2 * d + 1];
#pragma unroll
        for (int t = 0; t < 10; ++t) t22_lds[t * 64 + lane] = pack<OP>(D[t]);
    }
}

// Everything up to the two waves' shares of the inverse.  lds: the workgroup's C128Lds bytes.
// keys_loaded(): called between the issue of the key loads and their first use (a place for further independent memory
// operations).  block_done(): called right after the workgroup barrier that follows the diagonal blocks, when this
// wave's block D is final (a place to send it on its way while the off-diagonal block is formed).
// keys_done(): called in the second phase once this wave's tiles of A21 exist: the keys' registers and the gate's are
// free from there on, and 40 tile products follow (a place to start loads whose data is needed after them).
template <int KD, int OP, int METHOD, int DKS, int W, bool WITH_MAIL = true, bool NOGATE = false, class Hook, class Hook2, class Hook3 = NoHook>
__device__ __forceinline__ void c128_invert(char* lds, const void* Kc, int64_t row_stride, const float* bc, const float* gc,
                                            int64_t tok_stride, int valid, int aux, Lane ln, v4f (&D)[10], v4f (&Wc)[2][4],
                                            Hook keys_loaded, Hook2 block_done, Hook3 keys_done = Hook3())
{
    typedef typename KeyVec<KD>::type kvec;
    typedef C128Lds<KD, OP, DKS, METHOD, WITH_MAIL> LY;
    const int lane = 16 * ln.q + ln.n;
    float* small = reinterpret_cast<float*>(lds + (W == 0 ? LY::PRIVATE0 : LY::PRIVATE1));
    kvec* keys_bot = reinterpret_cast<kvec*>(lds + LY::KEYS_BOT);   // [tile row 0..3][k-step][lane]
    kvec* keys_top = reinterpret_cast<kvec*>(lds + LY::KEYS_TOP);   // [tile row 1..3][k-step][lane]
    Opnd<OP>* t22_lds = reinterpret_cast<Opnd<OP>*>(lds + LY::T22);
    Opnd<OP>* t11_lds = reinterpret_cast<Opnd<OP>*>(lds + LY::T11);
    GateVec<8, NOGATE> gate;
    gate.issue(bc, gc, tok_stride, ln, valid);
    HalfKeys<KD, DKS> hk;
    hk.load(Kc, row_stride, valid, 64 * W, ln);
    keys_loaded();
    gate.stage(small, ln);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int s = 0; s < DKS; ++s) {
            if (W == 1)
                keys_bot[(i * DKS + s) * 64 + lane] = hk.k[i][s];
            else if (i >= 1)
                keys_top[((i - 1) * DKS + s) * 64 + lane] = hk.k[i][s];
        }

    const DiagA<KD, DKS, W, NOGATE> diag{hk, gate, ln};
    c128_diagonal_block<OP, METHOD, W>(diag, D, small, t11_lds, t22_lds, aux, ln);
    __syncthreads();  // the keys and the diagonal-block inverses the other wave needs are in LDS
    block_done();

    // tiles of A21 this wave needs (columns d >= its smallest column), T orientation: a21[b][d] = A(4 + b, d)^T
    constexpr int DMIN = W == 0 ? 0 : 1;
    Opnd<OP> a21[4][4];
    if (W == 0) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            kvec kb[DKS];
#pragma unroll
            for (int s = 0; s < DKS; ++s) kb[s] = keys_bot[(b * DKS + s) * 64 + lane];
#pragma unroll
            for (int d = DMIN; d < 4; ++d) {
                v4f g = zero4();
#pragma unroll
                for (int s = 0; s < DKS; ++s) g = gram_step<KD>(hk.k[d][s], kb[s], g);
                a21[b][d] = pack<OP>(gate.template apply<true>(4 + b, d, g, ln));
            }
        }
    } else {
#pragma unroll
        for (int d = DMIN; d < 4; ++d) {
            kvec kt[DKS];
#pragma unroll
            for (int s = 0; s < DKS; ++s) kt[s] = keys_top[((d - 1) * DKS + s) * 64 + lane];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                v4f g = zero4();
#pragma unroll
                for (int s = 0; s < DKS; ++s) g = gram_step<KD>(kt[s], hk.k[b][s], g);
                a21[b][d] = pack<OP>(gate.template apply<true>(4 + b, d, g, ln));
            }
        }
    }
    keys_done();
    c128_merge<OP, W>(a21, D, Wc, t11_lds, t22_lds, ln);
}

// The off-diagonal block: this wave's two tile columns of W = -T22 (A21 T11), from its tiles of A21 (a21[b][d] =
// A(4 + b, d) in T orientation, columns d >= its smallest column), its own diagonal block D and the other wave's in LDS.
template <int OP, int W>
__device__ __forceinline__ void c128_merge(const Opnd<OP> (&a21)[4][4], const v4f (&D)[10], v4f (&Wc)[2][4], const Opnd<OP>* t11_lds,
                                           const Opnd<OP>* t22_lds, Lane ln)
{
    const int lane = 16 * ln.q + ln.n;
    // the factors: own block from registers, the other wave's from LDS
    Opnd<OP> t11[10], t22[10];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int d = c; d < 4; ++d) {
            if (W == 0)
                t11[tix(d, c)] = pack<OP>(D[tix(d, c)]);
            else if (c == 1 || c == 2)
                t11[tix(d, c)] = t11_lds[c128_t11_slot(d, c) * 64 + lane];
        }
#pragma unroll
    for (int t = 0; t < 10; ++t) t22[t] = W == 1 ? pack<OP>(D[t]) : t22_lds[t * 64 + lane];
    // W(:, c) = -T22 (A21 T11(:, c)) for this wave's two columns
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        constexpr int c0 = c128_col<W>(0), c1 = c128_col<W>(1);
        const int c = k == 0 ? c0 : c1;
        Opnd<OP> P[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            v4f acc = zero4();
#pragma unroll
            for (int d = 0; d < 4; ++d)
                if (d >= c) acc = tn<OP>(a21[b][d], t11[tix(d, c)], acc);
            P[b] = negated<OP>(pack<OP>(acc));  // the sign of -T22 (A21 T11)
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            v4f acc = zero4();
#pragma unroll
            for (int b = 0; b <= a; ++b) acc = tn<OP>(t22[tix(a, b)], P[b], acc);
            Wc[k][a] = acc;
        }
    }
}

// The dense result in whole 512-byte rows (1 KB-contiguous stores), both waves at the end and at the same time (wave 0
// rows 0..63, wave 1 rows 64..127 with wave 0's tiles of W fetched from LDS): 32 KB per wave.  Measured slower: wave 0
// storing its rows as soon as T11 is final (149 against 142 us on the stress workload), and 256-byte half rows written
// as soon as each 64 x 64 block is final (148 us).
template <int W>
__device__ __forceinline__ void c128_store_result(v4f* mail, float* strip, Out Tm, const v4f (&D)[10], const v4f (&Wc)[2][4], Lane ln);

template <int KD, int OP, int METHOD, int DKS, int W, bool NOGATE>
__device__ __forceinline__ void c128_invert_and_store(char* lds, const void* Kc, int64_t row_stride, const float* bc, const float* gc,
                                                      int64_t tok_stride, int valid, int aux, Out Tm, Lane ln)
{
    typedef C128Lds<KD, OP, DKS, METHOD> LY;
    v4f D[10], Wc[2][4];
    c128_invert<KD, OP, METHOD, DKS, W, true, NOGATE>(lds, Kc, row_stride, bc, gc, tok_stride, valid, aux, ln, D, Wc, NoHook(), NoHook());
    c128_store_result<W>(reinterpret_cast<v4f*>(lds + LY::MAIL), reinterpret_cast<float*>(lds + LY::STRIPS) + W * STORE_LDS_FLOATS, Tm, D,
                         Wc, ln);
}

// mail: 8 KB of LDS for wave 0's tiles of W; strip: this wave's store strip (may take the place of anything the waves have
// finished with before the barrier inside).
template <int W>
__device__ __forceinline__ void c128_store_result(v4f* mail, float* strip, Out Tm, const v4f (&D)[10], const v4f (&Wc)[2][4], Lane ln)
{
    const int lane = 16 * ln.q + ln.n;
    if (W == 0) {
#pragma unroll
        for (int k = 0; k < 2; ++k)
#pragma unroll
            for (int a = 0; a < 4; ++a) mail[(4 * k + a) * 64 + lane] = Wc[k][a];
    }
    __syncthreads();  // wave 0's tiles of W are in LDS, and nobody reads the keys any more
    zero_strip_patch(strip, ln);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v4f row[8];
        if (W == 0) {
#pragma unroll
            for (int j = 0; j <= i; ++j) row[j] = D[tix(i, j)];
            store_strip<8, true>(Tm, i, row, [](int) { return false; }, strip, ln);
        } else {
            row[0] = mail[i * 64 + lane];
            row[1] = Wc[0][i];
            row[2] = Wc[1][i];
            row[3] = mail[(4 + i) * 64 + lane];
#pragma unroll
            for (int j = 0; j <= i; ++j) row[4 + j] = D[tix(i, j)];
            store_strip<8, true>(Tm, 4 + i, row, [](int j) { return j >= 4; }, strip, ln);
        }
    }
}

// Fused kernel, scalar / no-gate kinds, C = 128, d_k = 64 or 128 (DKS k-steps): blocked, mixed (b0 = 16, 32) and
// direct-leaf recursion.  One workgroup of two wavefronts per matrix; workgroups of the H heads of one (batch, chunk)
// run back to back on one XCD (head_group_swizzle).
template <int KD, int OP, int METHOD, int DKS, bool NOGATE>
__global__ __launch_bounds__(128) void k_gdn_tri_inv_c128(const void* __restrict__ K, const float* __restrict__ beta,
                                                          const float* __restrict__ g, float* __restrict__ T, int64_t n_chunk,
                                                          ChunkMap map, int H, int d_k, int aux, int out_dt)
{
    constexpr int C = 128;
    __shared__ __attribute__((aligned(16))) char lds[C128Lds<KD, OP, DKS, METHOD>::BYTES];
    const int64_t m = head_group_swizzle(blockIdx.x, n_chunk, H);
    const uint32_t bc = (uint32_t)m / (uint32_t)H;
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const Lane ln = lane_id();
    const int64_t esz = (KD == OP_F32) ? 4 : 2;
    const void* Kc = static_cast<const char*>(K) + (tok0 * H + h) * (int64_t)d_k * esz;
    const float* bcp = beta + tok0 * H + h;
    const float* gcp = g ? g + tok0 * H + h : nullptr;
    const Out Tm = out_matrix(T, m, C, out_dt);
    if (w == 0)
        c128_invert_and_store<KD, OP, METHOD, DKS, 0, NOGATE>(lds, Kc, (int64_t)H * d_k, bcp, gcp, H, pos.valid, aux, Tm, ln);
    else
        c128_invert_and_store<KD, OP, METHOD, DKS, 1, NOGATE>(lds, Kc, (int64_t)H * d_k, bcp, gcp, H, pos.valid, aux, Tm, ln);
}

}  // namespace triinv
