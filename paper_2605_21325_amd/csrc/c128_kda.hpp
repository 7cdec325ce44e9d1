// C = 128 with the per-channel gate (paper Table 1, KDA row) on the two-wavefront layout of c128.hpp:
//     A_ij = beta_i sum_c k_ic k_jc exp(g_ic - g_jc) = beta_i [(K * exp(G - a)) (K * exp(a - G))^T]_ij   for any anchor a.
// Each wave streams its own 64 rows of K and G once, 32 channels at a time, and accumulates on the matrix cores
//   - the tiles of its 64 x 64 diagonal block, with one anchor per 16-row tile row (the first row of that tile row of
//     G, exactly as the C <= 64 kernels do: every exponent is <= 0 or within the decay of 16 tokens);
//   - its tiles of the off-diagonal block A21 with ONE anchor, the chunk's row 64: the bottom rows' factor
//     k_i exp(g_i - a) and the top rows' factor k_j exp(a - g_j) both have exponents <= 0 (log-decays only fall along a
//     chunk), so neither can overflow however strong the decay is.  The bottom wave forms the first kind of factor from
//     its rows, the top wave the second; the two exchange them through LDS, 32 channels at a time (double-buffered,
//     one workgroup barrier per step), and each accumulates two tile columns of A21 (exchanged, packed, at the end).
// Then the recursion, the merge and the store of c128.hpp.  The gated keys are rounded to the operand type OP.
#pragma once
#include "c128.hpp"

namespace triinv {

// Which tiles of its diagonal block (and in which orientation) the C = 64 recursion of wave W asks for: its root block
// is produced in N orientation by wave 0 and in T orientation by wave 1 (see c128_diagonal_block).
template <int METHOD, bool ROOT_IS_T> __host__ __device__ constexpr bool c128_need_tile(int i, int j, bool tr)
{
    if (METHOD == M_MIXED32 && i / 2 == j / 2) return true;
    if (i == j) return METHOD == M_BLOCK_DIRECT ? tr : true;
    const bool block_t = (i / 2 == j / 2) ? ((i / 2) & 1) != 0 : ROOT_IS_T;
    return block_t ? !tr : tr;
}

template <int OP, int METHOD> struct C128KdaLds {
    static constexpr int GOP = (int)sizeof(GOp<OP>);                       // one k-step operand per lane: 16 or 32 bytes
    static constexpr int XCHG = 0;                                         // [buffer 0..1][wave][tile row 0..3][lane]
    static constexpr int XCHG_BYTES = 2 * 2 * 4 * 64 * GOP;
    static constexpr int STRIPS = 0;                                       // the store strips take its place at the end
    static constexpr int SHARED_END = XCHG_BYTES > 2 * STORE_LDS_FLOATS * 4 ? XCHG_BYTES : 2 * STORE_LDS_FLOATS * 4;
    static constexpr int OPND = (int)sizeof(Opnd<OP>);
    static constexpr int T22 = SHARED_END;
    static constexpr int T11 = T22 + 10 * 64 * OPND;
    static constexpr int MAIL = T11 + 5 * 64 * OPND;                       // before the merge: wave 0's private area
    static constexpr int PRIVATE1 = MAIL + 8 * 1024;
    static constexpr int PRIVATE1_FLOATS = METHOD == M_BLOCK_DIRECT ? LEAF_FWD_FLOATS : XPOSE_FLOATS;
    static constexpr int ANCHORS = PRIVATE1 + PRIVATE1_FLOATS * 4;         // per wave: anchors [q][5][8], factors [q][10][8]
    static constexpr int ANCHOR_FLOATS = 4 * 5 * 8 + 4 * 10 * 8;
    static constexpr int BYTES = ANCHORS + 2 * ANCHOR_FLOATS * 4;
};

// Index of the pair (i, j), i > j, of tile rows in the factor table.
__host__ __device__ constexpr int c128_pair(int i, int j) { return i * (i - 1) / 2 + j; }

// The Gram passes of wave W.  pre: the tiles of its diagonal block (fp32, both orientations where asked for);
// a21[b][d]: A(4 + b, d) in T orientation for this wave's columns d (wave 0: d = 0, 1; wave 1: d = 2, 3); all still
// without beta and the mask.
// Exponentials.  With e_i = (g_i - a_I) log2 e (row i, its tile row's anchor a_I), u_i = k_i 2^(e_i) is the left factor of
// every tile in tile row I and v_j = k_j 2^(-e_j) the right factor of the diagonal tile (J, J).  Every other right
// factor differs from v_j by a factor that depends on the channel only, not on the row: tile (I, J), J < I, needs
// v_j 2^((a_I - a_J) log2 e), the off-diagonal block u_i 2^((a_I - a_mid) log2 e) and v_j 2^((a_mid - a_J) log2 e).  Those
// 10 x 32 channel-only factors are computed once per k-step by the whole wave (five per lane, through LDS) instead of once
// per row: 69 exponentials per lane and k-step instead of 144.
// Kc / gc: element (chunk row 0, this head, channel 0); row_stride in elements (the same for both).
// tab: this wave's ANCHOR_FLOATS floats of LDS.
template <int OP, int METHOD, bool K16, int W>
__device__ __forceinline__ void c128_kda_gram(char* xchg, float* tab, PreA<4>& pre, v4f (&a21)[4][2], const void* Kc, bool is_f16,
                                              const float* gc, int64_t row_stride, int d_k, Lane ln, int valid)
{
    constexpr float LOG2E = 1.44269504088896340736f;
    constexpr int STEPS = K16 ? 2 : 1;  // 16-bit keys: both k-steps of a 128-byte line of keys are requested together
    const int lane = 16 * ln.q + ln.n;
    GOp<OP>* xb = reinterpret_cast<GOp<OP>*>(xchg);
    float* anc = tab + ln.q * 40;            // [5][8]: anchors of tile rows 0..3 of this half, then the chunk's row 64
    float* fac = tab + 160 + ln.q * 80;      // [10][8]: pairs (i > j) by c128_pair, then the off-diagonal block's four
    int rowc[4];
    float keep[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = 64 * W + 16 * i + ln.n;
        rowc[i] = row < valid ? row : valid - 1;
        keep[i] = row < valid ? 1.f : 0.f;
    }
    const int mid = 64 < valid ? 64 : valid - 1;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            pre.n[tix(i, j)] = zero4();
            pre.t[tix(i, j)] = zero4();
        }
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int d = 0; d < 2; ++d) a21[b][d] = zero4();

    const int n_step = d_k / 32;
    for (int s0 = 0; s0 < n_step; s0 += STEPS) {
        RawKey8<K16> raw[STEPS][4];
#pragma unroll
        for (int t = 0; t < STEPS; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (s0 + t < n_step) raw[t][i] = load_key8<K16>(Kc, (int64_t)rowc[i] * row_stride + 32 * (s0 + t) + 8 * ln.q);
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            const int s = s0 + t;
            if (s >= n_step) break;
            const int ch = 32 * s + 8 * ln.q;
            // gate rows, tile-row anchors and the chunk's row 64 for this k-step, all loads first
            v4f G[4][2], An[5][2];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t off = (int64_t)rowc[i] * row_stride + ch;
                G[i][0] = *reinterpret_cast<const v4f*>(gc + off);
                G[i][1] = *reinterpret_cast<const v4f*>(gc + off + 4);
                const int ar = 64 * W + 16 * i < valid ? 64 * W + 16 * i : valid - 1;
                An[i][0] = *reinterpret_cast<const v4f*>(gc + (int64_t)ar * row_stride + ch);
                An[i][1] = *reinterpret_cast<const v4f*>(gc + (int64_t)ar * row_stride + ch + 4);
            }
            An[4][0] = *reinterpret_cast<const v4f*>(gc + (int64_t)mid * row_stride + ch);
            An[4][1] = *reinterpret_cast<const v4f*>(gc + (int64_t)mid * row_stride + ch + 4);
            // the channel-only factors: anchors to LDS (every lane of a row group holds the same values; one writes), five
            // table entries per lane, back through LDS
            if (ln.n == 0) {
#pragma unroll
                for (int i = 0; i < 5; ++i) {
                    *reinterpret_cast<v4f*>(&anc[8 * i]) = An[i][0];
                    *reinterpret_cast<v4f*>(&anc[8 * i + 4]) = An[i][1];
                }
            }
            wave_lds_sync();
#pragma unroll
            for (int k = 0; k < 5; ++k) {
                const int e = ln.n + 16 * k, p = e >> 3, r = e & 7;
                int hi, lo;                                      // the factor is 2^((anchor hi - anchor lo) log2 e)
                if (p < 6) {
                    hi = p >= 3 ? 3 : (p >= 1 ? 2 : 1);
                    lo = p - hi * (hi - 1) / 2;
                } else {
                    hi = W == 1 ? p - 6 : 4;
                    lo = W == 1 ? 4 : p - 6;
                }
                fac[e] = __builtin_amdgcn_exp2f((anc[8 * hi + r] - anc[8 * lo + r]) * LOG2E);
            }
            wave_lds_sync();
            // pass 1 over the rows: u (left factors, packed), v (right factors of the diagonal tiles, fp32), and this wave's
            // factor of the off-diagonal block, which goes to the other wave
            GOp<OP> ppi[4], mine[4];
            float v[4][8];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float kv[8], u[8], m[8];
                widen_key8<K16>(raw[t][i], is_f16, kv);
                const v4f f0 = *reinterpret_cast<const v4f*>(&fac[8 * (6 + i)]), f1 = *reinterpret_cast<const v4f*>(&fac[8 * (6 + i) + 4]);
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const float kk = kv[r] * keep[i];
                    const float e = (G[i][r / 4][r % 4] - An[i][r / 4][r % 4]) * LOG2E;
                    u[r] = kk * __builtin_amdgcn_exp2f(e);
                    v[i][r] = kk * __builtin_amdgcn_exp2f(-e);
                    m[r] = (W == 1 ? u[r] : v[i][r]) * (r < 4 ? f0[r] : f1[r - 4]);
                }
                ppi[i] = gpack<OP>(u);
                mine[i] = gpack<OP>(m);
                if (W == 1 || i >= 2) xb[(((s & 1) * 2 + W) * 4 + i) * 64 + lane] = mine[i];  // (the top wave's rows 0, 1 stay at home)
            }
            // pass 2: the diagonal block
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j <= i; ++j) {
                    float dn[8];
                    if (i == j) {
#pragma unroll
                        for (int r = 0; r < 8; ++r) dn[r] = v[j][r];
                    } else {
                        const v4f f0 = *reinterpret_cast<const v4f*>(&fac[8 * c128_pair(i, j)]);
                        const v4f f1 = *reinterpret_cast<const v4f*>(&fac[8 * c128_pair(i, j) + 4]);
#pragma unroll
                        for (int r = 0; r < 8; ++r) dn[r] = v[j][r] * (r < 4 ? f0[r] : f1[r - 4]);
                    }
                    const GOp<OP> pmj = gpack<OP>(dn);
                    if (c128_need_tile<METHOD, W == 1>(i, j, false)) pre.n[tix(i, j)] = gstep<OP>(ppi[i], pmj, pre.n[tix(i, j)]);
                    if (c128_need_tile<METHOD, W == 1>(i, j, true)) pre.t[tix(i, j)] = gstep<OP>(pmj, ppi[i], pre.t[tix(i, j)]);
                }
            __syncthreads();  // both waves' factors of this k-step are in LDS (the buffer of the step before last is free again)
            // A(4 + b, d)^T += (top factor d)(bottom factor b)^T for this wave's two columns d
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                if (W == 0) {  // o = bottom tile row b, from the other wave; own top rows d = 0, 1
                    const GOp<OP> up_b = xb[(((s & 1) * 2 + 1) * 4 + o) * 64 + lane];
#pragma unroll
                    for (int d = 0; d < 2; ++d) a21[o][d] = gstep<OP>(mine[d], up_b, a21[o][d]);
                } else if (o >= 2) {  // o = top tile row d = 2, 3, from the other wave; own bottom rows b
                    const GOp<OP> dn_d = xb[(((s & 1) * 2 + 0) * 4 + o) * 64 + lane];
#pragma unroll
                    for (int b = 0; b < 4; ++b) a21[b][o - 2] = gstep<OP>(dn_d, mine[b], a21[b][o - 2]);
                }
            }
        }
    }
}

template <int OP, int METHOD, int W>
__device__ __forceinline__ void c128_kda_invert(char* lds, const void* Kc, int kd, const float* gc, int64_t row_stride, const float* bc,
                                                int64_t tok_stride, int d_k, int valid, int aux, Lane ln, v4f (&D)[10], v4f (&Wc)[2][4])
{
    typedef C128KdaLds<OP, METHOD> LY;
    const int lane = 16 * ln.q + ln.n;
    float* small = reinterpret_cast<float*>(lds + (W == 0 ? LY::MAIL : LY::PRIVATE1));
    float* tab = reinterpret_cast<float*>(lds + LY::ANCHORS) + W * LY::ANCHOR_FLOATS;
    Opnd<OP>* t22_lds = reinterpret_cast<Opnd<OP>*>(lds + LY::T22);
    Opnd<OP>* t11_lds = reinterpret_cast<Opnd<OP>*>(lds + LY::T11);
    Opnd<OP>* a21_lds = reinterpret_cast<Opnd<OP>*>(lds + LY::XCHG);  // after the Gram passes: [b][d][lane], 16 packed tiles of A21
    // beta of this lane's two tokens: in flight during the Gram passes
    float raw_b[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int row = lane + 64 * t;
        raw_b[t] = row < valid ? bc[row * tok_stride] : 0.f;
    }
    PreA<4> pre;
    v4f acc21[4][2];
    if (kd == OP_F32)
        c128_kda_gram<OP, METHOD, false, W>(lds + LY::XCHG, tab, pre, acc21, Kc, false, gc, row_stride, d_k, ln, valid);
    else
        c128_kda_gram<OP, METHOD, true, W>(lds + LY::XCHG, tab, pre, acc21, Kc, kd == OP_F16, gc, row_stride, d_k, ln, valid);
    // beta_i row scaling and the strictly-lower mask
    small[lane] = raw_b[0];
    small[lane + 64] = raw_b[1];
    wave_lds_sync();
    Opnd<OP> a21[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float bn = small[64 * W + 16 * i + ln.n];
        const v4f bq = *reinterpret_cast<const v4f*>(&small[64 * W + 16 * i + 4 * ln.q]);
#pragma unroll
        for (int j = 0; j <= i; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool lowN = (i != j) || (4 * ln.q + r > ln.n), lowT = (i != j) || (ln.n > 4 * ln.q + r);
                pre.n[tix(i, j)][r] = lowN ? bq[r] * pre.n[tix(i, j)][r] : 0.f;
                pre.t[tix(i, j)][r] = lowT ? bn * pre.t[tix(i, j)][r] : 0.f;
            }
        const float bn_bot = small[64 + 16 * i + ln.n];  // tile row 4 + i of the chunk, T orientation: its row index is the lane's n
#pragma unroll
        for (int d = 0; d < 2; ++d) a21[i][2 * W + d] = pack<OP>(acc21[i][d] * bn_bot);
    }
    wave_lds_sync();
    __syncthreads();  // the last k-step's factors have been read: the exchange area is free
    // the packed tiles of A21 the other wave's columns of the merge need: wave 0 (columns 0, 3) takes d = 2, 3 from wave 1,
    // wave 1 (columns 1, 2) takes d = 1 from wave 0
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (W == 0) {
            a21_lds[(b * 4 + 1) * 64 + lane] = a21[b][1];
        } else {
            a21_lds[(b * 4 + 2) * 64 + lane] = a21[b][2];
            a21_lds[(b * 4 + 3) * 64 + lane] = a21[b][3];
        }
    }
    c128_diagonal_block<OP, METHOD, W>(pre, D, small, t11_lds, t22_lds, aux, ln);
    __syncthreads();  // the diagonal-block inverses and the tiles of A21 the other wave needs are in LDS
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        if (W == 0) {
            a21[b][2] = a21_lds[(b * 4 + 2) * 64 + lane];
            a21[b][3] = a21_lds[(b * 4 + 3) * 64 + lane];
        } else {
            a21[b][1] = a21_lds[(b * 4 + 1) * 64 + lane];
            a21[b][0] = a21[b][1];  // (never used: wave 1's columns start at 1)
        }
    }
    c128_merge<OP, W>(a21, D, Wc, t11_lds, t22_lds, ln);
}

// Fused kernel, per-channel gate, C = 128, any d_k (multiple of 32): blocked, mixed (b0 = 16, 32) and direct-leaf
// recursion.  One workgroup of two wavefronts per matrix.
template <int OP, int METHOD>
__global__ __launch_bounds__(128) void k_kda_tri_inv_c128(const void* __restrict__ K, const float* __restrict__ beta,
                                                          const float* __restrict__ g, float* __restrict__ T, int64_t n_chunk,
                                                          ChunkMap map, int H, int d_k, int k_dt, int aux, int out_dt)
{
    constexpr int C = 128;
    typedef C128KdaLds<OP, METHOD> LY;
    __shared__ __attribute__((aligned(16))) char lds[LY::BYTES];
    const int64_t m = head_group_swizzle(blockIdx.x, n_chunk, H);
    const uint32_t bc = (uint32_t)m / (uint32_t)H;
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const Lane ln = lane_id();
    const int64_t esz = (k_dt == OP_F32) ? 4 : 2;
    const int64_t e0 = (tok0 * H + h) * (int64_t)d_k;
    const void* Kc = static_cast<const char*>(K) + e0 * esz;
    const Out Tm = out_matrix(T, m, C, out_dt);
    v4f D[10], Wc[2][4];
    if (w == 0) {
        c128_kda_invert<OP, METHOD, 0>(lds, Kc, k_dt, g + e0, (int64_t)H * d_k, beta + tok0 * H + h, H, d_k, pos.valid, aux, ln, D, Wc);
        c128_store_result<0>(reinterpret_cast<v4f*>(lds + LY::MAIL), reinterpret_cast<float*>(lds + LY::STRIPS), Tm, D, Wc, ln);
    } else {
        c128_kda_invert<OP, METHOD, 1>(lds, Kc, k_dt, g + e0, (int64_t)H * d_k, beta + tok0 * H + h, H, d_k, pos.valid, aux, ln, D, Wc);
        c128_store_result<1>(reinterpret_cast<v4f*>(lds + LY::MAIL), reinterpret_cast<float*>(lds + LY::STRIPS) + STORE_LDS_FLOATS, Tm, D,
                             Wc, ln);
    }
}

}  // namespace triinv
