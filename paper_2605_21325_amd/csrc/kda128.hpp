// Per-channel gate (paper Table 1, KDA row) at C = 128 for the four-wavefront kernels of kernels.hpp: Newton-Schulz,
// the Neumann product and the refinement pass.  The chunk matrix is built by the four waves together:
//   A_ij = beta_i [(K * exp(G - a)) (K * exp(a - G))^T]_ij,  a = one anchor row of G (row 64),
// 32 channels per step.  Wave w gates the keys of its own tile rows w and 7 - w (both factors, rounded to the operand
// type), leaves them in LDS for the others (double-buffered: one barrier per step) and accumulates its own nine tiles.
// With a single anchor both factors stay within exp(+-the fall of g over half the chunk): the bound the other
// non-recursive per-channel paths at C = 128 have.
#pragma once
#include "kernels.hpp"

namespace triinv {

// The right ("down") factors of one step, every tile row: [tile row][lane], one operand of 8 channels each.  The left
// factor of a tile is its own row's, which never leaves the wave that gated it.
template <int OPG> struct KdaStep128 {
    static constexpr int SLOT = 64 * (int)sizeof(GOp<OPG>);
    static constexpr int BYTES = 8 * SLOT;  // 8 KB for 16-bit operands, 16 KB for fp32
    static __device__ __forceinline__ GOp<OPG>* slot(char* buf, int row, int lane)
    {
        return reinterpret_cast<GOp<OPG>*>(buf + row * SLOT) + lane;
    }
};

// Wave W's nine tiles (slot order of n128_row / n128_col) in N and / or T orientation, fp32, beta-scaled and masked.
// xch: 2 * KdaStep128<OPG>::BYTES that every wave is done with when the call returns AND a barrier has passed (the
// caller's next barrier).  Kc / gc: element (chunk row 0, this head, channel 0); bc: beta of chunk row 0, this head.
template <int OPG, int W, bool K16, bool WANT_N, bool WANT_T>
__device__ __forceinline__ void kda128_rows(char* xch, v4f (&an)[9], v4f (&at)[9], const void* Kc, bool is_f16, const float* gc,
                                            int64_t row_stride, const float* bc, int64_t tok_stride, int d_k, Lane ln, int valid)
{
    typedef KdaStep128<OPG> Step;
    constexpr float LOG2E = 1.44269504088896340736f;
    const int lane = 16 * ln.q + ln.n;
    int rowc[2];
    float keep[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int row = 16 * (h == 0 ? W : 7 - W) + ln.n;
        rowc[h] = row < valid ? row : valid - 1;
        keep[h] = row < valid ? 1.f : 0.f;
    }
    const int anchor = 64 < valid ? 64 : valid - 1;
#pragma unroll
    for (int s = 0; s < 9; ++s) {
        an[s] = zero4();
        at[s] = zero4();
    }
#pragma unroll 1
    for (int s = 0; s < d_k / 32; ++s) {
        const int ch = 32 * s + 8 * ln.q;
        RawKey8<K16> raw[2];
        v4f G[2][2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            raw[h] = load_key8<K16>(Kc, (int64_t)rowc[h] * row_stride + ch);
            G[h][0] = *reinterpret_cast<const v4f*>(gc + (int64_t)rowc[h] * row_stride + ch);
            G[h][1] = *reinterpret_cast<const v4f*>(gc + (int64_t)rowc[h] * row_stride + ch + 4);
        }
        const v4f a0 = *reinterpret_cast<const v4f*>(gc + (int64_t)anchor * row_stride + ch);
        const v4f a1 = *reinterpret_cast<const v4f*>(gc + (int64_t)anchor * row_stride + ch + 4);
        char* const buf = xch + (s & 1) * Step::BYTES;
        GOp<OPG> pp[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float kv[8], up[8], dn[8];
            widen_key8<K16>(raw[h], is_f16, kv);
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const float d = ((r < 4) ? (G[h][0][r] - a0[r]) : (G[h][1][r - 4] - a1[r - 4])) * LOG2E;
                const float kk = kv[r] * keep[h];
                up[r] = kk * __builtin_amdgcn_exp2f(d);
                dn[r] = kk * __builtin_amdgcn_exp2f(-d);
            }
            pp[h] = gpack<OPG>(up);
            *Step::slot(buf, h == 0 ? W : 7 - W, lane) = gpack<OPG>(dn);
        }
        __syncthreads();  // this step's down factors of every tile row are in LDS (the buffer of two steps ago is free)
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int i = n128_row<W>(t), j = n128_col<W>(t);
            const GOp<OPG> pmj = *Step::slot(buf, j, lane);
            if (WANT_N) an[t] = gstep<OPG>(pp[i == W ? 0 : 1], pmj, an[t]);
            if (WANT_T) at[t] = gstep<OPG>(pmj, pp[i == W ? 0 : 1], at[t]);
        }
    }
    // beta_i row scaling and the strictly-lower mask
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int i = h == 0 ? W : 7 - W;
        const int rn = 16 * i + ln.n;
        const float bn = rn < valid ? bc[rn * tok_stride] : 0.f;
        v4f bq;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int rq = 16 * i + 4 * ln.q + r;
            bq[r] = rq < valid ? bc[rq * tok_stride] : 0.f;
        }
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            const int t = i == W ? j : (W + 1) + j;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool lowN = (i != j) || (4 * ln.q + r > ln.n), lowT = (i != j) || (ln.n > 4 * ln.q + r);
                an[t][r] = lowN ? bq[r] * an[t][r] : 0.f;
                at[t][r] = lowT ? bn * at[t][r] : 0.f;
            }
        }
    }
}

// The nine tiles of one wave behind the tile-source interface.
template <int W> struct RowsA128 {
    const v4f (&n)[9];
    const v4f (&t)[9];
    template <bool TR> __device__ __forceinline__ v4f get(int i, int j) const
    {
        return TR ? t[i == W ? j : (W + 1) + j] : n[i == W ? j : (W + 1) + j];
    }
};

// All 36 tiles of A in N orientation, packed, in mailbox form (MailTiles): the refinement pass's source.
template <int OP> struct MailA128 {
    const char* base;
    Lane ln;
};
template <int OP> __device__ __forceinline__ Opnd<OP> left_operand(const MailA128<OP>& A, int k, int j)
{
    return MailTiles<OP>::get(A.base, tix(k, j), A.ln);
}

struct KdaHead128 {
    int64_t m, tok0;
    int h, valid, w;
    const void* Kc;
    const float* gc;
    const float* bc;
};
__device__ __forceinline__ KdaHead128 kda_head128(const void* K, const float* beta, const float* g, int64_t n_chunk, const ChunkMap& map,
                                                  int H, int d_k, int k_dt)
{
    KdaHead128 o;
    o.m = head_group_swizzle(blockIdx.x, n_chunk, H);
    const uint32_t bc = (uint32_t)o.m / (uint32_t)H;
    o.h = (int)((uint32_t)o.m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<128>(map, bc);
    o.tok0 = pos.tok0;
    o.valid = pos.valid;
    o.w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t e0 = (o.tok0 * H + o.h) * (int64_t)d_k;
    o.Kc = static_cast<const char*>(K) + e0 * (k_dt == OP_F32 ? 4 : 2);
    o.gc = g + e0;
    o.bc = beta + o.tok0 * H + o.h;
    return o;
}

template <int OPG, int W, bool WANT_N, bool WANT_T>
__device__ __forceinline__ void kda128_rows_any(char* xch, v4f (&an)[9], v4f (&at)[9], const KdaHead128& hd, int k_dt, int H, int d_k, Lane ln)
{
    if (k_dt == OP_F32)
        kda128_rows<OPG, W, false, WANT_N, WANT_T>(xch, an, at, hd.Kc, false, hd.gc, (int64_t)H * d_k, hd.bc, H, d_k, ln, hd.valid);
    else
        kda128_rows<OPG, W, true, WANT_N, WANT_T>(xch, an, at, hd.Kc, k_dt == OP_F16, hd.gc, (int64_t)H * d_k, hd.bc, H, d_k, ln, hd.valid);
}

// Wave W's nine tiles, N orientation, packed, into the mailbox of all 36.
template <int OP, int W>
__device__ __forceinline__ void kda128_publish_rows(char* xch, char* amail, const KdaHead128& hd, int k_dt, int H, int d_k, Lane ln)
{
    v4f an[9], at[9];
    kda128_rows_any<OP, W, true, false>(xch, an, at, hd, k_dt, H, d_k, ln);
#pragma unroll
    for (int s = 0; s < 9; ++s) MailTiles<OP>::put(amail, tix(n128_row<W>(s), n128_col<W>(s)), pack<OP>(an[s]), ln);
}

template <int OP> constexpr int kda128_lds_bytes(int rest)
{
    return rest > 2 * KdaStep128<OP>::BYTES ? rest : 2 * KdaStep128<OP>::BYTES;
}

// Newton-Schulz, per-channel gate, C = 128, any d_k (multiple of 32).
template <int OP>
__global__ __launch_bounds__(256) void k_kda_tri_inv_ns128(const void* __restrict__ K, const float* __restrict__ beta,
                                                           const float* __restrict__ g, float* __restrict__ T, int64_t n_chunk,
                                                           ChunkMap map, int H, int d_k, int k_dt, int n_iter, int out_dt)
{
    __shared__ __attribute__((aligned(16))) char lds[kda128_lds_bytes<OP>(ns128_lds_bytes<OP>())];
    const KdaHead128 hd = kda_head128(K, beta, g, n_chunk, map, H, d_k, k_dt);
    const Lane ln = lane_id();
    v4f an[9], at[9];
    Opnd<OP> At[9];
    TRIINV_PER_WAVE(hd.w, (kda128_rows_any<OP, W, false, true>(lds, an, at, hd, k_dt, H, d_k, ln)))
#pragma unroll
    for (int s = 0; s < 9; ++s) At[s] = pack<OP>(at[s]);
    __syncthreads();  // the gated keys in LDS are dead: X and Y take their place
    TRIINV_PER_WAVE(hd.w, (ns128_run<OP, W>(At, out_matrix(T, hd.m, 128, out_dt), lds, ln, n_iter, hd.w)))
}

// Neumann product, per-channel gate, C = 128.
template <int OP>
__global__ __launch_bounds__(256) void k_kda_tri_inv_neumann128(const void* __restrict__ K, const float* __restrict__ beta,
                                                                const float* __restrict__ g, float* __restrict__ T, int64_t n_chunk,
                                                                ChunkMap map, int H, int d_k, int k_dt, int out_dt)
{
    typedef MailTiles<OP> Mail;
    __shared__ __attribute__((aligned(16))) char lds[kda128_lds_bytes<OP>(ns128_lds_bytes<OP>())];
    const KdaHead128 hd = kda_head128(K, beta, g, n_chunk, map, H, d_k, k_dt);
    const Lane ln = lane_id();
    v4f an[9], at[9];
    TRIINV_PER_WAVE(hd.w, (kda128_rows_any<OP, W, true, true>(lds, an, at, hd, k_dt, H, d_k, ln)))
    __syncthreads();  // the gated keys in LDS are dead: the mailbox buffers take their place
    v4f Xt[9];
    Opnd<OP> yt[9];
    float* const patch = reinterpret_cast<float*>(lds) + hd.w * STORE_LDS_FLOATS;
    TRIINV_PER_WAVE(hd.w, (neumann128_prepare<OP, W>(RowsA128<W>{an, at}, Xt, yt, lds, ln)))
    TRIINV_PER_WAVE(hd.w, (neumann128_run<OP, W>(Xt, yt, out_matrix(T, hd.m, 128, out_dt), lds, lds + Mail::BYTES, patch, ln)))
}

// Refinement pass (paper Alg. 6) over an fp32 result in T, in place, per-channel gate, C = 128: the four waves rebuild A,
// leave its 36 tiles in LDS (N orientation, packed) and run the pass of refine128_run with them.
template <int OP>
__global__ __launch_bounds__(256) void k_kda_tri_inv_refine128(const void* __restrict__ K, const float* __restrict__ beta,
                                                               const float* __restrict__ g, float* T, int64_t n_chunk, ChunkMap map,
                                                               int H, int d_k, int k_dt)
{
    typedef MailTiles<OP> Mail;
    constexpr int Y_BYTES = N128_LDS_FLOATS * 4;  // refine128_run's copy of the first result; the key exchange comes before it
    __shared__ __attribute__((aligned(16))) char lds[kda128_lds_bytes<OP>(Y_BYTES) + Mail::BYTES];
    char* const amail = lds + kda128_lds_bytes<OP>(Y_BYTES);
    const KdaHead128 hd = kda_head128(K, beta, g, n_chunk, map, H, d_k, k_dt);
    const Lane ln = lane_id();
    TRIINV_PER_WAVE(hd.w, (kda128_publish_rows<OP, W>(lds, amail, hd, k_dt, H, d_k, ln)))
    __syncthreads();  // every tile of A is in LDS; the gated keys are dead
    const MailA128<OP> src{amail, ln};
    TRIINV_PER_WAVE(hd.w, (refine128_run<OP, W>(src, T + hd.m * 128 * 128, reinterpret_cast<float*>(lds), ln, hd.w)))
}

}  // namespace triinv
