// Kernels.  One 64-lane wavefront inverts one chunk matrix (C = 16 * NB) entirely in registers:
//   k_tri_inv             A given in global memory                          -> T
//   k_gdn_tri_inv         K, beta, g -> Gram on the matrix cores, scalar gate -> T   (A never leaves the registers;
//                         four wavefronts = four adjacent heads per workgroup at C <= 64)
//   k_kda_tri_inv         per-channel gate: gated keys contracted 32 channels at a time
//   k_gdn_any_dk_tri_inv  head dimensions without a specialised build (channel loop)
//   k_tri_inv_fwd_shuffle64  forward substitution with wavefront shuffles (baseline variant)
// and, at C = 128, four wavefronts per matrix with tiles in LDS for the methods whose state does not fit
// one wavefront: k_*_neumann128 (Neumann product), k_*_ns128 (Newton-Schulz).
// Methods: forward substitution (fp32 vector arithmetic, A broadcast through LDS), blocked recursion, mixed
// recursion, blocked recursion from directly solved blocks, Neumann product, Newton-Schulz, refinement
// (inv_core.hpp).  csrc/chunk_map.hpp says where a chunk's tokens are.
#pragma once
#include "chunk_map.hpp"
#include "inv_core.hpp"

namespace triinv {

enum : int { M_FWD = 0, M_BLOCK = 1, M_NEUMANN = 2, M_MIXED = 3, M_BLOCK_DIRECT = 4, M_NEWTON_SCHULZ = 5, M_MIXED32 = 6,
             M_BUILD_A = 100 /* no inversion: the chunk matrix A itself is written (not a triinv_method) */ };
enum : int { G_SCALAR = 0, G_CHANNEL = 1, G_NONE = 2 };

__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---------------------------------------------------------------------------------------------
// Tile source 1: A in global memory (row-major C x C, element type chosen at run time).
// ---------------------------------------------------------------------------------------------
template <int NB> struct GlobalA {
    static constexpr int C = 16 * NB;
    static constexpr bool kFromMemory = true;   // a tile is a plain load: fetch it when it is needed
    const void* base;  // first element of this matrix
    int dt;            // OP_F32 / OP_F16 / OP_BF16 storage
    Lane ln;

    __device__ __forceinline__ float elem16(uint16_t u) const { return dt == OP_F16 ? f16_to_f32(u) : bf16_to_f32(u); }

    template <bool TR> __device__ __forceinline__ v4f get(int i, int j) const
    {
        v4f v;
        if (!TR) {  // v[r] = A[16i + 4q + r][16j + n]
            const int64_t off = (int64_t)(16 * i + 4 * ln.q) * C + 16 * j + ln.n;
            if (dt == OP_F32) {
                const float* p = static_cast<const float*>(base) + off;
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = p[r * C];
            } else {
                const uint16_t* p = static_cast<const uint16_t*>(base) + off;
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = elem16(p[r * C]);
            }
            if (i == j) {
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = (4 * ln.q + r > ln.n) ? v[r] : 0.f;
            }
        } else {  // v[r] = A[16i + n][16j + 4q + r]
            const int64_t off = (int64_t)(16 * i + ln.n) * C + 16 * j + 4 * ln.q;
            if (dt == OP_F32) {
                v = *reinterpret_cast<const v4f*>(static_cast<const float*>(base) + off);
            } else {
                const uint2 u = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(base) + off);
                v[0] = elem16((uint16_t)(u.x & 0xffff));
                v[1] = elem16((uint16_t)(u.x >> 16));
                v[2] = elem16((uint16_t)(u.y & 0xffff));
                v[3] = elem16((uint16_t)(u.y >> 16));
            }
            if (i == j) {
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = (ln.n > 4 * ln.q + r) ? v[r] : 0.f;
            }
        }
        return v;
    }
};

// ---------------------------------------------------------------------------------------------
// Tile source 2: A built from the keys.  S = K_c K_c^T on the matrix cores with the stored key
// values as operands (16x16x32 for 16-bit keys, 16x16x4 for fp32 keys), then
// A_ij = beta_i exp(g_i - g_j) S_ij in fp32 (paper Table 1, GDN / DeltaNet rows).
// KD: storage type of K.  DKS: number of k-steps (32 channels each for 16-bit keys, 16 for fp32).
// ---------------------------------------------------------------------------------------------
template <int KD> struct KeyVec;
template <> struct KeyVec<OP_F32> { typedef v4f type; };
template <> struct KeyVec<OP_F16> { typedef v8h type; };
template <> struct KeyVec<OP_BF16> { typedef v8bf type; };

template <int KD> __device__ __forceinline__ v4f gram_step(typename KeyVec<KD>::type a, typename KeyVec<KD>::type b, v4f acc);
template <> __device__ __forceinline__ v4f gram_step<OP_F32>(v4f a, v4f b, v4f acc)
{
#pragma unroll
    for (int r = 0; r < 4; ++r) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[r], b[r], acc, 0, 0, 0);
    return acc;
}
template <> __device__ __forceinline__ v4f gram_step<OP_F16>(v8h a, v8h b, v4f acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc, 0, 0, 0);
}
template <> __device__ __forceinline__ v4f gram_step<OP_BF16>(v8bf a, v8bf b, v4f acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
}

// beta / g of one chunk's tokens in the two index patterns a lane needs (by its column n, by its
// rows 4q + r), and the scalar gate applied to a Gram tile:
//   A_ij = beta_i exp(g_i - g_j) S_ij for i > j, else 0      (paper Table 1, GDN / DeltaNet rows).
// g is kept multiplied by log2(e) (done once per token when the values are staged), so that the gate of an element is
// one subtraction and one exp2; without a gate g = 0 and exp2(0) = 1 exactly, so that kind needs no code of its own.
// NOGATE: the launch is known to have no gate (gc null): the factor exp(g_i - g_j) is 1 and its exponentials are left out.
template <int NB, bool NOGATE = false> struct GateVec {
    static constexpr int C = 16 * NB;
    float beta_n[NB], g_n[NB];   // g_*: g log2(e)
    v4f beta_q[NB], g_q[NB];
    bool gated;

    // Loading is split in two so that the caller can put its other global loads between the halves:
    // issue() starts the loads of this lane's beta / g values (C / 64 tokens per lane) and stage()
    // redistributes them through LDS into the two index patterns.  Vector-memory loads return in
    // order, so issuing these first lets stage() wait for them alone while later loads stay in flight.
    // bc, gc: first element of (chunk row 0, this head); tok_stride in elements; gc may be null.
    static constexpr int RAW = C >= 64 ? C / 64 : 1;
    float raw_b[RAW], raw_g[RAW];

    // valid: number of tokens the chunk really has; the rows beyond read the last real token (a valid
    // address, and a g that keeps every exponent of the gate <= 0) and get beta = 0.
    __device__ __forceinline__ void issue(const float* bc, const float* gc, int64_t tok_stride, Lane ln, int valid = C)
    {
        const int l = 16 * ln.q + ln.n;
        gated = (gc != nullptr);
        const float* gp = gated ? gc : bc;  // always a valid address: the load is unconditional, the value is not
#pragma unroll
        for (int k = 0; k < RAW; ++k) {
            const int t = l + 64 * k;
            if (C < 64 && t >= C) {  // more lanes than tokens
                raw_b[k] = 0.f;
                raw_g[k] = 0.f;
                continue;
            }
            const int tc = t < valid ? t : valid - 1;
            const float b = bc[tc * tok_stride];
            raw_b[k] = t < valid ? b : 0.f;
            raw_g[k] = gp[tc * tok_stride];
        }
    }

    // lds: wave-private, 2 * C floats.
    __device__ __forceinline__ void stage(float* lds, Lane ln)
    {
        const int l = 16 * ln.q + ln.n;
#pragma unroll
        for (int k = 0; k < RAW; ++k) {
            if (C < 64 && l >= C) continue;
            lds[l + 64 * k] = raw_b[k];
            lds[C + l + 64 * k] = gated ? raw_g[k] * 1.44269504088896340736f : 0.f;
        }
        wave_lds_sync();
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            beta_n[i] = lds[16 * i + ln.n];
            g_n[i] = lds[C + 16 * i + ln.n];
            beta_q[i] = *reinterpret_cast<const v4f*>(&lds[16 * i + 4 * ln.q]);
            g_q[i] = *reinterpret_cast<const v4f*>(&lds[C + 16 * i + 4 * ln.q]);
        }
        wave_lds_sync();
    }

    __device__ __forceinline__ void load(const float* bc, const float* gc, int64_t tok_stride, float* lds, Lane ln, int valid = C)
    {
        issue(bc, gc, tok_stride, ln, valid);
        stage(lds, ln);
    }

    // s: Gram tile (i, j) in N (TR = false) or T orientation.
    template <bool TR> __device__ __forceinline__ v4f apply(int i, int j, v4f s, Lane ln) const
    {
        v4f a;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            // N: element (row 16i + 4q + r, col 16j + n);  T: element (row 16i + n, col 16j + 4q + r)
            const float b = TR ? beta_n[i] : beta_q[i][r];
            const float d = TR ? (g_n[i] - g_q[j][r]) : (g_q[i][r] - g_n[j]);  // (g_i - g_j) log2 e
            const float w = NOGATE ? b : b * __builtin_amdgcn_exp2f(d);        // beta_i exp(g_i - g_j)
            const bool low = (i != j) || (TR ? (ln.n > 4 * ln.q + r) : (4 * ln.q + r > ln.n));
            a[r] = low ? w * s[r] : 0.f;
        }
        return a;
    }
};

template <int KD, int NB, int DKS> struct GramA {
    static constexpr bool kFromMemory = false;  // a tile costs matrix-core work and pins the key registers
    typedef typename KeyVec<KD>::type kvec;
    static constexpr int C = 16 * NB;
    static constexpr int KSTEP = (KD == OP_F32) ? 16 : 32;  // channels per k-step
    kvec k[NB][DKS];
    GateVec<NB> gate;
    Lane ln;

    // Kc: first key element of (chunk row 0, this head); row_stride in elements.
    // valid: number of tokens the chunk really has; rows beyond it read the last real token (a valid
    // address) and are then replaced by zero keys.
    __device__ __forceinline__ void load_keys(const void* Kc, int64_t row_stride, int valid = C)
    {
        constexpr int per_lane = (KD == OP_F32) ? 4 : 8;
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int s = 0; s < DKS; ++s) {
                const int row = 16 * i + ln.n;
                const int64_t off = (int64_t)(row < valid ? row : valid - 1) * row_stride + KSTEP * s + per_lane * ln.q;
                // plain loads: the non-temporal hint measured ~5 % slower here
                if (KD == OP_F32)
                    k[i][s] = *reinterpret_cast<const kvec*>(static_cast<const float*>(Kc) + off);
                else
                    k[i][s] = *reinterpret_cast<const kvec*>(static_cast<const uint16_t*>(Kc) + off);
            }
        if (valid < C) {  // wave-uniform: only a sequence's last chunk comes here
            const kvec zero = __builtin_bit_cast(kvec, v4u{0u, 0u, 0u, 0u});
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int s = 0; s < DKS; ++s)
                    if (16 * i + ln.n >= valid) k[i][s] = zero;
        }
    }

    __device__ __forceinline__ void issue_gate(const float* bc, const float* gc, int64_t tok_stride, int valid = C)
    {
        gate.issue(bc, gc, tok_stride, ln, valid);
    }
    __device__ __forceinline__ void stage_gate(float* lds) { gate.stage(lds, ln); }

    template <bool TR> __device__ __forceinline__ v4f get(int i, int j) const
    {
        v4f s = zero4();
#pragma unroll
        for (int t = 0; t < DKS; ++t) s = TR ? gram_step<KD>(k[j][t], k[i][t], s) : gram_step<KD>(k[i][t], k[j][t], s);
        return gate.template apply<TR>(i, j, s, ln);
    }
};

// ---------------------------------------------------------------------------------------------
// Which tiles of A, in which orientation, a method asks for (used by sources that have to form
// every tile up front).  The blocked recursion wants an off-diagonal tile in the orientation
// opposite to that of the merge that consumes it; that merge belongs to the smallest aligned
// block pair containing tile rows i and j.
// ---------------------------------------------------------------------------------------------
constexpr bool ROOT_T = true;  // the last merge of the blocked recursion is produced in T orientation

template <int NB> __host__ __device__ constexpr bool merge_block_is_T(int i, int j)
{
    int h = 1;
    while ((i / (2 * h)) != (j / (2 * h))) h *= 2;
    return (2 * h == NB) ? ROOT_T : (((i / (2 * h)) & 1) != 0);
}

constexpr int WITH_REFINE = 1000;  // METHOD + WITH_REFINE: the tiles of METHOD plus every tile in N orientation (Alg. 6's Y A)

template <int NB, int METHOD> __host__ __device__ constexpr bool need_tile(int i, int j, bool tr)
{
    if constexpr (METHOD >= WITH_REFINE) return !tr || need_tile<NB, METHOD - WITH_REFINE>(i, j, tr);
    if (METHOD == M_FWD || METHOD == M_NEWTON_SCHULZ || METHOD == M_BUILD_A) return tr;
    if (METHOD == M_NEUMANN) return true;
    if (METHOD == M_MIXED32 && i / 2 == j / 2) return true;  // the 32 x 32 Neumann blocks want both orientations
    if (i == j) return METHOD == M_BLOCK_DIRECT ? tr : true;
    return merge_block_is_T<NB>(i, j) ? !tr : tr;
}

// Tile source 3: all tiles precomputed in registers.
template <int NB> struct PreA {
    static constexpr bool kFromMemory = false;
    v4f n[NB * (NB + 1) / 2], t[NB * (NB + 1) / 2];
    template <bool TR> __device__ __forceinline__ v4f get(int i, int j) const { return TR ? t[tix(i, j)] : n[tix(i, j)]; }
};

// One k-step (32 channels; lane (q, n) holds channels 8q..8q+7 of row n) as a matrix-core operand.
template <int OPG> struct GOp;
template <> struct GOp<OP_F32> { float x[8]; };
template <> struct GOp<OP_F16> { v8h x; };
template <> struct GOp<OP_BF16> { v8bf x; };

template <int OPG> __device__ __forceinline__ GOp<OPG> gpack(const float (&v)[8]);
template <> __device__ __forceinline__ GOp<OP_F32> gpack<OP_F32>(const float (&v)[8])
{
    GOp<OP_F32> o;
#pragma unroll
    for (int r = 0; r < 8; ++r) o.x[r] = v[r];
    return o;
}
template <> __device__ __forceinline__ GOp<OP_F16> gpack<OP_F16>(const float (&v)[8])
{
    const v4u u = {pack2_f16(v[0], v[1]), pack2_f16(v[2], v[3]), pack2_f16(v[4], v[5]), pack2_f16(v[6], v[7])};
    return {__builtin_bit_cast(v8h, u)};
}
template <> __device__ __forceinline__ GOp<OP_BF16> gpack<OP_BF16>(const float (&v)[8])
{
    const v4u u = {pack2_bf16(v[0], v[1]), pack2_bf16(v[2], v[3]), pack2_bf16(v[4], v[5]), pack2_bf16(v[6], v[7])};
    return {__builtin_bit_cast(v8bf, u)};
}

template <int OPG> __device__ __forceinline__ v4f gstep(const GOp<OPG>& a, const GOp<OPG>& b, v4f acc);
template <> __device__ __forceinline__ v4f gstep<OP_F32>(const GOp<OP_F32>& a, const GOp<OP_F32>& b, v4f acc)
{
#pragma unroll
    for (int r = 0; r < 8; ++r) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x[r], b.x[r], acc, 0, 0, 0);
    return acc;
}
template <> __device__ __forceinline__ v4f gstep<OP_F16>(const GOp<OP_F16>& a, const GOp<OP_F16>& b, v4f acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.x, b.x, acc, 0, 0, 0);
}
template <> __device__ __forceinline__ v4f gstep<OP_BF16>(const GOp<OP_BF16>& a, const GOp<OP_BF16>& b, v4f acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.x, b.x, acc, 0, 0, 0);
}

// Eight consecutive key channels of one row as stored (16-bit: one 16-byte load; fp32: two).
template <bool K16> struct RawKey8;
template <> struct RawKey8<true> { uint4 u; };
template <> struct RawKey8<false> { v4f a, b; };

template <bool K16> __device__ __forceinline__ RawKey8<K16> load_key8(const void* Kc, int64_t off)
{
    RawKey8<K16> o;
    if constexpr (K16) {
        o.u = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(Kc) + off);
    } else {
        o.a = *reinterpret_cast<const v4f*>(static_cast<const float*>(Kc) + off);
        o.b = *reinterpret_cast<const v4f*>(static_cast<const float*>(Kc) + off + 4);
    }
    return o;
}

template <bool K16> __device__ __forceinline__ void widen_key8(const RawKey8<K16>& k, bool is_f16, float (&v)[8])
{
    if constexpr (K16) {
        const uint32_t w[4] = {k.u.x, k.u.y, k.u.z, k.u.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint16_t lo = (uint16_t)(w[r] & 0xffff), hi = (uint16_t)(w[r] >> 16);
            v[2 * r] = is_f16 ? f16_to_f32(lo) : bf16_to_f32(lo);
            v[2 * r + 1] = is_f16 ? f16_to_f32(hi) : bf16_to_f32(hi);
        }
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) { v[r] = k.a[r]; v[4 + r] = k.b[r]; }
    }
}

// Per-channel gate (paper Table 1, KDA row): A_ij = beta_i sum_c k_ic k_jc exp(g_ic - g_jc)
//   = beta_i [(K * exp(G - a)) (K * exp(a - G))^T]_ij   for any per-channel anchor a.
// C <= 64: one anchor per 16-row tile row I, a_I = the first row of that tile row of G: for a tile (I, J),
// J <= I, the left factor k_i exp(g_i - a_I) has an exponent within the decay of 16 tokens and <= 0, the
// right factor k_j exp(a_I - g_j) an exponent <= 0 for J < I and within the decay of 16 tokens for J = I
// (log-decays only fall along a chunk), so neither factor can overflow however strong the decay over the
// whole chunk is; the price is a right factor per (I, J) instead of per J, which costs one multiplication by a
// channel-only factor each (see below), not an exponential.
// C = 128 (no registers for that): a single anchor, row C/2, both factors within exp(+-half the chunk's decay).
// The gated keys are rounded to OPG and contracted on the matrix cores, 32 channels per step,
// accumulating every tile the method needs; nothing but K, G, beta is read, nothing stored.
// One iteration covers one whole 128-byte line of keys per row (64 channels of 16-bit keys, i.e.
// two k-steps, or 32 channels of fp32 keys): all of a line's key loads are issued together, so
// its second half is still cached when needed (requested one k-step apart, lines were found
// evicted in between and fetched from HBM twice).
// Kc / gc: element (chunk row 0, this head, channel 0); row_stride in elements (same for both).
// GATED = false: no per-channel gate; the stored keys themselves are the operands (OPG = their type,
// exact products) and gc is not read -- the any-d_k path of the scalar / no-gate kinds.
template <int OPG, int NB, int METHOD, bool K16, bool GATED = true>
__device__ __forceinline__ void accumulate_gated_gram(PreA<NB>& out, const void* Kc, bool is_f16, const float* gc,
                                                      int64_t row_stride, int d_k, Lane ln, int valid, float* tab = nullptr)
{
    constexpr int C = 16 * NB;
    constexpr float LOG2E = 1.44269504088896340736f;
    constexpr int STEPS = (K16 && NB <= 4) ? 2 : 1;  // C = 128 has no registers to spare for the pairing
    // rows beyond the chunk's real tokens read the last real one (valid addresses, finite exponents)
    // and contribute zero keys; the anchor is a real row too
    int rowc[NB];
    float keep[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int row = 16 * i + ln.n;
        rowc[i] = row < valid ? row : valid - 1;
        keep[i] = row < valid ? 1.f : 0.f;
    }
    const int anchor = C / 2 < valid ? C / 2 : valid - 1;
    for (int s0 = 0; s0 < d_k / 32; s0 += STEPS) {
        RawKey8<K16> raw[STEPS][NB];
#pragma unroll
        for (int t = 0; t < STEPS; ++t)
#pragma unroll
            for (int i = 0; i < NB; ++i)
                if (s0 + t < d_k / 32) raw[t][i] = load_key8<K16>(Kc, (int64_t)rowc[i] * row_stride + 32 * (s0 + t) + 8 * ln.q);
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            if (s0 + t >= d_k / 32) break;
            const int ch = 32 * (s0 + t) + 8 * ln.q;
            if constexpr (GATED && NB <= 4) {
                // gate rows and tile-row anchors of this k-step, all loads first
                v4f G[NB][2], An[NB][2];
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const int64_t off = (int64_t)rowc[i] * row_stride + ch;
                    G[i][0] = *reinterpret_cast<const v4f*>(gc + off);
                    G[i][1] = *reinterpret_cast<const v4f*>(gc + off + 4);
                    const int ar = 16 * i < valid ? 16 * i : valid - 1;
                    An[i][0] = *reinterpret_cast<const v4f*>(gc + (int64_t)ar * row_stride + ch);
                    An[i][1] = *reinterpret_cast<const v4f*>(gc + (int64_t)ar * row_stride + ch + 4);
                }
                // With e_i = (g_i - a_I) log2 e (row i, its tile row's anchor a_I), u_i = k_i 2^(e_i) is the left factor of every
                // tile in tile row I and v_j = k_j 2^(-e_j) the right factor of the diagonal tile (J, J).  The right factor of
                // tile (I, J), J < I, differs from v_j by 2^((a_I - a_J) log2 e), which depends on the channel only, not on the
                // row: those NB (NB - 1) / 2 x 32 factors are computed once per k-step by the whole wave (through LDS: the 16
                // lanes of a row group hold the same anchors; one writes them, each computes a share of the table) instead
                // of once per row: 67 exponentials per lane and k-step at C = 64 instead of 112, and no subtraction or scaling
                // of the exponent per pair either.
                constexpr int NP = NB * (NB - 1) / 2, NE = 8 * NP;
                float* anc = tab + ln.q * (8 * NB + NE);  // [NB][8] anchors, then [NP][8] factors, per row group
                float* fac = anc + 8 * NB;
                if constexpr (NP > 0) {
                    if (ln.n == 0) {
#pragma unroll
                        for (int i = 0; i < NB; ++i) {
                            *reinterpret_cast<v4f*>(&anc[8 * i]) = An[i][0];
                            *reinterpret_cast<v4f*>(&anc[8 * i + 4]) = An[i][1];
                        }
                    }
                    wave_lds_sync();
#pragma unroll
                    for (int k = 0; k < (NE + 15) / 16; ++k) {
                        const int e = ln.n + 16 * k, p = e >> 3, r = e & 7;
                        if (e < NE) {  // pair p = (hi, lo), hi > lo, in the order (1,0) (2,0) (2,1) (3,0) (3,1) (3,2)
                            const int hi = p >= 3 ? 3 : (p >= 1 ? 2 : 1), lo = p - hi * (hi - 1) / 2;
                            fac[e] = __builtin_amdgcn_exp2f((anc[8 * hi + r] - anc[8 * lo + r]) * LOG2E);
                        }
                    }
                    wave_lds_sync();
                }
                GOp<OPG> ppi[NB];
                float v[NB][8];
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    float kv[8], u[8];
                    widen_key8<K16>(raw[t][i], is_f16, kv);
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        const float kk = kv[r] * keep[i];
                        const float e = (G[i][r / 4][r % 4] - An[i][r / 4][r % 4]) * LOG2E;
                        u[r] = kk * __builtin_amdgcn_exp2f(e);
                        v[i][r] = kk * __builtin_amdgcn_exp2f(-e);
                    }
                    ppi[i] = gpack<OPG>(u);
                }
#pragma unroll
                for (int i = 0; i < NB; ++i)
#pragma unroll
                    for (int j = 0; j <= i; ++j) {
                        float dn[8];
                        if (i == j) {
#pragma unroll
                            for (int r = 0; r < 8; ++r) dn[r] = v[j][r];
                        } else {
                            const int p = i * (i - 1) / 2 + j;
                            const v4f f0 = *reinterpret_cast<const v4f*>(&fac[8 * p]), f1 = *reinterpret_cast<const v4f*>(&fac[8 * p + 4]);
#pragma unroll
                            for (int r = 0; r < 8; ++r) dn[r] = v[j][r] * (r < 4 ? f0[r] : f1[r - 4]);
                        }
                        const GOp<OPG> pmj = gpack<OPG>(dn);
                        if (need_tile<NB, METHOD>(i, j, false)) out.n[tix(i, j)] = gstep<OPG>(ppi[i], pmj, out.n[tix(i, j)]);
                        if (need_tile<NB, METHOD>(i, j, true)) out.t[tix(i, j)] = gstep<OPG>(pmj, ppi[i], out.t[tix(i, j)]);
                    }
                if constexpr (NP > 0) wave_lds_sync();  // (the table is rewritten by the next k-step)
                continue;
            }
            GOp<OPG> pp[NB], pm[NB];
            if constexpr (GATED) {
                const v4f a0 = *reinterpret_cast<const v4f*>(gc + (int64_t)anchor * row_stride + ch);
                const v4f a1 = *reinterpret_cast<const v4f*>(gc + (int64_t)anchor * row_stride + ch + 4);
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const int64_t off = (int64_t)rowc[i] * row_stride + ch;
                    const v4f g0 = *reinterpret_cast<const v4f*>(gc + off);
                    const v4f g1 = *reinterpret_cast<const v4f*>(gc + off + 4);
                    float kv[8], up[8], dn[8];
                    widen_key8<K16>(raw[t][i], is_f16, kv);
#pragma unroll
                    for (int r = 0; r < 8; ++r) {
                        const float d = ((r < 4) ? (g0[r] - a0[r]) : (g1[r - 4] - a1[r - 4])) * LOG2E;
                        const float kk = kv[r] * keep[i];
                        up[r] = kk * __builtin_amdgcn_exp2f(d);
                        dn[r] = kk * __builtin_amdgcn_exp2f(-d);
                    }
                    pp[i] = gpack<OPG>(up);
                    pm[i] = gpack<OPG>(dn);
                }
            } else {
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    float kv[8];
                    widen_key8<K16>(raw[t][i], is_f16, kv);
#pragma unroll
                    for (int r = 0; r < 8; ++r) kv[r] *= keep[i];
                    pp[i] = gpack<OPG>(kv);  // exact: OPG is the keys' own type
                    pm[i] = pp[i];
                }
            }
#pragma unroll
            for (int i = 0; i < NB; ++i)
#pragma unroll
                for (int j = 0; j <= i; ++j) {
                    if (need_tile<NB, METHOD>(i, j, false)) out.n[tix(i, j)] = gstep<OPG>(pp[i], pm[j], out.n[tix(i, j)]);
                    if (need_tile<NB, METHOD>(i, j, true)) out.t[tix(i, j)] = gstep<OPG>(pm[j], pp[i], out.t[tix(i, j)]);
                }
        }
    }
}

template <int OPG, int NB, int METHOD>
__device__ __forceinline__ void build_A_per_channel(PreA<NB>& out, const void* Kc, int kd, const float* gc, int64_t row_stride,
                                                    const float* bc, int64_t tok_stride, int d_k, float* lds, Lane ln, int valid)
{
    constexpr int C = 16 * NB;
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            out.n[tix(i, j)] = zero4();
            out.t[tix(i, j)] = zero4();
        }
    if (kd == OP_F32)
        accumulate_gated_gram<OPG, NB, METHOD, false>(out, Kc, false, gc, row_stride, d_k, ln, valid, lds);
    else
        accumulate_gated_gram<OPG, NB, METHOD, true>(out, Kc, kd == OP_F16, gc, row_stride, d_k, ln, valid, lds);
    // beta_i row scaling and the strictly-lower mask
    const int l = 16 * ln.q + ln.n;
#pragma unroll
    for (int t = l; t < C; t += 64) lds[t] = t < valid ? bc[t * tok_stride] : 0.f;
    wave_lds_sync();
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const float bn = lds[16 * i + ln.n];
        const v4f bq = *reinterpret_cast<const v4f*>(&lds[16 * i + 4 * ln.q]);
#pragma unroll
        for (int j = 0; j <= i; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool lowN = (i != j) || (4 * ln.q + r > ln.n), lowT = (i != j) || (ln.n > 4 * ln.q + r);
                out.n[tix(i, j)][r] = lowN ? bq[r] * out.n[tix(i, j)][r] : 0.f;
                out.t[tix(i, j)][r] = lowT ? bn * out.t[tix(i, j)][r] : 0.f;
            }
    }
    wave_lds_sync();
}

// Scalar / no-gate kinds for any d_k (multiple of 32): Gram tiles accumulated 32 channels at a time
// in a run-time loop with the stored keys as operands, then the scalar gate.  KD = type of K.
template <int KD, int NB, int METHOD>
__device__ __forceinline__ void build_A_scalar_any_dk(PreA<NB>& out, const void* Kc, int64_t row_stride, const float* bc,
                                                      const float* gc, int64_t tok_stride, int d_k, float* lds, Lane ln, int valid)
{
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            out.n[tix(i, j)] = zero4();
            out.t[tix(i, j)] = zero4();
        }
    accumulate_gated_gram<KD, NB, METHOD, KD != OP_F32, false>(out, Kc, KD == OP_F16, nullptr, row_stride, d_k, ln, valid);
    GateVec<NB> gate;
    gate.load(bc, gc, tok_stride, lds, ln, valid);
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            if (need_tile<NB, METHOD>(i, j, false)) out.n[tix(i, j)] = gate.template apply<false>(i, j, out.n[tix(i, j)], ln);
            if (need_tile<NB, METHOD>(i, j, true)) out.t[tix(i, j)] = gate.template apply<true>(i, j, out.t[tix(i, j)], ln);
        }
}

// ---------------------------------------------------------------------------------------------
// Result store.  Tm: first element of this matrix's T.  The register tiles (N or T orientation,
// IS_T(i, j)) of one 16-row strip are transposed through a wave-private LDS patch into plain
// rows, and the strip leaves as four 1 KB-contiguous streaming stores (16 B per lane): whole
// cache lines written by one instruction stream to HBM markedly faster than the 64-byte pieces
// a tile-shaped store produces.  Diagonal tiles get an exact unit diagonal and exact zeros above
// it; columns right of the diagonal tile are zero-filled.
// lds: STORE_LDS_FLOATS floats.
// ---------------------------------------------------------------------------------------------
// Streaming stores of the result.  Whole 16-byte pieces of full rows go out non-temporal and at
// system scope (written through the caches: T is consumed by a later kernel, never re-read here);
// measured with a same-pattern data mover ~4 % faster than the non-temporal hint alone and ~11 %
// faster than plain stores.  They are raw buffer stores over a descriptor that spans exactly this
// matrix (the cache-policy bits are an argument of the builtin, and the compiler, which sees the
// instruction, keeps the wait states a wide store needs before its data registers are rewritten;
// offsets outside the matrix would be dropped by the hardware's range check).  The 4-byte stores of
// forward substitution keep the plain non-temporal hint (partial lines written through measured slower).
constexpr int CACHE_SC0_SC1_NT = 1 | 2 | 16;  // gfx950 buffer-instruction cache-policy bits: sc0, nt, sc1

// One output matrix: its first byte and its element type (OP_F32, or OP_F16 / OP_BF16 when the caller
// asked for a 16-bit result: the fp32 values are rounded to nearest even on the way out).
struct Out {
    void* base;
    int dt;
};
__device__ __forceinline__ Out out_matrix(float* T, int64_t m, int C, int out_dt)
{
    return Out{reinterpret_cast<char*>(T) + m * C * C * (out_dt == OP_F32 ? 4 : 2), out_dt};
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t matrix_buffer(Out Tm, int C)
{
    return __builtin_amdgcn_make_buffer_rsrc(Tm.base, 0, C * C * (Tm.dt == OP_F32 ? 4 : 2), 0x00020000);  // raw buffer
}
// byte offset = lane_offset (the same for every store of a strip) + uniform_offset (a constant of the strip and row group).
// Both go into the vector offset, the instruction's scalar offset stays the immediate zero.  A 16-byte store whose scalar
// offset is a register is not safe here: the compiler places no wait state between such a store and a vector-ALU write
// of its data registers (it guards only the immediate form), and with a write in the very next slot the store now and
// then sent the new value of its first data register: about one matrix in 10^6 came out with the next strip's values
// in 16 of its elements.  With the immediate form the compiler inserts the wait state itself.  (The scalar form followed by
// an explicit two-slot wait that keeps the data registers alive measured the same: +0.9 % at C = 64, -0.9 % at C = 128.)
__device__ __forceinline__ void stream_store(v4u v, __amdgpu_buffer_rsrc_t out, int lane_offset, int uniform_offset = 0)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, out, lane_offset + uniform_offset, 0, CACHE_SC0_SC1_NT);
}
__device__ __forceinline__ void stream_store(v4f v, __amdgpu_buffer_rsrc_t out, int lane_offset, int uniform_offset = 0)
{
    stream_store(__builtin_bit_cast(v4u, v), out, lane_offset, uniform_offset);
}
__device__ __forceinline__ void stream_store(float v, float* p) { __builtin_nontemporal_store(v, p); }
// Element idx of a result matrix whose element size ESZ is known at compile time (so that the row part of the address
// folds into the store's immediate offset): fp32, or rounded to nearest even into the 16-bit type the caller asked for.
// ESZ = 0: the element size is read at run time, one address for both widths.
template <int ESZ> __device__ __forceinline__ void stream_store(float v, Out Tm, int64_t idx)
{
    if constexpr (ESZ == 4) {
        __builtin_nontemporal_store(v, static_cast<float*>(Tm.base) + idx);
    } else if constexpr (ESZ == 2) {
        __builtin_nontemporal_store((uint16_t)(Tm.dt == OP_F16 ? pack2_f16(v, 0.f) : pack2_bf16(v, 0.f)),
                                    static_cast<uint16_t*>(Tm.base) + idx);
    } else {
        const int sh = Tm.dt == OP_F32 ? 2 : 1;
        char* const p = static_cast<char*>(Tm.base) + (idx << sh);
        if (sh == 2)
            __builtin_nontemporal_store(v, reinterpret_cast<float*>(p));
        else
            __builtin_nontemporal_store((uint16_t)(Tm.dt == OP_F16 ? pack2_f16(v, 0.f) : pack2_bf16(v, 0.f)), reinterpret_cast<uint16_t*>(p));
    }
}

constexpr int STORE_LD = 16 * 8 + 4;                  // row stride of the patch (fits C = 128), floats
constexpr int STORE_LDS_FLOATS = 16 * STORE_LD;

// Zero the strip patch.  Strips stored afterwards in ascending order then find zeros right of their diagonal tile (strip
// i only writes tiles 0..i), which spares them a select per stored element.
__device__ __forceinline__ void zero_strip_patch(float* lds, Lane ln)
{
    const int lane = 16 * ln.q + ln.n;
#pragma unroll
    for (int k = 0; k < (STORE_LDS_FLOATS / 4 + 63) / 64; ++k) {
        const int p = 64 * k + lane;
        if (p < STORE_LDS_FLOATS / 4) *reinterpret_cast<v4f*>(&lds[4 * p]) = zero4();
    }
    wave_lds_sync();
}

// One strip: tiles (i, 0..i) in row[0..i], tile j in T orientation when row_is_t(j).
// ZEROED: the patch holds zeros right of tile i (zero_strip_patch, then strips in ascending order).
template <int NB, bool ZEROED = false, class RowIsT>
__device__ __forceinline__ void store_strip(Out Tm, int i, const v4f (&row)[NB], RowIsT row_is_t, float* lds, Lane ln,
                                            float diag = 1.f)
{
    constexpr int C = 16 * NB;
    const int lane = 16 * ln.q + ln.n;
    const __amdgpu_buffer_rsrc_t out = matrix_buffer(Tm, C);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        if (j > i) break;
        v4f v = row[j];
        if (row_is_t(j)) {  // v[r] = T[16i + n][16j + 4q + r]
            if (i == j) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int rr = ln.n, cc = 4 * ln.q + r;
                    v[r] = (rr == cc) ? diag : ((rr > cc) ? v[r] : 0.f);
                }
            }
            *reinterpret_cast<v4f*>(&lds[ln.n * STORE_LD + 16 * j + 4 * ln.q]) = v;
        } else {            // v[r] = T[16i + 4q + r][16j + n]
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int rr = 4 * ln.q + r, cc = ln.n;
                float x = v[r];
                if (i == j) x = (rr == cc) ? diag : ((rr > cc) ? x : 0.f);
                lds[rr * STORE_LD + 16 * j + cc] = x;
            }
        }
    }
    wave_lds_sync();
    if (Tm.dt == OP_F32) {
        // rows 16i .. 16i+15, C floats each: C/4 lanes per row, 256/C rows per instruction
        constexpr int LPR = C / 4, RPI = 64 / LPR;
#pragma unroll
        for (int k = 0; k < 16 / RPI; ++k) {
            const int rr = RPI * k + lane / LPR, cc = 4 * (lane % LPR);
            // unconditional read (columns right of the diagonal tile hold stale patch contents), then a select
            v4f v = *reinterpret_cast<const v4f*>(&lds[rr * STORE_LD + cc]);
            if (!ZEROED && cc >= 16 * (i + 1)) v = zero4();
            stream_store(v, out, ((lane / LPR) * C + cc) * 4, (16 * i + RPI * k) * C * 4);
        }
    } else {
        // 16-bit result: 8 elements (16 bytes) per lane, C/8 lanes per row
        constexpr int LPR = C / 8, RPI = 64 / LPR, ITER = RPI >= 16 ? 1 : 16 / RPI;
#pragma unroll
        for (int k = 0; k < ITER; ++k) {
            const int rr = RPI * k + lane / LPR, cc = 8 * (lane % LPR);
            if (RPI > 16 && rr >= 16) continue;  // C = 16: more lanes than the strip has 16-byte pieces
            v4f a = *reinterpret_cast<const v4f*>(&lds[rr * STORE_LD + cc]);
            v4f b = *reinterpret_cast<const v4f*>(&lds[rr * STORE_LD + cc + 4]);
            if (!ZEROED && cc >= 16 * (i + 1)) a = zero4();
            if (!ZEROED && cc + 4 >= 16 * (i + 1)) b = zero4();
            const v4u p = Tm.dt == OP_F16 ? v4u{pack2_f16(a[0], a[1]), pack2_f16(a[2], a[3]), pack2_f16(b[0], b[1]), pack2_f16(b[2], b[3])}
                                          : v4u{pack2_bf16(a[0], a[1]), pack2_bf16(a[2], a[3]), pack2_bf16(b[0], b[1]), pack2_bf16(b[2], b[3])};
            stream_store(p, out, ((lane / LPR) * C + cc) * 2, (16 * i + RPI * k) * C * 2);
        }
    }
    wave_lds_sync();
}

template <int NB, class IsT>
__device__ __forceinline__ void store_result(Out Tm, const v4f (&Tt)[NB * (NB + 1) / 2], IsT is_t, float* lds, Lane ln,
                                             float diag = 1.f)
{
    zero_strip_patch(lds, ln);
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        v4f row[NB];
#pragma unroll
        for (int j = 0; j <= i; ++j) row[j] = Tt[tix(i, j)];
        store_strip<NB, true>(Tm, i, row, [&](int j) { return is_t(i, j); }, lds, ln, diag);
    }
}

// ---------------------------------------------------------------------------------------------
// Forward substitution, row by row, in fp32 vector arithmetic.  Lane = one column c of T:
//   T[i][c] = [i == c] - sum_{j < i} A[i][j] T[j][c]
// so every lane needs the same A[i][j]: the rows of A are staged through LDS, 16 rows at a
// time (double-buffered), and read back with wave-uniform addresses (LDS broadcast).
// C = 128 runs two passes of 64 columns; pass p only involves rows and columns >= 64 p.
// Cost per matrix: C(C-1)/2 FMAs per lane plus one 16-byte LDS broadcast read per four of them; a
// single running sum per row measured faster than four interleaved partial sums.
// lds: wave-private, 2 * 16 * (C + 4) floats.
// ---------------------------------------------------------------------------------------------
template <int NB> constexpr int fwd_lds_floats() { return 2 * 16 * (16 * NB + 4); }

template <int NB, int ESZ, class ASrc>
__device__ __forceinline__ void forward_substitution(const ASrc& A, Out Tm, float* lds, Lane ln)
{
    constexpr int C = 16 * NB;
    constexpr int LD = C + 4;
    constexpr int PASSES = C >= 64 ? C / 64 : 1;  // C < 64: one pass, lanes >= C idle along (they store nothing)
    const int lane = 16 * ln.q + ln.n;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int c = 64 * p + lane;  // this lane's column
        const bool mine = C >= 64 || c < C;
        float Tc[C];                  // Tc[k] = T[64p + k][c]
        if (p > 0) {
            // rows above this pass's diagonal block: columns >= 64p are zero there
#pragma unroll 8
            for (int i = 0; i < 64 * p; ++i) stream_store<ESZ>(0.f, Tm, (int64_t)i * C + c);
        }
        v4f stage[NB];  // tiles (s, 4p..s) of the strip being staged, T orientation = row-major pieces
        stage[4 * p] = A.template get<true>(4 * p, 4 * p);
#pragma unroll
        for (int s = 4 * p; s < NB; ++s) {
            float* buf = lds + (s & 1) * 16 * LD;
#pragma unroll
            for (int j = 4 * p; j <= s; ++j) *reinterpret_cast<v4f*>(&buf[ln.n * LD + 16 * j + 4 * ln.q]) = stage[j];
            wave_lds_sync();
            if (s + 1 < NB) {
#pragma unroll
                for (int j = 4 * p; j <= s + 1; ++j) stage[j] = A.template get<true>(s + 1, j);
            }
#pragma unroll
            for (int ii = 0; ii < 16; ++ii) {
                const int i = 16 * s + ii;
                float acc = 0.f;
#pragma unroll
                for (int j4 = 64 * p; j4 < i; j4 += 4) {
                    const v4f a = *reinterpret_cast<const v4f*>(&buf[ii * LD + j4]);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (j4 + r < i) acc += a[r] * Tc[j4 + r - 64 * p];
                }
                const float t = (c < i) ? -acc : ((c == i) ? 1.f : 0.f);
                Tc[i - 64 * p] = t;
                if (mine) stream_store<ESZ>(t, Tm, (int64_t)i * C + c);
            }
        }
    }
}

// Forward substitution at C = 64 with the row of A broadcast by wavefront shuffles instead of LDS: lane l
// holds A[i][l] of every row i (one coalesced 256-byte load per row, all 63 issued up front) and
// T[:, l]; A[i][j] reaches every lane through a v_readlane of lane j.  One shuffle per multiply-add
// makes this variant issue about twice the vector instructions of the LDS-broadcast form above
// (measured: see the benchmark table); it is kept as the plain shuffle baseline.
__device__ __forceinline__ void forward_substitution_shuffle64(const void* Am, int in_dt, float* Tm, Lane ln)
{
    constexpr int C = 64;
    const int c = 16 * ln.q + ln.n;
    float a[C];  // a[i] = A[i][c] for c < i, else 0
#pragma unroll
    for (int i = 1; i < C; ++i) {
        float v;
        if (in_dt == OP_F32) {
            v = static_cast<const float*>(Am)[i * C + c];
        } else {
            const uint16_t u = static_cast<const uint16_t*>(Am)[i * C + c];
            v = in_dt == OP_F16 ? f16_to_f32(u) : bf16_to_f32(u);
        }
        a[i] = c < i ? v : 0.f;
    }
    float Tc[C];
    Tc[0] = c == 0 ? 1.f : 0.f;
    stream_store(Tc[0], Tm + c);
#pragma unroll
    for (int i = 1; i < C; ++i) {
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < i; ++j) {
            const float aij = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a[i]), j));
            acc += aij * Tc[j];
        }
        Tc[i] = (c < i) ? -acc : ((c == i) ? 1.f : 0.f);
        stream_store(Tc[i], Tm + i * C + c);
    }
}

template <int UNUSED = 0>  // a template only so that the header may define it in every translation unit
__global__ __launch_bounds__(64) void k_tri_inv_fwd_shuffle64(const void* __restrict__ A, float* __restrict__ T, int64_t n_mat, int in_dt)
{
    const int64_t m = blockIdx.x;
    if (m >= n_mat) return;
    forward_substitution_shuffle64(static_cast<const char*>(A) + m * 64 * 64 * (in_dt == OP_F32 ? 4 : 2), in_dt, T + m * 64 * 64,
                                   lane_id());
}

// The same substitution with all of A resident in LDS (tile-packed, 1 KB per lower tile): used at
// C >= 64 when the tiles come out of registers (Gram products), so that the key registers and the
// tile registers are free before the running values of T take theirs (C = 64: 10 KB per wavefront,
// four wavefronts per SIMD; 140 -> 122 us on the 16 384-matrix workload against the strip-staged form).
template <int NB> constexpr int fwd_resident_lds_floats() { return NB * (NB + 1) / 2 * 256; }

template <int NB, int ESZ, class ASrc>
__device__ __forceinline__ void forward_substitution_resident(const ASrc& A, Out Tm, float* lds, Lane ln)
{
    constexpr int C = 16 * NB;
    const int lane = 16 * ln.q + ln.n;
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j <= i; ++j)
            *reinterpret_cast<v4f*>(&lds[tix(i, j) * 256 + ln.n * 16 + 4 * ln.q]) = A.template get<true>(i, j);
    wave_lds_sync();
#pragma unroll
    for (int p = 0; p < C / 64; ++p) {
        const int c = 64 * p + lane;
        float Tc[C];
        if (p > 0) {
#pragma unroll 8
            for (int i = 0; i < 64 * p; ++i) stream_store<ESZ>(0.f, Tm, (int64_t)i * C + c);
        }
#pragma unroll
        for (int i = 64 * p; i < C; ++i) {
            float acc = 0.f;
#pragma unroll
            for (int j4 = 64 * p; j4 < i; j4 += 4) {
                const v4f a = *reinterpret_cast<const v4f*>(&lds[tix(i / 16, j4 / 16) * 256 + (i % 16) * 16 + (j4 % 16)]);
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (j4 + r < i) acc += a[r] * Tc[j4 + r - 64 * p];
            }
            const float t = (c < i) ? -acc : ((c == i) ? 1.f : 0.f);
            Tc[i - 64 * p] = t;
            stream_store<ESZ>(t, Tm, (int64_t)i * C + c);
            // keep the scheduler from hoisting later rows' LDS reads over this row (they do not depend on
            // it, and hoisted by the hundred they would spill the running values of T)
            if (i % 4 == 3) __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Kernels
// ---------------------------------------------------------------------------------------------
template <int NB> constexpr int gate_lds_floats() { return 2 * 16 * NB; }

// REFINE: one iterative-refinement step after a matrix-product method (C = 64 only).
template <int OP, int NB, int METHOD, class ASrc, bool REFINE = false>
__device__ __forceinline__ void invert_and_store(const ASrc& src, Out Tm, float* lds, Lane ln, int aux = 0)
{
    constexpr int NT = NB * (NB + 1) / 2;
    if constexpr (METHOD == M_BUILD_A) {
        // the strictly-lower chunk matrix itself (zero diagonal), strip by strip: at most NB tiles alive at a time
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            v4f row[NB];
#pragma unroll
            for (int j = 0; j <= i; ++j) row[j] = src.template get<true>(i, j);
            store_strip<NB>(Tm, i, row, [](int) { return true; }, lds, ln, 0.f);
        }
        return;
    }
    if (METHOD == M_FWD) {
        // The strip-staged form (standalone entry point, small C) gets one copy per element size of the result: the
        // wave-uniform branch costs nothing, a run-time element size costs every store its immediate offset (107 against
        // 116 us on 16 384 matrices of C = 64).  The fused, LDS-resident form keeps one copy with a run-time size: two
        // copies behind the Gram prologue nearly double its registers (100 -> 193 at C = 64: 122 -> 136 us).
        if constexpr (NB >= 4 && !ASrc::kFromMemory) {
            forward_substitution_resident<NB, 0>(src, Tm, lds, ln);
        } else {
            if (Tm.dt == OP_F32)
                forward_substitution<NB, 4>(src, Tm, lds, ln);
            else
                forward_substitution<NB, 2>(src, Tm, lds, ln);
        }
    } else if (METHOD == M_NEWTON_SCHULZ) {
        v4f Xt[NT];
        newton_schulz<OP, NB>(src, Xt, aux, ln);  // aux = number of iterations
        if constexpr (REFINE) refine_once<OP, NB>(src, Xt, [](int, int) { return true; }, lds, ln);
        store_result<NB>(Tm, Xt, [](int, int) { return true; }, lds, ln);
    } else if (METHOD == M_NEUMANN) {
        v4f Xt[NT];
        neumann<OP, NB>(src, Xt, ln);
        if constexpr (REFINE) refine_once<OP, NB>(src, Xt, [](int, int) { return true; }, lds, ln);
        store_result<NB>(Tm, Xt, [](int, int) { return true; }, lds, ln);
    } else {
        v4f Tt[NT];
        constexpr int LEAF = METHOD == M_MIXED ? LEAF_NEUMANN : METHOD == M_MIXED32 ? LEAF_NEUMANN32 : METHOD == M_BLOCK_DIRECT ? LEAF_FORWARD : LEAF_BLOCK_RECURSIVE;
        block_recursive<OP, NB, ROOT_T, LEAF>(src, Tt, lds, ln, aux);  // aux = refinement steps on the leaves (mixed recursion)
        if constexpr (REFINE) {
            refine_once<OP, NB>(src, Tt, [](int i, int j) { return result_is_T<NB, ROOT_T>(i, j); }, lds, ln);
            store_result<NB>(Tm, Tt, [](int, int) { return true; }, lds, ln);
        } else {
            store_result<NB>(Tm, Tt, [](int i, int j) { return result_is_T<NB, ROOT_T>(i, j); }, lds, ln);
        }
    }
}

template <int NB, int METHOD, bool FUSED = false> constexpr int core_lds_floats()
{
    static_assert(STORE_LDS_FLOATS >= XPOSE_FLOATS && STORE_LDS_FLOATS >= LEAF_FWD_FLOATS, "the store patch is the largest user");
    return METHOD != M_FWD ? STORE_LDS_FLOATS : (FUSED && NB >= 4) ? fwd_resident_lds_floats<NB>() : fwd_lds_floats<NB>();
}

// The matrix-product kernels may be run in place (A and T the same memory: the composed path of the fused entry points),
// so only forward substitution, which never is, declares its two pointers non-aliasing.
template <int METHOD> struct TriInvPointers {
    typedef const void* in;
    typedef float* out;
};
template <> struct TriInvPointers<M_FWD> {
    typedef const void* __restrict__ in;
    typedef float* __restrict__ out;
};

template <int OP, int NB, int METHOD, bool REFINE = false>
__global__ __launch_bounds__(64) void k_tri_inv(typename TriInvPointers<METHOD>::in A, typename TriInvPointers<METHOD>::out T, int64_t n_mat,
                                                int in_dt, int aux, int out_dt)
{
    constexpr int C = 16 * NB;
    __shared__ __attribute__((aligned(16))) float lds[core_lds_floats<NB, METHOD>()];
    const int64_t m = blockIdx.x;
    if (m >= n_mat) return;
    const Lane ln = lane_id();
    GlobalA<NB> src;
    src.base = static_cast<const char*>(A) + m * C * C * (in_dt == OP_F32 ? 4 : 2);
    src.dt = in_dt;
    src.ln = ln;
    invert_and_store<OP, NB, METHOD, GlobalA<NB>, REFINE>(src, out_matrix(T, m, C, out_dt), lds, ln, aux);
}

// Workgroup -> matrix map of the fused kernels.  Workgroups are handed to the 8 XCDs round-robin
// (workgroup id mod 8); the H heads of one (batch, chunk) read the same beta / g cache lines, so
// they are given to one XCD, back to back, and share those lines in its L2.  Groups beyond the
// last multiple of 8 keep the identity map.
__device__ __forceinline__ int64_t head_group_swizzle(int64_t bid, int64_t n_group, int H)
{
    const int64_t full = (n_group / 8) * 8;
    if (bid >= full * H) return bid;
    const int64_t x = bid % 8, q = bid / 8;
    return ((q / H) * 8 + x) * H + (q % H);
}

// WPB wavefronts per workgroup, each with its own matrix.
// spread = 0 (many heads): wave w of workgroup u takes head unit * WPB + w of one (batch, chunk), so a workgroup reads
// WPB adjacent 256-byte key rows of every token (measured a few percent faster than one head per workgroup); falls back
// to the plain order when H is not a multiple of WPB.
// spread = S > 0 (few heads, H < 8: the layout a tensor-parallel shard sees): with the map above a workgroup's whole
// traffic would fall into one contiguous 64 KB stretch of K and one of T -- few memory channels at a time; measured 8-12 %
// slower, with 10 % higher read latency and 4.5x the DRAM credit stalls.  Instead a workgroup takes ONE head of WPB chunks
// S chunks apart (S = max(1, 4 / H), so its four key regions are at least 64 KB apart), and the S * H workgroups that share
// those 4 S chunks run back to back on one XCD.  Chunks beyond the last full group of 4 S keep the plain order.
// The waves never synchronise with each other.  Returns chunk id * H + head, or -1 for a wave without a matrix.
template <int WPB>
__device__ __forceinline__ int64_t fused_matrix_index(int64_t n_chunk, int H, int64_t n_mat, int spread)
{
    const int w = (WPB == 1) ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (WPB > 1 && spread > 0) {
        const int64_t per_group = (int64_t)spread * H;                 // workgroups per group of WPB * spread chunks
        const int64_t n_group = n_chunk / (WPB * spread);
        const int64_t full = n_group * per_group;
        const int64_t bid = blockIdx.x;
        if (bid < full) {
            const int64_t gh = head_group_swizzle(bid, n_group, (int)per_group);
            const int64_t grp = gh / per_group;
            const int r = (int)(gh - grp * per_group);                 // j * H + head, j = offset inside the stride
            const int64_t chunk = grp * (WPB * spread) + r / H + (int64_t)spread * w;
            return chunk * H + r % H;
        }
        const int64_t m = (full + (bid - full)) * WPB + w;             // the tail: WPB consecutive matrices per workgroup
        return m < n_mat ? m : -1;
    }
    if (H % WPB != 0) {
        const int64_t m = (int64_t)blockIdx.x * WPB + w;
        return m < n_mat ? m : -1;
    }
    return head_group_swizzle(blockIdx.x, n_chunk, H / WPB) * WPB + w;
}

template <int KD, int OP, int NB, int METHOD, int DKS, bool REFINE = false, int WPB = 1>
__global__ __launch_bounds__(64 * WPB) void k_gdn_tri_inv(const void* __restrict__ K, const float* __restrict__ beta,
                                                          const float* __restrict__ g, float* __restrict__ T,
                                                          int64_t n_chunk, ChunkMap map, int H, int d_k, int aux, int out_dt, int spread)
{
    constexpr int C = 16 * NB;
    constexpr int CORE = core_lds_floats<NB, METHOD, true>();
    constexpr int GATE = gate_lds_floats<NB>();
    constexpr int PER_WAVE = CORE > GATE ? CORE : GATE;
    __shared__ __attribute__((aligned(16))) float lds_all[WPB * PER_WAVE];
    float* lds = lds_all + ((WPB == 1) ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))) * PER_WAVE;
    const int64_t m = fused_matrix_index<WPB>(n_chunk, H, n_chunk * H, spread);  // chunk id * H + h
    if (m < 0) return;
    const uint32_t bc = (uint32_t)m / (uint32_t)H;  // m < 2^31 (checked by the host)
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const Lane ln = lane_id();
    GramA<KD, NB, DKS> src;
    src.ln = ln;
    const int64_t esz = (KD == OP_F32) ? 4 : 2;
    src.issue_gate(beta + tok0 * H + h, g ? g + tok0 * H + h : nullptr, H, pos.valid);
    src.load_keys(static_cast<const char*>(K) + (tok0 * H + h) * (int64_t)d_k * esz, (int64_t)H * d_k, pos.valid);
    src.stage_gate(lds);
    invert_and_store<OP, NB, METHOD, GramA<KD, NB, DKS>, REFINE>(src, out_matrix(T, m, C, out_dt), lds, ln, aux);
}

// Fused kernel of the scalar / no-gate kinds for head dimensions without a specialised build.
template <int KD, int OP, int NB, int METHOD>
__global__ __launch_bounds__(64) void k_gdn_any_dk_tri_inv(const void* __restrict__ K, const float* __restrict__ beta,
                                                           const float* __restrict__ g, float* __restrict__ T,
                                                           int64_t n_chunk, ChunkMap map, int H, int d_k, int aux, int out_dt)
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
    build_A_scalar_any_dk<KD, NB, METHOD>(src, static_cast<const char*>(K) + (tok0 * H + h) * (int64_t)d_k * esz,
                                          (int64_t)H * d_k, beta + tok0 * H + h, g ? g + tok0 * H + h : nullptr, H, d_k, lds, ln,
                                          pos.valid);
    invert_and_store<OP, NB, METHOD, PreA<NB>, false>(src, out_matrix(T, m, C, out_dt), lds, ln, aux);
}

// Fused kernel for the per-channel gate: g is [B, Tlen, H, d_k]; the gated keys are rounded to OP.
template <int OP, int NB, int METHOD, int WPB = 1, bool REFINE = false>
__global__ __launch_bounds__(64 * WPB) void k_kda_tri_inv(const void* __restrict__ K, const float* __restrict__ beta,
                                                          const float* __restrict__ g, float* __restrict__ T,
                                                          int64_t n_chunk, ChunkMap map, int H, int d_k, int k_dt, int aux, int out_dt, int spread)
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
    const int64_t e0 = (tok0 * H + h) * (int64_t)d_k;  // element offset of (token 0, head h, channel 0)
    PreA<NB> src;
    build_A_per_channel<OP, NB, REFINE ? METHOD + WITH_REFINE : METHOD>(src, static_cast<const char*>(K) + e0 * esz, k_dt, g + e0,
                                                                        (int64_t)H * d_k, beta + tok0 * H + h, H, d_k, lds, ln,
                                                                        pos.valid);
    invert_and_store<OP, NB, METHOD, PreA<NB>, REFINE>(src, out_matrix(T, m, C, out_dt), lds, ln, aux);
}

// ---------------------------------------------------------------------------------------------
// C = 128 on one workgroup of four wavefronts per matrix (Neumann product, Newton-Schulz, refinement pass):
// wave w owns tile rows w and 7 - w of every matrix involved.  The refinement pass keeps its Y in LDS as 36 fp32
// tiles (16 x 20 floats each), readable in either orientation.
// ---------------------------------------------------------------------------------------------
constexpr int N128_NB = 8;
constexpr int N128_NT = 36;
constexpr int N128_LDS_FLOATS = N128_NT * XPOSE_FLOATS;   // 46 080 bytes

__device__ __forceinline__ v4f lds_tile_read_n(const float* t, Lane ln)
{
    v4f v;
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = t[(4 * ln.q + r) * XPOSE_LD + ln.n];
    return v;
}
// slot s of wave W: tile (i, j) with i = W for s <= W, else i = 7 - W
template <int W> __host__ __device__ constexpr int n128_row(int s) { return s <= W ? W : 7 - W; }
template <int W> __host__ __device__ constexpr int n128_col(int s) { return s <= W ? s : s - (W + 1); }

template <int W>
__device__ __forceinline__ void n128_store(Out Tm, const v4f (&Xt)[9], float* patch, Lane ln)
{
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int i = half == 0 ? W : 7 - W, s0 = half == 0 ? 0 : W + 1;
        v4f row[N128_NB];
#pragma unroll
        for (int j = 0; j < N128_NB; ++j)
            if (j <= i) row[j] = Xt[s0 + j];
        store_strip<N128_NB>(Tm, i, row, [](int) { return true; }, patch, ln);
    }
}

#define TRIINV_PER_WAVE(w, CALL) \
    switch (w) {                 \
    case 0: { constexpr int W = 0; CALL; } break; \
    case 1: { constexpr int W = 1; CALL; } break; \
    case 2: { constexpr int W = 2; CALL; } break; \
    default: { constexpr int W = 3; CALL; } break; \
    }

// ---------------------------------------------------------------------------------------------
// Newton-Schulz at C = 128 (paper Alg. 3, Eq. 8, for I + A): the same four-wavefront workgroup.
//   X <- I / C;  n_iter times:  Y <- X + A X;  X <- 2 X - X Y.
// Wave w owns tile rows w and 7 - w: it keeps its rows of A (T orientation, packed operands) and of X (both
// orientations, fp32) in registers and reads the right factor of every product (a tile of X, then of Y, in N
// orientation) from LDS.  A right factor in N orientation is exactly the register image its producer holds,
// so a tile crosses between waves as a mailbox: 64 consecutive slots of one packed operand each, lane l of the
// reader taking what lane l of the writer left.  No transposition, no bank conflicts, and the rounding to the
// operand type happens once, at the writer.  X and Y take 2 x 36 tiles: 36 KB for 16-bit operands, 72 KB for fp32.
// ---------------------------------------------------------------------------------------------
template <int OP> struct MailTiles {
    static constexpr int TILE_BYTES = 64 * (int)sizeof(Opnd<OP>);
    static constexpr int BYTES = N128_NT * TILE_BYTES;
    static __device__ __forceinline__ void put(char* base, int tile, Opnd<OP> v, Lane ln)
    {
        *reinterpret_cast<Opnd<OP>*>(base + tile * TILE_BYTES + (16 * ln.q + ln.n) * (int)sizeof(Opnd<OP>)) = v;
    }
    static __device__ __forceinline__ Opnd<OP> get(const char* base, int tile, Lane ln)
    {
        return *reinterpret_cast<const Opnd<OP>*>(base + tile * TILE_BYTES + (16 * ln.q + ln.n) * (int)sizeof(Opnd<OP>));
    }
};

template <int OP> constexpr int ns128_lds_bytes()
{
    return 2 * MailTiles<OP>::BYTES > 4 * STORE_LDS_FLOATS * 4 ? 2 * MailTiles<OP>::BYTES : 4 * STORE_LDS_FLOATS * 4;
}

template <int W> __host__ __device__ constexpr int n128_slot(int i, int k) { return i == W ? k : (W + 1) + k; }

// At: this wave's nine tiles of A in T orientation (slot order of n128_row / n128_col).  lds: ns128_lds_bytes<OP>() bytes
// that no wave uses for anything else any more.
template <int OP, int W>
__device__ __forceinline__ void ns128_run(const Opnd<OP> (&At)[9], Out Tm, char* lds, Lane ln, int n_iter, int w)
{
    typedef MailTiles<OP> Mail;
    char* const X = lds;
    char* const Y = lds + Mail::BYTES;
    v4f Xn[9], Xt[9];
#pragma unroll
    for (int s = 0; s < 9; ++s) {
        const int i = n128_row<W>(s), j = n128_col<W>(s);
        v4f x;
#pragma unroll
        for (int r = 0; r < 4; ++r) x[r] = (i == j && 4 * ln.q + r == ln.n) ? 1.f / 128.f : 0.f;
        Xn[s] = x;
        Xt[s] = x;
        Mail::put(X, tix(i, j), pack<OP>(x), ln);
    }
    __syncthreads();
#pragma unroll 1
    for (int it = 0; it < n_iter; ++it) {
        // Y(i,j) = X(i,j) + sum_k A(i,k) X(k,j) on this wave's rows
#pragma unroll
        for (int s = 0; s < 9; ++s) {
            const int i = n128_row<W>(s), j = n128_col<W>(s);
            const v4f acc = tn_sum<OP>(
                j, i, [&](int k) { return At[n128_slot<W>(i, k)]; }, [&](int k) { return Mail::get(X, tix(k, j), ln); }, Xn[s]);
            Mail::put(Y, tix(i, j), pack<OP>(acc), ln);
        }
        __syncthreads();  // Y complete; nobody reads X from LDS any more in this iteration
        // X(i,j) <- 2 X(i,j) - sum_k X(i,k) Y(k,j), both orientations; the packed old row first
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int i = half == 0 ? W : 7 - W, s0 = half == 0 ? 0 : W + 1;
            Opnd<OP> xo[N128_NB];
#pragma unroll
            for (int k = 0; k < N128_NB; ++k)
                if (k <= i) xo[k] = pack<OP>(Xt[s0 + k]);
#pragma unroll
            for (int j = 0; j < N128_NB; ++j) {
                if (j > i) continue;
                Opnd<OP> y[N128_NB];
#pragma unroll
                for (int k = 0; k < N128_NB; ++k)
                    if (k >= j && k <= i) y[k] = Mail::get(Y, tix(k, j), ln);
                const v4f pn = tn_sum<OP>(j, i, [&](int k) { return xo[k]; }, [&](int k) { return y[k]; }, zero4());
                const v4f pt = tn_sum<OP>(j, i, [&](int k) { return y[k]; }, [&](int k) { return xo[k]; }, zero4());
                Xn[s0 + j] = 2.f * Xn[s0 + j] - pn;
                Xt[s0 + j] = 2.f * Xt[s0 + j] - pt;
                Mail::put(X, tix(i, j), pack<OP>(Xn[s0 + j]), ln);
            }
        }
        __syncthreads();  // X complete; nobody reads Y any more
    }
    // X and Y in LDS are dead: their memory becomes the four store patches
    n128_store<W>(Tm, Xt, reinterpret_cast<float*>(lds) + w * STORE_LDS_FLOATS, ln);
}

// The fused kernel's tiles of A: the four waves load the chunk's keys once between them (wave w its tile rows w and
// 7 - w), pass them through LDS in mailbox form (slot [tile row][k-step][lane], one 16-byte
// key vector each) and every wave forms only its own nine tiles.
template <int KD, int DKS> struct SharedKeys128 {
    typedef typename KeyVec<KD>::type kvec;
    static constexpr int KSTEP = (KD == OP_F32) ? 16 : 32;
    static constexpr int BYTES = 8 * DKS * 64 * 16;
    kvec own[2][DKS];

    // Kc: first key element of (chunk row 0, this head); row_stride in elements; rows beyond valid read the last real token and become zero.
    __device__ __forceinline__ void load(const void* Kc, int64_t row_stride, int valid, int w, Lane ln)
    {
        constexpr int per_lane = (KD == OP_F32) ? 4 : 8;
        const kvec zero = __builtin_bit_cast(kvec, v4u{0u, 0u, 0u, 0u});
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int s = 0; s < DKS; ++s) {
                const int row = 16 * (h == 0 ? w : 7 - w) + ln.n;
                const int64_t off = (int64_t)(row < valid ? row : valid - 1) * row_stride + KSTEP * s + per_lane * ln.q;
                kvec v;
                if (KD == OP_F32)
                    v = *reinterpret_cast<const kvec*>(static_cast<const float*>(Kc) + off);
                else
                    v = *reinterpret_cast<const kvec*>(static_cast<const uint16_t*>(Kc) + off);
                own[h][s] = row < valid ? v : zero;
            }
    }
    __device__ __forceinline__ void publish(char* lds, int w, Lane ln) const
    {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int s = 0; s < DKS; ++s)
                *reinterpret_cast<kvec*>(lds + (((h == 0 ? w : 7 - w) * DKS + s) * 64 + 16 * ln.q + ln.n) * 16) = own[h][s];
    }
    // Tile s of wave W (slot order of n128_row / n128_col) in N (TR = false) or T orientation; after a barrier that
    // follows every wave's publish().
    template <int W, bool TR>
    __device__ __forceinline__ v4f tile(const char* lds, const GateVec<N128_NB>& gate, int s, Lane ln) const
    {
        const int i = n128_row<W>(s), j = n128_col<W>(s);
        v4f acc = zero4();
#pragma unroll
        for (int t = 0; t < DKS; ++t) {
            // both from LDS: the loaded keys' registers are free again once they are published
            const kvec kj = *reinterpret_cast<const kvec*>(lds + ((j * DKS + t) * 64 + 16 * ln.q + ln.n) * 16);
            const kvec ki = *reinterpret_cast<const kvec*>(lds + ((i * DKS + t) * 64 + 16 * ln.q + ln.n) * 16);
            acc = TR ? gram_step<KD>(kj, ki, acc) : gram_step<KD>(ki, kj, acc);
        }
        return gate.template apply<TR>(i, j, acc, ln);
    }
};

// SharedKeys128 behind the tile-source interface, for the tiles of wave W only.
template <int KD, int DKS, int W> struct SharedA128 {
    const SharedKeys128<KD, DKS>& keys;
    const GateVec<N128_NB>& gate;
    const char* lds;
    Lane ln;
    template <bool TR> __device__ __forceinline__ v4f get(int i, int j) const
    {
        return keys.template tile<W, TR>(lds, gate, i == W ? j : (W + 1) + j, ln);
    }
};

template <int OP, int W, class ASrc> __device__ __forceinline__ void ns128_tiles_of(const ASrc& A, Opnd<OP> (&At)[9])
{
#pragma unroll
    for (int s = 0; s < 9; ++s) At[s] = pack<OP>(A.template get<true>(n128_row<W>(s), n128_col<W>(s)));
}

// ---------------------------------------------------------------------------------------------
// Neumann product at C = 128, (I + A)^-1 = (I - A) (I + A^2) (I + A^4) ... (I + A^64): the four-wavefront workgroup
// and the mailbox tiles of the Newton-Schulz kernel above.  Wave w owns tile rows w and 7 - w.  It keeps X^T (fp32)
// and its rows of the running power Y = A^(2^k) in T orientation (packed) in registers; every product takes its
// other factor, a tile of Y in N orientation, from the mailbox.  Squaring forms both orientations of the new tile
// (two matrix-core instructions per product instead of one transposing read through LDS); the N image goes to the
// other of two mailbox buffers, which leaves one barrier per iteration:
//   Y' <- Y Y (cur -> nxt);  barrier;  X^T += Y'^T X^T (reads nxt);  swap.
// ---------------------------------------------------------------------------------------------
// Wave W's share of the start: X^T = I - A^T and Y = A in T orientation into registers, Y in N orientation into the mailbox.
template <int OP, int W, class ASrc>
__device__ __forceinline__ void neumann128_prepare(const ASrc& A, v4f (&Xt)[9], Opnd<OP> (&yt)[9], char* cur, Lane ln)
{
#pragma unroll
    for (int s = 0; s < 9; ++s) {
        const int i = n128_row<W>(s), j = n128_col<W>(s);
        MailTiles<OP>::put(cur, tix(i, j), pack<OP>(A.template get<false>(i, j)), ln);
        const v4f at = A.template get<true>(i, j);
#pragma unroll
        for (int r = 0; r < 4; ++r) Xt[s][r] = ((i == j && 4 * ln.q + r == ln.n) ? 1.f : 0.f) - at[r];
        yt[s] = pack<OP>(at);
    }
}

// cur, nxt: the two mailbox buffers (MailTiles<OP>::BYTES each), cur filled by neumann128_prepare; patch: this wave's
// store patch, anywhere in LDS that no wave uses for anything but the two buffers.
template <int OP, int W>
__device__ __forceinline__ void neumann128_run(v4f (&Xt)[9], Opnd<OP> (&yt)[9], Out Tm, char* cur, char* nxt, float* patch, Lane ln)
{
    typedef MailTiles<OP> Mail;
    __syncthreads();
#pragma unroll 1
    for (int it = 0; it < 6; ++it) {  // log2(128 / 2)
        const int p = 1 << it, pn = 2 << it;
        Opnd<OP> ytn[9];
#pragma unroll
        for (int s = 0; s < 9; ++s) {
            const int i = n128_row<W>(s), j = n128_col<W>(s);
            // structural zeros of A^p (tile (a, b) vanishes when 16 (a - b) + 15 < p); p is uniform
            const auto live = [&](int k) { return 16 * (i - k) + 15 >= p && 16 * (k - j) + 15 >= p; };
            const auto mine = [&](int k) { return yt[n128_slot<W>(i, k)]; };
            Opnd<OP> y[N128_NB];
#pragma unroll
            for (int k = 0; k < N128_NB; ++k)
                if (k >= j && k <= i) y[k] = Mail::get(cur, tix(k, j), ln);
            const auto theirs = [&](int k) { return y[k]; };
            const v4f an = tn_sum_if<OP>(j, i, mine, theirs, live, zero4());
            const v4f at = tn_sum_if<OP>(j, i, theirs, mine, live, zero4());
            ytn[s] = pack<OP>(at);
            Mail::put(nxt, tix(i, j), pack<OP>(an), ln);
        }
#pragma unroll
        for (int s = 0; s < 9; ++s) yt[s] = ytn[s];
        __syncthreads();  // the new power is complete; nobody reads the old one any more
        // X^T(i,j) += sum_k Y(k,j)^T X(i,k)^T over this wave's two tile rows; the packed old row first
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int i = half == 0 ? W : 7 - W, s0 = half == 0 ? 0 : W + 1;
            Opnd<OP> xo[N128_NB];
#pragma unroll
            for (int k = 0; k < N128_NB; ++k)
                if (k <= i) xo[k] = pack<OP>(Xt[s0 + k]);
#pragma unroll
            for (int j = 0; j < N128_NB; ++j) {
                if (j > i) continue;
                Xt[s0 + j] = tn_sum_if<OP>(
                    j, i, [&](int k) { return Mail::get(nxt, tix(k, j), ln); }, [&](int k) { return xo[k]; },
                    [&](int k) { return 16 * (k - j) + 15 >= pn; }, Xt[s0 + j]);
            }
        }
        char* const t = cur;
        cur = nxt;
        nxt = t;
    }
    __syncthreads();  // both mailbox buffers are dead: their memory becomes the four store patches
    n128_store<W>(Tm, Xt, patch, ln);
}

// ---------------------------------------------------------------------------------------------
// One step of iterative refinement at C = 128 (paper Alg. 6, Eq. 9, for I + A), as a second pass over
// a result Y that an earlier kernel left in T (fp32), in place:
//   R <- I - Y (I + A);   X <- Y + R Y.
// The same four-wavefront workgroup: Y goes to LDS (36 fp32 tiles, N layout); wave w keeps its tile
// rows w and 7 - w of Y^T and R^T in registers and forms
//   R^T(i,j) = [i==j] I - Y^T(i,j) - sum_k A(k,j)^T Y(i,k)^T,     X^T(i,j) = Y^T(i,j) + sum_k Y(k,j)^T R(i,k)^T.
// A wave reads and writes only its own rows of T in global memory, so the pass is safe in place.
// ---------------------------------------------------------------------------------------------
// Tile (k, j) of A as a left factor (N orientation, packed): formed on the spot by the sources that hold keys or read memory.
template <int OP, class ASrc> __device__ __forceinline__ Opnd<OP> left_operand(const ASrc& A, int k, int j)
{
    return pack<OP>(A.template get<false>(k, j));
}

template <int OP, int W, class ASrc>
__device__ __forceinline__ void refine128_run(const ASrc& A, float* Tm, float* Y, Lane ln, int w)
{
    v4f Yt[9];
#pragma unroll
    for (int s = 0; s < 9; ++s) {
        const int i = n128_row<W>(s), j = n128_col<W>(s);
        // row-major 16-byte pieces = the tile in T orientation: v[r] = Y[16i + n][16j + 4q + r]
        Yt[s] = *reinterpret_cast<const v4f*>(Tm + (16 * i + ln.n) * 128 + 16 * j + 4 * ln.q);
        *reinterpret_cast<v4f*>(&Y[tix(i, j) * XPOSE_FLOATS + ln.n * XPOSE_LD + 4 * ln.q]) = Yt[s];
    }
    __syncthreads();
    Opnd<OP> Rt[9];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int i = half == 0 ? W : 7 - W, s0 = half == 0 ? 0 : W + 1;
        Opnd<OP> yo[N128_NB];
#pragma unroll
        for (int k = 0; k < N128_NB; ++k)
            if (k <= i) yo[k] = pack<OP>(Yt[s0 + k]);
#pragma unroll
        for (int j = 0; j < N128_NB; ++j) {
            if (j > i) continue;
            v4f acc = zero4();
#pragma unroll
            for (int k = 0; k < N128_NB; ++k) {
                if (k < j || k > i) continue;
                acc = tn<OP>(left_operand<OP>(A, k, j), yo[k], acc);
            }
            v4f r;
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = ((i == j && 4 * ln.q + e == ln.n) ? 1.f : 0.f) - Yt[s0 + j][e] - acc[e];
            Rt[s0 + j] = pack<OP>(r);
        }
    }
    v4f Xt[9];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int i = half == 0 ? W : 7 - W, s0 = half == 0 ? 0 : W + 1;
#pragma unroll
        for (int j = 0; j < N128_NB; ++j) {
            if (j > i) continue;
            v4f acc = Yt[s0 + j];
#pragma unroll
            for (int k = 0; k < N128_NB; ++k) {
                if (k < j || k > i) continue;
                acc = tn<OP>(pack<OP>(lds_tile_read_n(Y + tix(k, j) * XPOSE_FLOATS, ln)), Rt[s0 + k], acc);
            }
            Xt[s0 + j] = acc;
        }
    }
    __syncthreads();  // Y is dead: its memory becomes the four store patches
    n128_store<W>(Out{Tm, OP_F32}, Xt, Y + w * STORE_LDS_FLOATS, ln);
}

template <int OP>
__global__ __launch_bounds__(256) void k_tri_inv_refine128(const void* __restrict__ A, float* T, int64_t n_mat, int in_dt)
{
    __shared__ __attribute__((aligned(16))) float Y[N128_LDS_FLOATS];
    const int64_t m = blockIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Lane ln = lane_id();
    GlobalA<N128_NB> src;
    src.base = static_cast<const char*>(A) + m * 128 * 128 * (in_dt == OP_F32 ? 4 : 2);
    src.dt = in_dt;
    src.ln = ln;
    (void)n_mat;
    TRIINV_PER_WAVE(w, (refine128_run<OP, W>(src, T + m * 128 * 128, Y, ln, w)))
}

template <int KD, int OP, int DKS>
__global__ __launch_bounds__(256) void k_gdn_tri_inv_refine128(const void* __restrict__ K, const float* __restrict__ beta,
                                                               const float* __restrict__ g, float* T, int64_t n_chunk,
                                                               ChunkMap map, int H, int d_k)
{
    constexpr int C = 128;
    __shared__ __attribute__((aligned(16))) float Y[N128_LDS_FLOATS];
    const int64_t m = head_group_swizzle(blockIdx.x, n_chunk, H);
    const uint32_t bc = (uint32_t)m / (uint32_t)H;
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Lane ln = lane_id();
    GramA<KD, N128_NB, DKS> src;
    src.ln = ln;
    const int64_t esz = (KD == OP_F32) ? 4 : 2;
    src.issue_gate(beta + tok0 * H + h, g ? g + tok0 * H + h : nullptr, H, pos.valid);
    src.load_keys(static_cast<const char*>(K) + (tok0 * H + h) * (int64_t)d_k * esz, (int64_t)H * d_k, pos.valid);
    src.stage_gate(Y + w * 2 * C);  // a private 2 * C floats inside the (not yet used) Y buffer
    __syncthreads();
    TRIINV_PER_WAVE(w, (refine128_run<OP, W>(src, T + m * C * C, Y, ln, w)))
}

template <int OP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OP == OP_F32 ? 2 : 3))) void k_tri_inv_ns128(const void* A, float* T, int64_t n_mat, int in_dt, int n_iter, int out_dt)  // may run in place
{
    __shared__ __attribute__((aligned(16))) char lds[ns128_lds_bytes<OP>()];
    const int64_t m = blockIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Lane ln = lane_id();
    GlobalA<N128_NB> src;
    src.base = static_cast<const char*>(A) + m * 128 * 128 * (in_dt == OP_F32 ? 4 : 2);
    src.dt = in_dt;
    src.ln = ln;
    (void)n_mat;
    Opnd<OP> At[9];
    TRIINV_PER_WAVE(w, (ns128_tiles_of<OP, W>(src, At)))
    // in place: every wave has read its rows of A before any wave stores (the iteration's barriers lie between)
    TRIINV_PER_WAVE(w, (ns128_run<OP, W>(At, out_matrix(T, m, 128, out_dt), lds, ln, n_iter, w)))
}

template <int KD, int OP, int DKS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OP == OP_F32 ? 2 : 3))) void k_gdn_tri_inv_ns128(const void* __restrict__ K, const float* __restrict__ beta,
                                                           const float* __restrict__ g, float* __restrict__ T,
                                                           int64_t n_chunk, ChunkMap map, int H, int d_k, int n_iter, int out_dt)
{
    constexpr int C = 128;
    typedef SharedKeys128<KD, DKS> Keys;
    constexpr int GATE_BYTES = 4 * 2 * C * 4;  // beta and g of the chunk, staged by every wave for itself
    constexpr int LDS_BYTES = ns128_lds_bytes<OP>() > Keys::BYTES + GATE_BYTES ? ns128_lds_bytes<OP>() : Keys::BYTES + GATE_BYTES;
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    const int64_t m = head_group_swizzle(blockIdx.x, n_chunk, H);
    const uint32_t bc = (uint32_t)m / (uint32_t)H;
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Lane ln = lane_id();
    const int64_t esz = (KD == OP_F32) ? 4 : 2;
    GateVec<N128_NB> gate;
    Keys keys;
    gate.issue(beta + tok0 * H + h, g ? g + tok0 * H + h : nullptr, H, ln, pos.valid);
    keys.load(static_cast<const char*>(K) + (tok0 * H + h) * (int64_t)d_k * esz, (int64_t)H * d_k, pos.valid, w, ln);
    gate.stage(reinterpret_cast<float*>(lds + Keys::BYTES) + w * 2 * C, ln);
    keys.publish(lds, w, ln);
    __syncthreads();
    Opnd<OP> At[9];
    TRIINV_PER_WAVE(w, (ns128_tiles_of<OP, W>(SharedA128<KD, DKS, W>{keys, gate, lds, ln}, At)))
    __syncthreads();  // the keys in LDS are dead: X and Y take their place
    TRIINV_PER_WAVE(w, (ns128_run<OP, W>(At, out_matrix(T, m, C, out_dt), lds, ln, n_iter, w)))
}

template <int OP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OP == OP_F32 ? 2 : 3))) void k_tri_inv_neumann128(const void* A, float* T, int64_t n_mat, int in_dt, int out_dt)  // may run in place
{
    __shared__ __attribute__((aligned(16))) char lds[ns128_lds_bytes<OP>()];
    const int64_t m = blockIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Lane ln = lane_id();
    GlobalA<N128_NB> src;
    src.base = static_cast<const char*>(A) + m * 128 * 128 * (in_dt == OP_F32 ? 4 : 2);
    src.dt = in_dt;
    src.ln = ln;
    (void)n_mat;
    v4f Xt[9];
    Opnd<OP> yt[9];
    char* const nxt = lds + MailTiles<OP>::BYTES;
    float* const patch = reinterpret_cast<float*>(lds) + w * STORE_LDS_FLOATS;
    TRIINV_PER_WAVE(w, (neumann128_prepare<OP, W>(src, Xt, yt, lds, ln)))
    // in place: every wave has read its rows of A before any wave stores (the iteration's barriers lie between)
    TRIINV_PER_WAVE(w, (neumann128_run<OP, W>(Xt, yt, out_matrix(T, m, 128, out_dt), lds, nxt, patch, ln)))
}

template <int KD, int OP, int DKS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(OP == OP_F32 ? 2 : 3))) void k_gdn_tri_inv_neumann128(const void* __restrict__ K, const float* __restrict__ beta,
                                                                const float* __restrict__ g, float* __restrict__ T,
                                                                int64_t n_chunk, ChunkMap map, int H, int d_k, int out_dt)
{
    constexpr int C = 128;
    typedef SharedKeys128<KD, DKS> Keys;
    typedef MailTiles<OP> Mail;
    // [keys | first mailbox buffer]; the second buffer takes the keys' place (first written after the barrier that ends
    // the keys' use), beta and g are staged, by every wave for itself, where the first buffer will be
    constexpr int CUR = Keys::BYTES > Mail::BYTES ? Keys::BYTES : Mail::BYTES;
    constexpr int LDS_BYTES = CUR + Mail::BYTES;
    static_assert(4 * 2 * C * 4 <= Mail::BYTES && 4 * STORE_LDS_FLOATS * 4 <= LDS_BYTES, "staging area and store patches fit");
    __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];
    const int64_t m = head_group_swizzle(blockIdx.x, n_chunk, H);
    const uint32_t bc = (uint32_t)m / (uint32_t)H;
    const int h = (int)((uint32_t)m - bc * (uint32_t)H);
    const ChunkPos pos = locate_chunk<C>(map, bc);
    const int64_t tok0 = pos.tok0;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const Lane ln = lane_id();
    const int64_t esz = (KD == OP_F32) ? 4 : 2;
    GateVec<N128_NB> gate;
    Keys keys;
    gate.issue(beta + tok0 * H + h, g ? g + tok0 * H + h : nullptr, H, ln, pos.valid);
    keys.load(static_cast<const char*>(K) + (tok0 * H + h) * (int64_t)d_k * esz, (int64_t)H * d_k, pos.valid, w, ln);
    gate.stage(reinterpret_cast<float*>(lds + CUR) + w * 2 * C, ln);
    keys.publish(lds, w, ln);
    __syncthreads();  // keys published, and every wave is done with its staging area
    v4f Xt[9];
    Opnd<OP> yt[9];
    float* const patch = reinterpret_cast<float*>(lds) + w * STORE_LDS_FLOATS;
    TRIINV_PER_WAVE(w, (neumann128_prepare<OP, W>(SharedA128<KD, DKS, W>{keys, gate, lds, ln}, Xt, yt, lds + CUR, ln)))
    TRIINV_PER_WAVE(w, (neumann128_run<OP, W>(Xt, yt, out_matrix(T, m, C, out_dt), lds + CUR, lds, patch, ln)))
}

}  // namespace triinv
