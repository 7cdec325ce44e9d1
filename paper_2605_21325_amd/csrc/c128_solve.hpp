// C = 128, the inverse applied instead of stored (W = (I + A)^{-1} diag(s) X, paper Sec. 1 Eq. 3; direction of the fused
// layer kernel of Sec. 5.2) on the two-wavefront layout of c128.hpp.  After the recursion the 36 lower tiles of the
// inverse are spread over the two waves; each wave scales its 18 tiles' columns by s, rounds them to the operand type
// and publishes them in LDS (row-major 16 x 16 tiles: a tile written in either orientation is read back in T
// orientation, the left-factor form of tn(), with one access per lane).  Two right-hand sides are split by COLUMNS
// (c128_apply): a lane owns the 8 bytes of consecutive columns one load brings (4 for 16-bit elements, 2 for fp32), 16
// lanes cover one 128-byte line of a row, and the 64- (32-) column groups go to the two waves alternately, so that at
// d_x = 128 each wave reads half of every row of X, multiplies all 36 tiles into it and writes half of every row of W:
// the same bytes and the same number of tile products on both waves.  A single right-hand side is split by ROWS
// (c128_apply_rows): each wave loads and stores whole 256-byte row pieces of its 64 rows, and the top rows of X
// reach the wave that computes the bottom rows through LDS.
#pragma once
#include <type_traits>
#include "c128.hpp"
#include "solve.hpp"

namespace triinv {

// Eight bytes of one row of X as stored.
template <int OP> struct XHalf;
template <> struct XHalf<OP_F32> { v2f f; };
template <> struct XHalf<OP_F16> { v2u u; };
template <> struct XHalf<OP_BF16> { v2u u; };

// Column tile c of a 16-row tile row of X as a matrix-core operand: rows 4q + r of this lane's column VEC n + c.
template <int OP> __device__ __forceinline__ Opnd<OP> xh_operand(const XHalf<OP> (&row)[4], int c)
{
    if constexpr (OP == OP_F32) {
        return {v4f{row[0].f[c], row[1].f[c], row[2].f[c], row[3].f[c]}};
    } else {
        const int d = c >> 1;
        const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;  // the lower / upper halves of two rows' dwords
        const uint32_t lo = __builtin_amdgcn_perm(row[1].u[d], row[0].u[d], sel);
        const uint32_t hi = __builtin_amdgcn_perm(row[3].u[d], row[2].u[d], sel);
        Opnd<OP> o;
        o.x = __builtin_bit_cast(decltype(o.x), v2u{lo, hi});
        return o;
    }
}

// One right-hand side, seen by one wave: 128 rows, column groups of 16 * VEC columns.  X and W are addressed through
// buffer descriptors based at the chunk's first row of this head with 32-bit byte offsets (128 rows of H * d_x elements
// stay far below 2^31 bytes; the launcher checks): one offset register per row instead of a 64-bit pointer.
template <int OP> struct RhsHalf {
    static constexpr int ESZ = OP == OP_F32 ? 4 : 2;
    static constexpr int VEC = 8 / ESZ;
    static constexpr int GW = 16 * VEC;
    static constexpr int CACHE_NT = 2;  // non-temporal stores of W (the streaming policy of T's stores measured slower here)
    __amdgpu_buffer_rsrc_t xb, wb;
    int row_bytes;
    int d_x, valid;
    Lane ln;
    XHalf<OP> raw[8][4];

    __device__ __forceinline__ void init(const RhsArgs& a, int64_t tok0, int h, int H, int valid_, Lane ln_)
    {
        ln = ln_;
        d_x = a.d_x;
        valid = valid_;
        row_bytes = H * d_x * ESZ;
        const int64_t e0 = (tok0 * H + h) * (int64_t)d_x * ESZ;
        // the descriptors span the chunk's real rows: whatever lies beyond is neither read nor written
        const int span = (valid - 1) * row_bytes + d_x * ESZ;
        xb = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(a.X)) + e0, 0, span, 0x00020000);
        wb = __builtin_amdgcn_make_buffer_rsrc(static_cast<char*>(a.W) + e0, 0, span, 0x00020000);
    }
    __device__ __forceinline__ bool active(int gi) const { return GW * gi + VEC * ln.n < d_x; }
    __device__ __forceinline__ int n_group() const { return (d_x + GW - 1) / GW; }

    // Byte offset of (row 16 j + 4 q + r, this lane's columns) = lane part (one register) + uniform part (a scalar; the
    // hardware's range check does not see it, so it is only used for tile rows that lie inside the chunk entirely).
    // The one tile row a short last chunk may cut is handled lane by lane (rows beyond the last token read that token:
    // they only meet zero columns of the inverse); tile rows beyond it are not touched at all.
    __device__ __forceinline__ int lane_offset(int gi) const
    {
        return 4 * ln.q * row_bytes + (active(gi) ? (GW * gi + VEC * ln.n) * ESZ : 0);
    }

    __device__ __forceinline__ void issue(int gi)
    {
        const int lo = lane_offset(gi);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (16 * j + 16 <= valid) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    raw[j][r] = __builtin_bit_cast(XHalf<OP>, __builtin_amdgcn_raw_buffer_load_b64(xb, lo, (16 * j + r) * row_bytes, 0));
            } else if (16 * j < valid) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = 16 * j + 4 * ln.q + r;
                    const int rc = row < valid ? row : valid - 1;
                    raw[j][r] = __builtin_bit_cast(XHalf<OP>, __builtin_amdgcn_raw_buffer_load_b64(xb, lo + (rc - 4 * ln.q) * row_bytes, 0, 0));
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) raw[j][r] = __builtin_bit_cast(XHalf<OP>, v2u{0u, 0u});
            }
        }
    }

    __device__ __forceinline__ void store(int gi, int i, const v4f (&acc)[VEC])
    {
        if (!active(gi) || 16 * i >= valid) return;
        const int lo = lane_offset(gi);
        const bool whole = 16 * i + 16 <= valid;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            v2u v;
            if constexpr (OP == OP_F32) {
                v = __builtin_bit_cast(v2u, v2f{acc[0][r], acc[1][r]});
            } else if constexpr (OP == OP_F16) {
                v = v2u{pack2_f16(acc[0][r], acc[1][r]), pack2_f16(acc[2][r], acc[3][r])};
            } else {
                v = v2u{pack2_bf16(acc[0][r], acc[1][r]), pack2_bf16(acc[2][r], acc[3][r])};
            }
            if (whole || 16 * i + 4 * ln.q + r < valid) __builtin_amdgcn_raw_buffer_store_b64(v, wb, lo, (16 * i + r) * row_bytes, CACHE_NT);
        }
    }
};

// Column tile c of a 16-row tile row of X held as 16-byte row pieces (solve.hpp's XRow), as a matrix-core operand: one
// byte-permute per register takes the lower (c even) or upper (c odd) halves of two rows' dwords.
template <int OP> __device__ __forceinline__ Opnd<OP> xrow_operand(const XRow<OP> (&row)[4], int c)
{
    if constexpr (OP == OP_F32) {
        return {v4f{row[0].f[c], row[1].f[c], row[2].f[c], row[3].f[c]}};
    } else {
        const int d = c >> 1;
        const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
        Opnd<OP> o;
        o.x = __builtin_bit_cast(decltype(o.x), v2u{__builtin_amdgcn_perm(row[1].u[d], row[0].u[d], sel),
                                                    __builtin_amdgcn_perm(row[3].u[d], row[2].u[d], sel)});
        return o;
    }
}

// One right-hand side split by ROWS: wave W owns rows 64 W .. 64 W + 63 of X and of the result, in whole 256-byte row
// pieces (a lane owns the 16 bytes one load brings, 16 lanes one row piece, four rows per instruction: the layout of the
// one-wavefront kernels, solve.hpp).  Column groups of 16 * VEC columns.
template <int OP> struct RhsRows {
    static constexpr int ESZ = OP == OP_F32 ? 4 : 2;
    static constexpr int VEC = 16 / ESZ;
    static constexpr int GW = 16 * VEC;
    static constexpr int CACHE_NT = 2;
    __amdgpu_buffer_rsrc_t xb, wb;
    int row_bytes;
    int d_x, valid;
    Lane ln;
    XRow<OP> raw[4][4];  // tile row 4 W + j, row 4 q + r of it

    __device__ __forceinline__ void init(const RhsArgs& a, int64_t tok0, int h, int H, int valid_, Lane ln_)
    {
        ln = ln_;
        d_x = a.d_x;
        valid = valid_;
        row_bytes = H * d_x * ESZ;
        const int64_t e0 = (tok0 * H + h) * (int64_t)d_x * ESZ;
        const int span = (valid - 1) * row_bytes + d_x * ESZ;  // the chunk's real rows: nothing beyond is read or written
        xb = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(a.X)) + e0, 0, span, 0x00020000);
        wb = __builtin_amdgcn_make_buffer_rsrc(static_cast<char*>(a.W) + e0, 0, span, 0x00020000);
    }
    __device__ __forceinline__ bool active(int gi) const { return GW * gi + VEC * ln.n < d_x; }
    __device__ __forceinline__ int n_group() const { return (d_x + GW - 1) / GW; }
    __device__ __forceinline__ int lane_offset(int gi) const
    {
        return 4 * ln.q * row_bytes + (active(gi) ? (GW * gi + VEC * ln.n) * ESZ : 0);
    }

    // Loads of this wave's 64 rows of column group gi.  A tile row inside the chunk entirely takes the row's offset as the
    // uniform part of the address (the hardware's range check does not see that part); the one a short last chunk cuts is
    // clamped lane by lane (rows beyond the last token read that token: they only meet zero columns of the inverse);
    // tile rows beyond it are zero.
    template <int W> __device__ __forceinline__ void issue(int gi)
    {
        const int lo = lane_offset(gi);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int J = 4 * W + j;
            if (16 * J + 16 <= valid) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    raw[j][r] = __builtin_bit_cast(XRow<OP>, __builtin_amdgcn_raw_buffer_load_b128(xb, lo, (16 * J + r) * row_bytes, 0));
            } else if (16 * J < valid) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = 16 * J + 4 * ln.q + r;
                    const int rc = row < valid ? row : valid - 1;
                    raw[j][r] = __builtin_bit_cast(XRow<OP>, __builtin_amdgcn_raw_buffer_load_b128(xb, lo + (rc - 4 * ln.q) * row_bytes, 0, 0));
                }
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) raw[j][r] = __builtin_bit_cast(XRow<OP>, v4u{0u, 0u, 0u, 0u});
            }
        }
    }

    // Rows 16 J + 4 q + r of the result, VEC columns per lane: acc[c][r].  The row's offset goes into the per-lane part
    // of the address (a 16-byte buffer store with a register as its uniform offset is not followed by the wait state its
    // data registers need before they are written again).
    __device__ __forceinline__ void store(int gi, int J, const v4f (&acc)[VEC])
    {
        if (!active(gi) || 16 * J >= valid) return;
        const int lo = lane_offset(gi);
        const bool whole = 16 * J + 16 <= valid;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            v4u v;
            if constexpr (OP == OP_F32) {
                v = __builtin_bit_cast(v4u, v4f{acc[0][r], acc[1][r], acc[2][r], acc[3][r]});
            } else if constexpr (OP == OP_F16) {
                v = v4u{pack2_f16(acc[0][r], acc[1][r]), pack2_f16(acc[2][r], acc[3][r]), pack2_f16(acc[4][r], acc[5][r]),
                        pack2_f16(acc[6][r], acc[7][r])};
            } else {
                v = v4u{pack2_bf16(acc[0][r], acc[1][r]), pack2_bf16(acc[2][r], acc[3][r]), pack2_bf16(acc[4][r], acc[5][r]),
                        pack2_bf16(acc[6][r], acc[7][r])};
            }
            if (whole || 16 * J + 4 * ln.q + r < valid)
                __builtin_amdgcn_raw_buffer_store_b128(v, wb, lo + (16 * J + r) * row_bytes, 0, CACHE_NT);
        }
    }
};

// Published tiles: element type = operand type, 16 rows of TILE_LD elements.  16-bit tiles go without padding (a set is
// 18 KB, two sets and the recursion fit four workgroups per compute unit): the 8-byte row pieces read_t / write_t move
// stay conflict-free, the 2-byte column writes of write_n become two-way conflicts.  fp32 tiles keep a stride of 20.
template <int OP> struct TileLds {
    typedef typename std::conditional<OP == OP_F32, float, uint16_t>::type elem;
    static constexpr int TILE_LD = OP == OP_F32 ? 20 : 16;
    static constexpr int TILE_ELEMS = 16 * TILE_LD;
    static constexpr int BYTES = 36 * TILE_ELEMS * (int)sizeof(elem);

    static __device__ __forceinline__ elem narrow(float x)
    {
        if constexpr (OP == OP_F32) {
            return x;
        } else if constexpr (OP == OP_F16) {
            return (uint16_t)(pack2_f16(x, 0.f) & 0xffffu);
        } else {
            return (uint16_t)(pack2_bf16(x, 0.f) & 0xffffu);
        }
    }
    // t in N orientation (t[r] = M[4q + r][n])
    static __device__ __forceinline__ void write_n(elem* tile, v4f t, Lane ln)
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) tile[(4 * ln.q + r) * TILE_LD + ln.n] = narrow(t[r]);
    }
    // t in T orientation (t[r] = M[n][4q + r])
    static __device__ __forceinline__ void write_t(elem* tile, v4f t, Lane ln)
    {
        const Opnd<OP> o = pack<OP>(t);
        *reinterpret_cast<Opnd<OP>*>(&tile[ln.n * TILE_LD + 4 * ln.q]) = o;
    }
    static __device__ __forceinline__ Opnd<OP> read_t(const elem* tile, Lane ln)
    {
        return *reinterpret_cast<const Opnd<OP>*>(&tile[ln.n * TILE_LD + 4 * ln.q]);
    }
};

template <int KD, int OP, int DKS, int METHOD, int NRHS> struct C128SolveLds {
    typedef C128Lds<KD, OP, DKS, METHOD, false> INV;
    static constexpr int TILES = 0;  // after the recursion, in place of the keys: one set of 36 tiles per right-hand side
    static constexpr int SCALE = INV::BYTES > NRHS * TileLds<OP>::BYTES ? INV::BYTES : NRHS * TileLds<OP>::BYTES;  // 128 floats per wave
    static constexpr int BYTES = SCALE + 2 * 128 * 4;
};

// The row scales of this lane's two tokens, every right-hand side.
template <int NRHS>
__device__ __forceinline__ void c128_load_scales(float (&raw_s)[NRHS][2], const RhsList& rhs, int64_t tok0, int h, int H, int valid, int lane)
{
#pragma unroll
    for (int k = 0; k < NRHS; ++k)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int row = lane + 64 * t;
            const int rc = row < valid ? row : valid - 1;
            raw_s[k][t] = rhs.r[k].scale ? rhs.r[k].scale[(tok0 + rc) * H + h] : 1.f;
        }
}

// The diagonal tiles of a wave's block in exact unit-triangular form (wave 0 holds them in N, wave 1 in T orientation).
template <int W> __device__ __forceinline__ void c128_unit_diagonal(v4f (&D)[10], Lane ln)
{
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int rr = W == 0 ? 4 * ln.q + r : ln.n, cc = W == 0 ? ln.n : 4 * ln.q + r;
            D[tix(d, d)][r] = (rr == cc) ? 1.f : ((rr > cc) ? D[tix(d, d)][r] : 0.f);
        }
}

// s of one right-hand side by the two index patterns the tiles' columns need: s_n[j] = s[16 j + n] (all eight tile
// columns), s_q[j][r] = s[64 + 16 j + 4 q + r] (the bottom block's).  sc: this wave's 128 floats of LDS.
__device__ __forceinline__ void c128_scale_patterns(float* sc, const float (&raw)[2], float (&s_n)[8], v4f (&s_q)[4], Lane ln)
{
    const int lane = 16 * ln.q + ln.n;
    sc[lane] = raw[0];
    sc[lane + 64] = raw[1];
    wave_lds_sync();
#pragma unroll
    for (int j = 0; j < 8; ++j) s_n[j] = sc[16 * j + ln.n];
#pragma unroll
    for (int j = 0; j < 4; ++j) s_q[j] = *reinterpret_cast<const v4f*>(&sc[64 + 16 * j + 4 * ln.q]);
    wave_lds_sync();
}

// This wave's 18 tiles of the inverse, columns scaled by s, rounded to the operand type, into one published set.
template <int OP, int W>
__device__ __forceinline__ void c128_publish_tiles(typename TileLds<OP>::elem* set, const v4f (&D)[10], const v4f (&Wc)[2][4],
                                                   const float (&s_n)[8], const v4f (&s_q)[4], Lane ln)
{
    typedef TileLds<OP> TL;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j <= i; ++j) {
            if (W == 0)
                TL::write_n(set + tix(i, j) * TL::TILE_ELEMS, D[tix(i, j)] * s_n[j], ln);
            else
                TL::write_t(set + tix(4 + i, 4 + j) * TL::TILE_ELEMS, D[tix(i, j)] * s_q[j], ln);
        }
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int col = c128_col<W>(c);
            TL::write_n(set + tix(4 + i, col) * TL::TILE_ELEMS, Wc[c][i] * s_n[col], ln);
        }
        __builtin_amdgcn_sched_barrier(0);  // tile row by tile row: scaled all at once the tiles take twice their registers
    }
}

// The inverse (D: this wave's diagonal block, Wc: its two tile columns of the off-diagonal block, as the recursion leaves
// them) applied to NRHS right-hand sides.  The sides share the inverse: its tiles are published once per right-hand side
// (their columns scaled by that side's s), all sets before the one barrier, so that nothing of the inverse stays in
// registers afterwards.  x: initialised for the first right-hand side, its first column group (W) already requested
// (taken by value: through a reference its row registers ended up in scratch memory for fp32 operands).
// tiles_lds: NRHS * TileLds<OP>::BYTES that both waves are done with when they arrive here (a barrier comes first);
// scale_lds: 128 floats per wave.
template <int OP, int W, int NRHS>
__device__ __forceinline__ void c128_apply(char* tiles_lds, char* scale_lds, v4f (&D)[10], v4f (&Wc)[2][4], const float (&raw_s)[NRHS][2],
                                           RhsHalf<OP> x, const RhsList& rhs, int64_t tok0, int h, int H, int valid, Lane ln)
{
    typedef TileLds<OP> TL;
    typedef typename TL::elem elem;
    c128_unit_diagonal<W>(D, ln);
    elem* tiles = reinterpret_cast<elem*>(tiles_lds);
    float* sc = reinterpret_cast<float*>(scale_lds) + 128 * W;
    constexpr int VEC = RhsHalf<OP>::VEC;
    __syncthreads();  // nobody reads what the recursion kept where the tiles go
#pragma unroll
    for (int k = 0; k < NRHS; ++k) {
        float s_n[8];
        v4f s_q[4];
        c128_scale_patterns(sc, raw_s[k], s_n, s_q, ln);
        c128_publish_tiles<OP, W>(tiles + k * 36 * TL::TILE_ELEMS, D, Wc, s_n, s_q, ln);
    }
    __syncthreads();  // every tile is in LDS
#pragma unroll
    for (int k = 0; k < NRHS; ++k) {
        if (k > 0) {
            x.init(rhs.r[k], tok0, h, H, valid, ln);
            __builtin_amdgcn_sched_barrier(0);
            if (W < x.n_group()) x.issue(W);
        }
        const int n_group = x.n_group();
#pragma unroll 1
        for (int gi = W; gi < n_group;) {
            Opnd<OP> xo[8][VEC];
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int c = 0; c < VEC; ++c) xo[j][c] = xh_operand<OP>(x.raw[j], c);
            const int cur = gi;
            gi += 2;
            // the tiles are read back strip by strip (held in registers they would cost a wavefront per SIMD; the opaque
            // offset keeps the reads inside this loop -- an offset, not the pointer: behind an opaque pointer the compiler
            // no longer knows that it reads LDS, and the generic loads it then uses wait for every store of W before them)
            int hide = 0;
            asm volatile("" : "+v"(hide));
            const elem* set = tiles + k * 36 * TL::TILE_ELEMS + hide;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v4f acc[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = zero4();
#pragma unroll
                for (int j = 0; j <= i; ++j) {
                    const Opnd<OP> t = TL::read_t(set + tix(i, j) * TL::TILE_ELEMS, ln);
#pragma unroll
                    for (int c = 0; c < VEC; ++c) acc[c] = tn<OP>(t, xo[j][c], acc[c]);
                }
                x.store(cur, i, acc);
                __builtin_amdgcn_sched_barrier(0);  // one strip's tile reads at a time (all 36 hoisted to the top cost 72 registers)
            }
            if (gi < n_group) x.issue(gi);  // (d_x > 128 only; started earlier it would cost the registers of a second group)
        }
    }
}

template <int KD, int OP, int METHOD, int DKS, int W, int NRHS, bool NOGATE>
__device__ __forceinline__ void c128_invert_and_apply(char* lds, const void* Kc, int64_t row_stride, const float* bc, const float* gc,
                                                      int64_t tok_stride, const RhsList& rhs, int64_t tok0, int h, int H, int valid,
                                                      int aux, Lane ln)
{
    typedef C128SolveLds<KD, OP, DKS, METHOD, NRHS> LY;
    float raw_s[NRHS][2];  // in flight while the chunk is inverted
    c128_load_scales<NRHS>(raw_s, rhs, tok0, h, H, valid, 16 * ln.q + ln.n);
    v4f D[10], Wc[2][4];
    RhsHalf<OP> x;
    x.init(rhs.r[0], tok0, h, H, valid, ln);
    c128_invert<KD, OP, METHOD, DKS, W, false, NOGATE>(lds, Kc, row_stride, bc, gc, tok_stride, valid, aux, ln, D, Wc, NoHook(), NoHook(), [&]() {
        // X's first column group: requested as soon as the keys' registers are free, in flight during the last 40 tile
        // products of the recursion and while the inverse's tiles are published
        __builtin_amdgcn_sched_barrier(0);
        if (W < x.n_group()) x.issue(W);
        __builtin_amdgcn_sched_barrier(0);
    });
    c128_apply<OP, W, NRHS>(lds + LY::TILES, lds + LY::SCALE, D, Wc, raw_s, x, rhs, tok0, h, H, valid, ln);
}

// LDS of the row-split form: one set of tiles and the top 64 rows of one column group of X as operand tiles
// ([tile row][column tile][lane]), both in place of what the recursion kept there.
template <int KD, int OP, int DKS, int METHOD> struct C128SolveRowsLds {
    typedef C128Lds<KD, OP, DKS, METHOD, false> INV;
    static constexpr int TILES = 0;
    static constexpr int XTOP = TileLds<OP>::BYTES;
    static constexpr int END = XTOP + 16 * 64 * 16;
    static constexpr int SCALE = INV::BYTES > END ? INV::BYTES : END;  // 128 floats per wave
    static constexpr int BYTES = SCALE + 2 * 128 * 4;
    static_assert(XTOP % 16 == 0, "16-byte accesses");
};

// One right-hand side split by rows: wave 0 computes the top 64 rows of W from its own rows of X; wave 1 the bottom 64
// from the top rows of X, which wave 0 hands over through LDS, and its own.  Each wave turns the rows it loaded into
// operand tiles once (a byte-permute per register) and wave 0 publishes its tiles as they are; one tile row of W (VEC
// accumulators) is formed at a time.  Both waves read and write whole 256-byte row pieces.
// x: its first column group requested.
template <int OP, int W>
__device__ __forceinline__ void c128_apply_rows(char* tiles_lds, char* xtop_lds, char* scale_lds, v4f (&D)[10], v4f (&Wc)[2][4],
                                                const float (&raw_s)[2], RhsRows<OP> x, Lane ln)
{
    typedef TileLds<OP> TL;
    typedef typename TL::elem elem;
    constexpr int VEC = RhsRows<OP>::VEC;
    c128_unit_diagonal<W>(D, ln);
    elem* tiles = reinterpret_cast<elem*>(tiles_lds);
    Opnd<OP>* xtop = reinterpret_cast<Opnd<OP>*>(xtop_lds) + (16 * ln.q + ln.n);  // tile (j, c) at [(VEC j + c) * 64]
    __syncthreads();  // nobody reads what the recursion kept where the tiles and the rows go
    {
        float s_n[8];
        v4f s_q[4];
        c128_scale_patterns(reinterpret_cast<float*>(scale_lds) + 128 * W, raw_s, s_n, s_q, ln);
        c128_publish_tiles<OP, W>(tiles, D, Wc, s_n, s_q, ln);
    }
    const int n_group = x.n_group();
#pragma unroll 1
    for (int gi = 0; gi < n_group; ++gi) {
        Opnd<OP> xo[4][VEC];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                xo[j][c] = xrow_operand<OP>(x.raw[j], c);
                if (W == 0) xtop[(VEC * j + c) * 64] = xo[j][c];
            }
        __syncthreads();  // the tiles (first group) and the top rows are in LDS
        int hide = 0;
        asm volatile("" : "+v"(hide));  // keeps the tile reads inside the loop (an offset: the pointer stays an LDS pointer)
        const elem* set = tiles + hide;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int I = 4 * W + i;
            v4f acc[VEC];
#pragma unroll
            for (int c = 0; c < VEC; ++c) acc[c] = zero4();
            if (W == 1) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const Opnd<OP> t = TL::read_t(set + tix(I, j) * TL::TILE_ELEMS, ln);
#pragma unroll
                    for (int c = 0; c < VEC; ++c) acc[c] = tn<OP>(t, xtop[(VEC * j + c) * 64 + hide], acc[c]);
                }
            }
#pragma unroll
            for (int j = 0; j <= i; ++j) {
                const Opnd<OP> t = TL::read_t(set + tix(I, 4 * W + j) * TL::TILE_ELEMS, ln);
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = tn<OP>(t, xo[j][c], acc[c]);
            }
            x.store(gi, I, acc);
            __builtin_amdgcn_sched_barrier(0);  // one tile row's reads at a time
        }
        if (gi + 1 < n_group) {  // (d_x beyond one group only)
            __syncthreads();     // wave 1 is done with the top rows
            x.template issue<W>(gi + 1);
        }
    }
}

template <int KD, int OP, int METHOD, int DKS, int W, bool NOGATE>
__device__ __forceinline__ void c128_invert_and_apply_rows(char* lds, const void* Kc, int64_t row_stride, const float* bc, const float* gc,
                                                           int64_t tok_stride, const RhsList& rhs, int64_t tok0, int h, int H, int valid,
                                                           int aux, Lane ln)
{
    typedef C128SolveRowsLds<KD, OP, DKS, METHOD> LY;
    float raw_s[1][2];  // in flight while the chunk is inverted
    c128_load_scales<1>(raw_s, rhs, tok0, h, H, valid, 16 * ln.q + ln.n);
    v4f D[10], Wc[2][4];
    RhsRows<OP> x;
    x.init(rhs.r[0], tok0, h, H, valid, ln);
    c128_invert<KD, OP, METHOD, DKS, W, false, NOGATE>(lds, Kc, row_stride, bc, gc, tok_stride, valid, aux, ln, D, Wc, NoHook(), NoHook(), [&]() {
        // this wave's rows of X: requested as soon as the keys' registers are free
        __builtin_amdgcn_sched_barrier(0);
        x.template issue<W>(0);
        __builtin_amdgcn_sched_barrier(0);
    });
    c128_apply_rows<OP, W>(lds + LY::TILES, lds + LY::XTOP, lds + LY::SCALE, D, Wc, raw_s[0], x, ln);
}

// Fused kernel, scalar / no-gate kinds, C = 128: blocked or mixed recursion, then the inverse applied to one right-hand side
// split by rows (c128_apply_rows).  One workgroup of two wavefronts per chunk matrix.
template <int KD, int OP, int METHOD, int DKS, bool NOGATE>
__global__ __launch_bounds__(128) void k_gdn_tri_solve_c128_rows(const void* __restrict__ K, const float* __restrict__ beta,
                                                                 const float* __restrict__ g, RhsList rhs, int64_t n_chunk, ChunkMap map,
                                                                 int H, int d_k, int aux)
{
    constexpr int C = 128;
    __shared__ __attribute__((aligned(16))) char lds[C128SolveRowsLds<KD, OP, DKS, METHOD>::BYTES];
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
    if (w == 0)
        c128_invert_and_apply_rows<KD, OP, METHOD, DKS, 0, NOGATE>(lds, Kc, (int64_t)H * d_k, bcp, gcp, H, rhs, tok0, h, H, pos.valid, aux, ln);
    else
        c128_invert_and_apply_rows<KD, OP, METHOD, DKS, 1, NOGATE>(lds, Kc, (int64_t)H * d_k, bcp, gcp, H, rhs, tok0, h, H, pos.valid, aux, ln);
}

// Fused kernel, scalar / no-gate kinds, C = 128, d_k = 64 or 128: blocked or mixed recursion, then the inverse applied to
// one or two right-hand sides.  One workgroup of two wavefronts per chunk matrix.
template <int KD, int OP, int METHOD, int DKS, int NRHS, bool NOGATE>
__global__ __launch_bounds__(128) void k_gdn_tri_solve_c128(const void* __restrict__ K, const float* __restrict__ beta,
                                                            const float* __restrict__ g, RhsList rhs, int64_t n_chunk, ChunkMap map,
                                                            int H, int d_k, int aux)
{
    constexpr int C = 128;
    __shared__ __attribute__((aligned(16))) char lds[C128SolveLds<KD, OP, DKS, METHOD, NRHS>::BYTES];
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
    if (w == 0)
        c128_invert_and_apply<KD, OP, METHOD, DKS, 0, NRHS, NOGATE>(lds, Kc, (int64_t)H * d_k, bcp, gcp, H, rhs, tok0, h, H, pos.valid, aux, ln);
    else
        c128_invert_and_apply<KD, OP, METHOD, DKS, 1, NRHS, NOGATE>(lds, Kc, (int64_t)H * d_k, bcp, gcp, H, rhs, tok0, h, H, pos.valid, aux, ln);
}

}  // namespace triinv
