// 16 x 16 register tiles and the one matrix-core primitive everything is built from (gfx950).
//
// A logical 16 x 16 fp32 matrix M lives in 4 VGPRs of one 64-lane wavefront in the accumulator
// layout of the 16x16 MFMA instructions: lane l = 16*q + n (q = l / 16, n = l % 16) holds
//     v[r] = M[4*q + r][n],  r = 0..3.
// The same four registers, narrowed to the operand type, are a valid B operand of M (contraction
// over M's ROW index) and a valid A operand of M^T.  Hence the single primitive
//     tn(X, Y) = X^T * Y          (X, Y, result all in the layout above)
// needs no cross-lane movement between dependent products.  A matrix that must act as a LEFT
// factor is therefore kept transposed ("T orientation": the tile registers hold M^T), a RIGHT
// factor as is ("N orientation").
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace triinv {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

enum : int { OP_F32 = 0, OP_F16 = 1, OP_BF16 = 2 };

struct Lane {
    int q;  // lane / 16 : row group (rows 4q..4q+3 of a tile)
    int n;  // lane % 16 : column of a tile
};

__device__ __forceinline__ Lane lane_id()
{
    int l = __lane_id();
    return Lane{l >> 4, l & 15};
}

// Two fp32 -> two bf16 / fp16 in one register, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack2_bf16(float a, float b)
{
    const v2f f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2bf));
}
__device__ __forceinline__ uint32_t pack2_f16(float a, float b)
{
    const v2f f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2h));
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b)
{
    return __builtin_bit_cast(float, ((uint32_t)b) << 16);
}

__device__ __forceinline__ float f16_to_f32(uint16_t h)
{
    return (float)__builtin_bit_cast(_Float16, h);
}

// Packed matrix-core operand of one tile.
template <int OP> struct Opnd;
template <> struct Opnd<OP_F32> { v4f x; };
template <> struct Opnd<OP_F16> { v4h x; };
template <> struct Opnd<OP_BF16> { v4s x; };

template <int OP> __device__ __forceinline__ Opnd<OP> pack(v4f t);
template <> __device__ __forceinline__ Opnd<OP_F32> pack<OP_F32>(v4f t) { return {t}; }
template <> __device__ __forceinline__ Opnd<OP_F16> pack<OP_F16>(v4f t)
{
    const v2u u = {pack2_f16(t[0], t[1]), pack2_f16(t[2], t[3])};
    return {__builtin_bit_cast(v4h, u)};
}
template <> __device__ __forceinline__ Opnd<OP_BF16> pack<OP_BF16>(v4f t)
{
    const v2u u = {pack2_bf16(t[0], t[1]), pack2_bf16(t[2], t[3])};
    return {__builtin_bit_cast(v4s, u)};
}

// Element masks of one tile as bit patterns on the packed operand: keeping an element is an AND
// with all ones, dropping it an AND with zero (which also kills NaN / Inf).
template <int OP> struct Mask;
template <> struct Mask<OP_F32> { v4u m; };
template <> struct Mask<OP_F16> { v2u m; };
template <> struct Mask<OP_BF16> { v2u m; };

template <int OP> __device__ __forceinline__ Mask<OP> make_mask(bool k0, bool k1, bool k2, bool k3)
{
    Mask<OP> o;
    if constexpr (OP == OP_F32) {
        o.m = v4u{k0 ? ~0u : 0u, k1 ? ~0u : 0u, k2 ? ~0u : 0u, k3 ? ~0u : 0u};
    } else {
        o.m = v2u{(k0 ? 0xffffu : 0u) | (k1 ? 0xffff0000u : 0u), (k2 ? 0xffffu : 0u) | (k3 ? 0xffff0000u : 0u)};
    }
    return o;
}

template <int OP> __device__ __forceinline__ Opnd<OP> masked(Opnd<OP> x, Mask<OP> k)
{
    if constexpr (OP == OP_F32) {
        return {__builtin_bit_cast(v4f, __builtin_bit_cast(v4u, x.x) & k.m)};
    } else {
        Opnd<OP> o;
        o.x = __builtin_bit_cast(decltype(o.x), __builtin_bit_cast(v2u, x.x) & k.m);
        return o;
    }
}

// -x: a sign flip on the packed operand (two instructions for the 16-bit types, half of what negating the fp32 tile costs).
template <int OP> __device__ __forceinline__ Opnd<OP> negated(Opnd<OP> x)
{
    if constexpr (OP == OP_F32) {
        return {-x.x};
    } else {
        Opnd<OP> o;
        o.x = __builtin_bit_cast(decltype(o.x), __builtin_bit_cast(v2u, x.x) ^ v2u{0x80008000u, 0x80008000u});
        return o;
    }
}

// acc + X^T * Y   (x packed from X, y packed from Y)
template <int OP> __device__ __forceinline__ v4f tn(Opnd<OP> x, Opnd<OP> y, v4f acc);
template <> __device__ __forceinline__ v4f tn<OP_F32>(Opnd<OP_F32> x, Opnd<OP_F32> y, v4f acc)
{
    // 16x16x4 fp32: k slot q of step r stands for contraction index 4q + r on both operands
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x[0], y.x[0], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x[1], y.x[1], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x[2], y.x[2], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x[3], y.x[3], acc, 0, 0, 0);
    return acc;
}
template <> __device__ __forceinline__ v4f tn<OP_F16>(Opnd<OP_F16> x, Opnd<OP_F16> y, v4f acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x16f16(x.x, y.x, acc, 0, 0, 0);
}
template <> __device__ __forceinline__ v4f tn<OP_BF16>(Opnd<OP_BF16> x, Opnd<OP_BF16> y, v4f acc)
{
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(x.x, y.x, acc, 0, 0, 0);
}

// acc + sum over k in [lo, hi] of X(k)^T * Y(k); live(k): a wave-uniform run-time test that may drop terms whose tiles
// are known to hold zeros.
template <int OP, class FX, class FY, class Live>
__device__ __forceinline__ v4f tn_sum_if(int lo, int hi, FX x, FY y, Live live, v4f acc)
{
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (k < lo || k > hi) continue;
        if (live(k)) acc = tn<OP>(x(k), y(k), acc);
    }
    return acc;
}
template <int OP, class FX, class FY> __device__ __forceinline__ v4f tn_sum(int lo, int hi, FX x, FY y, v4f acc)
{
    return tn_sum_if<OP>(lo, hi, x, y, [](int) { return true; }, acc);
}

__device__ __forceinline__ v4f zero4() { return v4f{0.f, 0.f, 0.f, 0.f}; }

// Index of lower tile (i, j), i >= j, in a packed array of NB*(NB+1)/2 tiles.
__host__ __device__ constexpr int tix(int i, int j) { return i * (i + 1) / 2 + j; }

}  // namespace triinv
