// Per-channel gate at C = 128 with the inverse applied instead of stored: the two-wavefront recursion of
// c128_kda.hpp, then the apply stage of c128_solve.hpp (W = T diag(s) X, paper Sec. 3.5 / Eq. 3 with the
// KDA gate of Table 1).
#pragma once
#include "c128_kda.hpp"
#include "c128_solve.hpp"

namespace triinv {

template <int OP, int METHOD, int NRHS> struct C128KdaSolveLds {
    typedef C128KdaLds<OP, METHOD> INV;
    static constexpr int TILES = 0;  // after the recursion, in place of everything it kept: one set of 36 tiles per right-hand side
    static constexpr bool BY_ROWS = NRHS == 1;  // one right-hand side: split by rows (c128_apply_rows)
    static constexpr int XTOP = TileLds<OP>::BYTES;
    static constexpr int APPLY = BY_ROWS ? XTOP + 16 * 64 * 16 : NRHS * TileLds<OP>::BYTES;
    static constexpr int SCALE = INV::BYTES > APPLY ? INV::BYTES : APPLY;  // 128 floats per wave
    static constexpr int BYTES = SCALE + 2 * 128 * 4;
};

// The recursion needs nearly the whole register file, so the right-hand side's first loads and the row scales are
// requested after it, not during it as in the scalar-gate kernel.
template <int OP, int METHOD, int W, int NRHS>
__device__ __forceinline__ void c128_kda_invert_and_apply(char* lds, const void* Kc, int kd, const float* gc, int64_t row_stride,
                                                          const float* bc, int64_t tok_stride, int d_k, const RhsList& rhs,
                                                          int64_t tok0, int h, int H, int valid, int aux, Lane ln)
{
    typedef C128KdaSolveLds<OP, METHOD, NRHS> LY;
    v4f D[10], Wc[2][4];
    c128_kda_invert<OP, METHOD, W>(lds, Kc, kd, gc, row_stride, bc, tok_stride, d_k, valid, aux, ln, D, Wc);
    float raw_s[NRHS][2];
    c128_load_scales<NRHS>(raw_s, rhs, tok0, h, H, valid, 16 * ln.q + ln.n);
    if constexpr (LY::BY_ROWS) {
        RhsRows<OP> x;
        x.init(rhs.r[0], tok0, h, H, valid, ln);
        x.template issue<W>(0);
        c128_apply_rows<OP, W>(lds + LY::TILES, lds + LY::XTOP, lds + LY::SCALE, D, Wc, raw_s[0], x, ln);
    } else {
        RhsHalf<OP> x;
        x.init(rhs.r[0], tok0, h, H, valid, ln);
        if (W < x.n_group()) x.issue(W);
        c128_apply<OP, W, NRHS>(lds + LY::TILES, lds + LY::SCALE, D, Wc, raw_s, x, rhs, tok0, h, H, valid, ln);
    }
}

// Fused kernel, per-channel gate, C = 128, any d_k (multiple of 32): blocked or mixed recursion, then the inverse applied
// to one or two right-hand sides.  One workgroup of two wavefronts per chunk matrix.
template <int OP, int METHOD, int NRHS>
__global__ __launch_bounds__(128) void k_kda_tri_solve_c128(const void* __restrict__ K, const float* __restrict__ beta,
                                                            const float* __restrict__ g, RhsList rhs, int64_t n_chunk, ChunkMap map,
                                                            int H, int d_k, int k_dt, int aux)
{
    constexpr int C = 128;
    __shared__ __attribute__((aligned(16))) char lds[C128KdaSolveLds<OP, METHOD, NRHS>::BYTES];
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
    if (w == 0)
        c128_kda_invert_and_apply<OP, METHOD, 0, NRHS>(lds, Kc, k_dt, g + e0, (int64_t)H * d_k, beta + tok0 * H + h, H, d_k, rhs, tok0, h,
                                                       H, pos.valid, aux, ln);
    else
        c128_kda_invert_and_apply<OP, METHOD, 1, NRHS>(lds, Kc, k_dt, g + e0, (int64_t)H * d_k, beta + tok0 * H + h, H, d_k, rhs, tok0, h,
                                                       H, pos.valid, aux, ln);
}

}  // namespace triinv
