// Benchmark utility, not part of the method: data movers with the fused kernels' memory access patterns and
// nothing else, to measure what the memory system gives those patterns (the practical ceiling the real kernels
// are compared with).  Built into libtriinv_probe.so; only bench.py loads it.
//
//   triinv_probe_mover(K, T, n_chunk, H, C, lds_pad_bytes, store_kind, stream)
//     per matrix (chunk, head): reads C rows of 256 bytes (16-bit keys, d_k = 128) at a row stride of H * 256 bytes
//     with the lane -> address map of the Gram operand loads (lane (q, n): row 16 i + n, bytes 64 s + 16 q), and
//     writes C * C * 4 bytes (an fp32 T) as 1 KB-contiguous streaming buffer stores, 16 bytes per lane.
//     C = 64: four wavefronts = four adjacent heads per workgroup, head groups of one chunk on one XCD;
//     C = 128: one wavefront per workgroup; every loaded register is written twice (32 KB in, 64 KB out).
//     lds_pad_bytes: unused dynamic LDS, to set the number of resident workgroups as the real kernels do.
//     store_kind: 0 = raw buffer stores with the sc0 sc1 nt bits (what the library's kernels issue), 1 = global stores with
//     the same bits (inline assembly followed by the wait states a wide store needs before its data registers are rewritten).
//   Returns 0, or -1 for arguments it does not take.  Device pointers; nothing is allocated or synchronised.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
constexpr int CACHE_SC0_SC1_NT = 1 | 2 | 16;  // gfx950 buffer-instruction cache-policy bits: sc0, nt, sc1

__device__ __forceinline__ int64_t head_group_swizzle(int64_t bid, int64_t n_group, int H)
{
    const int64_t full = (n_group / 8) * 8;
    if (bid >= full * H) return bid;
    const int64_t x = bid % 8, q = bid / 8;
    return ((q / H) * 8 + x) * H + (q % H);
}

template <int C, int WPB, int STORE_KIND>
__global__ __launch_bounds__(64 * WPB) void k_mover(const char* __restrict__ K, float* __restrict__ T, int64_t n_chunk, int H)
{
    constexpr int NREG = C / 4;      // 16-byte registers per lane: C rows x 256 B / 64 lanes / 16 B
    constexpr int REP = C / 64;      // output bytes / input bytes
    const int w = (WPB == 1) ? 0 : __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int l = threadIdx.x & 63, q = l >> 4, n = l & 15;
    const int64_t m = head_group_swizzle(blockIdx.x, n_chunk, H / WPB) * WPB + w;  // chunk * H + head
    const int64_t chunk = m / H;
    const int h = (int)(m - chunk * H);
    const char* base = K + (chunk * C * H + h) * 256;
    v4f r[NREG];
#pragma unroll
    for (int k = 0; k < NREG; ++k) {
        const int i = k >> 2, s = k & 3;
        r[k] = *reinterpret_cast<const v4f*>(base + (int64_t)(16 * i + n) * (H * 256) + 64 * s + 16 * q);
    }
    const __amdgpu_buffer_rsrc_t out = __builtin_amdgcn_make_buffer_rsrc(T + m * C * C, 0, C * C * 4, 0x00020000);
    char* const outp = reinterpret_cast<char*>(T + m * C * C);
#pragma unroll
    for (int rep = 0; rep < REP; ++rep)
#pragma unroll
        for (int k = 0; k < NREG; ++k) {
            const int off = ((rep * NREG + k) * 64 + l) * 16;
            if (STORE_KIND == 0)
                __builtin_amdgcn_raw_buffer_store_b128(r[k], out, off, 0, CACHE_SC0_SC1_NT);
            else
                asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 2" : : "v"(outp + off), "v"(r[k]));
        }
}

}  // namespace

template <int STORE_KIND>
static int launch(const char* K, float* T, int64_t n_chunk, int H, int C, unsigned lds_pad_bytes, hipStream_t s)
{
    if (C == 64 && H % 4 == 0) {
        hipLaunchKernelGGL((k_mover<64, 4, STORE_KIND>), dim3((unsigned)(n_chunk * H / 4)), dim3(256), lds_pad_bytes, s, K, T, n_chunk, H);
    } else if (C == 128) {
        hipLaunchKernelGGL((k_mover<128, 1, STORE_KIND>), dim3((unsigned)(n_chunk * H)), dim3(64), lds_pad_bytes, s, K, T, n_chunk, H);
    } else {
        return -1;
    }
    return 0;
}

extern "C" int triinv_probe_mover(const void* K, float* T, int64_t n_chunk, int H, int C, unsigned lds_pad_bytes, int store_kind,
                                  void* hip_stream)
{
    if (!K || !T || n_chunk <= 0 || H <= 0 || n_chunk * H > 0x7fffffffLL || lds_pad_bytes > 160u * 1024u) return -1;
    if (store_kind != 0 && store_kind != 1) return -1;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const char* Kc = static_cast<const char*>(K);
    if ((store_kind == 0 ? launch<0>(Kc, T, n_chunk, H, C, lds_pad_bytes, s) : launch<1>(Kc, T, n_chunk, H, C, lds_pad_bytes, s)) != 0)
        return -1;
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
