// Where the tokens of a chunk sit (paper Sec. 1: a sequence of L tokens is cut into ceil(L / C)
// chunks of at most C tokens).  Two layouts:
//   fixed   B sequences of Tlen tokens each, token t of sequence b at row b * Tlen + t;
//           chunk id bc = b * cps + k, cps = ceil(Tlen / C);
//   varlen  sequences packed back to back; cu_seqlens[s] = first token row of sequence s,
//           cu_chunks[s] = id of its first chunk (both device arrays of n_seq + 1 entries).
// A last chunk with fewer than C tokens is treated as padded with tokens whose key and beta are
// zero: the padded rows and columns of A vanish and T has identity rows and columns there.
#pragma once
#include <stdint.h>
#ifdef __HIPCC__
#include <hip/hip_runtime.h>
#define TRIINV_HOST_DEVICE __host__ __device__ __forceinline__
#else
#define TRIINV_HOST_DEVICE inline  // plain C++: the map is host-testable
#endif

namespace triinv {

struct ChunkMap {
    int64_t Tlen;               // fixed layout: tokens per sequence; varlen: total number of tokens
    uint32_t cps;               // fixed layout: chunks per sequence
    uint32_t n_seq;             // varlen: number of sequences
    const int64_t* cu_seqlens;  // varlen (device), else null
    const int64_t* cu_chunks;   // varlen (device), else null
};

struct ChunkPos {
    int64_t tok0;  // row of the chunk's first token
    int valid;     // its number of tokens, 1..C
};

// The offset arrays of the varlen layout are trusted but not believed: whatever they hold (a chunk id at or beyond
// cu_chunks[n_seq], offsets that disagree with each other, trailing empty sequences), the returned first token lies
// inside [first token of the sequence found, its last token] and inside [0, total tokens - 1], and valid >= 1, so every
// row a kernel reads afterwards (tok0 .. tok0 + valid - 1) is a row of the caller's buffers.
template <int C> TRIINV_HOST_DEVICE ChunkPos locate_chunk(const ChunkMap& map, uint32_t bc)
{
    ChunkPos p;
    int64_t left;
    if (map.cu_seqlens == nullptr) {
        const uint32_t s = bc / map.cps, k = bc - s * map.cps;
        p.tok0 = (int64_t)s * map.Tlen + (int64_t)k * C;
        left = map.Tlen - (int64_t)k * C;
    } else {
        // the sequence s with cu_chunks[s] <= bc < cu_chunks[s + 1]; at most 32 halvings
        uint32_t lo = 0, hi = map.n_seq;
        for (int it = 0; it < 32 && hi - lo > 1; ++it) {
            const uint32_t mid = lo + (hi - lo) / 2;
            if (map.cu_chunks[mid] <= (int64_t)bc) lo = mid; else hi = mid;
        }
        const int64_t total = map.Tlen;
        int64_t first = map.cu_seqlens[lo], end = map.cu_seqlens[lo + 1];  // tokens [first, end) of the sequence
        if (end > total) end = total;
        if (first > end - 1) first = end - 1;
        if (first < 0) first = 0;
        int64_t tok0 = first + ((int64_t)bc - map.cu_chunks[lo]) * C;
        if (tok0 > end - 1) tok0 = end - 1;
        if (tok0 < first) tok0 = first;
        p.tok0 = tok0;
        left = end - tok0;
    }
    p.valid = left >= C ? C : (left < 1 ? 1 : (int)left);
    return p;
}

}  // namespace triinv
