// Host build of the chunk map (csrc/chunk_map.hpp) for the CPU tests: plain g++, no GPU.
#include "../../paper_2605_21325_amd/csrc/chunk_map.hpp"

extern "C" void chunk_map_locate(int C, int64_t Tlen_or_total, uint32_t cps, uint32_t n_seq, const int64_t* cu_seqlens,
                                 const int64_t* cu_chunks, uint32_t bc, int64_t* tok0, int* valid)
{
    const triinv::ChunkMap map{Tlen_or_total, cps, n_seq, cu_seqlens, cu_chunks};
    triinv::ChunkPos p;
    switch (C) {
    case 16: p = triinv::locate_chunk<16>(map, bc); break;
    case 32: p = triinv::locate_chunk<32>(map, bc); break;
    case 64: p = triinv::locate_chunk<64>(map, bc); break;
    default: p = triinv::locate_chunk<128>(map, bc); break;
    }
    *tok0 = p.tok0;
    *valid = p.valid;
}
