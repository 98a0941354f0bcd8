// One-directional passes over the switch's own tile table: every W_base tile read and
// discarded, or every W_work tile written with zeros.  Same workgroup per tile, same
// 16-byte pieces and the same row pieces as the switch and its copy, so the two rates
// bracket what a read-plus-write pass over these tiles can reach: a pass that moves N
// bytes each way cannot take less than N / read_rate + N / write_rate unless the two
// directions overlap in the memory system.  Measurement aid, not a step of the method.
#pragma once
#include "device_types.hpp"

namespace adafuse {

// PT pieces of 16 bytes per thread: tile_rows * tile_cols / 8 / 256
template <int PT, bool WRITE>
__global__ __launch_bounds__(256) void hbm_probe_kernel(const TileDev *tiles, int tile_cols, uint32_t *sink)
{
    const TileDev tile = tiles[blockIdx.x];
    const int ppr = tile_cols / 8;  // pieces per tile row
    uint4_t v[PT];
    uint32_t x = 0;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
        const int q = threadIdx.x + 256 * i;
        const int row = q / ppr, col = 8 * (q % ppr);
        const bool ok = row < tile.rows_left && col < tile.cols_left;
        const size_t off = (size_t)row * tile.ldw + col;
        if constexpr (WRITE) {
            if (ok) st_global_nt(uint4_t{0u, 0u, 0u, 0u}, reinterpret_cast<uint4_t *>(tile.w_dst + off));
        } else {
            v[i] = uint4_t{0u, 0u, 0u, 0u};
            if (ok) v[i] = ld_global_nt(reinterpret_cast<const uint4_t *>(tile.w_src + off));
        }
    }
    if constexpr (!WRITE) {
#pragma unroll
        for (int i = 0; i < PT; ++i) x ^= v[i][0] ^ v[i][1] ^ v[i][2] ^ v[i][3];
        // keeps the loads alive; a tile whose words cancel to this pattern writes one word, which nobody reads
        if (x == 0x9e3779b9u) sink[0] = x;
    }
}

}  // namespace adafuse
