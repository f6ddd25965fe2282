// Order in which the GEMM grids take their output tiles.
//
// Consecutive block ids go round-robin to the chip's 8 XCDs, each with an L2 of its own, so a tile order decides
// which tiles share an L2 and how evenly the XCDs are loaded.  Two orders, both a pure function of the block id:
//   token-major   XCD x owns the token tiles x, x + 8, ... and walks them eight at a time across the channel tiles
//                 (the eight blocks an XCD starts together share one weight tile; the activation tiles of its eight
//                 token tiles stay in its L2).  Even when there are many token tiles; with few, the XCDs whose
//                 residue classes are empty or short idle.
//   channel-major XCD x owns the channel tiles x, x + 8, ... and runs all token tiles of one before the next (its
//                 blocks share that weight tile).  For few token tiles and many channel tiles.
// The launcher takes the channel-major order when it lowers the largest share of an XCD by a tenth or more.
#pragma once
#include <hip/hip_runtime.h>

namespace svdq {

struct TileGrid {
    int mtiles, ntiles, nmajor;
};

inline TileGrid make_tile_grid(int mtiles, int ntiles) {
    const long long by_m = (long long)((mtiles + 7) / 8) * ntiles;       // blocks of the busiest XCD, token-major
    const long long by_n = (long long)((ntiles + 7) / 8) * mtiles;       // channel-major
    return TileGrid{mtiles, ntiles, by_n * 10 <= by_m * 9 ? 1 : 0};
}

// number of block ids (some of them name no tile: tile_of returns false)
__host__ __device__ inline int tile_ids(const TileGrid& g) {
    return g.nmajor ? ((g.ntiles + 7) / 8) * 8 * g.mtiles : ((g.mtiles + 63) / 64) * 64 * g.ntiles;
}

__device__ __forceinline__ bool tile_of(const TileGrid& g, int id, int& mt, int& nt) {
    const int xcd = id & 7, idx = id >> 3;
    if (g.nmajor) {
        const int q = idx / g.mtiles;
        nt = q * 8 + xcd;
        mt = idx - q * g.mtiles;
        return nt < g.ntiles;
    }
    const int sm = idx / (8 * g.ntiles), rem = idx - sm * (8 * g.ntiles);
    nt = rem >> 3;
    mt = (sm * 8 + (rem & 7)) * 8 + xcd;
    return mt < g.mtiles;
}

}  // namespace svdq
