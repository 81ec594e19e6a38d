// Assignment of tiles of stored entries to persistent workgroups.  Plain
// integer arithmetic, usable on the host (tests) and on the device.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define SGAP_HOST_DEVICE __host__ __device__ __forceinline__
#else
#define SGAP_HOST_DEVICE inline
#endif

namespace sgap {

// Which tiles a persistent workgroup takes.  The 8 dies (XCDs) of the chip
// have private L2s and receive workgroups round-robin (workgroup b runs on die
// b % 8).  Tiles are therefore handed out in chunks of consecutive tiles:
// chunk c goes to die c % 8, and the workgroups of a die take the tiles of the
// die's chunks in order, round-robin.  A die then works on one or a few
// stretches of neighbouring rows at a time, so a row of the dense operand that
// neighbouring rows of A share is fetched into one L2, not into all eight,
// while every die still receives an even sample of the whole matrix (stretches
// of short or empty rows cost several times more per entry than long rows).
// With fewer than 8 workgroups, a grid that is no multiple of 8, or no more
// tiles than workgroups, plain round-robin over the workgroups is used.
struct TileDeal {
    int64_t tiles;   // tiles of the matrix
    int32_t dies;    // 8 or 1
    int32_t chunk;   // tiles per chunk
    int32_t die;     // this workgroup's die
    int32_t wg;      // this workgroup's number on its die
    int32_t wgs;     // workgroups per die
    int64_t mine;    // tiles this workgroup takes

    // block = this workgroup's number in a grid of `grid` workgroups
    SGAP_HOST_DEVICE TileDeal(int64_t tiles_, uint32_t block, uint32_t grid) : tiles(tiles_)
    {
        // (a grid with a workgroup per tile just takes tile = workgroup)
        dies = (grid >= 8 && grid % 8 == 0 && tiles > grid) ? 8 : 1;
        die = (int32_t)(block % dies);
        wg = (int32_t)(block / dies);
        wgs = (int32_t)(grid / dies);
        // about 16 chunks per die, at most one round of the die's workgroups
        int64_t c = tiles / (dies * 16);
        if (c > wgs) c = wgs;
        if (c < 1) c = 1;
        chunk = (int32_t)c;
        const int64_t full = tiles / chunk, rem = tiles % chunk;
        const int64_t die_tiles = (full / dies + (die < full % dies ? 1 : 0)) * chunk + (die == full % dies ? rem : 0);
        mine = wg < die_tiles ? (die_tiles - wg + wgs - 1) / wgs : 0;
    }
    // global number of this workgroup's j-th tile, j < mine
    SGAP_HOST_DEVICE int64_t tile(int64_t j) const
    {
        const int64_t q = wg + j * wgs;  // q-th tile of this die
        return (die + (int64_t)dies * (q / chunk)) * chunk + q % chunk;
    }
};

}  // namespace sgap
