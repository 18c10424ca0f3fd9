// Index maps of the GEMM launches (host and device; no HIP dependency, so that they can be checked on the CPU):
// workgroup id -> output tile, and the block-by-block operand layout.
#pragma once
#include <cstddef>
#if !defined(__HIPCC__)
#define CPH_HD inline
#else
#define CPH_HD __host__ __device__ __forceinline__
#endif

// Workgroup id -> output tile.  Consecutive workgroup ids go round-robin over the 8 XCDs: XCD x runs ids x, x+8, ...
// The tile rows are cut into bands of 8*GM rows; within a band XCD x takes rows [x*GM, (x+1)*GM) and walks them
// column by column, so that the tiles in flight on one XCD share GM + 32/GM operand panels in its L2 and all eight
// XCDs sweep the same columns at the same time whatever the number of tile rows is (the B panels, common to all of
// them, then come out of the last-level cache once for the eight; with per-XCD ranges that start at different
// columns a product with a ragged number of tile rows ran 5 % slower).  The rows left after the last whole band are
// dealt as equal contiguous ranges of the same walk.
struct TileWalk {
    int band_tiles;      // tiles one XCD takes from the whole bands
    int rest_first_m;    // first tile row after the whole bands
    int rest_per_xcd;    // tiles one XCD takes from the rest
};
CPH_HD TileWalk tile_walk(int tiles_m, int tiles_n, int GM)
{
    const int bands = tiles_m / (8 * GM);
    const int rest_rows = tiles_m - bands * 8 * GM;
    return {bands * GM * tiles_n, bands * 8 * GM, (rest_rows * tiles_n + 7) / 8};
}
CPH_HD bool tile_of_block(int bid, int tiles_m, int tiles_n, int GM, int &tm, int &tn)
{
    const TileWalk w = tile_walk(tiles_m, tiles_n, GM);
    const int x = bid & 7, j = bid >> 3;
    const int per_group = GM * tiles_n;
    if (j < w.band_tiles) {
        const int band = j / per_group, in = j - band * per_group;
        tm = (band * 8 + x) * GM + in % GM;
        tn = in / GM;
        return true;
    }
    const int lid = x * w.rest_per_xcd + (j - w.band_tiles);
    const int rest_rows = tiles_m - w.rest_first_m;
    if (j - w.band_tiles >= w.rest_per_xcd || lid >= rest_rows * tiles_n) return false;
    const int group = lid / per_group;
    const int first_m = group * GM;
    const int gsize = (rest_rows - first_m < GM ? rest_rows - first_m : GM);
    const int in = lid - group * per_group;
    tm = w.rest_first_m + first_m + in % gsize;
    tn = in / gsize;
    return true;
}
// Workgroups of a launch: a multiple of 8, at most 7 of them without a tile.
inline int gemm_grid(int tiles_m, int tiles_n, int GM)
{
    const TileWalk w = tile_walk(tiles_m, tiles_n, GM);
    return 8 * (w.band_tiles + w.rest_per_xcd);
}

// Element (row, col) of a bf16 matrix stored block by block, [rows / 256][ld / 64][256][64] (ld a multiple of 64, the
// rows allocated up to a multiple of 256): the layout in which the main loop reads an operand flagged ABL / BBL, one
// K-step of a tile being 32 KB of consecutive memory.
CPH_HD size_t blocked64_index(size_t row, int col, long ld)
{
    return ((row >> 8) * (size_t)(ld >> 6) + (size_t)(col >> 6)) * 16384 + (row & 255) * 64 + (size_t)(col & 63);
}
