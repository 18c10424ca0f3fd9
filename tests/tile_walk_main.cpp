// Host check of the workgroup -> tile map of the GEMM launches: for every shape and group size each tile is
// produced by exactly one workgroup of the grid, the grid is a multiple of 8 with at most 7 idle workgroups, and
// while whole bands last the eight XCDs (workgroup id mod 8) are at the same tile column at the same step.
#include <cstdio>
#include <vector>
#include "tile_walk.hpp"

int main()
{
    long shapes = 0;
    const int gms[] = {1, 2, 4, 8, 16}, tns[] = {1, 2, 3, 16, 17, 125, 501};
    for (int gm : gms)
        for (int tm = 1; tm <= 150; ++tm)
            for (int tn : tns) {
                const int grid = gemm_grid(tm, tn, gm);
                if (grid % 8 || grid < tm * tn || grid > tm * tn + 7) {
                    std::printf("grid: gm %d tiles %d x %d -> %d\n", gm, tm, tn, grid);
                    return 1;
                }
                std::vector<int> seen((size_t)tm * tn, 0);
                const TileWalk w = tile_walk(tm, tn, gm);
                for (int j = 0; j < grid / 8; ++j) {
                    int col0 = -1;
                    for (int x = 0; x < 8; ++x) {
                        int a = -1, c = -1;
                        if (!tile_of_block(j * 8 + x, tm, tn, gm, a, c)) continue;
                        if (a < 0 || a >= tm || c < 0 || c >= tn) {
                            std::printf("range: gm %d tiles %d x %d block %d -> (%d, %d)\n", gm, tm, tn, j * 8 + x, a, c);
                            return 1;
                        }
                        ++seen[(size_t)a * tn + c];
                        if (j < w.band_tiles) {
                            if (x == 0) col0 = c;
                            if (c != col0 || a / gm % 8 != x) {
                                std::printf("lockstep: gm %d tiles %d x %d step %d xcd %d -> (%d, %d)\n", gm, tm, tn, j, x, a, c);
                                return 1;
                            }
                        }
                    }
                }
                for (size_t i = 0; i < seen.size(); ++i)
                    if (seen[i] != 1) {
                        std::printf("cover: gm %d tiles %d x %d tile %zu produced %d times\n", gm, tm, tn, i, seen[i]);
                        return 1;
                    }
                ++shapes;
            }
    // the block-by-block layout: a bijection onto [0, rows * ld) for rows a multiple of 256 and ld of 64, 8-column
    // pieces contiguous, and the 256 x 64 block of a tile's K-step contiguous
    for (long ld : {64L, 192L, 1024L})
        for (size_t rows : {(size_t)256, (size_t)768}) {
            std::vector<char> hit(rows * ld, 0);
            for (size_t r = 0; r < rows; ++r)
                for (int c = 0; c < ld; ++c) {
                    const size_t at = blocked64_index(r, c, ld);
                    if (at >= hit.size() || hit[at]) {
                        std::printf("blocked: ld %ld rows %zu (%zu, %d) -> %zu\n", ld, rows, r, c, at);
                        return 1;
                    }
                    hit[at] = 1;
                    if (c % 8 && at != blocked64_index(r, c - 1, ld) + 1) return 1;
                    const size_t block = ((r / 256) * (size_t)(ld / 64) + c / 64) * 16384;
                    if (at < block || at >= block + 16384 || at - block != (r % 256) * 64 + c % 64) return 1;
                }
        }
    std::printf("ok %ld\n", shapes);
    return 0;
}
