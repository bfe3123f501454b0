// Tile order of the upper triangle of a square matrix of nt x nt tiles, shared by the kernels that compute
// symmetric updates tile by tile (the Hessian's SYRK and the split-operand GEMM).
#pragma once
#include <cstdint>
#include <hip/hip_runtime.h>

namespace gptq {

constexpr int STRIP = 8;        // tile columns per strip

// Tile order of the upper triangle: strips of STRIP tile columns; a strip holds its full rows above the
// diagonal block (STRIP tiles each) and then the rows of the diagonal block, row q with its STRIP - q valid
// tiles.  Only valid tiles are numbered: the order is dealt to the XCDs in equal runs, and every XCD works
// through its run on its own, so runs that contained returned-from tiles would leave some XCDs with up to
// 20 % less work than others (on a 48-tile-row matrix) and the launch waiting for the fullest one.
__host__ __device__ inline int64_t syrk_strip_tiles(int nt, int s) {
    const int cols = (nt - s * STRIP) < STRIP ? (nt - s * STRIP) : STRIP;
    return (int64_t)s * STRIP * cols + (int64_t)cols * (cols + 1) / 2;
}
__host__ inline int64_t syrk_total_tiles(int nt) {
    int64_t total = 0;
    for (int s = 0; s * STRIP < nt; ++s) total += syrk_strip_tiles(nt, s);
    return total;
}
__device__ __forceinline__ void syrk_tile_of(int nt, int64_t L, int& bi, int& bj) {
    int s = 0;
    for (int64_t c = syrk_strip_tiles(nt, 0); L >= c; c = syrk_strip_tiles(nt, s)) { L -= c; ++s; }
    const int cols = min(STRIP, nt - s * STRIP);
    const int64_t above = (int64_t)s * STRIP * cols;
    if (L < above) {
        bi = (int)(L / cols);
        bj = s * STRIP + (int)(L % cols);
    } else {
        int l = (int)(L - above), q = 0;
        for (int c = cols; l >= c; c = cols - q) { l -= c; ++q; }
        bi = s * STRIP + q;
        bj = bi + l;
    }
}
}  // namespace gptq
