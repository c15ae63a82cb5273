// Host-side check of the workgroup-id -> tile mapping used by the token loss's matrix-core kernels
// (paper_2504_13818_amd/csrc/tile_map.h, compiled here for the CPU): for an n0 x n1 tile grid, the ids
// 0 .. super_grid_blocks(n0, n1) - 1 must name every tile exactly once and nothing outside the grid.
#include <cstddef>
#include <cstdint>
#include <vector>

#include "tile_map.h"

extern "C" {

// 0 if the mapping of an n0 x n1 grid is a bijection onto the tiles; otherwise a code:
// 1 = an id accepted with coordinates outside the grid, 2 = a tile named twice, 3 = a tile never named,
// 4 = the grid is not a whole number of rounds over the XCDs.
// `grid` is the number of ids enumerated (the launch size); tile_map_check_one passes the mapping's own.
int tile_map_check_ids(int64_t n0, int64_t n1, int64_t grid) {
    if (grid % pods::kXcds != 0) return 4;
    std::vector<unsigned char> seen((std::size_t)(n0 * n1), 0);
    for (int64_t bid = 0; bid < grid; ++bid) {
        int64_t t0 = -1, t1 = -1;
        if (!pods::decode_tile(bid, n0, n1, t0, t1)) continue;
        if (t0 < 0 || t0 >= n0 || t1 < 0 || t1 >= n1) return 1;
        if (seen[(std::size_t)(t0 * n1 + t1)]++) return 2;
    }
    for (unsigned char s : seen)
        if (s != 1) return 3;
    return 0;
}

int tile_map_check_one(int64_t n0, int64_t n1) {
    return tile_map_check_ids(n0, n1, pods::super_grid_blocks(n0, n1));
}

// Sweeps n0 in [n0_lo, n0_hi] (step n0_step) x n1 in [1, n1_hi]; returns the number of failing grids
// and writes the first failing (n0, n1, code) to first[3].
int64_t tile_map_check_range(int64_t n0_lo, int64_t n0_hi, int64_t n0_step, int64_t n1_hi, int64_t* first) {
    int64_t bad = 0;
#pragma omp parallel for schedule(dynamic) reduction(+ : bad)
    for (int64_t n0 = n0_lo; n0 <= n0_hi; n0 += n0_step)
        for (int64_t n1 = 1; n1 <= n1_hi; ++n1) {
            const int code = tile_map_check_one(n0, n1);
            if (code != 0) {
#pragma omp critical
                if (bad == 0 && first[2] == 0) { first[0] = n0; first[1] = n1; first[2] = code; }
                ++bad;
            }
        }
    return bad;
}

// The strip mapping of d_w_lm: ids 0 .. strip_grid_blocks - 1 name every tile exactly once; additionally the
// 32 ids an XCD gets in one round (ids r*256 + x, x congruent mod 8) must span at most two strips and 16
// operand columns on the two axes together (for n1 >= 8), which is what the mapping is for.
int strip_map_check_one(int64_t n0, int64_t n1) {
    const int64_t grid = pods::strip_grid_blocks(n0, n1);
    if (grid % pods::kRoundWorkgroups != 0 && grid % pods::kXcds != 0) return 4;
    std::vector<unsigned char> seen((std::size_t)(n0 * n1), 0);
    for (int64_t bid = 0; bid < grid; ++bid) {
        int64_t t0 = -1, t1 = -1;
        if (!pods::decode_strip_tile(bid, n0, n1, t0, t1)) continue;
        if (t0 < 0 || t0 >= n0 || t1 < 0 || t1 >= n1) return 1;
        if (seen[(std::size_t)(t0 * n1 + t1)]++) return 2;
    }
    for (unsigned char s : seen)
        if (s != 1) return 3;
    for (int64_t r0 = 0; r0 < grid; r0 += pods::kRoundWorkgroups)
        for (int64_t x = 0; x < pods::kXcds; ++x) {
            std::vector<int64_t> c0, c1;
            for (int64_t i = x; i < pods::kRoundWorkgroups && r0 + i < grid; i += pods::kXcds) {
                int64_t t0, t1;
                if (!pods::decode_strip_tile(r0 + i, n0, n1, t0, t1)) continue;
                bool f0 = false, f1 = false;
                for (int64_t v : c0) f0 |= v == t0;
                for (int64_t v : c1) f1 |= v == t1;
                if (!f0) c0.push_back(t0);
                if (!f1) c1.push_back(t1);
            }
            // n1 >= 8: at most two strips, 16 columns in all; narrower grids: the strips 32 workgroups fill
            const std::size_t strips = n1 >= 8 ? 2 : (std::size_t)((32 + 4 * n1 - 1) / (4 * n1) + 1);
            if (c0.size() > 4 * strips || (n1 >= 8 && c0.size() + c1.size() > 16) || c1.size() > (std::size_t)n1) return 5;
        }
    return 0;
}

int64_t strip_map_check_range(int64_t n0_lo, int64_t n0_hi, int64_t n0_step, int64_t n1_hi, int64_t* first) {
    int64_t bad = 0;
#pragma omp parallel for schedule(dynamic) reduction(+ : bad)
    for (int64_t n0 = n0_lo; n0 <= n0_hi; n0 += n0_step)
        for (int64_t n1 = 1; n1 <= n1_hi; ++n1) {
            const int code = strip_map_check_one(n0, n1);
            if (code != 0) {
#pragma omp critical
                if (bad == 0 && first[2] == 0) { first[0] = n0; first[1] = n1; first[2] = code; }
                ++bad;
            }
        }
    return bad;
}
int strip_map_used(int64_t n0) { return pods::use_strips(n0) ? 1 : 0; }

int64_t tile_map_blocks(int64_t n0, int64_t n1) { return pods::super_blocks(n0, n1); }
int64_t tile_map_few_blocks(void) { return pods::kFewBlocks; }
int64_t tile_map_grid(int64_t n0, int64_t n1) { return pods::super_grid_blocks(n0, n1); }

}  // extern "C"
