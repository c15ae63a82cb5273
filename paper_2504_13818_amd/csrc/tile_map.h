// Workgroup id -> output tile of the matrix-core kernels of the token loss.  Pure integer code, shared
// by the kernels (device), the launch sizing (host) and a host-side exhaustive check that every tile of
// a grid is taken by exactly one workgroup id.
#pragma once

#include <cstdint>

#if defined(__HIPCC__)
#define PODS_HOST_DEVICE __host__ __device__
#else
#define PODS_HOST_DEVICE
#endif

namespace pods {

constexpr int kXcds = 8;                           // XCDs (one L2 each); workgroup ids go round them
constexpr int kSuper0 = 4, kSuper1 = 8;            // tiles per XCD block along the two tile axes (at most)

// Workgroup id -> tile (t0, t1) of an n0 x n1 tile grid, so that ids congruent mod 8 (one XCD)
// walk blocks of 4 x s1 tiles (the 32 workgroups resident on an XCD then share operand rows in its L2).  s1 divides the second axis as evenly as blocks of at most 8 can
// (14 tiles -> 7 + 7, not 8 + 6): with an even number of unequal block columns the short column would
// always fall to the same XCDs, which then run out of work early.  Returns false for ids that fall
// outside the grid.
PODS_HOST_DEVICE inline int64_t super_width(int64_t n1) {
    const int64_t cols = (n1 + kSuper1 - 1) / kSuper1;
    return (n1 + cols - 1) / cols;
}
// The caller of decode_tile passes exactly the n0, n1 the launch was sized with (super_grid_blocks): the
// mapping of a launch with few blocks depends on both.
// Blocks go round the XCDs (block b to XCD b mod 8), which keeps the XCDs on neighbouring blocks at any
// time.  A launch with few blocks (d_w_lm: one or two rounds of long tiles) would leave the XCDs
// unevenly loaded that way, so there each XCD takes one contiguous eighth of the slots (tiles, and the
// holes of partial blocks) in block order instead: balanced to within one tile.
constexpr int64_t kFewBlocks = 64;
PODS_HOST_DEVICE inline int64_t super_blocks(int64_t n0, int64_t n1) {
    const int64_t s1 = super_width(n1);
    return ((n0 + kSuper0 - 1) / kSuper0) * ((n1 + s1 - 1) / s1);
}
PODS_HOST_DEVICE inline int64_t super_grid_blocks(int64_t n0, int64_t n1) {
    const int64_t nst = super_blocks(n0, n1), per_block = kSuper0 * super_width(n1);
    if (nst < kFewBlocks) return (nst * per_block + kXcds - 1) / kXcds * kXcds;
    return (nst + kXcds - 1) / kXcds * kXcds * per_block;
}
PODS_HOST_DEVICE inline bool decode_tile(int64_t bid, int64_t n0, int64_t n1, int64_t& t0, int64_t& t1) {
    const int64_t s1 = super_width(n1);
    const int64_t per_block = kSuper0 * s1;
    const int64_t nst1 = (n1 + s1 - 1) / s1;
    const int64_t nst = super_blocks(n0, n1);
    const int64_t xcd = bid % kXcds, q = bid / kXcds;   // workgroup ids go round the XCDs
    int64_t st;
    int w;
    if (nst < kFewBlocks) {
        const int64_t per_xcd = (nst * per_block + kXcds - 1) / kXcds;
        const int64_t seq = xcd * per_xcd + q;
        st = seq / per_block;
        w = (int)(seq % per_block);
    } else {
        st = (q / per_block) * kXcds + xcd;
        w = (int)(q % per_block);
    }
    t0 = (st / nst1) * kSuper0 + w / s1;
    t1 = (st % nst1) * s1 + w % s1;
    return st < nst && t0 < n0 && t1 < n1;
}

// d_w_lm's mapping for tile grids with many tiles on the first axis (the vocabulary): the workgroups of an XCD
// walk strips of 4 x n1 tiles, the first axis fastest inside a strip, strips going round the XCDs.  Any 32
// consecutive workgroups of an XCD then cover 4 x 8 tiles (or the end of one strip and the start of the XCD's
// next) whatever n1 is, and the host launches kRoundWorkgroups ids at a time: one workgroup per compute unit,
// all started together, so that those 32 walk the contraction axis in step and share operand tiles in the L2.
// (Inside one long launch the workgroups of a block start as compute units fall free, drift apart by more than
// the L2 holds, and fetch most operand tiles once each.)
constexpr int64_t kRoundWorkgroups = 256;
PODS_HOST_DEVICE inline bool use_strips(int64_t n0) { return (n0 + kSuper0 - 1) / kSuper0 >= kFewBlocks; }
PODS_HOST_DEVICE inline int64_t strip_grid_blocks(int64_t n0, int64_t n1) {
    const int64_t strips = (n0 + kSuper0 - 1) / kSuper0;
    return (strips + kXcds - 1) / kXcds * kXcds * kSuper0 * n1;
}
PODS_HOST_DEVICE inline bool decode_strip_tile(int64_t bid, int64_t n0, int64_t n1, int64_t& t0, int64_t& t1) {
    const int64_t xcd = bid % kXcds, s = bid / kXcds;   // workgroup ids go round the XCDs
    const int64_t per_strip = kSuper0 * n1;
    const int64_t strip = (s / per_strip) * kXcds + xcd;
    const int64_t w = s % per_strip;
    t0 = strip * kSuper0 + w % kSuper0;
    t1 = w / kSuper0;
    return t0 < n0;
}

}  // namespace pods
