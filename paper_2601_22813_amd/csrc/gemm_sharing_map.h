// Index arithmetic of the GEMM's shared last round (gemm.hip): the K tiles of the `rem` shared
// output tiles form one tile-major sequence of U = rem * ktotal units that G blocks cut into equal
// contiguous ranges.  Host and device use the same functions (the host side only through the
// library's test aids), so the mapping can be checked on a CPU by brute force.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define QII_HD __host__ __device__
#else
#define QII_HD
#endif

namespace qii {

// number of a block among the G sharing blocks, from its hardware block id: consecutive ids go to
// different XCDs, so each XCD gets a contiguous run of numbers (hence of units and of tiles)
QII_HD inline int sharing_block_number(int block_id, int G)
{
    return (G & 7) == 0 ? (block_id & 7) * (G >> 3) + (block_id >> 3) : block_id;
}

// units [u0, u1) of block number blk
QII_HD inline void sharing_block_units(int64_t U, int G, int blk, int64_t &u0, int64_t &u1)
{
    u0 = U * blk / G;
    u1 = U * (blk + 1) / G;
}

// the block whose range holds unit u: the largest b with floor(U b / G) <= u
QII_HD inline int sharing_block_of_unit(int64_t u, int64_t U, int G)
{
    return (int)(((u + 1) * G - 1) / U);
}

// the piece of [u, u_end) that lies in one tile: shared tile lt, K tiles [kt0, kt0 + ktiles)
QII_HD inline void sharing_segment(int64_t u, int64_t u_end, int ktotal, int &lt, int &kt0, int &ktiles)
{
    lt = (int)(u / ktotal);
    kt0 = (int)(u % ktotal);
    ktiles = (int)(u_end - u) < ktotal - kt0 ? (int)(u_end - u) : ktotal - kt0;
}

// partial-tile slot of block blk's segment in shared tile lt.  Along the unit sequence every new
// segment advances the block, the tile or both, so blk + lt is unique, and the segments of one
// tile occupy consecutive slots in the order of their K ranges.
QII_HD inline int sharing_slot(int blk, int lt) { return blk + lt; }

// launch position of shared tile lt (positions `base` .. `base + rem - 1` follow the full rounds),
// numbered so that the blocks of one XCD work on positions of that XCD's own run of tiles
QII_HD inline int sharing_position(int lt, int rem, int base)
{
    return base + ((rem & 7) == 0 ? (lt % (rem >> 3)) * 8 + lt / (rem >> 3) : lt);
}

}  // namespace qii
