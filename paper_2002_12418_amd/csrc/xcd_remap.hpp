// Workgroup order that follows the chip's eight XCDs.
//
// The hardware deals consecutive workgroup ids round-robin to the 8 XCDs of an MI355X, each with an L2 of its own.
// xcd_contiguous turns a workgroup id into a position in the work list such that the workgroups one XCD receives
// cover a contiguous range of that list: neighbours in the list -- tiles that share an operand panel, image rows or
// a tile halo -- then meet in one L2 instead of eight.  `total` is the grid size; the map is a bijection on
// [0, total) for any total.
#pragma once
#include <hip/hip_runtime.h>

namespace mnnconv {

constexpr unsigned kXcds = 8;

__device__ __forceinline__ unsigned xcd_contiguous(unsigned bid, unsigned total)
{
    const unsigned per = total / kXcds, rem = total % kXcds, xcd = bid % kXcds, loc = bid / kXcds;
    return xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
}

}  // namespace mnnconv
