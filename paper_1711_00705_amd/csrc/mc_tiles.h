// Which tile a workgroup takes.
//
// The hardware hands the workgroups of a launch to the chip's eight accelerator dies (XCDs)
// round-robin: workgroup b runs on die b % 8, and each die has an L2 of its own.  With the plain
// mapping tile = b, neighbouring tiles therefore always sit on different dies, and whatever two
// neighbours share -- the cache line a tile boundary cuts through when a tensor does not start
// on a line boundary, a line of the lookup table -- is fetched from memory once per die.
// xcd_tile() permutes the tiles inside runs of 8 * run workgroups so that each die walks `run`
// consecutive tiles, one after the other in dispatch order; the ragged end of the launch keeps
// the plain mapping.  A permutation of tiles cannot change any result: tiles are independent.
#pragma once

#include <hip/hip_runtime.h>

namespace mc {

constexpr int kXcds = 8;

__host__ __device__ __forceinline__ int xcd_tile(int b, int n_blocks, int run) {
    if (run <= 1) return b;
    const int span = kXcds * run;
    if (b >= n_blocks - n_blocks % span) return b;
    const int r = b % span;
    return b - r + (r % kXcds) * run + r / kXcds;
}

}  // namespace mc
