// Compile-time constants shared by the host format builder, the launchers and the device code
// (which is also compiled at run time, so nothing here may need a host header).
#pragma once

namespace spmv {

// Lanes of a wavefront on CDNA4.  The paper's "warp" (32 lanes, Section IV-A) maps to this.
constexpr int kWave = 64;
// Blocked SELL with an LDS x window: slices per workgroup, and the LDS budget of a window.
constexpr int kXwinGroup = 32;
constexpr long long kXwinMaxBytes = 160 * 1024;
// Rows per workgroup of the striped parts' reduce launch (their sums live in LDS).
constexpr int kReduceBlockRows = 1024;
// Wavefront-bitmap part: steps of 64 entries per wavefront (a tile is 64 * kWbmTileSteps entries).
constexpr int kWbmTileSteps = 8;
// Two-pass part with x windows in LDS: entries per group (the unit of padding and of the reduce
// launch's group list), and the LDS budget of an x window or of a block's accumulators.
constexpr int kXlGroup = 16;
constexpr long long kXlMaxLds = 128 * 1024;

}  // namespace spmv
