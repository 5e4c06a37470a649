// Constants shared by the host-side layout builder and the gather kernels.
#pragma once

namespace pcg {

constexpr int kGatherThreads = 1024;     // one workgroup per compute unit (LDS-bound)
constexpr int kTileMax = 40704;          // floats of LDS a workgroup stages (159 of the 160 KiB)
constexpr int kMaxRounds = 16;           // slices a wave handles per tile pass
constexpr int kMaxChunkGroups = kMaxRounds * kGatherThreads;   // 16384 groups per workgroup

}  // namespace pcg
