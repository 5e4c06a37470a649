// Constants shared by the host-side layout builder and the gather kernels.
#pragma once

namespace pcg {

constexpr int kGatherThreads = 1024;     // one workgroup per compute unit (LDS-bound)
constexpr int kGatherWaves = kGatherThreads / 64;
constexpr int kTileMax = 40704;          // floats of LDS a workgroup stages (159 of the 160 KiB)
constexpr int kBanks = 32;               // LDS banks (4 bytes wide); a half-wave of 32 lanes is
                                         // served in one pass when its addresses fall in 32 banks
constexpr int kTileTokensMax = kTileMax - kBanks;   // the last kBanks floats of a tile read as zero
constexpr int kLaneGroups = 4;           // groups a lane handles side by side (one 16-byte load)
constexpr int kBlockGroups = 64 * kLaneGroups;                 // groups per block: 256
constexpr int kMaxBlocksPerWave = 4;     // blocks a wave handles per tile pass
constexpr int kMaxAcc = kLaneGroups * kMaxBlocksPerWave;       // running sums per lane: 16
constexpr int kChunkStep = kGatherWaves * kBlockGroups;        // 4096 groups: one block per wave
constexpr int kMaxChunkGroups = kMaxBlocksPerWave * kChunkStep;   // 16384 groups per workgroup
constexpr int kRunGroups = 16;           // consecutive groups whose clamped sums the gather adds up into one run sum

// Block of a chunk that wave w handles in its q-th turn.  Blocks are sorted by list length, so
// alternating the direction evens out the work of the waves.
__host__ __device__ inline int block_of(int q, int w) {
  return q * kGatherWaves + ((q & 1) ? kGatherWaves - 1 - w : w);
}

}  // namespace pcg
