// Host-side view of the scratch memory and the launch functions of each stage.
#pragma once
#include "s3gd_common.h"

namespace s3gd {

constexpr u32 kTargetBlocks = 256 * 16;  // blocks of a streaming launch: 16 per compute unit

inline u32 encode_tiles(u64 N) { return (u32)((N + 3 + kTile - 1) / kTile); }  // rows may start up to 3 slots late
inline u32 tile_stride(u64 N) { return (encode_tiles(N) + 1 + 3) & ~3u; }
inline u32 vote_tiles(u64 N) { return (u32)((N + kVoteTile - 1) / kVoteTile); }

struct Workspace {
  RowState* rs;   // [M]
  u32* status;    // [4]: 0 = NaN seen, 1 = rows on the general path
  u32* hist;      // [M][kHistBins]
  u64* tile_cnt;  // [M][tile_stride]
  u32* seg;       // [M][vote_tiles + 1]
};

hipError_t launch_encode(const Workspace& ws, const float* grads, u32 M, u64 N, u64 K, u32* words, u32* counts,
                         hipStream_t s);
hipError_t launch_vote(const Workspace& ws, const u32* words, const u32* counts, u32 M, u64 N, u64 K, int32_t* tally,
                       int8_t* votes, float* x, float lr, hipStream_t s);
hipError_t launch_update(float* x, const int8_t* votes, float lr, u64 N, hipStream_t s);

}  // namespace s3gd
