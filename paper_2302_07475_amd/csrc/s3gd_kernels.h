// Host-side view of the scratch memory and the launch functions of each stage.
#pragma once
#include "s3gd_common.h"

namespace s3gd {

constexpr u32 kMaxStreamBlocks = 256 * 16;  // upper bound on the blocks of one streaming launch (256 CUs x 8 resident blocks)

inline u32 encode_tiles(u64 N) { return (u32)((N + 3 + kTile - 1) / kTile); }  // rows may start up to 3 slots late
inline u32 tile_stride(u64 N) { return (encode_tiles(N) + 1 + 3) & ~3u; }
inline u32 wave_tiles(u64 N) { return (u32)((N + 3 + kWaveTile - 1) / kWaveTile); }
inline u32 blk_stride(u64 N) { return ((wave_tiles(N) + 15) / 16 + 1 + 3) & ~3u; }  // per-row scratch of the random-K scan
inline u32 wave_stride(u32 gx) { return gx * kWaves + 4; }  // per-row stride of the per-wave tables of a launch with gx blocks per row
// entries of the per-wave tables: gx * M <= max(resident blocks, M) for every launch
// segment lists a row has after a filter pass in chunks: kChain chunks of kWaves * kChunkTiles wave tiles each
inline u32 chunk_count(u64 N) { return (u32)(((N + 3 + kWaveTile - 1) / kWaveTile + kWaves * kChunkTiles - 1) / (kWaves * kChunkTiles)); }
inline u32 chunk_lists(u64 N) { return (chunk_count(N) + kChain - 1) / kChain; }
// entries of the per-list tables: enough for the persistent filter pass (a list per wave) and for the chunked one
inline size_t wave_table_entries(u32 M_max, u64 N_max) {
  const size_t waves = (size_t)(kMaxStreamBlocks + M_max) * kWaves + 4 * (size_t)M_max;
  const size_t lists = (size_t)M_max * ((size_t)chunk_lists(N_max) + 4);
  return waves > lists ? waves : lists;
}
inline u32 coding_blk_stride(u64 N) { return 2 * tile_stride(N); }  // u32 entries per row when tile_cnt serves the coding kernels
// entries per row of the segment table: one per tile of the finest tiling, plus the end
inline size_t seg_row_entries(u64 N) { return (size_t)((N + kMomTile - 1) / kMomTile) + 1; }

// Kernel ids for the optional per-kernel timing (HIP events on the caller's stream).
enum KernelId : int {
  KID_ENCODE_INIT = 0,
  KID_HIST0, KID_HIST1, KID_HIST2, KID_RESOLVE, KID_TILE_COUNT, KID_SCAN_TILES, KID_EMIT,
  KID_SAMPLE, KID_FILTER, KID_CAND_SELECT, KID_CAND_EMIT,
  KID_SEG_BOUNDS, KID_VOTE_DENSE, KID_VOTE_SPARSE, KID_UPDATE,
  KID_COMPENSATE, KID_FILTER_MEM, KID_VOTE_MOMENTUM, KID_UPDATE_MOMENTUM,
  KID_PACK, KID_UNPACK, KID_VOTES_TO_MESSAGE, KID_RANDK,
  KID_PLAIN_READ, KID_PLAIN_RMW,
  KID_COUNT
};

// Records a start/stop event pair around a launch when profiling is on.
struct Profiler {
  static constexpr int kPairs = 4096;
  int mode = 0;  // 0 off, 1 every kernel, 2 only the selection pass over the gradients (two events per step: each is a packet of its own and idles the stream for about 4 us; launching the pass with its events attached to its dispatch, hipExtLaunchKernelGGL, cost the same)
  bool open = false;
  int used = 0;
  hipEvent_t* ev = nullptr;  // 2 * kPairs events, created when profiling is first enabled
  int kid[kPairs];
  void begin(int k, hipStream_t s) {
    open = mode != 0 && used < kPairs && (mode == 1 || k == KID_FILTER || k == KID_FILTER_MEM || k == KID_RANDK || k == KID_PLAIN_READ || k == KID_PLAIN_RMW);
    if (open) { kid[used] = k; (void)hipEventRecord(ev[2 * used], s); }
  }
  void end(hipStream_t s) {
    if (open) { (void)hipEventRecord(ev[2 * used + 1], s); ++used; open = false; }
  }
};

// bits of status[3], set by the coding kernels
constexpr u32 kCodingFormat = 1;    // a packed vector did not decode (bad header, too many ones, index >= N)
constexpr u32 kCodingCapacity = 2;  // an output buffer was too small for the vector

struct Workspace {
  Profiler* prof;
  RowState* rs;   // [2][M_max]  the two state buffers the kernels of a call alternate between; the final state ends in the first
  RowCounters* rc;  // [M]
  u32* status;    // [8]: 0 = NaN seen, 1 = rows on the general path, 2 = rows of the last encode, 3 = coding flags,
                  //      4 = candidate rows whose radix select ran over all levels, 5 = rows whose words came from the
                  //      row passes with a threshold known beforehand (K = N), 6 = unused, 7 = rows that left the
                  //      candidate route before the filter pass (decided from the sample)
  u32* hist;      // [kHistStages][M][kHistBins]: all zero between calls (the last kernel of a call clears what it used)
  bool hist_dirty;  // the histograms may hold data (scratch shared with other shapes): clear them before the call
  u32 M_max;
  u64* tile_cnt;  // [M][tile_stride]  (the coding kernels use it as u32 block sums)
  u32* seg;       // [M][tiles of the launch's tiling + 1], at most seg_row_entries(N) per row
  u64* blk_sum;   // [M][blk_stride]   scratch of the random-K scan
  u64* wave_seg;  // [M][wave_stride][kChain]  candidate route: (first slot << 32) | count of each segment of candidate words
  u64* wave_segb; // [M][wave_stride][kChain]  the same for the segment's bracket records
  u32* wave_nseg; // [M][wave_stride]  candidate route: segments in each list
  u64* wave_sum;  // [M][wave_stride]  candidate route: (ties << 32) | (selected without ties) of each list against the threshold
  char* pool;     // candidate route: the candidate words of all rows, then their bracket records (carved per call);
                  // random-K: (word, arrival number) records
  u64 pool_bytes;
  u32 stream_blocks;  // blocks of a streaming launch = blocks resident on the device at once (one round, no tail)
  u32 stream_blocks_mem;  // the same for the filter pass that also carries the error-compensation memory
};

// What one encode call launches; a pure function of the shapes and the pool size.
struct EncodePlan {
  bool candidates;   // try the candidate route first
  bool chunks;       // the filter pass runs in chunks (one block each, in index order) instead of persistent waves
  bool zero_sure;    // that pass stores +0.0 over the entries at or above U and keeps their bits beside their words
  u32 n_chunks, n_lists;  // chunked filter pass: blocks per row, segment lists per row
  u32 n_tiles, gx;   // 4096-entry tiles per row, streaming blocks per row
  u32 n_wtiles, tiles_per_wave;  // candidate route: 1024-entry wave tiles per row, and per wave of the filter
  u32 n_units;       // sample units (16 entries each) per row
  u64 unit_stride;   // row entries per sample unit window
  u32 sample_rank;   // rank, among the sample, of the key that becomes the lower bound L
  u32 sample_rank_hi;  // rank of the key that becomes the bracket's upper end U (0: no entry is sure)
  u32 cand_stride;   // candidate word slots per row
  u32 brk_shift;     // a segment of n word slots has room for n >> brk_shift bracket records
  u32 brk_stride;    // bracket record slots per row
  u32 slab;          // candidate slots a wave of the filter pass owns at a time (a multiple of 256)
  double bound;      // upper estimate of the candidates per row, without slab slack
};
EncodePlan plan_encode(u32 M, u64 N, u64 K, u64 pool_bytes, u32 stream_blocks, bool chunks);
u64 sample_unit_position(u32 u, u64 unit_stride);  // first entry of sample unit u of a row (host copy of the kernels' rule)
u32 resident_stream_blocks(int device, bool with_memory);  // from the occupancy of the filter kernel; at most kMaxStreamBlocks
u64 candidate_pool_bytes(u32 M_max, u64 N_max, u64 K_max);

// `nan_flag` (device, nullable): receives 1 if the call saw a NaN, else 0, when its last kernel runs.
hipError_t launch_encode(const Workspace& ws, const float* grads, float* err, float eta, u32 M, u64 N, u64 K, u32* words,
                         u32* counts, hipStream_t s, u32* nan_flag = nullptr);
// Plain non-temporal read of `n` fp32 entries with the filter pass's launch shape: what this memory system gives a read stream.
hipError_t launch_plain_read(const Workspace& ws, const float* buf, u64 n, hipStream_t s);
hipError_t launch_plain_rmw(const Workspace& ws, const float* a, float* b, u64 n, hipStream_t s);
hipError_t launch_vote(const Workspace& ws, const u32* words, const u32* counts, u32 M, u64 N, u64 K, int32_t* tally,
                       int8_t* votes, float* x, float lr, hipStream_t s);
hipError_t launch_update(const Workspace& ws, float* x, const int8_t* votes, float lr, u64 N, hipStream_t s);
u64 packed_row_capacity(u64 N, u64 K);
hipError_t launch_pack(const Workspace& ws, const u32* words, const u32* counts, u32 M, u64 N, u64 K, u32* packed, u64 row_words,
                       hipStream_t s);
hipError_t launch_unpack(const Workspace& ws, const u32* packed, u64 row_words, u32 M, u64 N, u64 K, u32* words, u32* counts,
                         hipStream_t s);
hipError_t launch_votes_to_message(const Workspace& ws, const int8_t* votes, u64 N, u64 cap, u32* words, u32* count, hipStream_t s);
hipError_t launch_randk_encode(const Workspace& ws, const float* grads, u32 M, u64 N, u64 K, u64 seed, u32 t, u32* words,
                               u32* counts, hipStream_t s);
hipError_t launch_vote_momentum(const Workspace& ws, const u32* words, const u32* counts, u32 M, u64 N, u64 K, float* x, float* v,
                                float lr, float mu, hipStream_t s);
hipError_t launch_update_momentum(const Workspace& ws, float* x, float* v, const int8_t* votes, float lr, float mu, u64 N,
                                  hipStream_t s);

}  // namespace s3gd
