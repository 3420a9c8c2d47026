// Shared declarations of the S3GD-MV HIP library (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "s3gd.h"

namespace s3gd {

typedef uint32_t u32;
typedef uint64_t u64;

// ---- geometry -------------------------------------------------------------------------------
constexpr int kBlock = 256;                 // threads of the streaming kernels (4 waves)
constexpr int kWaves = kBlock / 64;
constexpr int kLoads = 4;                   // 16-byte loads per thread and tile
constexpr int kTile = kBlock * 4 * kLoads;  // 4096 gradient entries per tile
constexpr int kHistBins = 2048;             // first radix digit: key bits [30:20]
constexpr int kHistStages = 6;              // histograms of one encode call: sample (two levels), filter bins, radix select (three levels)
constexpr unsigned kMomTile = 4096;         // coordinates one wave of the momentum sweep owns (the finest vote tiling)
constexpr int kScanBlock = 1024;

// Radix digits of the 31-bit magnitude key, most significant first.
__host__ __device__ constexpr int digit_shift(int level) { return level == 0 ? 20 : (level == 1 ? 10 : 0); }
__host__ __device__ constexpr int digit_bits(int level) { return level == 0 ? 11 : 10; }

// Per-row selection state, device resident.  Every kernel of an encode call reads the state its
// predecessor left (one buffer), advances it by one resolve step where a histogram has been filled
// since (every block on its own, all to the same result) and its first block writes it to the other
// buffer for the successor: no kernel reads a state that is being written.
struct RowState {
  u32 prefix;     // key bits fixed so far (right aligned)
  u32 k_rem;      // rank still sought inside the current prefix, 1-based from the largest
  u32 T;          // K-th largest key: the threshold rho taken at the K-th value (eq. "topk")
                  // (while the sample is resolved: the prefix of the sample key that becomes U)
  u32 q;          // entries with key == T that are selected (lowest indices first); 0 when T == 0
                  // (while the sample is resolved: the rank still sought for U; 0 = there is no U)
  u32 c_gt;       // entries with key > T
  u32 count;      // words the row emits = c_gt + q
  u32 mode;       // kModeGeneral, kModeCandidates, kModeCandWide or kModeCandDone
  u32 L;          // candidate route: every entry with key >= L is a candidate; a multiple of 1024
  u32 U;          // candidate route: a candidate with key >= U is selected whatever the threshold turns out to
                  // be; the others (L <= key < U, the bracket) take part in the radix select.  A multiple of
                  // 1024, or 0x80000000 when no entry is sure
  u32 row_emit;   // the row passes (count, emit) serve the row with a threshold that is already known:
                  // 2 = K = N (threshold 0, count from the scan)
  u32 n_cand;     // candidate route, for diagnostics: candidates the filter pass kept ...
  u32 n_brk;      // ... and those of them inside the bracket
  u32 pad[4];
};
static_assert(sizeof(RowState) == 64, "RowState is one 64-byte line");

// Per-row counters that the blocks of one kernel add to (never rewritten as a whole).
struct RowCounters {
  u32 n_cand;     // candidates the filter pass kept ...
  u32 n_brk;      // ... and those of them inside the bracket (the two are added to as one 64-bit word)
  u32 n_alloc;    // candidate slots handed out (slab allocator / exact reservations) ...
  u32 n_alloc_b;  // ... and, by the filter pass in chunks, bracket slots (reserved together, as one 64-bit word)
  u32 overflow;   // a wave or block found no room for its candidates
  u32 pad[3];
};
static_assert(sizeof(RowCounters) == 32, "RowCounters is half a 64-byte line");
static_assert(offsetof(RowCounters, n_cand) % 8 == 0 && offsetof(RowCounters, n_alloc) % 8 == 0, "the counter pairs are aligned 64-bit words");

constexpr u32 kModeGeneral = 0;     // multi-pass radix select over the whole row
constexpr u32 kModeCandidates = 1;  // sampled bounds, one filter pass, last ten key bits resolved among the bracket's candidates
constexpr u32 kModeCandWide = 2;    // as above, but the bracket is wider than the filter's bins: full radix select among its candidates
constexpr u32 kModeCandDone = 3;    // candidate row whose threshold the filter pass already fixed (every selected entry lies above the bracket)
constexpr u32 kNoUpper = 0x80000000u;  // U when no entry is sure: above every key

constexpr int kWaveTile = 64 * 4 * kLoads;  // 1024 entries: the unit of the candidate route (one wave, no barriers)
constexpr int kChunkTiles = 2;      // wave tiles a wave of the chunked filter pass holds: a block covers 8192 entries
constexpr u32 kSlabMin = 256;       // candidate slots a wave reserves at a time: a multiple of this chosen per call ...
constexpr u32 kSlabMax = 1u << 20;  // ... up to this, from the candidates expected per wave
constexpr int kChain = 8;           // segments (slabs) a wave of the filter pass may leave behind
constexpr int kSampleUnit = 16;     // consecutive entries per sample unit (one 64-byte line)
constexpr int kSamplePerBlock = 4096;

// ---- wave / block primitives ----------------------------------------------------------------
__device__ __forceinline__ u32 lane_id() {
  return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}
// number of set bits of a wave ballot below the calling lane
__device__ __forceinline__ u32 ballot_rank(u64 b) {
  return __builtin_amdgcn_mbcnt_hi((u32)(b >> 32), __builtin_amdgcn_mbcnt_lo((u32)b, 0u));
}
__device__ __forceinline__ u64 ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// Orders the LDS accesses of the lanes of one wave: what a lane wrote before is visible to every
// lane after (a wave executes its LDS instructions in order; the fences only bind the compiler).
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T>
__device__ __forceinline__ T wave_incl_scan(T v) {
  const u32 lane = lane_id();
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    T o = __shfl_up(v, d, 64);
    if (lane >= (u32)d) v += o;
  }
  return v;
}

// Exclusive scan over the threads of a block (blockDim.x a multiple of 64, at most 1024).
// `lds` holds at least blockDim.x / 64 entries.  Returns the exclusive prefix; *total = block sum.
template <typename T>
__device__ __forceinline__ T block_excl_scan(T v, T* total, T* lds) {
  const u32 lane = lane_id();
  const u32 wave = threadIdx.x >> 6;
  const u32 nw = blockDim.x >> 6;
  T inc = wave_incl_scan(v);
  if (lane == 63) lds[wave] = inc;
  __syncthreads();
  T base = 0, tot = 0;
  for (u32 w = 0; w < nw; ++w) {
    T s = lds[w];
    if (w < wave) base += s;
    tot += s;
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

// ---- tile of one gradient row in registers ----------------------------------------------------
// A row starts at a 4-byte aligned address.  `a` = number of fp32 slots between the previous
// 16-byte boundary and the row start (0..3).  Tiles are laid over the "virtual" index
// v = n + a, so that every 16-byte load is aligned.  Entry (j, e) of thread t is
// v = tile*kTile + j*1024 + t*4 + e: ascending v is the order (j, wave, lane, e).
struct TileRegs {
  u32 b[kLoads * 4];  // raw fp32 bit patterns
  u32 valid;          // bit (4j+e) set when the entry lies inside the row
};

typedef u32 u32x4 __attribute__((ext_vector_type(4)));
// Streaming 16-byte load: the gradients are read once per pass and never reused, so the load is
// marked non-temporal (measured about 13 % faster than a plain load on a 19 GB stream).
__device__ __forceinline__ uint4 load_stream16(const u32* p) {
  const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(q.x, q.y, q.z, q.w);
}

// Careful path of one 16-byte group that may straddle the ends of the row.
__device__ __forceinline__ void load_edge4(const u32* __restrict__ rowv, u32 a, u64 vend, u64 v, int j, TileRegs& r) {
  if (v >= a && v + 4 <= vend) {
    const uint4 q = load_stream16(rowv + v);
    r.b[4 * j + 0] = q.x; r.b[4 * j + 1] = q.y; r.b[4 * j + 2] = q.z; r.b[4 * j + 3] = q.w;
    r.valid |= 0xFu << (4 * j);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const u64 ve = v + e;
      if (ve >= a && ve < vend) {
        r.b[4 * j + e] = rowv[ve];
        r.valid |= 1u << (4 * j + e);
      } else {
        r.b[4 * j + e] = 0;
      }
    }
  }
}

// Loads `span` entries starting at vbase; thread/lane `t` owns entries vbase + j*span/kLoads + t*4 + e.
// Tiles that lie wholly inside the row (all but the first and last of a row) take a branch-free
// path so that the four loads are in flight together.
template <int SPAN>
__device__ __forceinline__ void load_span(const u32* __restrict__ rowv, u32 a, u64 vend, u64 vbase, u32 t, TileRegs& r) {
  constexpr int STEP = SPAN / kLoads;
  if (vbase >= a && vbase + SPAN <= vend) {  // uniform over the block (SPAN = kTile) or wave (SPAN = kWaveTile)
    uint4 q[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) q[j] = load_stream16(rowv + vbase + (u64)j * STEP + (u64)t * 4);
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      r.b[4 * j + 0] = q[j].x; r.b[4 * j + 1] = q[j].y; r.b[4 * j + 2] = q[j].z; r.b[4 * j + 3] = q[j].w;
    }
    r.valid = 0xFFFFu;
  } else {
    r.valid = 0;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) load_edge4(rowv, a, vend, vbase + (u64)j * STEP + (u64)t * 4, j, r);
  }
}

__device__ __forceinline__ void load_tile(const u32* __restrict__ rowv /* row start minus a slots */,
                                          u32 a, u64 vend /* N + a */, u64 vbase, TileRegs& r) {
  load_span<kTile>(rowv, a, vend, vbase, threadIdx.x, r);
}

// Ranks of flagged entries of a tile in ascending index order.
// mask: bit (4j+e) of this thread's entries.  base[j] = number of flagged entries of the block that
// precede this thread's load j.  *total = flagged entries in the block.  lds: kLoads*kWaves entries.
__device__ __forceinline__ void tile_rank(u32 mask, u32 base[kLoads], u32* total, u32* lds) {
  const u32 wave = threadIdx.x >> 6;
  const u32 lane = lane_id();
  u32 pre[kLoads];
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    const u32 c = __popc((mask >> (4 * j)) & 0xFu);  // 0..4
    const u64 b0 = ballot(c & 1u), b1 = ballot(c & 2u), b2 = ballot(c & 4u);
    pre[j] = ballot_rank(b0) + 2u * ballot_rank(b1) + 4u * ballot_rank(b2);
    if (lane == 0) lds[j * kWaves + wave] = __popcll(b0) + 2u * __popcll(b1) + 4u * __popcll(b2);
  }
  __syncthreads();
  u32 run = 0;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      if ((u32)w == wave) base[j] = run + pre[j];
      run += lds[j * kWaves + w];
    }
  }
  *total = run;
  __syncthreads();
}

}  // namespace s3gd
