// Server side of Algorithm 1: signed tally of the workers' messages per coordinate, its sign
// (sgn(0) = 0 for ties and for coordinates nobody voted on; Section 2.2 "Majority vote") and the
// model update x <- x - lr * vote (eq. "s3gd").
//
// Messages are sorted by index, so each row is cut once into per-tile segments by binary search;
// a block (or, for the dense outputs and the momentum sweep, a wave) then owns a tile of
// consecutive coordinates, tallies them with LDS integer atomics and is the only writer of that
// stretch of the outputs.
#include "s3gd_common.h"
#include "s3gd_kernels.h"

namespace s3gd {

constexpr int kRowChunk = 256;  // rows whose segment bounds sit in LDS at once

// seg[m][t] = first position of row m whose index is >= t * tile_coords (t = 0 .. n_vt).
__global__ void k_seg_bounds(const u32* __restrict__ words, const u32* __restrict__ counts, u64 K, u32 n_vt, u32 seg_stride,
                             u32 tile_coords, u32* __restrict__ seg) {
  const u32 m = blockIdx.y;
  const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t > n_vt) return;
  const u32* w = words + (size_t)m * K;
  const u64 target = ((u64)t * tile_coords) << 1;
  u32 lo = 0, hi = counts[m];
  if ((u64)hi > K) hi = (u32)K;  // a count above the row length is a caller error; stay in bounds
  while (lo < hi) {
    const u32 mid = lo + ((hi - lo) >> 1);
    if ((u64)w[mid] < target) lo = mid + 1; else hi = mid;
  }
  seg[(size_t)m * seg_stride + t] = lo;
}

__device__ __forceinline__ void load_bounds(const u32* __restrict__ seg, u32 seg_stride, u32 m0, u32 M, u32 tile, u32* lo, u32* hi) {
  const u32 m = m0 + threadIdx.x;
  if (threadIdx.x < kRowChunk && m < M) {
    lo[threadIdx.x] = seg[(size_t)m * seg_stride + tile];
    hi[threadIdx.x] = seg[(size_t)m * seg_stride + tile + 1];
  }
}

// Sparse variant: only x is produced, and only where somebody voted.
//
// The tally of a coordinate lives in an FB-bit field of an LDS word (FB = 8 while M <= 63, 16 while
// M <= 16383, else 32), so one block covers 32768 / 16384 / 8192 coordinates: at the sparsities of
// interest a tile holds few messages and the cost of a tile is a chain of memory latencies, so
// fewer, larger tiles are what counts.  A field holds BIAS + tally, which stays inside
// [BIAS - M, BIAS + M] and so never carries into its neighbour; its top bit is a "claimed" flag.
// Per tile: fill the fields with BIAS; add every vote; then every message tries to set the flag
// of its coordinate, and the one that finds it clear owns the coordinate and applies the update.
constexpr int kVoteWords = 8192;  // LDS words of the packed tally (32 KB)

template <int FB>
struct VoteField {
  static constexpr int kPer = 32 / FB;
  static constexpr u32 kFlag = 1u << (FB - 1);
  static constexpr u32 kBias = 1u << (FB - 2);
  static constexpr u32 kFill = FB == 8 ? 0x40404040u : (FB == 16 ? 0x40004000u : 0x40000000u);
  static constexpr u32 kTile = kVoteWords * kPer;
};

// ---- a wave's own tile ---------------------------------------------------------------------------
// One wave owns kMomTile consecutive coordinates and a slice of LDS holding their packed tally;
// nothing is shared between waves, so no block-wide barrier is needed and a block is just four
// independent waves.  The wave fills its slice, fetches the segment bounds of all rows (one row
// per lane) and adds the messages in.  Where a row has only a few messages in the tile (small K/N)
// they are numbered flat across the rows, so that every lane fetches its messages with independent
// loads instead of one dependent, nearly empty load per row; where rows have dozens each, lanes run
// over the messages of a row, a few rows at a time.
constexpr int kMomPass = 4;  // messages a lane fetches before it adds them to the tally

template <int FB>
__device__ __forceinline__ void tally_wave_tile(const u32* __restrict__ words, u64 K, const u32* __restrict__ seg, u32 seg_stride,
                                                u32 M, u64 N, u32 tile, u32* t) {
  typedef VoteField<FB> F;
  constexpr u32 kSlice = kMomTile / F::kPer;
  const u32 lane = lane_id();
  const u64 base = (u64)tile * kMomTile;
  // the bounds of the first 64 rows are requested before the slice is filled: the fill hides their latency
  u32 lo0 = 0, hi0 = 0;
  if (lane < M) {
    const u32* sg = seg + (size_t)lane * seg_stride + tile;
    lo0 = sg[0];
    hi0 = sg[1];
  }
  for (u32 i = lane * 4; i < kSlice; i += 256) *reinterpret_cast<uint4*>(&t[i]) = make_uint4(F::kFill, F::kFill, F::kFill, F::kFill);
  wave_sync();

  for (u32 m0 = 0; m0 < M; m0 += 64) {
    const u32 rows = M - m0 < 64u ? M - m0 : 64u;
    u32 lo = lo0, cnt = hi0 > lo0 ? hi0 - lo0 : 0u;
    if (m0 > 0) {
      lo = 0; cnt = 0;
      if (lane < rows) {
        const u32* sg = seg + (size_t)(m0 + lane) * seg_stride + tile;
        lo = sg[0];
        const u32 hi = sg[1];
        cnt = hi > lo ? hi - lo : 0u;
      }
    }
    const u32 incl = wave_incl_scan(cnt);
    const u32 first = incl - cnt;  // number of this row's first message in the tile's flat numbering
    const u32 total = __builtin_amdgcn_readlane(incl, 63);
    if (total >= 32u * rows) {
      // rows with dozens of messages each in this tile: lanes over the messages of a row, kMomPass rows at a time
      for (u32 r0 = 0; r0 < rows; r0 += kMomPass) {
        u32 rl[kMomPass], rc[kMomPass], longest = 0;
#pragma unroll
        for (int p = 0; p < kMomPass; ++p) {
          const u32 r = r0 + (u32)p < rows ? r0 + (u32)p : rows - 1;  // r is wave-uniform
          rl[p] = __builtin_amdgcn_readlane(lo, r);
          rc[p] = r0 + (u32)p < rows ? __builtin_amdgcn_readlane(cnt, r) : 0u;
          longest = rc[p] > longest ? rc[p] : longest;
        }
        for (u32 i = lane; i < longest + lane; i += 64) {  // the same trip count in every lane
          u32 wd[kMomPass];
#pragma unroll
          for (int p = 0; p < kMomPass; ++p) wd[p] = i < rc[p] ? words[(size_t)(m0 + r0 + (u32)p) * K + rl[p] + i] : S3GD_PAD;
#pragma unroll
          for (int p = 0; p < kMomPass; ++p) {
            const u32 c = (u32)((u64)(wd[p] >> 1) - base);
            if (wd[p] == S3GD_PAD || c >= kMomTile || base + c >= N) continue;
            const u32 sh = (c % F::kPer) * FB;
            atomicAdd(&t[c / F::kPer], (wd[p] & 1u) ? (0u - (1u << sh)) : (1u << sh));
          }
        }
      }
      continue;
    }
    for (u32 j0 = 0; j0 < total; j0 += 64u * kMomPass) {
      size_t at[kMomPass];
#pragma unroll
      for (int p = 0; p < kMomPass; ++p) at[p] = ~(size_t)0;
      for (u32 r = 0; r < rows; ++r) {  // r is wave-uniform: the three values come from lane r
        const u32 rf = __builtin_amdgcn_readlane(first, r), rc = __builtin_amdgcn_readlane(cnt, r),
                  rl = __builtin_amdgcn_readlane(lo, r);
        if (rc == 0) continue;
#pragma unroll
        for (int p = 0; p < kMomPass; ++p) {
          const u32 d = j0 + (u32)p * 64u + lane - rf;  // wraps to a huge value for messages of earlier rows
          if (d < rc) at[p] = (size_t)(m0 + r) * K + rl + d;
        }
      }
      u32 wd[kMomPass];
#pragma unroll
      for (int p = 0; p < kMomPass; ++p) wd[p] = at[p] != ~(size_t)0 ? words[at[p]] : S3GD_PAD;
#pragma unroll
      for (int p = 0; p < kMomPass; ++p) {
        const u32 c = (u32)((u64)(wd[p] >> 1) - base);
        if (wd[p] == S3GD_PAD || c >= kMomTile || base + c >= N) continue;  // the last two never hold for sorted rows
        const u32 sh = (c % F::kPer) * FB;
        atomicAdd(&t[c / F::kPer], (wd[p] & 1u) ? (0u - (1u << sh)) : (1u << sh));
      }
    }
  }
  wave_sync();
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream_f4(const float* p) {
  const f32x4 q = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
  return make_float4(q.x, q.y, q.z, q.w);
}
__device__ __forceinline__ void store_stream_f4(float* p, float4 a) {
  f32x4 q;
  q.x = a.x; q.y = a.y; q.z = a.z; q.w = a.w;
  __builtin_nontemporal_store(q, reinterpret_cast<f32x4*>(p));
}

// Dense variant: writes every element of tally and/or votes, optionally updates x.  A wave per
// kMomTile coordinates: tally in its own LDS slice, then 16 votes (one 16-byte store) per lane and
// round, and four tally entries (one 16-byte store) per lane and round.
template <int FB>
__global__ __launch_bounds__(kBlock) void k_vote_dense(const u32* __restrict__ words, u64 K, const u32* __restrict__ seg,
                                                       u32 seg_stride, u32 M, u64 N, u32 n_vt, int32_t* __restrict__ tally,
                                                       int8_t* __restrict__ votes, float* __restrict__ x, float lr) {
  typedef VoteField<FB> F;
  constexpr u32 kSlice = kMomTile / F::kPer;
  __shared__ __attribute__((aligned(16))) u32 lds[kWaves * kSlice];
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  const u32 tile = blockIdx.x * kWaves + wave;
  if (tile >= n_vt) return;  // whole waves leave; nothing below synchronises across waves
  u32* t = lds + wave * kSlice;
  const u64 base = (u64)tile * kMomTile;
  tally_wave_tile<FB>(words, K, seg, seg_stride, M, N, tile, t);
  auto tally_of = [&](u32 c) -> int {
    const u32 f = (t[c / F::kPer] >> ((c % F::kPer) * FB)) & (F::kFlag - 1u);
    return (int)f - (int)F::kBias;
  };
  if (votes) {
    for (u32 c0 = lane * 16u; c0 < kMomTile; c0 += 1024u) {
      const u64 n = base + c0;
      if (n >= N) break;
      u32 w[4] = {0, 0, 0, 0};
      if (FB == 8) {
        // four fields per word, each 0x40 + tally: the four vote bytes of a word at once.  A field above
        // 0x40 carries into its top bit when 0x3F is added, a field below 0x40 does not when 0x40 is
        // (fields stay below 0x80, so no carry crosses into the neighbour).
        const uint4 f4 = *reinterpret_cast<const uint4*>(&t[c0 / 4]);
        const u32 f[4] = {f4.x, f4.y, f4.z, f4.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const u32 v = f[k] & 0x7F7F7F7Fu;
          const u32 pos = ((v + 0x3F3F3F3Fu) >> 7) & 0x01010101u;
          const u32 neg = (~(v + 0x40404040u) >> 7) & 0x01010101u;
          w[k] = pos | (neg * 0xFFu);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int d = tally_of(c0 + (u32)i);
          w[i / 4] |= (u32)(((d > 0) - (d < 0)) & 0xFF) << (8 * (i % 4));
        }
      }
      if (n + 16 <= N) {
        u32x4 q;  // streamed out: 1 byte per coordinate is never read back by this kernel
        q.x = w[0]; q.y = w[1]; q.z = w[2]; q.w = w[3];
        __builtin_nontemporal_store(q, reinterpret_cast<u32x4*>(votes + n));
      } else {
        for (int i = 0; i < 16 && n + i < N; ++i) votes[n + i] = (int8_t)((w[i / 4] >> (8 * (i % 4))) & 0xFF);
      }
    }
  }
  if (x && !tally && base + kMomTile <= N) {
    // The fused sweep over a tile that lies inside the vector: four groups of four coordinates per lane
    // at a time, the parameters of all four requested before any is written back.  Every lane runs
    // through every group whether anybody voted there or not (a wave only skips what all its lanes
    // skip), so the work per group is kept small: with 8-bit fields the four votes of a word come out
    // of a few bit operations on the whole word, and the step is applied as x - d with d one of
    // lr, -lr, 0 (x - 0 keeps the bits of x, also of -0.0).
    constexpr int kGroups = 4;
    const u32 lr_bits = __float_as_uint(lr);
    for (u32 cb = lane * 4u; cb < kMomTile; cb += 256u * kGroups) {
      u32 pos[kGroups], neg[kGroups];  // bit 8e: coordinate e of the group is voted up / down
      bool line[kGroups];
      float4 xv[kGroups];
#pragma unroll
      for (int u = 0; u < kGroups; ++u) {
        const u32 c0 = cb + (u32)u * 256u;
        if (FB == 8) {
          const u32 v = t[c0 / 4] & 0x7F7F7F7Fu;  // four fields of 0x40 + tally
          pos[u] = ((v + 0x3F3F3F3Fu) >> 7) & 0x01010101u;
          neg[u] = (~(v + 0x40404040u) >> 7) & 0x01010101u;
        } else {
          pos[u] = 0;
          neg[u] = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int d = tally_of(c0 + (u32)e);
            pos[u] |= (u32)(d > 0) << (8 * e);
            neg[u] |= (u32)(d < 0) << (8 * e);
          }
        }
        // four lanes share 64 bytes of x: if one of them has a vote all four rewrite their part (the same
        // bits where nothing moves), so that memory sees whole 64-byte writes and not 16-byte pieces,
        // which it would have to merge by reading first
        line[u] = ((ballot((pos[u] | neg[u]) != 0) >> (lane & 60u)) & 0xFull) != 0;
        if (line[u]) xv[u] = load_stream_f4(x + base + c0);
      }
#pragma unroll
      for (int u = 0; u < kGroups; ++u) {
        if (!line[u]) continue;
        float* xe = &xv[u].x;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const u32 d = ((pos[u] >> (8 * e)) & 1u) ? lr_bits : (((neg[u] >> (8 * e)) & 1u) ? (lr_bits ^ 0x80000000u) : 0u);
          xe[e] = xe[e] - __uint_as_float(d);
        }
        store_stream_f4(x + base + cb + (u32)u * 256u, xv[u]);
      }
    }
    return;
  }
  if (tally || x) {
    for (u32 c0 = lane * 4u; c0 < kMomTile; c0 += 256u) {
      const u64 n = base + c0;
      if (n >= N) break;
      // nobody voted on these four coordinates (one word of 8-bit fields still holds the fill): nothing moves
      if (FB == 8 && !tally && (t[c0 / 4] & 0x7F7F7F7Fu) == F::kFill) continue;
      const int d[4] = {tally_of(c0), tally_of(c0 + 1), tally_of(c0 + 2), tally_of(c0 + 3)};
      const int v[4] = {(d[0] > 0) - (d[0] < 0), (d[1] > 0) - (d[1] < 0), (d[2] > 0) - (d[2] < 0), (d[3] > 0) - (d[3] < 0)};
      if (n + 4 <= N) {
        if (tally) *reinterpret_cast<int4*>(tally + n) = make_int4(d[0], d[1], d[2], d[3]);
        if (x && (v[0] | v[1] | v[2] | v[3])) {
          float4 xv = *reinterpret_cast<float4*>(x + n);
          if (v[0]) xv.x = xv.x - lr * (float)v[0];
          if (v[1]) xv.y = xv.y - lr * (float)v[1];
          if (v[2]) xv.z = xv.z - lr * (float)v[2];
          if (v[3]) xv.w = xv.w - lr * (float)v[3];
          *reinterpret_cast<float4*>(x + n) = xv;
        }
      } else {
        for (int e = 0; e < 4 && n + e < N; ++e) {
          if (tally) tally[n + e] = d[e];
          if (x && v[e]) x[n + e] = x[n + e] - lr * (float)v[e];
        }
      }
    }
  }
}

template <int FB, int PHASE>
__device__ __forceinline__ void vote_rows(const u32* __restrict__ words, u64 K, u32 m0, u32 rows, const u32* lo, const u32* hi,
                                          u32* t, u64 base, u64 N, float* __restrict__ x, float lr) {
  typedef VoteField<FB> F;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  for (u32 r = wave; r < rows; r += kWaves) {
    const u32* w = words + (size_t)(m0 + r) * K;
    for (u32 i = lo[r] + lane; i < hi[r]; i += 64) {
      const u32 wd = w[i];
      const u32 c = (u32)((u64)(wd >> 1) - base);
      if (c >= F::kTile || base + c >= N) continue;  // never true for sorted rows with indices < N
      const u32 sh = (c % F::kPer) * FB;
      if (PHASE == 0) {
        atomicAdd(&t[c / F::kPer], (wd & 1u) ? (0u - (1u << sh)) : (1u << sh));
      } else {
        const u32 old = atomicOr(&t[c / F::kPer], F::kFlag << sh) >> sh;
        if (!(old & F::kFlag)) {
          const int s = (int)(old & (F::kFlag - 1u)) - (int)F::kBias;
          if (s != 0) {
            float* p = x + (base + c);
            *p = *p - lr * (float)((s > 0) - (s < 0));
          }
        }
      }
    }
  }
}

// A light tile: at most kKeep rows per wave and at most 64 messages per row (the usual case at small
// K/N: a tile holds a few dozen messages per worker).  Every lane then holds its messages in
// registers across both phases, and the parameter of each message is fetched right away, so that
// a tile costs two memory latencies in a row (messages, parameters) instead of four.
constexpr int kKeep = 8;

template <int FB>
__device__ __forceinline__ void vote_tile_light(const u32* __restrict__ words, u64 K, u32 M, const u32* lo, const u32* hi, u32* t,
                                                u64 base, u64 N, float* __restrict__ x, float lr) {
  typedef VoteField<FB> F;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  u32 wd[kKeep];
  float xv[kKeep];
#pragma unroll
  for (int k = 0; k < kKeep; ++k) {
    const u32 r = wave + (u32)k * kWaves;
    wd[k] = S3GD_PAD;
    xv[k] = 0.0f;
    if (r < M) {
      const u32 i = lo[r] + lane;
      if (i < hi[r]) wd[k] = words[(size_t)r * K + i];
    }
    const u32 c = (u32)((u64)(wd[k] >> 1) - base);
    if (wd[k] == S3GD_PAD || c >= F::kTile || base + c >= N) {  // the last two never hold for sorted rows with indices < N
      wd[k] = S3GD_PAD;
    } else {
      xv[k] = x[base + c];
      const u32 sh = (c % F::kPer) * FB;
      atomicAdd(&t[c / F::kPer], (wd[k] & 1u) ? (0u - (1u << sh)) : (1u << sh));
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kKeep; ++k) {
    if (wd[k] == S3GD_PAD) continue;
    const u32 c = (u32)((u64)(wd[k] >> 1) - base);
    const u32 sh = (c % F::kPer) * FB;
    const u32 old = atomicOr(&t[c / F::kPer], F::kFlag << sh) >> sh;
    if (!(old & F::kFlag)) {  // first to claim the coordinate: apply its update
      const int sgn = (int)(old & (F::kFlag - 1u)) - (int)F::kBias;
      if (sgn != 0) x[base + c] = xv[k] - lr * (float)((sgn > 0) - (sgn < 0));
    }
  }
}

template <int FB>
__global__ __launch_bounds__(kBlock) void k_vote_sparse(const u32* __restrict__ words, u64 K, const u32* __restrict__ seg,
                                                        u32 seg_stride, u32 M, u64 N, u32 n_vt, float* __restrict__ x, float lr) {
  typedef VoteField<FB> F;
  __shared__ __attribute__((aligned(16))) u32 t[kVoteWords];
  __shared__ u32 lo[2][kRowChunk], hi[2][kRowChunk];
  const bool one_chunk = M <= (u32)kRowChunk;  // bounds of the next tile are then fetched a tile ahead
  u32 buf = 0;
  if (one_chunk && blockIdx.x < n_vt) load_bounds(seg, seg_stride, 0, M, blockIdx.x, lo[0], hi[0]);
  for (u32 tile = blockIdx.x; tile < n_vt; tile += gridDim.x) {
    const u64 base = (u64)tile * F::kTile;
    for (int i = threadIdx.x * 4; i < kVoteWords; i += kBlock * 4) *reinterpret_cast<uint4*>(&t[i]) = make_uint4(F::kFill, F::kFill, F::kFill, F::kFill);
    __syncthreads();
    if (one_chunk) {
      if (tile + gridDim.x < n_vt) load_bounds(seg, seg_stride, 0, M, tile + gridDim.x, lo[buf ^ 1], hi[buf ^ 1]);
      const bool heavy = M > (u32)(kWaves * kKeep) || (threadIdx.x < M && hi[buf][threadIdx.x] - lo[buf][threadIdx.x] > 64u);
      if (!__syncthreads_or(heavy)) {  // block-uniform
        vote_tile_light<FB>(words, K, M, lo[buf], hi[buf], t, base, N, x, lr);
      } else {
        vote_rows<FB, 0>(words, K, 0, M, lo[buf], hi[buf], t, base, N, x, lr);
        __syncthreads();
        vote_rows<FB, 1>(words, K, 0, M, lo[buf], hi[buf], t, base, N, x, lr);
      }
      buf ^= 1;
    } else {
      for (int phase = 0; phase < 2; ++phase) {
        for (u32 m0 = 0; m0 < M; m0 += kRowChunk) {
          __syncthreads();
          load_bounds(seg, seg_stride, m0, M, tile, lo[0], hi[0]);
          __syncthreads();
          const u32 rows = M - m0 < (u32)kRowChunk ? M - m0 : (u32)kRowChunk;
          if (phase == 0) vote_rows<FB, 0>(words, K, m0, rows, lo[0], hi[0], t, base, N, x, lr);
          else vote_rows<FB, 1>(words, K, m0, rows, lo[0], hi[0], t, base, N, x, lr);
        }
      }
    }
    __syncthreads();  // all claims made before the fields are refilled
  }
}

// Standalone update from a materialised vote vector.  A lane takes 16 consecutive votes (one
// 16-byte load) at a time, kUpd such groups with all their loads in flight together; a group that
// holds a vote has the whole 64 bytes of x that belong to it rewritten (memory merges a smaller write
// by reading first).
constexpr int kUpd = 4;

typedef u32 u32x4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void load_votes(const int8_t* __restrict__ votes, u64 i0, u64 stride, u64 n16, u32x4v (&v)[kUpd]) {
#pragma unroll
  for (int u = 0; u < kUpd; ++u) {
    const u64 i = i0 + (u64)u * stride;
    v[u] = 0;
    if (i < n16) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4v*>(votes + i * 16));
  }
}

// One block per 256 * kUpd consecutive groups of 16 coordinates, launched in coordinate order, so that
// the blocks running at any time touch a compact window of x (scattered accesses spread over the
// whole vector cost address translation and DRAM page misses on top of the transfer).  Few groups
// hold a vote (one in sixteen on a 1.2e9-coordinate model with four workers), so a lane that updated
// its own groups would issue four loads and four stores for a handful of active lanes each time.
// Instead the lanes of a wave queue their voted groups in LDS (the 16 votes and the group's number)
// and the wave works the queue off sixteen groups at a time, four lanes per group: one 16-byte load
// and one 16-byte store per lane, every lane busy, the four lanes of a group rewriting its 64 bytes
// together.
__global__ __launch_bounds__(kBlock) void k_apply_update(float* __restrict__ x, const int8_t* __restrict__ votes, float lr, u64 N) {
  __shared__ u32 queue_votes[kWaves][4][64 * kUpd], queue_group[kWaves][64 * kUpd];
  const u32 lane = lane_id();
  u32 (*qv)[64 * kUpd] = queue_votes[threadIdx.x >> 6];
  u32* qg = queue_group[threadIdx.x >> 6];
  const u64 n16 = N / 16;
  const u64 i0 = (u64)blockIdx.x * (kBlock * kUpd) + threadIdx.x;  // slot u of this thread: group i0 + u * kBlock
  u32x4v v[kUpd];
  load_votes(votes, i0, kBlock, n16, v);
  u32 total = 0;
#pragma unroll
  for (int u = 0; u < kUpd; ++u) {
    const bool live = (v[u].x | v[u].y | v[u].z | v[u].w) != 0;  // groups past the end were loaded as zeros
    const u64 m = ballot(live);
    if (live) {
      const u32 at = total + ballot_rank(m);
      qv[0][at] = v[u].x; qv[1][at] = v[u].y; qv[2][at] = v[u].z; qv[3][at] = v[u].w;
      qg[at] = (u32)(i0 + (u64)u * kBlock);
    }
    total += (u32)__popcll(m);
  }
  wave_sync();
  for (u32 r0 = 0; r0 < total; r0 += 16) {  // wave-uniform
    const u32 k = r0 + (lane >> 2), part = lane & 3u;
    if (k < total) {
      const u32 vw = qv[part][k];
      float* p = x + (u64)qg[k] * 16 + part * 4;
      float4 xv = load_stream_f4(p);
      const int a = (int8_t)(vw & 0xFF), b = (int8_t)((vw >> 8) & 0xFF), c = (int8_t)((vw >> 16) & 0xFF), d = (int8_t)(vw >> 24);
      if (a) xv.x = xv.x - lr * (float)a;
      if (b) xv.y = xv.y - lr * (float)b;
      if (c) xv.z = xv.z - lr * (float)c;
      if (d) xv.w = xv.w - lr * (float)d;
      store_stream_f4(p, xv);
    }
  }
  if (blockIdx.x == 0) {
    for (u64 n = n16 * 16 + threadIdx.x; n < N; n += blockDim.x) {
      const int vt = votes[n];
      if (vt) x[n] = x[n] - lr * (float)vt;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Momentum form of the update (Section 4 "Effects of optimization hyper-parameters"):
//   v <- mu * v + vote,  x <- x - lr * v,
// every operation rounded once in fp32 (no fused multiply-add).  Unlike the plain update this one
// moves every coordinate whose momentum is non-zero, so v is streamed in full; x is read and both
// are written only for runs of 16 coordinates (64 bytes) that hold a vote or a non-zero momentum (a
// coordinate with +0.0 momentum and no vote stays exactly as it is: mu * 0 + 0 = 0, x - lr * 0 = x).
// Whole 64-byte runs, not the 16 bytes of one lane: memory merges a smaller write by reading first.
__device__ __forceinline__ void momentum_apply(float& x, float& v, int s, float lr, float mu) {
  v = __fadd_rn(__fmul_rn(mu, v), (float)s);
  x = __fsub_rn(x, __fmul_rn(lr, v));
}

// Four consecutive coordinates whose momenta `vv` are already loaded; consecutive lanes hold
// consecutive groups.
__device__ __forceinline__ void momentum_group4(float* __restrict__ x, float* __restrict__ v, u64 n, float4 vv, const int (&s)[4],
                                                float lr, float mu) {
  const u32 any = __float_as_uint(vv.x) | __float_as_uint(vv.y) | __float_as_uint(vv.z) | __float_as_uint(vv.w) |
                  (u32)(s[0] | s[1] | s[2] | s[3]);
  if (((ballot(any != 0) >> (lane_id() & 60u)) & 0xFull) == 0) return;  // nothing to do in these 64 bytes
  float4 xv = *reinterpret_cast<const float4*>(x + n);
  momentum_apply(xv.x, vv.x, s[0], lr, mu);
  momentum_apply(xv.y, vv.y, s[1], lr, mu);
  momentum_apply(xv.z, vv.z, s[2], lr, mu);
  momentum_apply(xv.w, vv.w, s[3], lr, mu);
  *reinterpret_cast<float4*>(v + n) = vv;
  *reinterpret_cast<float4*>(x + n) = xv;
}

// The last, partial group of the vector.
__device__ __forceinline__ void momentum_tail(float* __restrict__ x, float* __restrict__ v, u64 n, u64 N, const int (&s)[4], float lr,
                                              float mu) {
  for (int e = 0; e < 4 && n + e < N; ++e) {
    float xe = x[n + e], ve = v[n + e];
    momentum_apply(xe, ve, s[e], lr, mu);
    v[n + e] = ve;
    x[n + e] = xe;
  }
}

__device__ __forceinline__ void momentum_group(float* __restrict__ x, float* __restrict__ v, u64 n, u64 N, const int (&s)[4],
                                               float lr, float mu) {
  if (n + 4 <= N) momentum_group4(x, v, n, *reinterpret_cast<const float4*>(v + n), s, lr, mu);
  else momentum_tail(x, v, n, N, s, lr, mu);
}

// ---- the fused vote + momentum sweep -----------------------------------------------------------
// One wave owns kMomTile consecutive coordinates and nothing is shared between waves: no block-wide
// barrier, a block is just four independent waves, and one block per 16384 coordinates is launched
// in coordinate order, so that the running blocks cover a compact window of x and v (a read-modify-
// write stream is measurably faster that way than with far-apart persistent streams).  A wave
//   1. issues the loads of its momenta (nothing depends on them before step 4),
//   2. fills its slice of the packed LDS tally, fetches the segment bounds of all rows (one row per
//      lane) and flattens the messages of its tile into one numbering, so that every lane fetches
//      its messages with independent loads instead of one dependent load per row,
//   3. adds the messages into the tally,
//   4. sweeps: per group of four coordinates, skip if all four momenta are +0.0 and nobody voted
//      (mu * 0 + 0 = 0 and x - lr * 0 = x), else fetch x, update, store both.
constexpr int kMomRounds = 4;                      // groups of four coordinates a lane has in flight
constexpr u32 kMomBatch = 256u * kMomRounds;       // coordinates of a wave per batch of rounds
constexpr int kMomBatches = kMomTile / kMomBatch;  // batches per tile; the momenta of the next are fetched a batch ahead

template <int FB>
__global__ __launch_bounds__(kBlock) void k_vote_momentum(const u32* __restrict__ words, u64 K, const u32* __restrict__ seg,
                                                          u32 seg_stride, u32 M, u64 N, u32 n_vt, float* __restrict__ x,
                                                          float* __restrict__ v, float lr, float mu) {
  typedef VoteField<FB> F;
  constexpr u32 kSlice = kMomTile / F::kPer;  // LDS words of one wave's tally
  __shared__ __attribute__((aligned(16))) u32 lds[kWaves * kSlice];
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  const u32 tile = blockIdx.x * kWaves + wave;
  if (tile >= n_vt) return;  // whole waves leave; nothing below synchronises across waves
  u32* t = lds + wave * kSlice;
  const u64 base = (u64)tile * kMomTile;

  float4 vv[kMomRounds];
#pragma unroll
  for (int u = 0; u < kMomRounds; ++u) {
    const u64 n = base + (u32)u * 256u + lane * 4u;
    vv[u] = n + 4 <= N ? load_stream_f4(v + n) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  tally_wave_tile<FB>(words, K, seg, seg_stride, M, N, tile, t);

  for (int bt = 0; bt < kMomBatches; ++bt) {
    const u32 c0 = (u32)bt * kMomBatch + lane * 4u;
    float4 nv[kMomRounds];  // the next batch's momenta, requested before this batch waits for anything
#pragma unroll
    for (int u = 0; u < kMomRounds; ++u) {
      const u64 n = base + c0 + kMomBatch + (u32)u * 256u;
      nv[u] = (bt + 1 < kMomBatches && n + 4 <= N) ? load_stream_f4(v + n) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    int sg[kMomRounds][4];
    bool live[kMomRounds];
    float4 xv[kMomRounds];
#pragma unroll
    for (int u = 0; u < kMomRounds; ++u) {
      const u32 c = c0 + (u32)u * 256u;
      const u64 n = base + c;
      u32 any = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const u32 f = (t[(c + e) / F::kPer] >> (((c + e) % F::kPer) * FB)) & (F::kFlag - 1u);
        const int d = (int)f - (int)F::kBias;
        sg[u][e] = (d > 0) - (d < 0);
        any |= (u32)sg[u][e];
      }
      any |= __float_as_uint(vv[u].x) | __float_as_uint(vv[u].y) | __float_as_uint(vv[u].z) | __float_as_uint(vv[u].w);
      // four lanes share 64 bytes of v and of x: if one of them has work, all four rewrite their part
      // (the same bits where nothing moves), so that memory sees whole 64-byte writes and not 16-byte
      // pieces, which it would have to merge by reading first (measured: 10 % to 30 % of the sweep
      // while the momentum is sparse; groups of 8 lanes do the same, 16 lanes lose)
      const bool line = ((ballot(any != 0) >> (lane & 60u)) & 0xFull) != 0;
      live[u] = line && n + 4 <= N;
      if (live[u]) xv[u] = load_stream_f4(x + n);
      if (n < N && n + 4 > N) momentum_tail(x, v, n, N, sg[u], lr, mu);  // the one group that straddles the end
    }
#pragma unroll
    for (int u = 0; u < kMomRounds; ++u) {
      if (live[u]) {
        const u64 n = base + c0 + (u32)u * 256u;
        momentum_apply(xv[u].x, vv[u].x, sg[u][0], lr, mu);
        momentum_apply(xv[u].y, vv[u].y, sg[u][1], lr, mu);
        momentum_apply(xv[u].z, vv[u].z, sg[u][2], lr, mu);
        momentum_apply(xv[u].w, vv[u].w, sg[u][3], lr, mu);
        store_stream_f4(v + n, vv[u]);
        store_stream_f4(x + n, xv[u]);
      }
      vv[u] = nv[u];
    }
  }
}

// The same from a materialised vote vector.
__global__ __launch_bounds__(kBlock) void k_apply_momentum(float* __restrict__ x, float* __restrict__ v, const int8_t* __restrict__ votes,
                                                           float lr, float mu, u64 N) {
  const u64 n4 = (N + 3) / 4;
  for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (u64)gridDim.x * blockDim.x) {
    const u64 n = i * 4;
    int s[4] = {0, 0, 0, 0};
    if (n + 4 <= N) {
      const u32 w = *reinterpret_cast<const u32*>(votes + n);
      s[0] = (int8_t)(w & 0xFF); s[1] = (int8_t)((w >> 8) & 0xFF); s[2] = (int8_t)((w >> 16) & 0xFF); s[3] = (int8_t)(w >> 24);
    } else {
      for (int e = 0; e < 4 && n + e < N; ++e) s[e] = votes[n + e];
    }
    momentum_group(x, v, n, N, s, lr, mu);
  }
}

hipError_t launch_vote_momentum(const Workspace& ws, const u32* words, const u32* counts, u32 M, u64 N, u64 K, float* x, float* v,
                                float lr, float mu, hipStream_t s) {
  Profiler& P = *ws.prof;
  const int fb = M <= 63 ? 8 : (M <= 16383 ? 16 : 32);
  const u32 n_vt = (u32)((N + kMomTile - 1) / kMomTile);
  const u32 stride = n_vt + 1;
  P.begin(KID_SEG_BOUNDS, s);
  k_seg_bounds<<<dim3((n_vt + 1 + 255) / 256, M), 256, 0, s>>>(words, counts, K, n_vt, stride, kMomTile, ws.seg);
  P.end(s);
  const u32 g = (n_vt + kWaves - 1) / kWaves;
  P.begin(KID_VOTE_MOMENTUM, s);
  if (fb == 8) k_vote_momentum<8><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, x, v, lr, mu);
  else if (fb == 16) k_vote_momentum<16><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, x, v, lr, mu);
  else k_vote_momentum<32><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, x, v, lr, mu);
  P.end(s);
  return hipGetLastError();
}

hipError_t launch_update_momentum(const Workspace& ws, float* x, float* v, const int8_t* votes, float lr, float mu, u64 N,
                                  hipStream_t s) {
  u64 blocks = ((N + 3) / 4 + kBlock - 1) / kBlock;
  if (blocks > ws.stream_blocks * 4ull) blocks = ws.stream_blocks * 4ull;
  if (blocks < 1) blocks = 1;
  ws.prof->begin(KID_UPDATE_MOMENTUM, s);
  k_apply_momentum<<<(u32)blocks, kBlock, 0, s>>>(x, v, votes, lr, mu, N);
  ws.prof->end(s);
  return hipGetLastError();
}

hipError_t launch_vote(const Workspace& ws, const u32* words, const u32* counts, u32 M, u64 N, u64 K, int32_t* tally,
                       int8_t* votes, float* x, float lr, hipStream_t s) {
  Profiler& P = *ws.prof;
  // The sweep over every coordinate also serves the fused call once there is a message per twenty
  // coordinates: the sparse kernel walks the messages twice (tally, then claim) and pays per message
  // (measured crossover between M*K/N = 0.03, where the sparse kernel is 1.4 times faster, and
  // 0.08, where the sweep is; at one message per coordinate the sweep is 5 times faster).
  const bool dense = tally || votes || (u64)M * K * 20 >= N;
  const int fb = M <= 63 ? 8 : (M <= 16383 ? 16 : 32);
  const u32 tile_coords = dense ? kMomTile : (u32)kVoteWords * (32u / fb);
  const u32 n_vt = (u32)((N + tile_coords - 1) / tile_coords);  // a tiling no finer than kMomTile: the table row fits
  const u32 stride = n_vt + 1;
  P.begin(KID_SEG_BOUNDS, s);
  k_seg_bounds<<<dim3((n_vt + 1 + 255) / 256, M), 256, 0, s>>>(words, counts, K, n_vt, stride, tile_coords, ws.seg);
  P.end(s);
  if (dense) {
    P.begin(KID_VOTE_DENSE, s);
    const u32 g = (n_vt + kWaves - 1) / kWaves;
    if (fb == 8) k_vote_dense<8><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, tally, votes, x, lr);
    else if (fb == 16) k_vote_dense<16><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, tally, votes, x, lr);
    else k_vote_dense<32><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, tally, votes, x, lr);
    P.end(s);
  } else {
    const u32 g = n_vt < ws.stream_blocks ? n_vt : ws.stream_blocks;
    P.begin(KID_VOTE_SPARSE, s);
    if (fb == 8) k_vote_sparse<8><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, x, lr);
    else if (fb == 16) k_vote_sparse<16><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, x, lr);
    else k_vote_sparse<32><<<g, kBlock, 0, s>>>(words, K, ws.seg, stride, M, N, n_vt, x, lr);
    P.end(s);
  }
  return hipGetLastError();
}

hipError_t launch_update(const Workspace& ws, float* x, const int8_t* votes, float lr, u64 N, hipStream_t s) {
  u64 blocks = (N / 16 + kBlock * kUpd - 1) / (kBlock * kUpd);  // at most 2^27 / 1024 blocks
  if (blocks < 1) blocks = 1;
  ws.prof->begin(KID_UPDATE, s);
  k_apply_update<<<(u32)blocks, kBlock, 0, s>>>(x, votes, lr, N);
  ws.prof->end(s);
  return hipGetLastError();
}

}  // namespace s3gd
