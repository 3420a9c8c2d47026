// Compact wire format of a sparse ternary vector: the messages of Algorithm 1 as they would cross
// a network.  The paper prices a worker's message at about K + K*log2(N/K) bits (K signs plus the
// support pattern; Section 2.2 "Gradient compression") and the server's answer at the same
// expression in the size of the voted support (Section 2.2 "Model update").  The 32-bit words the
// encode kernels emit are 3-4 times larger; the kernels here convert between the two.
//
// Code: Elias-Fano on the ascending index set, one sign bit per entry.  With n entries below N and
// L = floor(log2(N / n)):
//     word 0        n
//     word 1        L
//     sign section  ceil(n/64) x 64 bits: bit l of group g = entry 64g + l is negative
//     low section   ceil(n/64) * L x 64 bits: group g*L + b = bit b of the low L index bits of the
//                   entries 64g .. 64g+63, one entry per lane ("bit planes")
//     high section  n + ((N-1) >> L) + 1 bits (none when n = 0): bit (index_i >> L) + i set for the i-th entry
// The 64-entry groups are wave ballots: a wave turns 64 consecutive entries into one sign group
// and L low groups with L + 1 ballots, and reads them back with one shift per plane.
#include "s3gd_common.h"
#include "s3gd_kernels.h"

namespace s3gd {

constexpr u32 kHeaderWords = 2;
constexpr int kHighPerThread = 1;                               // high-section words per thread
constexpr u32 kHighWordsPerBlock = kBlock * kHighPerThread;      // 8192 bits of a high section per block

__host__ __device__ inline u32 ef_low_bits(u64 N, u64 n) {
  if (n == 0) return 0;
  const u64 q = N / n;  // >= 1
  u32 L = 0;
  while ((q >> (L + 1)) != 0) ++L;
  return L;
}

struct EfLayout {
  u32 n, L, G;
  u64 sign_off, low_off, high_off, high_bits, high_words, total_words;  // offsets in 32-bit words
};

__host__ __device__ inline EfLayout ef_layout(u64 N, u32 n) {
  EfLayout e;
  e.n = n;
  e.L = ef_low_bits(N, n);
  e.G = (n + 63) / 64;
  e.sign_off = kHeaderWords;
  e.low_off = e.sign_off + 2ull * e.G;
  e.high_off = e.low_off + 2ull * e.G * e.L;
  e.high_bits = n ? (u64)n + ((N - 1) >> e.L) + 1 : 0;
  e.high_words = (e.high_bits + 31) / 32;
  e.total_words = e.high_off + e.high_words;
  return e;
}

u64 packed_row_capacity(u64 N, u64 K) {
  if (K > N) K = N;
  u64 low_max;  // max over n <= K of n * L(n) <= n * log2(N / n), which grows with n while n <= N / e
  if (K == 0) low_max = 0;
  else if (4 * K <= N) low_max = K * (ef_low_bits(N, K) + 1);
  else low_max = N / 2 + N / 32 + 1;  // max of n * log2(N / n) over all n is N / (e ln 2) = 0.5307 N
  const u64 sign = 2 * ((K + 63) / 64);
  const u64 low = (low_max + 31) / 32 + 64;  // + up to one partly filled 64-entry group per plane
  const u64 high = (3 * K + 1 + 31) / 32 + 1;  // (N-1) >> L < 2n
  const u64 w = kHeaderWords + sign + low + high;
  return (w + 1) & ~1ull;
}

// ------------------------------------------------------------------------------------------------
// pack
__global__ __launch_bounds__(kBlock) void k_ef_clear_high(const u32* __restrict__ counts, u64 N, u64 K, u32* __restrict__ packed,
                                                          u64 row_words, u32* __restrict__ status) {
  const u32 m = blockIdx.y;
  u32 n = counts[m];
  if ((u64)n > K) n = (u32)K;
  const EfLayout e = ef_layout(N, n);
  u32* row = packed + (size_t)m * row_words;
  // the flags of the previous coding call go first, whatever row 0 turns out to be
  if (m == 0 && blockIdx.x == 0 && threadIdx.x == 0) status[3] = 0;
  if (e.total_words > row_words) return;  // reported by the pack kernel
  for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < e.high_words; i += (u64)gridDim.x * blockDim.x) row[e.high_off + i] = 0;
}

__global__ __launch_bounds__(kBlock) void k_ef_pack(const u32* __restrict__ words, const u32* __restrict__ counts, u64 N, u64 K,
                                                    u32* __restrict__ packed, u64 row_words, u32* __restrict__ status) {
  const u32 m = blockIdx.y;
  u32 n = counts[m];
  if ((u64)n > K) n = (u32)K;
  const EfLayout e = ef_layout(N, n);
  u32* row = packed + (size_t)m * row_words;
  if (e.total_words > row_words) {  // cannot happen with the capacity the library reports
    if (blockIdx.x == 0 && threadIdx.x == 0) { atomicOr(&status[3], kCodingCapacity); row[0] = 0; row[1] = 0; }
    return;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) { row[0] = n; row[1] = e.L; }
  u64* sign = reinterpret_cast<u64*>(row + e.sign_off);
  u64* low = reinterpret_cast<u64*>(row + e.low_off);
  u32* high = row + e.high_off;
  const u32* w = words + (size_t)m * K;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  for (u32 g = blockIdx.x * kWaves + wave; g < e.G; g += gridDim.x * kWaves) {
    const u32 i = g * 64 + lane;
    const bool ok = i < n;
    const u32 wd = ok ? w[i] : 0u;
    const u32 idx = wd >> 1;
    const u64 sg = ballot(ok && (wd & 1u));
    if (lane == 0) sign[g] = sg;
    u64 mine = 0;
    for (u32 b = 0; b < e.L; ++b) {
      const u64 bal = ballot(ok && ((idx >> b) & 1u));
      if (lane == b) mine = bal;
    }
    if (lane < e.L) low[(size_t)g * e.L + lane] = mine;
    // high section: one bit per entry at (idx >> L) + i.  Positions ascend with the lane, so lanes
    // that share a 32-bit word are neighbours: OR them together and let the last one write.
    const u64 p = ok ? (u64)(idx >> e.L) + i : ~0ull;
    u64 key = p >> 5;
    u32 val = ok ? 1u << (p & 31u) : 0u;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const u64 ok_key = __shfl_up(key, d, 64);
      const u32 ov = __shfl_up(val, d, 64);
      if (lane >= (u32)d && ok_key == key) val |= ov;
    }
    const u64 next_key = __shfl_down(key, 1, 64);
    if (ok && (lane == 63 || next_key != key) && p < e.high_bits) atomicOr(&high[key], val);
  }
}

// ------------------------------------------------------------------------------------------------
// unpack: ranks of the ones of the high section come from popcounts per block, scanned per row
__device__ __forceinline__ bool ef_read_header(const u32* __restrict__ row, u64 N, u64 K, u64 row_words, EfLayout& e) {
  const u32 n = row[0], L = row[1];
  if ((u64)n > K || (u64)n > N) return false;
  e = ef_layout(N, n);
  return L == e.L && e.total_words <= row_words;
}

__global__ __launch_bounds__(kBlock) void k_ef_count(const u32* __restrict__ packed, u64 row_words, u64 N, u64 K, u32* __restrict__ blk,
                                                     u32 blk_stride, u32* __restrict__ status) {
  const u32 m = blockIdx.y;
  const u32* row = packed + (size_t)m * row_words;
  if (m == 0 && blockIdx.x == 0 && threadIdx.x == 0) status[3] = 0;
  EfLayout e;
  if (!ef_read_header(row, N, K, row_words, e)) return;
  __shared__ u32 lds[kWaves];
  const u32* high = row + e.high_off;
  for (u64 b = blockIdx.x; b * kHighWordsPerBlock < e.high_words; b += gridDim.x) {
    u32 c = 0;
#pragma unroll
    for (int k = 0; k < kHighPerThread; ++k) {
      const u64 i = b * kHighWordsPerBlock + (u64)threadIdx.x * kHighPerThread + k;
      if (i < e.high_words) c += __popc(high[i]);
    }
    u32 total;
    (void)block_excl_scan<u32>(c, &total, lds);
    if (threadIdx.x == 0) blk[(size_t)m * blk_stride + b] = total;
  }
}

__global__ __launch_bounds__(kScanBlock) void k_ef_scan(const u32* __restrict__ packed, u64 row_words, u64 N, u64 K,
                                                        u32* __restrict__ blk, u32 blk_stride) {
  const u32 m = blockIdx.x;
  const u32* row = packed + (size_t)m * row_words;
  EfLayout e;
  if (!ef_read_header(row, N, K, row_words, e)) return;
  __shared__ u32 lds[kScanBlock / 64];
  const u32 nb = (u32)((e.high_words + kHighWordsPerBlock - 1) / kHighWordsPerBlock);
  u32* t = blk + (size_t)m * blk_stride;
  u32 carry = 0;
  for (u32 base = 0; base < nb; base += kScanBlock) {
    const u32 i = base + threadIdx.x;
    const u32 v = i < nb ? t[i] : 0;
    u32 total;
    const u32 ex = carry + block_excl_scan<u32>(v, &total, lds);
    if (i < nb) t[i] = ex;
    carry += total;
  }
}

__global__ __launch_bounds__(kBlock) void k_ef_decode(const u32* __restrict__ packed, u64 row_words, u64 N, u64 K,
                                                      const u32* __restrict__ blk, u32 blk_stride, u32* __restrict__ words,
                                                      u32* __restrict__ counts, u32* __restrict__ status) {
  const u32 m = blockIdx.y;
  const u32* row = packed + (size_t)m * row_words;
  u32* out = words + (size_t)m * K;
  EfLayout e;
  if (!ef_read_header(row, N, K, row_words, e)) {  // a corrupt header: the row decodes to nothing
    if (blockIdx.x == 0 && threadIdx.x == 0) { counts[m] = 0; atomicOr(&status[3], kCodingFormat); }
    for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < K; i += (u64)gridDim.x * blockDim.x) out[i] = S3GD_PAD;
    return;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) counts[m] = e.n;
  for (u64 i = (u64)e.n + (u64)blockIdx.x * blockDim.x + threadIdx.x; i < K; i += (u64)gridDim.x * blockDim.x) out[i] = S3GD_PAD;
  __shared__ u32 lds[kWaves];
  const u64* sign = reinterpret_cast<const u64*>(row + e.sign_off);
  const u64* low = reinterpret_cast<const u64*>(row + e.low_off);
  const u32* high = row + e.high_off;
  bool bad = false;
  for (u64 b = blockIdx.x; b * kHighWordsPerBlock < e.high_words; b += gridDim.x) {
    u32 hw[kHighPerThread], c = 0;
    const u64 w0 = b * kHighWordsPerBlock + (u64)threadIdx.x * kHighPerThread;
#pragma unroll
    for (int k = 0; k < kHighPerThread; ++k) {
      hw[k] = w0 + k < e.high_words ? high[w0 + k] : 0u;
      c += __popc(hw[k]);
    }
    u32 total;
    u32 rank = blk[(size_t)m * blk_stride + b] + block_excl_scan<u32>(c, &total, lds);
#pragma unroll
    for (int k = 0; k < kHighPerThread; ++k) {
      u32 bits = hw[k];
      while (bits) {
        const u32 bit = __ffs(bits) - 1;
        bits &= bits - 1;
        const u64 p = (w0 + k) * 32 + bit;
        const u32 i = rank++;
        if (i >= e.n || p < i) { bad = true; continue; }  // more ones than entries
        const u32 g = i >> 6, l = i & 63u;
        u32 lo = 0;
        for (u32 bb = 0; bb < e.L; ++bb) lo |= (u32)((low[(size_t)g * e.L + bb] >> l) & 1ull) << bb;
        const u64 idx = ((p - i) << e.L) | lo;
        if (idx >= N) { bad = true; out[i] = S3GD_PAD; continue; }
        out[i] = ((u32)idx << 1) | (u32)((sign[g] >> l) & 1ull);
      }
    }
  }
  if (bad) atomicOr(&status[3], kCodingFormat);
}

// ------------------------------------------------------------------------------------------------
// the server's answer as a message: ordered compaction of the non-zero votes
constexpr u32 kVotesPerBlock = kBlock * 16;

__device__ __forceinline__ u32 nonzero_bytes(u32 w) {  // bit 8k set iff byte k of w is non-zero
  return ((w | ((w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu)) >> 7) & 0x01010101u;
}

__device__ __forceinline__ void load_votes16(const int8_t* __restrict__ votes, u64 N, u64 n0, u32 (&v)[4]) {
  if (n0 + 16 <= N) {
    const uint4 q = *reinterpret_cast<const uint4*>(votes + n0);
    v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
  } else {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      v[k] = 0;
      for (int e = 0; e < 4; ++e) {
        const u64 n = n0 + 4 * k + e;
        if (n < N) v[k] |= (u32)(uint8_t)votes[n] << (8 * e);
      }
    }
  }
}

__global__ __launch_bounds__(kBlock) void k_votes_count(const int8_t* __restrict__ votes, u64 N, u32* __restrict__ blk,
                                                        u32* __restrict__ status) {
  __shared__ u32 lds[kWaves];
  if (blockIdx.x == 0 && threadIdx.x == 0) status[3] = 0;
  const u64 nb = (N + kVotesPerBlock - 1) / kVotesPerBlock;
  for (u64 b = blockIdx.x; b < nb; b += gridDim.x) {
    u32 v[4], c = 0;
    const u64 n0 = b * kVotesPerBlock + (u64)threadIdx.x * 16;
    if (n0 < N) {
      load_votes16(votes, N, n0, v);
#pragma unroll
      for (int k = 0; k < 4; ++k) c += __popc(nonzero_bytes(v[k]));
    }
    u32 total;
    (void)block_excl_scan<u32>(c, &total, lds);
    if (threadIdx.x == 0) blk[b] = total;
  }
}

__global__ __launch_bounds__(kScanBlock) void k_votes_scan(u32* __restrict__ blk, u64 N, u32* __restrict__ count) {
  __shared__ u32 lds[kScanBlock / 64];
  const u32 nb = (u32)((N + kVotesPerBlock - 1) / kVotesPerBlock);
  u32 carry = 0;
  for (u32 base = 0; base < nb; base += kScanBlock) {
    const u32 i = base + threadIdx.x;
    const u32 v = i < nb ? blk[i] : 0;
    u32 total;
    const u32 ex = carry + block_excl_scan<u32>(v, &total, lds);
    if (i < nb) blk[i] = ex;
    carry += total;
  }
  if (threadIdx.x == 0) count[0] = carry;
}

__global__ __launch_bounds__(kBlock) void k_votes_emit(const int8_t* __restrict__ votes, u64 N, const u32* __restrict__ blk, u64 cap,
                                                       u32* __restrict__ words, const u32* __restrict__ count,
                                                       u32* __restrict__ status) {
  __shared__ u32 lds[kWaves];
  const u64 nb = (N + kVotesPerBlock - 1) / kVotesPerBlock;
  const u32 total_words = count[0];
  if (blockIdx.x == 0 && threadIdx.x == 0 && (u64)total_words > cap) atomicOr(&status[3], kCodingCapacity);
  for (u64 i = (u64)total_words + (u64)blockIdx.x * blockDim.x + threadIdx.x; i < cap; i += (u64)gridDim.x * blockDim.x) words[i] = S3GD_PAD;
  for (u64 b = blockIdx.x; b < nb; b += gridDim.x) {
    u32 v[4] = {0, 0, 0, 0}, c = 0;
    const u64 n0 = b * kVotesPerBlock + (u64)threadIdx.x * 16;
    if (n0 < N) {
      load_votes16(votes, N, n0, v);
#pragma unroll
      for (int k = 0; k < 4; ++k) c += __popc(nonzero_bytes(v[k]));
    }
    u32 total;
    u64 o = (u64)blk[b] + block_excl_scan<u32>(c, &total, lds);
    if (c == 0) continue;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const u32 byte = (v[k] >> (8 * e)) & 0xFFu;
        if (byte) {
          if (o < cap) words[o] = ((u32)(n0 + 4 * k + e) << 1) | (byte >> 7);
          ++o;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
static u32 coding_blocks(const Workspace& ws, u64 units) {
  u64 g = units < 1 ? 1 : units;
  if (g > ws.stream_blocks) g = ws.stream_blocks;
  return (u32)g;
}

hipError_t launch_pack(const Workspace& ws, const u32* words, const u32* counts, u32 M, u64 N, u64 K, u32* packed, u64 row_words,
                       hipStream_t s) {
  Profiler& P = *ws.prof;
  u32 gx = coding_blocks(ws, (K + 64 * kWaves - 1) / (64 * kWaves)) / M;
  if (gx < 1) gx = 1;
  P.begin(KID_PACK, s);
  k_ef_clear_high<<<dim3(gx, M), kBlock, 0, s>>>(counts, N, K, packed, row_words, ws.status);
  k_ef_pack<<<dim3(gx, M), kBlock, 0, s>>>(words, counts, N, K, packed, row_words, ws.status);
  P.end(s);
  return hipGetLastError();
}

hipError_t launch_unpack(const Workspace& ws, const u32* packed, u64 row_words, u32 M, u64 N, u64 K, u32* words, u32* counts,
                         hipStream_t s) {
  Profiler& P = *ws.prof;
  u32* blk = reinterpret_cast<u32*>(ws.tile_cnt);
  const u32 bstride = coding_blk_stride(N);
  const u64 max_high_words = (3 * K + 1 + 31) / 32 + 1;
  u32 gx = coding_blocks(ws, (max_high_words + kHighWordsPerBlock - 1) / kHighWordsPerBlock) / M;
  if (gx < 1) gx = 1;
  P.begin(KID_UNPACK, s);
  k_ef_count<<<dim3(gx, M), kBlock, 0, s>>>(packed, row_words, N, K, blk, bstride, ws.status);
  k_ef_scan<<<M, kScanBlock, 0, s>>>(packed, row_words, N, K, blk, bstride);
  k_ef_decode<<<dim3(gx, M), kBlock, 0, s>>>(packed, row_words, N, K, blk, bstride, words, counts, ws.status);
  P.end(s);
  return hipGetLastError();
}

hipError_t launch_votes_to_message(const Workspace& ws, const int8_t* votes, u64 N, u64 cap, u32* words, u32* count, hipStream_t s) {
  Profiler& P = *ws.prof;
  u32* blk = reinterpret_cast<u32*>(ws.tile_cnt);
  const u32 gx = coding_blocks(ws, (N + kVotesPerBlock - 1) / kVotesPerBlock);
  P.begin(KID_VOTES_TO_MESSAGE, s);
  k_votes_count<<<gx, kBlock, 0, s>>>(votes, N, blk, ws.status);
  k_votes_scan<<<1, kScanBlock, 0, s>>>(blk, N, count);
  k_votes_emit<<<gx, kBlock, 0, s>>>(votes, N, blk, cap, words, count, ws.status);
  P.end(s);
  return hipGetLastError();
}

}  // namespace s3gd
