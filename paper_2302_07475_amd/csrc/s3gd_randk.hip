// RandKSign, the worker side of Algorithm 2 (Section 3.4 "Effect of the random-K sparsification"):
// K coordinates drawn at random instead of the K largest, their signs sent, no error memory.
//
// The paper leaves the sampling law open.  Here worker m at iteration t selects
// {pi(0), ..., pi(K-1)} for a pseudo-random permutation pi of [0, N) keyed by (seed, t, m): exactly
// K distinct coordinates, each selected with probability K/N over the keys.  pi is a counter-based
// generator, so the work is O(K) per worker and never touches the other N - K gradient entries:
//   - b = bit length of N - 1 (at least 2), h = ceil(b / 2); a value below 4^h is split into a
//     left half (high h bits) and a right half (low h bits);
//   - 6 Feistel rounds (left, right) <- (right, left ^ (F(right ^ key_r) & (2^h - 1)));
//   - F(z): z ^= z >> 16; z *= 0x85EBCA6B; z ^= z >> 13; z *= 0xC2B2AE35; z ^= z >> 16 (mod 2^32);
//   - k0 = F(lo32(seed) + 0x9E3779B9 (t+1)); k1 = F(k0 ^ hi32(seed)); k2 = F(k1 ^ 0x85EBCA77 (m+1));
//     key_r = F(k2 + 0xC2B2AE3D (r+1));
//   - the network is applied again while the value is >= N (cycle walking; it is a bijection of
//     [0, 4^h), so the walk from a value below N comes back below N, and 4^h < 4N keeps it short).
//
// The message must list the selected coordinates in ascending order.  They arrive in the order of
// the permutation, so they are bucket-sorted: a bucket is 2048 consecutive coordinates (it can hold
// at most 2048 distinct entries, which fit the LDS of one wave whatever the data), a count pass and
// a scan give every bucket its slot range in the row, a second pass drops each word into its
// bucket, and each bucket is ordered in place: a handful of words by one lane in registers, more by
// one wave with a bitonic network in LDS.
#include "s3gd_common.h"
#include "s3gd_kernels.h"

namespace s3gd {

constexpr int kRounds = 6;
constexpr u32 kBucketShift = 11;
constexpr u32 kBucket = 1u << kBucketShift;  // coordinates per bucket

struct PermKey {
  u32 k[kRounds];
  u32 h, mask;
};

__host__ __device__ inline u32 fmix32(u32 z) {
  z ^= z >> 16; z *= 0x85EBCA6Bu; z ^= z >> 13; z *= 0xC2B2AE35u; z ^= z >> 16;
  return z;
}

__device__ __forceinline__ PermKey perm_key(u64 seed, u32 t, u32 m, u64 N) {
  PermKey p;
  const u32 k0 = fmix32((u32)seed + 0x9E3779B9u * (t + 1u));
  const u32 k1 = fmix32(k0 ^ (u32)(seed >> 32));
  const u32 k2 = fmix32(k1 ^ (0x85EBCA77u * (m + 1u)));
#pragma unroll
  for (int r = 0; r < kRounds; ++r) p.k[r] = fmix32(k2 + 0xC2B2AE3Du * (u32)(r + 1));
  u32 b = 64u - (u32)__clzll((unsigned long long)(N - 1) | 2ull);  // bit length of N - 1, at least 2
  p.h = (b + 1) / 2;
  p.mask = (1u << p.h) - 1u;  // h <= 16 because N < 2^31
  return p;
}

__device__ __forceinline__ u32 permute(u32 i, u64 N, const PermKey& p) {
  u32 v = i;
  do {
    u32 left = v >> p.h, right = v & p.mask;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      const u32 nr = left ^ (fmix32(right ^ p.k[r]) & p.mask);
      left = right;
      right = nr;
    }
    v = (left << p.h) | right;
  } while ((u64)v >= N);
  return v;
}

__global__ void k_randk_clear(u32* __restrict__ bucket, u32 nb, u32 bstride, u32* __restrict__ status, u32 M) {
  const u32 m = blockIdx.y;
  for (u32 i = blockIdx.x * blockDim.x + threadIdx.x; i < nb; i += gridDim.x * blockDim.x) bucket[(size_t)m * bstride + i] = 0;
  if (m == 0 && blockIdx.x == 0 && threadIdx.x == 0) { status[0] = 0; status[1] = 0; status[2] = M; status[4] = 0; }
}

// The selected entries reach their buckets in two steps around the scan of the bucket counts.
//   kCount    count the non-zero selected entries of each bucket
//   kRank     the same, and every entry keeps (word, its arrival number in its bucket) in `tmp`,
//             so that the second step neither evaluates the permutation nor touches the gradients again
//   kScatter  second step without `tmp`: bucket[] holds the first slot of each bucket; every entry
//             takes the next slot of its bucket (afterwards bucket[b] is the end of bucket b)
enum { kCount = 0, kRank = 1, kScatter = 2 };

template <int STEP>
__global__ __launch_bounds__(kBlock) void k_randk_pass(const float* __restrict__ grads, u64 N, u64 K, u64 seed, u32 t,
                                                       u32* __restrict__ bucket, u32 bstride, u32* __restrict__ words,
                                                       uint2* __restrict__ tmp, u32* __restrict__ status) {
  const u32 m = blockIdx.y;
  const PermKey p = perm_key(seed, t, m, N);
  const u32* row = reinterpret_cast<const u32*>(grads + (size_t)m * N);
  u32* bk = bucket + (size_t)m * bstride;
  u32* out = words + (size_t)m * K;
  bool nan = false;
  for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < K; i += (u64)gridDim.x * blockDim.x) {
    const u32 n = permute((u32)i, N, p);
    const u32 bits = row[n];
    const u32 key = bits & 0x7FFFFFFFu;
    if (key == 0) {  // sgn(0) = 0: nothing to send
      if (STEP == kRank) tmp[(size_t)m * K + i] = make_uint2(S3GD_PAD, 0u);
      continue;
    }
    nan |= key > 0x7F800000u;
    const u32 word = (n << 1) | (bits >> 31);
    if (STEP == kScatter) {
      const u32 pos = atomicAdd(&bk[n >> kBucketShift], 1u);
      if ((u64)pos < K) out[pos] = word;  // pos < K by construction
    } else if (STEP == kRank) {
      tmp[(size_t)m * K + i] = make_uint2(word, atomicAdd(&bk[n >> kBucketShift], 1u));
    } else {
      atomicAdd(&bk[n >> kBucketShift], 1u);
    }
  }
  if (STEP != kScatter && nan) status[0] = 1;
}

// Second step with `tmp`: bucket[] holds the first slot of each bucket.
__global__ __launch_bounds__(kBlock) void k_randk_place(const uint2* __restrict__ tmp, u64 K, const u32* __restrict__ bucket, u32 bstride,
                                                        u32* __restrict__ words) {
  const u32 m = blockIdx.y;
  const u32* bk = bucket + (size_t)m * bstride;
  u32* out = words + (size_t)m * K;
  for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < K; i += (u64)gridDim.x * blockDim.x) {
    const uint2 wr = tmp[(size_t)m * K + i];
    if (wr.x == S3GD_PAD) continue;
    const u64 pos = (u64)bk[wr.x >> (1 + kBucketShift)] + wr.y;
    if (pos < K) out[pos] = wr.x;  // pos < K by construction
  }
}

// Exclusive scan of a row's bucket counts in three steps, so that many blocks share the work: the
// sum of every chunk of kScanChunk counts, a scan of those sums by one block per row (which also
// yields counts[m]), and the scan inside each chunk started from its chunk's offset.
constexpr int kScanPer = 8;
constexpr u32 kScanChunk = kScanBlock * kScanPer;

__device__ __forceinline__ u32 load_chunk(const u32* __restrict__ t, u32 nb, u32 i0, u32 (&v)[kScanPer]) {
  u32 sum = 0;
#pragma unroll
  for (int k = 0; k < kScanPer; ++k) { v[k] = i0 + k < nb ? t[i0 + k] : 0; sum += v[k]; }
  return sum;
}

__global__ __launch_bounds__(kScanBlock) void k_randk_chunk_sums(const u32* __restrict__ bucket, u32 nb, u32 bstride,
                                                                 u32* __restrict__ sums, u32 sstride) {
  __shared__ u32 lds[kScanBlock / 64];
  const u32 m = blockIdx.y;
  u32 v[kScanPer], total;
  const u32 sum = load_chunk(bucket + (size_t)m * bstride, nb, blockIdx.x * kScanChunk + threadIdx.x * kScanPer, v);
  (void)block_excl_scan<u32>(sum, &total, lds);
  if (threadIdx.x == 0) sums[(size_t)m * sstride + blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanBlock) void k_randk_scan_sums(u32* __restrict__ sums, u32 n_chunks, u32 sstride,
                                                                u32* __restrict__ counts) {
  __shared__ u32 lds[kScanBlock / 64];
  u32* t = sums + (size_t)blockIdx.x * sstride;
  u32 carry = 0;
  for (u32 base = 0; base < n_chunks; base += kScanBlock) {
    const u32 i = base + threadIdx.x;
    const u32 v = i < n_chunks ? t[i] : 0;
    u32 total;
    const u32 ex = carry + block_excl_scan<u32>(v, &total, lds);
    if (i < n_chunks) t[i] = ex;
    carry += total;
  }
  if (threadIdx.x == 0) counts[blockIdx.x] = carry;
}

__global__ __launch_bounds__(kScanBlock) void k_randk_scan_chunks(u32* __restrict__ bucket, u32 nb, u32 bstride,
                                                                  const u32* __restrict__ sums, u32 sstride) {
  __shared__ u32 lds[kScanBlock / 64];
  const u32 m = blockIdx.y;
  u32* t = bucket + (size_t)m * bstride;
  const u32 i0 = blockIdx.x * kScanChunk + threadIdx.x * kScanPer;
  u32 v[kScanPer], total;
  const u32 sum = load_chunk(t, nb, i0, v);
  u32 ex = sums[(size_t)m * sstride + blockIdx.x] + block_excl_scan<u32>(sum, &total, lds);
#pragma unroll
  for (int k = 0; k < kScanPer; ++k) {
    if (i0 + k < nb) t[i0 + k] = ex;
    ex += v[k];
  }
}

// Orders every bucket's words in place.  A lane first takes a bucket of its own: buckets of up to
// kSmall words (the common case at small K/N, where a bucket holds a handful) are ordered in
// registers by that lane alone.  Larger ones (at most kBucket words, all distinct) are then taken
// one after the other by the whole wave, with a bitonic network in the wave's LDS slice.
constexpr int kSmall = 8;

__device__ __forceinline__ void cmp_swap(u32& x, u32& y) {
  const u32 lo = x < y ? x : y, hi = x < y ? y : x;
  x = lo; y = hi;
}

// `starts`: bucket[b] is the first slot of bucket b (and counts[m] the end of the last); otherwise
// bucket[b] is the end of bucket b.
__global__ __launch_bounds__(kBlock) void k_randk_sort(const u32* __restrict__ bucket, u32 nb, u32 bstride, u64 K,
                                                       u32* __restrict__ words, const u32* __restrict__ counts, u32 starts) {
  __shared__ u32 lds_all[kWaves][kBucket];
  const u32 m = blockIdx.y;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  u32* a = lds_all[wave];
  const u32* bk = bucket + (size_t)m * bstride;
  u32* out = words + (size_t)m * K;
  for (u32 base = (blockIdx.x * kWaves + wave) * 64; base < nb; base += gridDim.x * kWaves * 64) {
    const u32 b = base + lane;
    u32 s = 0, n = 0;
    if (b < nb) {
      s = starts ? bk[b] : (b ? bk[b - 1] : 0u);
      u32 e = starts ? (b + 1 < nb ? bk[b + 1] : counts[m]) : bk[b];
      if ((u64)e > K) e = (u32)K;
      if ((u64)s > K) s = (u32)K;
      n = e > s ? e - s : 0u;
    }
    if (n >= 2 && n <= (u32)kSmall) {
      u32 r[kSmall];
#pragma unroll
      for (int i = 0; i < kSmall; ++i) r[i] = (u32)i < n ? out[s + i] : 0xFFFFFFFFu;
      // odd-even merge sorting network for 8 keys (19 comparators)
      cmp_swap(r[0], r[1]); cmp_swap(r[2], r[3]); cmp_swap(r[4], r[5]); cmp_swap(r[6], r[7]);
      cmp_swap(r[0], r[2]); cmp_swap(r[1], r[3]); cmp_swap(r[4], r[6]); cmp_swap(r[5], r[7]);
      cmp_swap(r[1], r[2]); cmp_swap(r[5], r[6]);
      cmp_swap(r[0], r[4]); cmp_swap(r[1], r[5]); cmp_swap(r[2], r[6]); cmp_swap(r[3], r[7]);
      cmp_swap(r[2], r[4]); cmp_swap(r[3], r[5]);
      cmp_swap(r[1], r[2]); cmp_swap(r[3], r[4]); cmp_swap(r[5], r[6]);
#pragma unroll
      for (int i = 0; i < kSmall; ++i)
        if ((u32)i < n) out[s + i] = r[i];
    }
    u64 big = ballot(n > (u32)kSmall);
    while (big) {  // wave-uniform
      const int l = __ffsll((unsigned long long)big) - 1;
      big &= big - 1;
      const u32 bs = __shfl(s, l, 64);
      u32 bn = __shfl(n, l, 64);
      if (bn > kBucket) bn = kBucket;  // cannot happen: a bucket spans kBucket coordinates
      u32 P = 2;
      while (P < bn) P <<= 1;
      for (u32 i = lane; i < P; i += 64) a[i] = i < bn ? out[bs + i] : 0xFFFFFFFFu;
      wave_sync();
      for (u32 k = 2; k <= P; k <<= 1) {
        for (u32 j = k >> 1; j > 0; j >>= 1) {
          for (u32 i = lane; i < P / 2; i += 64) {
            // pair (lo, lo + j) of the block of size 2j that holds the i-th comparator
            const u32 lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
            const u32 hi = lo + j;
            const bool up = (lo & k) == 0;
            const u32 x = a[lo], y = a[hi];
            if ((x > y) == up) { a[lo] = y; a[hi] = x; }
          }
          wave_sync();
        }
      }
      for (u32 i = lane; i < bn; i += 64) out[bs + i] = a[i];
      wave_sync();
    }
  }
}

__global__ void k_randk_pad(const u32* __restrict__ counts, u64 K, u32* __restrict__ words) {
  const u32 m = blockIdx.y;
  u32* out = words + (size_t)m * K;
  for (u64 i = (u64)counts[m] + (u64)blockIdx.x * blockDim.x + threadIdx.x; i < K; i += (u64)gridDim.x * blockDim.x) out[i] = S3GD_PAD;
}

hipError_t launch_randk_encode(const Workspace& ws, const float* grads, u32 M, u64 N, u64 K, u64 seed, u32 t, u32* words,
                               u32* counts, hipStream_t s) {
  Profiler& P = *ws.prof;
  u32* bucket = reinterpret_cast<u32*>(ws.tile_cnt);
  const u32 bstride = coding_blk_stride(N);          // >= N / 2048 + 2 entries per row
  const u32 nb = (u32)((N + kBucket - 1) >> kBucketShift);
  u32 gk = (u32)((K + kBlock - 1) / kBlock);
  const u32 cap = ws.stream_blocks * 2 / M ? ws.stream_blocks * 2 / M : 1;
  if (gk > cap) gk = cap;
  if (gk < 1) gk = 1;
  u32 gb = (nb + kWaves * 64 - 1) / (kWaves * 64);
  if (gb > cap) gb = cap;
  // room for (word, arrival number) of every selected entry in the candidate pool, which this call does not use otherwise?
  const bool ranked = (u64)M * K * sizeof(uint2) <= ws.pool_bytes;
  uint2* tmp = reinterpret_cast<uint2*>(ws.pool);
  P.begin(KID_RANDK, s);
  k_randk_clear<<<dim3((nb + 255) / 256 < 64 ? (nb + 255) / 256 : 64, M), 256, 0, s>>>(bucket, nb, bstride, ws.status, M);
  if (K > 0) {
    if (ranked) k_randk_pass<kRank><<<dim3(gk, M), kBlock, 0, s>>>(grads, N, K, seed, t, bucket, bstride, words, tmp, ws.status);
    else k_randk_pass<kCount><<<dim3(gk, M), kBlock, 0, s>>>(grads, N, K, seed, t, bucket, bstride, words, tmp, ws.status);
  }
  u32* sums = reinterpret_cast<u32*>(ws.blk_sum);    // [M][2 * blk_stride] as u32: far more than n_chunks entries per row
  const u32 sstride = 2 * blk_stride(N);
  const u32 n_chunks = (nb + kScanChunk - 1) / kScanChunk;
  k_randk_chunk_sums<<<dim3(n_chunks, M), kScanBlock, 0, s>>>(bucket, nb, bstride, sums, sstride);
  k_randk_scan_sums<<<M, kScanBlock, 0, s>>>(sums, n_chunks, sstride, counts);
  k_randk_scan_chunks<<<dim3(n_chunks, M), kScanBlock, 0, s>>>(bucket, nb, bstride, sums, sstride);
  if (K > 0) {
    if (ranked) k_randk_place<<<dim3(gk, M), kBlock, 0, s>>>(tmp, K, bucket, bstride, words);
    else k_randk_pass<kScatter><<<dim3(gk, M), kBlock, 0, s>>>(grads, N, K, seed, t, bucket, bstride, words, tmp, ws.status);
    k_randk_sort<<<dim3(gb, M), kBlock, 0, s>>>(bucket, nb, bstride, K, words, counts, ranked ? 1u : 0u);
    k_randk_pad<<<dim3(gk < 64 ? gk : 64, M), 256, 0, s>>>(counts, K, words);
  }
  P.end(s);
  return hipGetLastError();
}

}  // namespace s3gd
