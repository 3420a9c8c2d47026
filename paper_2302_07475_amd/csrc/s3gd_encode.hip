// Worker side of Algorithm 1: batched top-K magnitude selection and sign encoding.
//
// The magnitude order of fp32 values equals the unsigned order of key = bits & 0x7FFFFFFF
// (true for denormals, +-0 and +-Inf).  The K-th largest key T of each row is found by radix
// select over the key's digits; the row then emits, in ascending index, every entry with
// key > T and the first q = K - #{key > T} entries with key == T (Section 2.1 eq. "topk": the
// threshold lies between the K-th and (K+1)-th magnitude; ties go to the lowest index).
#include "s3gd_common.h"
#include "s3gd_kernels.h"

namespace s3gd {

// ------------------------------------------------------------------------------------------------
// state reset (a kernel rather than a memset so that callers may capture the call into a graph)
__global__ void k_encode_init(RowState* rs, u32* hist, u32* status, u32 M, u32 K, u32 mode) {
  const u32 m = blockIdx.y;
  for (u32 i = blockIdx.x * blockDim.x + threadIdx.x; i < (u32)kHistBins; i += gridDim.x * blockDim.x)
    hist[(size_t)m * kHistBins + i] = 0;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    RowState s{};
    s.k_rem = K;
    s.mode = mode;
    rs[m] = s;
    if (m == 0) { status[0] = 0; status[1] = 0; status[2] = M; }
  }
}

// ------------------------------------------------------------------------------------------------
// General path, histogram pass of one radix level over the whole row.
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void k_hist_rows(const float* __restrict__ grads, u64 N, const RowState* __restrict__ rs,
                                                      u32* __restrict__ hist, u32 n_tiles, u32* __restrict__ status) {
  constexpr int NB = 1 << digit_bits(LEVEL);
  constexpr int SH = digit_shift(LEVEL);
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode != kModeGeneral) return;
  __shared__ u32 h[NB];
  for (int i = threadIdx.x; i < NB; i += kBlock) h[i] = 0;
  __syncthreads();
  const float* row = grads + (size_t)m * N;
  const u32 a = (u32)((reinterpret_cast<uintptr_t>(row) >> 2) & 3u);
  const u32* rowv = reinterpret_cast<const u32*>(row) - a;
  const u64 vend = N + a;
  bool nan = false;
  for (u32 tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    TileRegs r;
    load_tile(rowv, a, vend, (u64)tile * kTile, r);
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) {
      const u32 key = r.b[i] & 0x7FFFFFFFu;
      bool take = (r.valid >> i) & 1u;
      if (LEVEL == 0) nan |= take && key > 0x7F800000u;
      if (LEVEL > 0) take = take && (key >> (SH + digit_bits(LEVEL))) == st.prefix;
      if (take) atomicAdd(&h[(key >> SH) & (NB - 1)], 1u);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < NB; i += kBlock) {
    const u32 c = h[i];
    if (c) atomicAdd(&hist[(size_t)m * kHistBins + i], c);
  }
  if (LEVEL == 0 && nan) status[0] = 1;
}

// Picks the digit that holds the sought rank, narrows the prefix and clears the histogram.
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void k_resolve(RowState* rs, u32* hist, u32 K) {
  constexpr int NB = 1 << digit_bits(LEVEL);
  constexpr int PER = NB / kBlock;
  const u32 m = blockIdx.x;
  RowState st = rs[m];
  if (st.mode != kModeGeneral) return;
  __shared__ u32 lds[kWaves];
  u32* h = hist + (size_t)m * kHistBins;
  // thread 0 owns the highest bins
  const int top = NB - 1 - (int)threadIdx.x * PER;
  u32 c[PER];
  u32 s = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) { c[i] = h[top - i]; s += c[i]; }
  u32 total;
  const u32 above = block_excl_scan<u32>(s, &total, lds);
  const u32 k = st.k_rem;
  if (above < k && k <= above + s) {
    u32 acc = above;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      if (acc < k && k <= acc + c[i]) {
        st.prefix = (st.prefix << digit_bits(LEVEL)) | (u32)(top - i);
        st.k_rem = k - acc;
        if (LEVEL == 2) {
          st.T = st.prefix;
          st.q = st.T == 0 ? 0u : st.k_rem;
          st.c_gt = K - st.k_rem;
          st.count = st.c_gt + st.q;
        }
        rs[m] = st;
      }
      acc += c[i];
    }
  }
#pragma unroll
  for (int i = 0; i < PER; ++i) h[top - i] = 0;
}

// Per tile: entries above the threshold and entries equal to it, packed as (eq << 32) | gt.
__global__ __launch_bounds__(kBlock) void k_tile_count(const float* __restrict__ grads, u64 N, const RowState* __restrict__ rs,
                                                       u64* __restrict__ tile_cnt, u32 n_tiles, u32 tile_stride) {
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode != kModeGeneral) return;
  __shared__ u32 lds[2 * kWaves];
  const float* row = grads + (size_t)m * N;
  const u32 a = (u32)((reinterpret_cast<uintptr_t>(row) >> 2) & 3u);
  const u32* rowv = reinterpret_cast<const u32*>(row) - a;
  const u64 vend = N + a;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  for (u32 tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    TileRegs r;
    load_tile(rowv, a, vend, (u64)tile * kTile, r);
    u32 gt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) {
      const u32 key = r.b[i] & 0x7FFFFFFFu;
      const bool ok = (r.valid >> i) & 1u;
      gt += ok && key > st.T;
      eq += ok && key == st.T;
    }
    u32 pk = gt | (eq << 16);  // at most 1024 per wave each
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) pk += __shfl_down(pk, d, 64);
    if (lane == 0) { lds[wave] = pk & 0xFFFFu; lds[kWaves + wave] = pk >> 16; }
    __syncthreads();
    if (threadIdx.x == 0) {
      u32 g = 0, e = 0;
      for (int w = 0; w < kWaves; ++w) { g += lds[w]; e += lds[kWaves + w]; }
      tile_cnt[(size_t)m * tile_stride + tile] = ((u64)e << 32) | g;
    }
    __syncthreads();
  }
}

// In-place exclusive scan of a row's packed tile counts; entry n_tiles receives the row total.
__global__ __launch_bounds__(kScanBlock) void k_scan_tiles(u64* __restrict__ tile_cnt, u32 n_tiles, u32 tile_stride) {
  __shared__ u64 lds[kScanBlock / 64];
  u64* t = tile_cnt + (size_t)blockIdx.x * tile_stride;
  u64 carry = 0;
  for (u32 base = 0; base < n_tiles; base += kScanBlock * 4) {
    const u32 i0 = base + threadIdx.x * 4;
    u64 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = (i0 + k < n_tiles) ? t[i0 + k] : 0;
    const u64 s = v[0] + v[1] + v[2] + v[3];
    u64 total;
    u64 ex = carry + block_excl_scan<u64>(s, &total, lds);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (i0 + k < n_tiles) t[i0 + k] = ex;
      ex += v[k];
    }
    carry += total;
  }
  if (threadIdx.x == 0) t[n_tiles] = carry;
}

// Emits the words of every tile at its scanned offset, in ascending index.
__global__ __launch_bounds__(kBlock) void k_emit_rows(const float* __restrict__ grads, u64 N, u64 K, const RowState* __restrict__ rs,
                                                      const u64* __restrict__ tile_cnt, u32 n_tiles, u32 tile_stride,
                                                      u32* __restrict__ words) {
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode != kModeGeneral) return;
  __shared__ u32 lds[kLoads * kWaves];
  const float* row = grads + (size_t)m * N;
  const u32 a = (u32)((reinterpret_cast<uintptr_t>(row) >> 2) & 3u);
  const u32* rowv = reinterpret_cast<const u32*>(row) - a;
  const u64 vend = N + a;
  const u64* tc = tile_cnt + (size_t)m * tile_stride;
  u32* out = words + (size_t)m * K;
  for (u32 tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const u64 c0 = tc[tile], c1 = tc[tile + 1];
    const u32 gt_before = (u32)c0, eq_before = (u32)(c0 >> 32);
    const u32 gt_here = (u32)c1 - gt_before, eq_here = (u32)(c1 >> 32) - eq_before;
    const u32 ties_open = st.q > eq_before ? st.q - eq_before : 0u;  // tie slots left for this tile onwards
    const u32 ties_here = ties_open < eq_here ? ties_open : eq_here;
    if (gt_here + ties_here == 0) continue;  // block-uniform
    TileRegs r;
    load_tile(rowv, a, vend, (u64)tile * kTile, r);
    u32 gt_mask = 0, eq_mask = 0;
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) {
      const u32 key = r.b[i] & 0x7FFFFFFFu;
      const bool ok = (r.valid >> i) & 1u;
      gt_mask |= (u32)(ok && key > st.T) << i;
      eq_mask |= (u32)(ok && key == st.T) << i;
    }
    u32 sel = gt_mask;
    if (ties_here) {  // block-uniform
      if (ties_here == eq_here) {
        sel |= eq_mask;
      } else {
        u32 base[kLoads], total;
        tile_rank(eq_mask, base, &total, lds);
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
          u32 rk = base[j];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const u32 bit = 1u << (4 * j + e);
            if (eq_mask & bit) { if (rk < ties_here) sel |= bit; ++rk; }
          }
        }
      }
    }
    u32 base[kLoads], total;
    tile_rank(sel, base, &total, lds);
    const u32 o0 = gt_before + (eq_before < st.q ? eq_before : st.q);
    const u64 v0 = (u64)tile * kTile + (u64)threadIdx.x * 4 - a;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      u32 o = o0 + base[j];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = 4 * j + e;
        if ((sel >> i) & 1u) {
          const u32 n = (u32)(v0 + (u64)j * (kBlock * 4) + e);
          if (o < K) out[o] = (n << 1) | (r.b[i] >> 31);  // o < K by construction; guards a racing writer of grads
          ++o;
        }
      }
    }
  }
}

// counts[m] and the pad words of rows that selected zeros.
__global__ void k_finish_rows(const RowState* __restrict__ rs, u64 K, u32* __restrict__ words, u32* __restrict__ counts,
                              u32* __restrict__ status) {
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    counts[m] = st.count;
    if (st.mode == kModeGeneral) atomicAdd(&status[1], 1u);
  }
  u32* out = words + (size_t)m * K;
  for (u64 i = (u64)st.count + blockIdx.x * blockDim.x + threadIdx.x; i < K; i += (u64)gridDim.x * blockDim.x)
    out[i] = S3GD_PAD;
}

__global__ void k_zero_counts(u32* counts, u32 M) {
  const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < M) counts[i] = 0;
}

// ------------------------------------------------------------------------------------------------
hipError_t launch_encode(const Workspace& ws, const float* grads, u32 M, u64 N, u64 K, u32* words, u32* counts,
                         hipStream_t s) {
  if (K == 0) {
    k_zero_counts<<<(M + 255) / 256, 256, 0, s>>>(counts, M);
    return hipGetLastError();
  }
  const u32 n_tiles = encode_tiles(N);
  const u32 stride = tile_stride(N);
  u32 gx = (kTargetBlocks + M - 1) / M;
  if (gx > n_tiles) gx = n_tiles;
  if (gx < 1) gx = 1;
  const dim3 grid(gx, M);
  Profiler& P = *ws.prof;
#define S3GD_LAUNCH(KID, ...) do { P.begin(KID, s); __VA_ARGS__; P.end(s); } while (0)
  S3GD_LAUNCH(KID_ENCODE_INIT, (k_encode_init<<<dim3(2, M), 256, 0, s>>>(ws.rs, ws.hist, ws.status, M, (u32)K, kModeGeneral)));
  S3GD_LAUNCH(KID_HIST0, (k_hist_rows<0><<<grid, kBlock, 0, s>>>(grads, N, ws.rs, ws.hist, n_tiles, ws.status)));
  S3GD_LAUNCH(KID_RESOLVE, (k_resolve<0><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, (u32)K)));
  S3GD_LAUNCH(KID_HIST1, (k_hist_rows<1><<<grid, kBlock, 0, s>>>(grads, N, ws.rs, ws.hist, n_tiles, ws.status)));
  S3GD_LAUNCH(KID_RESOLVE, (k_resolve<1><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, (u32)K)));
  S3GD_LAUNCH(KID_HIST2, (k_hist_rows<2><<<grid, kBlock, 0, s>>>(grads, N, ws.rs, ws.hist, n_tiles, ws.status)));
  S3GD_LAUNCH(KID_RESOLVE, (k_resolve<2><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, (u32)K)));
  S3GD_LAUNCH(KID_TILE_COUNT, (k_tile_count<<<grid, kBlock, 0, s>>>(grads, N, ws.rs, ws.tile_cnt, n_tiles, stride)));
  S3GD_LAUNCH(KID_SCAN_TILES, (k_scan_tiles<<<M, kScanBlock, 0, s>>>(ws.tile_cnt, n_tiles, stride)));
  S3GD_LAUNCH(KID_EMIT, (k_emit_rows<<<grid, kBlock, 0, s>>>(grads, N, K, ws.rs, ws.tile_cnt, n_tiles, stride, words)));
  u32 fx = (u32)((K + 4095) / 4096);
  if (fx > 64) fx = 64;
  S3GD_LAUNCH(KID_FINISH, (k_finish_rows<<<dim3(fx, M), 256, 0, s>>>(ws.rs, K, words, counts, ws.status)));
#undef S3GD_LAUNCH
  return hipGetLastError();
}

}  // namespace s3gd
