// Worker side of Algorithm 1: batched top-K magnitude selection and sign encoding.
//
// The magnitude order of fp32 values equals the unsigned order of key = bits & 0x7FFFFFFF
// (true for denormals, +-0 and +-Inf).  The K-th largest key T of each row is found by radix
// select over the key's digits; the row then emits, in ascending index, every entry with
// key > T and the first q = K - #{key > T} entries with key == T (Section 2.1 eq. "topk": the
// threshold lies between the K-th and (K+1)-th magnitude; ties go to the lowest index).
//
// Two routes reach the same T, q and words:
//   candidate route  a strided sample of the row gives a lower bound L with, very likely,
//                    K <= #{key >= L} <= capacity.  ONE pass over the row copies those candidates
//                    (index, bits) into per-wave segments of a pool and histograms them; T is then
//                    resolved and the words are emitted from the candidates alone.
//                    If the K-th key lies far above L (a row whose magnitudes are spread widely
//                    around the threshold) the radix select simply runs over the candidates.
//                    At dense sparsity levels (K > N/16) the pass keeps only a bracket of keys above L
//                    and counts the entries above it; the words then come from a second pass over the
//                    row (two reads).  K = N selects nothing: count and emit (two reads).
//   general route    three histogram passes over the row (11 + 10 + 10 key bits), a per-tile count
//                    pass and an emit pass.  Any row for which the candidate route's checks fail
//                    (too few or too many candidates, tiny rows) takes it; the choice is made on
//                    the device, per row, with no host synchronisation.
#include <math.h>

#include "s3gd_common.h"
#include "s3gd_kernels.h"

namespace s3gd {

// ------------------------------------------------------------------------------------------------
// Error-compensation memory (Section 2.2 "Gradient update with sparsification error compensation";
// Algorithm 1, the two lines before "send"): the row that is compressed is g = g~ + eta * e, and the
// memory becomes e' = g - TopK(g), i.e. g off the selected set and zero on it.  With a memory the
// encode keeps g IN the memory buffer: the single pass over the row writes e <- g while it filters,
// and the emit kernels write +0.0 over every entry whose sign they send.  The general route then
// simply reads the memory buffer as its gradient row.
//
// g is evaluated in fp32 as written: a rounded product, then a rounded sum (no fused multiply-add).
__device__ __forceinline__ u32 compensate_bits(u32 g_tilde, u32 e, float eta) {
  return __float_as_uint(__fadd_rn(__uint_as_float(g_tilde), __fmul_rn(eta, __uint_as_float(e))));
}

__device__ __forceinline__ void store_stream16(u32* p, u32 a, u32 b, u32 c, u32 d) {
  u32x4 q; q.x = a; q.y = b; q.z = c; q.w = d;
  __builtin_nontemporal_store(q, reinterpret_cast<u32x4*>(p));
}

// e <- g~ + eta * e over the flat [M * N] array (rows are contiguous).  Used when no row of the call
// goes through the filter pass (tiny rows, a pool too small for the plan, K = 0).  `head` = elements before the first
// 16-byte boundary, the same for both arrays.
__global__ __launch_bounds__(kBlock) void k_compensate(const float* __restrict__ g_tilde, float* __restrict__ err, float eta, u64 total,
                                                       u32 head) {
  const u32* gt = reinterpret_cast<const u32*>(g_tilde);
  u32* e = reinterpret_cast<u32*>(err);
  const u64 tid = (u64)blockIdx.x * blockDim.x + threadIdx.x, nthr = (u64)gridDim.x * blockDim.x;
  const u64 h = head < total ? head : total;
  const u64 n4 = (total - h) / 4;
  for (u64 i = tid; i < n4; i += nthr) {
    const u64 o = h + i * 4;
    const uint4 a = load_stream16(gt + o), b = load_stream16(e + o);
    store_stream16(e + o, compensate_bits(a.x, b.x, eta), compensate_bits(a.y, b.y, eta), compensate_bits(a.z, b.z, eta),
                   compensate_bits(a.w, b.w, eta));
  }
  if (tid < h) e[tid] = compensate_bits(gt[tid], e[tid], eta);
  const u64 t0 = h + n4 * 4;
  if (t0 + tid < total) e[t0 + tid] = compensate_bits(gt[t0 + tid], e[t0 + tid], eta);
}

// ------------------------------------------------------------------------------------------------
// state reset (a kernel rather than a memset so that callers may capture the call into a graph)
__global__ void k_encode_init(RowState* rs, u32* hist, u32* status, u32 M, u32 first_rank, u32 mode, u32 first_alloc, u32 bracket, u32 all_selected) {
  const u32 m = blockIdx.y;
  for (u32 i = blockIdx.x * blockDim.x + threadIdx.x; i < (u32)kHistBins; i += gridDim.x * blockDim.x)
    hist[(size_t)m * kHistBins + i] = 0;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    RowState s{};
    s.k_rem = first_rank;  // K on the general route, the sample rank on the candidate route
    s.mode = mode;
    s.n_alloc = first_alloc;  // candidate slots already handed out: the first slab of every wave of the filter pass
    s.bracket = bracket;
    s.row_emit = all_selected ? 2u : 0u;  // K = N: threshold 0, no tie slots (the zero-filled T and q), count from the scan
    rs[m] = s;
    if (m == 0) { status[0] = 0; status[1] = 0; status[2] = M; status[4] = 0; status[5] = 0; status[6] = 0; status[7] = 0; }
  }
}

// ------------------------------------------------------------------------------------------------
// The candidates of a row, as the filter pass left them: a table of segment lists, each of at most
// kChain segments (first slot, count) of the row's pool.  Lists in order and segments in order
// enumerate the candidates in ascending index.  A ListWalk numbers the candidates of one list
// 0 .. total-1 across its segments, so that a wave takes them 64 (or more) at a time whatever the
// segment lengths are: a list may be two long slabs or eight short runs.
struct ListWalk {
  u32 first[kChain], count[kChain], slot[kChain];  // flat number of a segment's first candidate, its length, its first slot
  u32 total;
  bool single;  // the whole list is one run of the pool (the usual case: the wave's first slab sufficed); wave-uniform
  const uint2* pool;
  __device__ ListWalk(const u64* __restrict__ wave_seg, const u32* __restrict__ wave_nseg, u32 wave_stride, const uint2* cand,
                      u32 cand_stride, u32 m, u32 g)
      : total(0), pool(cand + (size_t)m * cand_stride) {
    const u64* segs = wave_seg + ((size_t)m * wave_stride + g) * kChain;
    const u32 n_seg = wave_nseg[(size_t)m * wave_stride + g];
#pragma unroll
    for (int c = 0; c < kChain; ++c) {
      const u64 sg = segs[c];  // the whole line is loaded; entries past n_seg are stale
      slot[c] = (u32)(sg >> 32);
      count[c] = (u32)c < n_seg ? (u32)sg : 0u;
      first[c] = total;
      total += count[c];
    }
    single = __builtin_amdgcn_readfirstlane(n_seg <= 1u ? 1 : 0) != 0;
  }
  // pool slot of candidate j < total
  __device__ __forceinline__ u32 locate(u32 j) const {
    if (single) return slot[0] + j;
    u32 at = 0;
#pragma unroll
    for (int c = 0; c < kChain; ++c) {
      const u32 d = j - first[c];  // wraps to a huge value for candidates of earlier segments
      if (d < count[c]) at = slot[c] + d;
    }
    return at;
  }
};
constexpr int kWalk = 4;  // candidates a lane has in flight where their order does not matter

// Adds one to h[bin] for every lane with `take`.  Where most lanes of a wave add to ONE bin (the
// rows of the general route are mostly degenerate ones: mostly zeros, all equal, heavy ties) LDS
// serialises them: the lanes that share the first lane's bin add once, through that lane, when
// there are at least eight of them.  (Over the candidates of a row, which share their leading
// digits, the same was measured to gain nothing.)
__device__ __forceinline__ void hist_add(u32* h, u32 bin, bool take) {
  const u32 b0 = __builtin_amdgcn_readfirstlane(take ? bin : 0xFFFFFFFFu);
  const bool same = take && bin == b0;
  const u64 sm = ballot(same);
  const u32 n_same = (u32)__popcll(sm);
  if (n_same >= 8u) {  // wave-uniform
    if (same) {
      if (ballot_rank(sm) == 0) atomicAdd(&h[b0], n_same);
    } else if (take) {
      atomicAdd(&h[bin], 1u);
    }
  } else if (take) {
    atomicAdd(&h[bin], 1u);
  }
}

// Histogram pass of one radix level (11 + 10 + 10 key bits, most significant first).
//   general rows            over the whole row
//   wide candidate rows     over the row's candidates, every level
//   other candidate rows    over the candidates at the last level only: the filter pass has already
//                           fixed the upper 21 bits
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void k_hist_rows(const float* __restrict__ grads, u64 N, const RowState* __restrict__ rs,
                                                      u32* __restrict__ hist, u32 n_tiles, u32* __restrict__ status,
                                                      const uint2* __restrict__ cand, u32 cand_stride, const u64* __restrict__ wave_seg,
                                                      const u32* __restrict__ wave_nseg, u32 wave_stride, u32 n_waves, u32 parts) {
  constexpr int NB = 1 << digit_bits(LEVEL);
  constexpr int SH = digit_shift(LEVEL);
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode == kModeCandidates && LEVEL != 2) return;
  __shared__ u32 h[NB];
  for (int i = threadIdx.x; i < NB; i += kBlock) h[i] = 0;
  __syncthreads();
  bool nan = false;
  if (st.mode == kModeGeneral) {
    const float* row = grads + (size_t)m * N;
    const u32 a = (u32)((reinterpret_cast<uintptr_t>(row) >> 2) & 3u);
    const u32* rowv = reinterpret_cast<const u32*>(row) - a;
    const u64 vend = N + a;
    for (u32 tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
      TileRegs r;
      load_tile(rowv, a, vend, (u64)tile * kTile, r);
#pragma unroll
      for (int i = 0; i < kLoads * 4; ++i) {
        const u32 key = r.b[i] & 0x7FFFFFFFu;
        bool take = (r.valid >> i) & 1u;
        if (LEVEL == 0) nan |= take && key > 0x7F800000u;
        if (LEVEL > 0) take = take && (key >> (SH + digit_bits(LEVEL))) == st.prefix;
        hist_add(h, (key >> SH) & (NB - 1), take);
      }
    }
  } else {  // `parts` waves per segment list, each with a share of its candidates (their order does not matter here)
    const u32 lane = lane_id();
    for (u32 w = blockIdx.x * kWaves + (threadIdx.x >> 6); w < n_waves * parts; w += gridDim.x * kWaves) {
      const u32 g = w / parts, part = w - g * parts;
      const ListWalk lw(wave_seg, wave_nseg, wave_stride, cand, cand_stride, m, g);
      const u32 share = ((lw.total + parts - 1) / parts + 63u) & ~63u;
      const u32 lo = part * share;
      const u32 hi = lo + share < lw.total ? lo + share : lw.total;
      for (u32 i0 = lo + lane; i0 < hi; i0 += 64 * kWalk) {
        u32 key[kWalk];
#pragma unroll
        for (int u = 0; u < kWalk; ++u) {
          const u32 j = i0 + (u32)u * 64u;
          key[u] = j < hi ? (lw.pool[lw.locate(j)].y & 0x7FFFFFFFu) : 0xFFFFFFFFu;
        }
#pragma unroll
        for (int u = 0; u < kWalk; ++u)
          if (key[u] != 0xFFFFFFFFu && (LEVEL == 0 || (key[u] >> (SH + digit_bits(LEVEL))) == st.prefix))
            atomicAdd(&h[(key[u] >> SH) & (NB - 1)], 1u);
      }
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
//   kResolveRadix      a level of the radix select filled by k_hist_rows: every level for general
//                      and wide candidate rows, the last level for the other candidate rows
//   kResolveSample     levels 0..1 over the sample: ends with L = 21-bit prefix << 10
//   kResolveFilter     2048 bins of (key - L) >> 10 filled by the filter pass: checks the candidate
//                      route and fixes the 21-bit prefix, or starts a radix select over the
//                      candidates (K-th key in the open top bin), or hands the row to the general route
// `have_bins` is 0 when the filter pass is the chunked one (with a memory): that pass fills no bins
// (kResolveFilter), and it must run over every row to form g, so no row leaves the candidate route
// before it (kResolveSample).
enum { kResolveRadix = 0, kResolveSample = 1, kResolveFilter = 2 };

template <int LEVEL, int WHAT>
__global__ __launch_bounds__(kBlock) void k_resolve(RowState* rs, u32* hist, u32 K, u32 have_bins, u32 sample_cap, u32* status) {
  constexpr int NB = WHAT == kResolveFilter ? kHistBins : (1 << digit_bits(LEVEL));
  constexpr int PER = NB / kBlock;
  const u32 m = blockIdx.x;
  RowState st = rs[m];
  if (WHAT == kResolveRadix ? (st.mode == kModeCandidates && LEVEL != 2) : (st.mode != kModeCandidates)) return;
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
#pragma unroll
  for (int i = 0; i < PER; ++i) h[top - i] = 0;
  // With a bracket the n_sure entries above it come first in the order: the K-th overall is the
  // (K - n_sure)-th of the candidates (n_sure is 0 without a bracket).
  const u32 k = WHAT == kResolveFilter ? (K > st.n_sure ? K - st.n_sure : 0u) : st.k_rem;
  if (WHAT == kResolveFilter) {
    // The candidate route stands only if no wave ran out of room and the K-th largest key is among
    // the candidates.  If it sits in the open-ended top bin (thread 0's c[0]) the bins say nothing
    // about it: the radix select then starts over, among the candidates.
    __shared__ u32 verdict;
    // (A filter pass in chunks fills no bins: its candidates are the slots it handed out.)
    if (!have_bins) st.n_cand = st.n_alloc;
    if (threadIdx.x == 0) {
      const bool usable = !st.overflow && k >= 1 && st.n_cand >= k && (!have_bins || total == st.n_cand);
      // a bracket has no way on if the K-th key lies above it (k == 0): those entries were not kept
      // (with bins; without them the radix select over the candidates finds the (K - n_sure)-th)
      verdict = usable ? ((have_bins && c[0] < k) ? 2u : ((st.bracket && have_bins) ? 0u : 1u)) : 0u;
    }
    __syncthreads();
    if (verdict != 2u) {
      if (threadIdx.x == 0) {
        st.mode = verdict ? kModeCandWide : kModeGeneral;
        st.prefix = 0;
        st.k_rem = verdict ? k : K;
        rs[m] = st;
      }
      return;
    }
  }
  if (above < k && k <= above + s) {
    u32 acc = above;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      if (acc < k && k <= acc + c[i]) {
        const u32 digit = (u32)(top - i);
        if (WHAT == kResolveFilter) st.prefix = (st.L >> 10) + digit;
        else st.prefix = (st.prefix << digit_bits(LEVEL)) | digit;
        st.k_rem = k - acc;
        if (WHAT == kResolveSample && LEVEL == 1) {
          st.L = st.prefix << 10;
          st.prefix = 0;
          st.k_rem = K;
          // L = 0: the sample holds fewer than its share of non-zero entries (a mostly-zero row with K
          // above its non-zeros), every entry would be a candidate.  The row goes to the general route
          // before the filter pass instead of after it, unless that pass must still form g in the memory.
          if (st.L == 0 && have_bins) st.mode = kModeGeneral;
          // Likewise a row with so many entries at or above L that they cannot fit its share of the
          // pool (all entries equal, heavy ties at the threshold): `sample_cap` is the number of
          // sampled entries that stands for a full pool (0: no such check).
          if (sample_cap && have_bins && acc + c[i] > sample_cap) st.mode = kModeGeneral;
          if (st.mode == kModeGeneral) atomicAdd(&status[7], 1u);
        }
        if (LEVEL == 2) {
          st.T = st.prefix;
          st.q = st.T == 0 ? 0u : st.k_rem;
          st.c_gt = K - st.k_rem;
          st.count = st.c_gt + st.q;
          if (st.mode == kModeCandidates && st.bracket) {
            st.mode = kModeRangeEmit;  // the candidates do not hold every selected entry: a second pass over the waves' ranges emits
          } else if (st.mode == kModeCandWide && st.bracket) {
            st.mode = kModeGeneral;    // chunked pass: the row passes count and emit with this T
            st.row_emit = 1;
          }
        }
        rs[m] = st;
      }
      acc += c[i];
    }
  }
}

// Per tile: entries above the threshold and entries equal to it, packed as (eq << 32) | gt.
__global__ __launch_bounds__(kBlock) void k_tile_count(const float* __restrict__ grads, u64 N, const RowState* __restrict__ rs,
                                                       u64* __restrict__ tile_cnt, u32 n_tiles, u32 tile_stride,
                                                       u32* __restrict__ status) {
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
    bool nan = false;
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) {
      const u32 key = r.b[i] & 0x7FFFFFFFu;
      const bool ok = (r.valid >> i) & 1u;
      gt += ok && key > st.T;
      eq += ok && key == st.T;
      nan |= ok && key > 0x7F800000u;
    }
    if (nan) status[0] = 1;  // the only pass that sees every entry when K = N skips the radix select
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
__global__ __launch_bounds__(kScanBlock) void k_scan_tiles(u64* __restrict__ tile_cnt, u32 n_tiles, u32 tile_stride,
                                                           RowState* __restrict__ rs, u32 candidate_rows) {
  if ((rs[blockIdx.x].mode != kModeGeneral) != (candidate_rows != 0)) return;
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
  if (threadIdx.x == 0) {
    t[n_tiles] = carry;
    if (!candidate_rows && rs[blockIdx.x].row_emit == 2u) {  // K = N: every non-zero entry is sent
      rs[blockIdx.x].c_gt = (u32)carry;
      rs[blockIdx.x].count = (u32)carry;
    }
  }
}

// Emits the words of every tile at its scanned offset, in ascending index.
// With a memory (`err` non-NULL) `grads` IS the memory buffer holding g, and every entry whose sign
// is sent is overwritten with +0.0; a tile is read and rewritten by the same block only.
__global__ __launch_bounds__(kBlock) void k_emit_rows(const float* grads, u64 N, u64 K, const RowState* __restrict__ rs,
                                                      const u64* __restrict__ tile_cnt, u32 n_tiles, u32 tile_stride,
                                                      u32* __restrict__ words, float* err) {
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
    if (err) {
      // +0.0 over every entry whose sign is sent.  Four lanes share 64 bytes of the row: if one of them
      // has such an entry all four rewrite their 16 bytes (memory merges a smaller write by reading
      // first; with dense K nearly every run is touched).  Groups that reach outside the row store
      // their selected entries one by one.
      u32* erow = reinterpret_cast<u32*>(err + (size_t)m * N) - a;
      const u32 lane = lane_id();
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        const u32 s4 = (sel >> (4 * j)) & 0xFu, ok4 = (r.valid >> (4 * j)) & 0xFu;
        const u64 live = ballot(s4 != 0);
        if (((live >> (lane & 60u)) & 0xFull) == 0) continue;
        u32* p = erow + (u64)tile * kTile + (u64)j * (kBlock * 4) + (u64)threadIdx.x * 4;
        if (ok4 == 0xFu) {
          *reinterpret_cast<uint4*>(p) = make_uint4((s4 & 1u) ? 0u : r.b[4 * j], (s4 & 2u) ? 0u : r.b[4 * j + 1],
                                                    (s4 & 4u) ? 0u : r.b[4 * j + 2], (s4 & 8u) ? 0u : r.b[4 * j + 3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if ((s4 >> e) & 1u) p[e] = 0u;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Candidate route.

// Position of sample unit u of a row: one unit per stride window, at a hashed offset inside it,
// so that a periodic pattern in the row cannot line up with the sample.
__host__ __device__ __forceinline__ u64 sample_unit_start(u32 u, u64 stride) {
  u32 h = u * 0x9E3779B1u;
  h ^= h >> 15; h *= 0x85EBCA77u; h ^= h >> 13;
  return (u64)u * stride + (u64)h % (stride - (kSampleUnit - 1));
}

u64 sample_unit_position(u32 u, u64 stride) { return sample_unit_start(u, stride); }

// Histogram of one radix level over the sample of each row (gathered straight from the row).
// With a memory (`err` non-NULL) the sampled value is g~ + eta * e.
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void k_sample_hist(const float* __restrict__ grads, const float* __restrict__ err, float eta, u64 N,
                                                        const RowState* __restrict__ rs, u32* __restrict__ hist, u32 n_units,
                                                        u64 unit_stride) {
  constexpr int NB = 1 << digit_bits(LEVEL);
  constexpr int SH = digit_shift(LEVEL);
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode != kModeCandidates) return;
  __shared__ u32 h[NB];
  for (int i = threadIdx.x; i < NB; i += kBlock) h[i] = 0;
  __syncthreads();
  const u32* row = reinterpret_cast<const u32*>(grads + (size_t)m * N);
  const u32* erow = err ? reinterpret_cast<const u32*>(err + (size_t)m * N) : nullptr;
  const u32 n_samples = n_units * kSampleUnit;
#pragma unroll 4
  for (u32 i = blockIdx.x * kSamplePerBlock + threadIdx.x; i < (blockIdx.x + 1) * kSamplePerBlock && i < n_samples; i += kBlock) {
    const u32 u = i / kSampleUnit, e = i % kSampleUnit;
    const u64 pos = sample_unit_start(u, unit_stride) + e;
    u32 bits = row[pos];
    if (erow) bits = compensate_bits(bits, erow[pos], eta);
    const u32 key = bits & 0x7FFFFFFFu;
    if (LEVEL == 0 || (key >> (SH + digit_bits(LEVEL))) == st.prefix) atomicAdd(&h[(key >> SH) & (NB - 1)], 1u);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < NB; i += kBlock) {
    const u32 c = h[i];
    if (c) atomicAdd(&hist[(size_t)m * kHistBins + i], c);
  }
}

// The one pass over the gradients: every entry with key >= L becomes a candidate (index, bits).
// Waves work independently (no block barrier inside the loop): a wave owns a contiguous run of
// wave tiles (1024 entries each) and appends its candidates, in ascending index, to slabs of the
// row's candidate pool.  What a wave leaves behind is its SEGMENT LIST: up to kChain pairs
// (first slot, count), written once when the wave ends.  Waves in order, and each wave's segments
// in order, list the row's candidates in ascending index; the kernels after the pass walk them
// that way, one wave per list.  The block also histograms (key - L) >> 10 into 2048 bins, the
// last of which is open-ended.
//
// Slabs.  Every wave starts with a slab of its own, assigned by position (no atomic), sized to
// about twice the candidates a wave expects; only a wave that fills it (skewed rows) reserves
// another, twice as large each time, with a returning atomic on the row's counter.  A wave that
// would need more than kChain segments (more than a hundred times its share) marks the row for
// the general route.  Those atomics are what must stay rare:
// all waves of a row hit ONE address, a few thousand of them per millisecond queue up behind each
// other, and a wave waiting for its atomic also waits for its prefetched tile (measured with
// 256-entry slabs reserved on demand: 26 000 atomics cost 0.4 ms of a 3.2 ms pass).
//
// Stores are rare and non-temporal: on this memory system ANY store traffic mixed into the read
// stream costs several per cent of read bandwidth, whatever its volume (measured: one 8-byte store
// per 4 KB read, or one 512-byte store per 256 KB read, both cost 9 %; non-temporal stores issued
// every 2 MB read cost 2.5 %).  So candidates are staged in LDS and written about nine hundred at a
// time, and nothing else is stored per tile.
constexpr int kStage = 1024;       // staged candidates per wave
constexpr int kStageFlush = 896;   // flush once this many are staged

struct FilterWave {
  u32 cur, end, total;  // slab cursor, slab end, candidates so far (wave-uniform)
  u32 fill;             // candidates staged in LDS; they belong to out[cur - fill, cur)
  u32 seg_base, n_seg;  // first slot of the segment being filled; segments already closed
  u64* segs;            // the wave's segment list in global memory, kChain entries
  u32 sure;  // bracket: entries at or above the bracket's upper end seen by this wave
  bool overflow, nan;
};

// Ends the segment being filled: its (first slot, count) goes to the wave's list.
__device__ __forceinline__ void close_segment(FilterWave& w, u32 lane) {
  const u32 count = w.cur - w.seg_base;
  if (count == 0) return;  // wave-uniform
  if (w.n_seg < (u32)kChain) {
    if (lane == 0) w.segs[w.n_seg] = ((u64)w.seg_base << 32) | count;
    ++w.n_seg;
  } else {
    w.overflow = true;
  }
}

__device__ __forceinline__ void store_stream8(u64* p, u64 v) { __builtin_nontemporal_store(v, p); }

// Writes the staged candidates to the wave's slab and enters them into the block's bins.  Binning
// here, a candidate per lane, rather than where a candidate is found (a lane or two at a time under
// its own branch) takes the bin arithmetic and the NaN test out of the per-tile code: a quarter of
// the pass's instructions once a tile holds ten candidates (K = N / 100).
__device__ __forceinline__ void flush_stage(FilterWave& w, const u64* stage, uint2* __restrict__ out, u32 lane, u32 L, u32* h) {
  __builtin_amdgcn_wave_barrier();
  u64* dst = reinterpret_cast<u64*>(out) + (w.cur - w.fill);
  const u32 Lq = L >> 10;
  for (u32 i = lane; i < w.fill; i += 64) {
    const u64 cd = stage[i];
    store_stream8(dst + i, cd);
    const u32 key = (u32)(cd >> 32) & 0x7FFFFFFFu;
    w.nan |= key > 0x7F800000u;
    const u32 bin = (key >> 10) - Lq;
    // the open top bin takes most candidates of a heavy-tailed row: one add per wave for those
    const bool top = bin >= (u32)kHistBins - 1;
    const u64 tm = ballot(top);
    if (!top) atomicAdd(&h[bin], 1u);
    else if (ballot_rank(tm) == 0) atomicAdd(&h[kHistBins - 1], (u32)__popcll(tm));
  }
  __builtin_amdgcn_wave_barrier();
  w.fill = 0;
}

// Writes the candidates of one tile, in ascending index, to the LDS stage or (DIRECT) to memory.
template <bool DIRECT, bool BINS, bool NANS>
__device__ __forceinline__ void place_candidates(const TileRegs& r, const bool (&pr)[kLoads * 4], const u64 (&mk)[kLoads * 4],
                                                 const u32 (&tot)[kLoads], u32 first_slot, u64 v0, u32 L, u32* h,
                                                 uint2* __restrict__ dst_global, u64* dst_stage, bool& nan) {
  const u32 Lq = L >> 10;
  u32 run = first_slot;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    if (tot[j] == 0) continue;  // wave-uniform
    // candidates of load j in lower lanes, then this lane's own in ascending e
    u32 o = run + ballot_rank(mk[4 * j]) + ballot_rank(mk[4 * j + 1]) + ballot_rank(mk[4 * j + 2]) + ballot_rank(mk[4 * j + 3]);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = 4 * j + e;
      if (pr[i]) {
        const u32 key = r.b[i] & 0x7FFFFFFFu;
        const uint2 cd = make_uint2((u32)(v0 + (u64)j * 256 + e), r.b[i]);
        if (DIRECT) dst_global[o] = cd; else dst_stage[o] = ((u64)cd.y << 32) | cd.x;
        ++o;
        if (NANS) nan |= key > 0x7F800000u;
        if (BINS) {
          const u32 bin = (key >> 10) - Lq;
          atomicAdd(&h[bin < (u32)kHistBins - 1 ? bin : (u32)kHistBins - 1], 1u);
        }
      }
    }
    run += tot[j];
  }
}

// INTERIOR tiles lie wholly inside the row: their loads are branch-free.
template <bool INTERIOR>
__device__ __forceinline__ void load_filter_tile(const u32* __restrict__ rowv, u32 a, u64 vend, u32 tile, u32 lane, TileRegs& r) {
  const u64 vbase = (u64)tile * kWaveTile;
  if (INTERIOR) {
    uint4 q[kLoads];
#pragma unroll
    for (int j = 0; j < kLoads; ++j) q[j] = load_stream16(rowv + vbase + (u64)j * 256 + (u64)lane * 4);
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
      r.b[4 * j + 0] = q[j].x; r.b[4 * j + 1] = q[j].y; r.b[4 * j + 2] = q[j].z; r.b[4 * j + 3] = q[j].w;
    }
    r.valid = 0xFFFFu;
  } else {
    r.valid = 0;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) load_edge4(rowv, a, vend, vbase + (u64)j * 256 + (u64)lane * 4, j, r);
  }
}

// Writes a wave tile back over the row it was loaded from (the memory row receiving g).
template <bool INTERIOR>
__device__ __forceinline__ void store_filter_tile(u32* __restrict__ rowv, u32 tile, u32 lane, const TileRegs& r) {
  const u64 vbase = (u64)tile * kWaveTile;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    u32* p = rowv + vbase + (u64)j * 256 + (u64)lane * 4;
    if (INTERIOR || ((r.valid >> (4 * j)) & 0xFu) == 0xFu) {
      store_stream16(p, r.b[4 * j], r.b[4 * j + 1], r.b[4 * j + 2], r.b[4 * j + 3]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if ((r.valid >> (4 * j + e)) & 1u) p[e] = r.b[4 * j + e];
    }
  }
}

template <bool INTERIOR, bool BRACKET>
__device__ __forceinline__ void filter_tile(const TileRegs& r, u32 a, u32 tile, u32 lane, u32 L, u32* h, u64* stage, u32* n_alloc,
                                            uint2* __restrict__ out, u32 cand_stride, u32 slab, FilterWave& w) {
  // One compare per entry; its lane mask doubles as the wave ballot, so counting and ranking the
  // candidates below is scalar work plus a few mbcnt.  With a bracket an entry at or above its upper
  // end U (the start of the open top bin) is only counted: it is selected whatever the threshold.
  const u32 U = L + ((u32)(kHistBins - 1) << 10);
  bool pr[kLoads * 4];
  u64 mk[kLoads * 4];
  u64 any = 0;
#pragma unroll
  for (int i = 0; i < kLoads * 4; ++i) {
    const u32 key = r.b[i] & 0x7FFFFFFFu;
    pr[i] = key >= L;
    if (!INTERIOR) pr[i] = pr[i] && ((r.valid >> i) & 1u);
    if (BRACKET) {
      const bool top = pr[i] && key >= U;
      w.sure += (u32)__popcll(ballot(top));
      w.nan |= top && key > 0x7F800000u;
      pr[i] = pr[i] && !top;
    }
    mk[i] = ballot(pr[i]);
    any |= mk[i];
  }
  if (any == 0) return;  // wave-uniform
  u32 tot[kLoads], total = 0;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    tot[j] = (u32)__popcll(mk[4 * j]) + (u32)__popcll(mk[4 * j + 1]) + (u32)__popcll(mk[4 * j + 2]) + (u32)__popcll(mk[4 * j + 3]);
    total += tot[j];
  }
  if (w.overflow) return;
  if (w.cur + total > w.end) {
    flush_stage(w, stage, out, lane, L, h);  // staged candidates belong to the old slab
    close_segment(w, lane);
    // the next slab: twice the previous one (slab, slab, 2 slab, 4 slab, ...), and at least what the tile needs
    const u32 grown = slab << (w.n_seg > 1 ? w.n_seg - 1 : 0);
    const u32 fit = (total + slab - 1) & ~(slab - 1);  // slab is a power of two
    const u32 need = grown > fit ? grown : fit;
    u32 b = 0;
    if (lane == 0) b = atomicAdd(n_alloc, need);
    w.cur = __builtin_amdgcn_readfirstlane(b);
    w.end = w.cur + need;
    w.seg_base = w.cur;
    if (w.end > cand_stride || w.end < w.cur) {  // pool exhausted (or the counter wrapped): nothing more is written
      w.overflow = true;
      w.end = w.cur;
      w.seg_base = w.cur;
    }
  }
  if (w.overflow) return;
  if (w.fill + total > (u32)kStage) flush_stage(w, stage, out, lane, L, h);
  const u64 v0 = (u64)tile * kWaveTile + (u64)lane * 4 - a;
  if (total > (u32)kStage) {  // a tile too dense to stage writes straight to memory (stage is empty here)
    place_candidates<true, true, true>(r, pr, mk, tot, w.cur, v0, L, h, out, stage, w.nan);
  } else {
    place_candidates<false, false, false>(r, pr, mk, tot, w.fill, v0, L, h, out, stage, w.nan);
    w.fill += total;
  }
  w.cur += total;
  w.total += total;
  if (w.fill >= (u32)kStageFlush) flush_stage(w, stage, out, lane, L, h);
}

// The filter pass over rows that are read only: persistent waves, each with a range of its own.
// BRACKET (dense K, where keeping every entry at or above L would need a pool as large as the row):
// only the entries inside the 2047 closed bins above L are kept, the ones above are counted.
template <bool BRACKET>
__global__ __launch_bounds__(kBlock) void k_filter(const float* __restrict__ grads, u64 N, RowState* __restrict__ rs, u32* __restrict__ hist, uint2* __restrict__ cand,
                                                   u32 cand_stride, u64* __restrict__ wave_seg, u32* __restrict__ wave_nseg,
                                                   u32 wave_stride, u32 n_wtiles, u32 tiles_per_wave, u32 slab,
                                                   u32* __restrict__ status, u32* __restrict__ wave_sure) {
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode != kModeCandidates) return;
  __shared__ u32 h[kHistBins];
  __shared__ u64 stage_all[kWaves][kStage];
  for (int i = threadIdx.x; i < kHistBins; i += kBlock) h[i] = 0;
  __syncthreads();
  const float* row = grads + (size_t)m * N;
  const u32 a = (u32)((reinterpret_cast<uintptr_t>(row) >> 2) & 3u);
  const u32* rowv = reinterpret_cast<const u32*>(row) - a;
  const u64 vend = N + a;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  uint2* out = cand + (size_t)m * cand_stride;
  u64* stage = stage_all[wave];
  const u32 g = blockIdx.x * kWaves + wave;  // the wave's position among the waves of its row
  FilterWave w{};
  w.cur = g * slab;  // the wave's first slab; rs[m].n_alloc starts past all of them
  w.end = w.cur + slab;
  w.seg_base = w.cur;
  w.segs = wave_seg + ((size_t)m * wave_stride + g) * kChain;
  const u32 t0 = (blockIdx.x * kWaves + wave) * tiles_per_wave;
  const u32 t1 = t0 + tiles_per_wave < n_wtiles ? t0 + tiles_per_wave : n_wtiles;
  // interior tiles: [first, last) where the tile neither starts before the row nor ends after it
  const u32 first = a ? 1u : 0u;
  const u32 last = (u32)(vend / kWaveTile);  // tiles below this index end inside the row
  // Software pipeline: the loads of tile t+1 are in flight while tile t is processed.
  TileRegs nxt;
  if (t0 < t1) {
    if (t0 >= first && t0 < last) load_filter_tile<true>(rowv, a, vend, t0, lane, nxt);
    else load_filter_tile<false>(rowv, a, vend, t0, lane, nxt);
  }
  for (u32 tile = t0; tile < t1; ++tile) {
    const TileRegs r = nxt;
    if (tile + 1 < t1) {
      if (tile + 1 >= first && tile + 1 < last) load_filter_tile<true>(rowv, a, vend, tile + 1, lane, nxt);
      else load_filter_tile<false>(rowv, a, vend, tile + 1, lane, nxt);
    }
    if (tile >= first && tile < last) filter_tile<true, BRACKET>(r, a, tile, lane, st.L, h, stage, &rs[m].n_alloc, out, cand_stride, slab, w);
    else filter_tile<false, BRACKET>(r, a, tile, lane, st.L, h, stage, &rs[m].n_alloc, out, cand_stride, slab, w);
  }
  if (!w.overflow) {
    flush_stage(w, stage, out, lane, st.L, h);
    close_segment(w, lane);
  }
  if (lane == 0) {
    wave_nseg[(size_t)m * wave_stride + g] = w.overflow ? 0u : w.n_seg;
    if (w.total) atomicAdd(&rs[m].n_cand, w.total);
    if (BRACKET) {
      wave_sure[(size_t)m * wave_stride + g] = w.sure;
      if (w.sure) atomicAdd(&rs[m].n_sure, w.sure);
    }
    if (w.overflow) rs[m].overflow = 1;
  }
  if (w.nan) status[0] = 1;
  __syncthreads();
  for (int i = threadIdx.x; i < kHistBins; i += kBlock) {
    const u32 c = h[i];
    if (c) atomicAdd(&hist[(size_t)m * kHistBins + i], c);
  }
}

// A plain read of a flat array with the launch shape and the loads of k_filter (persistent waves,
// a contiguous run of 1024-entry tiles each, the next tile requested before the current one is
// used) and none of its work: what the memory system gives a read stream of this shape.  The one
// compare per entry keeps the loads alive; `sink` receives a count nobody reads.
__global__ __launch_bounds__(kBlock) void k_plain_read(const float* __restrict__ buf, u32 n_wtiles, u32 tiles_per_wave, u32* __restrict__ sink) {
  const u32* rowv = reinterpret_cast<const u32*>(buf);
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  const u32 t0 = (blockIdx.x * kWaves + wave) * tiles_per_wave;
  const u32 t1 = t0 + tiles_per_wave < n_wtiles ? t0 + tiles_per_wave : n_wtiles;
  u32 seen = 0;
  TileRegs nxt;
  if (t0 < t1) load_filter_tile<true>(rowv, 0, 0, t0, lane, nxt);
  for (u32 tile = t0; tile < t1; ++tile) {
    const TileRegs r = nxt;
    if (tile + 1 < t1) load_filter_tile<true>(rowv, 0, 0, tile + 1, lane, nxt);
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) seen += (r.b[i] & 0x7FFFFFFFu) >= 0x7F800001u;
  }
  if (seen == 0x7FFFFFFFu) *sink = seen;  // never: a wave sees at most 2^22 entries per launch shape used here
}

// ---- the filter pass with a memory, in chunks --------------------------------------------------
// The row is g = grads + eta * err, and g is written over err as it is filtered (grads and err rows
// start at the same 16-byte phase, checked by the caller).  One block per chunk of 8192 consecutive
// entries, launched in index order; a wave holds its kChunkTiles consecutive wave tiles in
// registers.  The block counts its candidates, reserves exactly that many slots of the row's pool
// with one atomic, and its waves write them there in ascending index.  Chunk c leaves the segment
// (first slot, count) as entry c of the row's segment table, so that list g of the table (kChain
// entries) is chunks g*kChain .. g*kChain + kChain - 1 in order.  No bins are filled: the radix
// select then runs over the candidates at every level.
//
// Why not persistent waves as in k_filter: this pass reads two rows and writes one, and blocks
// dispatched in index order keep the running blocks inside a compact window of the three streams,
// which the memory system rewards (a bare read-modify-write stream: 5.9 TB/s against 5.2 TB/s for
// waves that each stream a far-apart range).  A read-only pass gains nothing from it, and the one
// returning atomic per block, harmless next to 96 KB of traffic, would bound it: atomics on one
// counter (or on the neighbouring counters of a few rows) complete at about 86 per microsecond.
// BRACKET: entries at or above U are counted in `sure` and not kept.
template <bool INTERIOR, bool BRACKET>
__device__ __forceinline__ u32 count_candidates(const TileRegs& r, u32 L, u32 U, u32& sure, bool& nan) {
  u32 total = 0;
#pragma unroll
  for (int i = 0; i < kLoads * 4; ++i) {
    const u32 key = r.b[i] & 0x7FFFFFFFu;
    bool p = key >= L;
    if (!INTERIOR) p = p && ((r.valid >> i) & 1u);
    if (BRACKET) {
      const bool top = p && key >= U;
      sure += (u32)__popcll(ballot(top));
      nan |= top && key > 0x7F800000u;
      p = p && !top;
    }
    total += (u32)__popcll(ballot(p));
  }
  return total;
}

template <bool INTERIOR, bool BRACKET>
__device__ __forceinline__ void place_chunk_tile(const TileRegs& r, u32 a, u32 tile, u32 lane, u32 L, u32 U, u32 first_slot,
                                                 uint2* __restrict__ out, bool& nan) {
  bool pr[kLoads * 4];
  u64 mk[kLoads * 4];
#pragma unroll
  for (int i = 0; i < kLoads * 4; ++i) {
    const u32 key = r.b[i] & 0x7FFFFFFFu;
    pr[i] = key >= L && (!BRACKET || key < U);
    if (!INTERIOR) pr[i] = pr[i] && ((r.valid >> i) & 1u);
    mk[i] = ballot(pr[i]);
  }
  u32 tot[kLoads];
#pragma unroll
  for (int j = 0; j < kLoads; ++j)
    tot[j] = (u32)__popcll(mk[4 * j]) + (u32)__popcll(mk[4 * j + 1]) + (u32)__popcll(mk[4 * j + 2]) + (u32)__popcll(mk[4 * j + 3]);
  const u64 v0 = (u64)tile * kWaveTile + (u64)lane * 4 - a;
  place_candidates<true, false, true>(r, pr, mk, tot, first_slot, v0, L, nullptr, out, nullptr, nan);
}

// Six waves per SIMD (80 registers, four of them spilled) measured 2 % to 6 % faster than the five the
// kernel would take by itself; seven lose again, and so do eight waves of one tile each.
template <bool BRACKET>
__global__ __launch_bounds__(kBlock, 6) void k_filter_chunks(const float* __restrict__ grads, float* __restrict__ err, float eta, u64 N,
                                                          RowState* __restrict__ rs, uint2* __restrict__ cand, u32 cand_stride,
                                                          u64* __restrict__ list_seg, u32* __restrict__ list_nseg, u32 list_stride,
                                                          u32 n_chunks, u32* __restrict__ status) {
  static_assert(kChunkTiles == 2, "the two wave tiles of a chunk are held in named registers");
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode != kModeCandidates) return;  // block-uniform
  __shared__ u32 wsum[kWaves], wsure[kWaves];
  __shared__ u32 sbase;
  const float* row = grads + (size_t)m * N;
  const u32 a = (u32)((reinterpret_cast<uintptr_t>(row) >> 2) & 3u);
  const u32* rowv = reinterpret_cast<const u32*>(row) - a;
  u32* errv = reinterpret_cast<u32*>(err + (size_t)m * N) - a;
  const u64 vend = N + a;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  const u32 chunk = blockIdx.x;
  const u32 t0 = (chunk * kWaves + wave) * kChunkTiles, t1 = t0 + 1;
  const u32 first = a ? 1u : 0u;              // tiles from here on do not start before the row
  const u32 last = (u32)(vend / kWaveTile);   // tiles below this index end inside the row
  const bool in0 = t0 >= first && t0 < last, in1 = t1 >= first && t1 < last;  // wave-uniform
  TileRegs r0, r1, e0, e1;
  if (in0) { load_filter_tile<true>(rowv, a, vend, t0, lane, r0); load_filter_tile<true>(errv, a, vend, t0, lane, e0); }
  else { load_filter_tile<false>(rowv, a, vend, t0, lane, r0); load_filter_tile<false>(errv, a, vend, t0, lane, e0); }
  if (in1) { load_filter_tile<true>(rowv, a, vend, t1, lane, r1); load_filter_tile<true>(errv, a, vend, t1, lane, e1); }
  else { load_filter_tile<false>(rowv, a, vend, t1, lane, r1); load_filter_tile<false>(errv, a, vend, t1, lane, e1); }
  // g = grads + eta * err goes over err right away: the stores are under way while the candidates are counted
#pragma unroll
  for (int i = 0; i < kLoads * 4; ++i) r0.b[i] = compensate_bits(r0.b[i], e0.b[i], eta);
  if (in0) store_filter_tile<true>(errv, t0, lane, r0); else store_filter_tile<false>(errv, t0, lane, r0);
#pragma unroll
  for (int i = 0; i < kLoads * 4; ++i) r1.b[i] = compensate_bits(r1.b[i], e1.b[i], eta);
  if (in1) store_filter_tile<true>(errv, t1, lane, r1); else store_filter_tile<false>(errv, t1, lane, r1);
  // dense K: the same bracket as the persistent pass keeps (its 2047 closed bins), though no bins are filled here
  const u32 U = st.L + ((u32)(kHistBins - 1) << 10);
  u32 sure = 0;
  bool nan = false;
  const u32 c0 = in0 ? count_candidates<true, BRACKET>(r0, st.L, U, sure, nan) : count_candidates<false, BRACKET>(r0, st.L, U, sure, nan);
  const u32 c1 = in1 ? count_candidates<true, BRACKET>(r1, st.L, U, sure, nan) : count_candidates<false, BRACKET>(r1, st.L, U, sure, nan);
  if (lane == 0) {
    wsum[wave] = c0 + c1;
    if (BRACKET) wsure[wave] = sure;
  }
  if (nan) status[0] = 1;
  __syncthreads();
  u32 before = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const u32 c = wsum[w];
    if ((u32)w < wave) before += c;
    total += c;
  }
  if (threadIdx.x == 0) {
    if (BRACKET) {
      u32 block_sure = 0;
      for (int w = 0; w < kWaves; ++w) block_sure += wsure[w];
      if (block_sure) atomicAdd(&rs[m].n_sure, block_sure);
    }
    u32 base = 0;
    bool fits = true;
    if (total) {
      base = atomicAdd(&rs[m].n_alloc, total);
      fits = base + total <= cand_stride && base + total >= base;
      if (!fits) rs[m].overflow = 1;
    }
    sbase = fits ? base : 0xFFFFFFFFu;
    list_seg[(size_t)m * list_stride * kChain + chunk] = fits ? (((u64)base << 32) | total) : 0ull;
    if (chunk % kChain == 0) {
      const u32 left = n_chunks - chunk;
      list_nseg[(size_t)m * list_stride + chunk / kChain] = left < (u32)kChain ? left : (u32)kChain;
    }
  }
  __syncthreads();
  const u32 base = sbase;
  if (total == 0 || base == 0xFFFFFFFFu) return;
  uint2* out = cand + (size_t)m * cand_stride;
  if (c0) {
    if (in0) place_chunk_tile<true, BRACKET>(r0, a, t0, lane, st.L, U, base + before, out, nan);
    else place_chunk_tile<false, BRACKET>(r0, a, t0, lane, st.L, U, base + before, out, nan);
  }
  if (c1) {
    if (in1) place_chunk_tile<true, BRACKET>(r1, a, t1, lane, st.L, U, base + before + c0, out, nan);
    else place_chunk_tile<false, BRACKET>(r1, a, t1, lane, st.L, U, base + before + c0, out, nan);
  }
  if (nan) status[0] = 1;
}

// The kernels below walk the candidates of a row in ascending index (ListWalk): a wave per segment
// list.
// (eq << 32) | gt of each segment list against the final threshold; scanned afterwards.
__global__ __launch_bounds__(kBlock) void k_cand_count(const RowState* __restrict__ rs, const uint2* __restrict__ cand, u32 cand_stride,
                                                       const u64* __restrict__ wave_seg, const u32* __restrict__ wave_nseg,
                                                       u32 wave_stride, u32 n_waves, u64* __restrict__ wave_sum,
                                                       const u32* __restrict__ wave_sure) {
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode == kModeGeneral) return;
  const u32 lane = lane_id();
  for (u32 g = blockIdx.x * kWaves + (threadIdx.x >> 6); g < n_waves; g += gridDim.x * kWaves) {  // wave-uniform
    const ListWalk lw(wave_seg, wave_nseg, wave_stride, cand, cand_stride, m, g);
    u32 gt = 0, eq = 0;
    u32 done = 0;
    if (lw.single && (lw.slot[0] & 1u) == 0) {  // wave-uniform: two candidates per lane and load, 16 bytes
      const uint4* p4 = reinterpret_cast<const uint4*>(lw.pool + lw.slot[0]);
      const u32 pairs = lw.total >> 1;
      for (u32 i0 = lane; i0 < pairs; i0 += 64 * kWalk) {
        uint4 c[kWalk];
#pragma unroll
        for (int u = 0; u < kWalk; ++u) {
          const u32 j = i0 + (u32)u * 64u;
          c[u] = j < pairs ? p4[j] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < kWalk; ++u) {
          const bool ok = i0 + (u32)u * 64u < pairs;
          const u32 k0 = c[u].y & 0x7FFFFFFFu, k1 = c[u].w & 0x7FFFFFFFu;
          gt += (ok && k0 > st.T) + (ok && k1 > st.T);
          eq += (ok && k0 == st.T) + (ok && k1 == st.T);
        }
      }
      done = pairs << 1;
    }
    for (u32 i0 = done + lane; i0 < lw.total; i0 += 64 * kWalk) {
      u32 key[kWalk];
#pragma unroll
      for (int u = 0; u < kWalk; ++u) {
        const u32 j = i0 + (u32)u * 64u;
        key[u] = j < lw.total ? (lw.pool[lw.locate(j)].y & 0x7FFFFFFFu) : 0xFFFFFFFFu;
      }
#pragma unroll
      for (int u = 0; u < kWalk; ++u) {
        gt += key[u] != 0xFFFFFFFFu && key[u] > st.T;
        eq += key[u] == st.T;  // T is a key, never the filler
      }
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) { gt += __shfl_xor(gt, d, 64); eq += __shfl_xor(eq, d, 64); }
    if (st.mode == kModeRangeEmit) gt += wave_sure[(size_t)m * wave_stride + g];  // above the bracket: all greater than T
    if (lane == 0) wave_sum[(size_t)m * wave_stride + g] = ((u64)eq << 32) | gt;
  }
}

// Emits the words of each segment list at its scanned offset, in ascending index, the tie quota
// applied in index order.  With a memory (`err` non-NULL), +0.0 goes over every entry whose sign is sent.
__global__ __launch_bounds__(kBlock) void k_cand_emit(const RowState* __restrict__ rs, const uint2* __restrict__ cand, u32 cand_stride,
                                                      const u64* __restrict__ wave_seg, const u32* __restrict__ wave_nseg,
                                                      u32 wave_stride, u32 n_waves, const u64* __restrict__ wave_sum, u64 K,
                                                      u32* __restrict__ words, float* __restrict__ err, u64 N) {
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode == kModeGeneral || st.mode == kModeRangeEmit) return;
  const u32 lane = lane_id();
  float* erow = err ? err + (size_t)m * N : nullptr;
  u32* out = words + (size_t)m * K;
  for (u32 g = blockIdx.x * kWaves + (threadIdx.x >> 6); g < n_waves; g += gridDim.x * kWaves) {  // wave-uniform
    const ListWalk lw(wave_seg, wave_nseg, wave_stride, cand, cand_stride, m, g);
    if (lw.total == 0) continue;
    const u64 before = wave_sum[(size_t)m * wave_stride + g];  // exclusive prefix over the lists before this one
    u32 eq_seen = (u32)(before >> 32);
    u32 o = (u32)before + (eq_seen < st.q ? eq_seen : st.q);
    for (u32 i0 = 0; i0 < lw.total; i0 += 64 * kWalk) {  // wave-uniform trip count
      // kWalk groups of 64 candidates are loaded together, then placed one group after the other
      uint2 cds[kWalk];
#pragma unroll
      for (int u = 0; u < kWalk; ++u) {
        const u32 j = i0 + (u32)u * 64u + lane;
        cds[u] = j < lw.total ? lw.pool[lw.locate(j)] : make_uint2(0, 0);
      }
#pragma unroll
      for (int u = 0; u < kWalk; ++u) {
        if (i0 + (u32)u * 64u >= lw.total) break;  // wave-uniform
        const bool ok = i0 + (u32)u * 64u + lane < lw.total;
        const uint2 cd = cds[u];
        const u32 key = cd.y & 0x7FFFFFFFu;
        const bool is_eq = ok && key == st.T;
        const u64 eq_mask = ballot(is_eq);
        const bool sel = ok && (key > st.T || (is_eq && eq_seen + ballot_rank(eq_mask) < st.q));
        const u64 sel_mask = ballot(sel);
        if (sel) {
          const u32 pos = o + ballot_rank(sel_mask);
          if (pos < K) {  // pos < K by construction
            out[pos] = (cd.x << 1) | (cd.y >> 31);
            if (erow) erow[cd.x] = 0.0f;
          }
        }
        o += (u32)__popcll(sel_mask);
        eq_seen += (u32)__popcll(eq_mask);
      }
    }
  }
}

// ---- dense K: the words from a second pass over the waves' ranges -------------------------------
// The filter pass with a bracket kept only the candidates inside it, so the words cannot come from
// the pool.  Every wave walks the same run of wave tiles as in the filter pass; its first output slot
// is the scanned count of its predecessors (candidates above T plus the entries above the bracket,
// and the ties before it), so no count pass over the row is needed.
template <bool INTERIOR>
__device__ __forceinline__ void emit_range_tile(const TileRegs& r, u32 a, u32 tile, u32 lane, u32 T, u32 q, u32& o, u32& eq_seen,
                                                u32* __restrict__ out, u64 K, u32* zero_row) {
  bool sel[kLoads * 4], eqb[kLoads * 4];
  u64 eqm[kLoads * 4];
  u64 eq_any = 0;
#pragma unroll
  for (int i = 0; i < kLoads * 4; ++i) {
    const u32 key = r.b[i] & 0x7FFFFFFFu;
    const bool ok = INTERIOR || ((r.valid >> i) & 1u);
    sel[i] = ok && key > T;
    eqb[i] = ok && key == T;
    eqm[i] = ballot(eqb[i]);
    eq_any |= eqm[i];
  }
  if (eq_any) {  // wave-uniform
    if (eq_seen < q) {  // tie slots are left: they go to the equal entries in ascending index
      u32 run = eq_seen;
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        u32 rk = run + ballot_rank(eqm[4 * j]) + ballot_rank(eqm[4 * j + 1]) + ballot_rank(eqm[4 * j + 2]) + ballot_rank(eqm[4 * j + 3]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (eqb[4 * j + e]) { sel[4 * j + e] = rk < q; ++rk; }
        }
        run += (u32)__popcll(eqm[4 * j]) + (u32)__popcll(eqm[4 * j + 1]) + (u32)__popcll(eqm[4 * j + 2]) + (u32)__popcll(eqm[4 * j + 3]);
      }
    }
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) eq_seen += (u32)__popcll(eqm[i]);
  }
  const u64 v0 = (u64)tile * kWaveTile + (u64)lane * 4 - a;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    const u64 m0 = ballot(sel[4 * j]), m1 = ballot(sel[4 * j + 1]), m2 = ballot(sel[4 * j + 2]), m3 = ballot(sel[4 * j + 3]);
    if ((m0 | m1 | m2 | m3) == 0) continue;  // wave-uniform
    u32 p = o + ballot_rank(m0) + ballot_rank(m1) + ballot_rank(m2) + ballot_rank(m3);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int i = 4 * j + e;
      if (sel[i]) {
        if (p < K) out[p] = ((u32)(v0 + (u64)j * 256 + e) << 1) | (r.b[i] >> 31);  // p < K by construction
        ++p;
      }
    }
    o += (u32)__popcll(m0) + (u32)__popcll(m1) + (u32)__popcll(m2) + (u32)__popcll(m3);
    if (zero_row) {  // the row is a memory: +0.0 over the sent entries, as whole 64-byte runs (see k_emit_rows)
      const u32 s4 = (u32)sel[4 * j] | ((u32)sel[4 * j + 1] << 1) | ((u32)sel[4 * j + 2] << 2) | ((u32)sel[4 * j + 3] << 3);
      if (((ballot(s4 != 0) >> (lane & 60u)) & 0xFull) == 0) continue;
      u32* p = zero_row + (u64)tile * kWaveTile + (u64)j * 256 + (u64)lane * 4;
      if (INTERIOR) {
        *reinterpret_cast<uint4*>(p) = make_uint4((s4 & 1u) ? 0u : r.b[4 * j], (s4 & 2u) ? 0u : r.b[4 * j + 1],
                                                  (s4 & 4u) ? 0u : r.b[4 * j + 2], (s4 & 8u) ? 0u : r.b[4 * j + 3]);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if ((s4 >> e) & 1u) p[e] = 0u;
      }
    }
  }
}

// `zero` non-NULL: `grads` is a memory holding g (the same buffer): every sent entry becomes +0.0.
__global__ __launch_bounds__(kBlock) void k_range_emit(const float* grads, u64 N, u64 K, const RowState* __restrict__ rs,
                                                       const u64* __restrict__ wave_sum, u32 wave_stride, u32 n_wtiles,
                                                       u32 tiles_per_wave, u32* __restrict__ words, float* zero) {
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (st.mode != kModeRangeEmit) return;
  const float* row = grads + (size_t)m * N;
  const u32 a = (u32)((reinterpret_cast<uintptr_t>(row) >> 2) & 3u);
  const u32* rowv = reinterpret_cast<const u32*>(row) - a;
  const u64 vend = N + a;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  const u32 g = blockIdx.x * kWaves + wave;  // the same wave, the same run of tiles as in the filter pass
  const u32 t0 = g * tiles_per_wave;
  const u32 t1 = t0 + tiles_per_wave < n_wtiles ? t0 + tiles_per_wave : n_wtiles;
  if (t0 >= t1) return;  // wave-uniform; nothing below synchronises across waves
  const u64 before = wave_sum[(size_t)m * wave_stride + g];
  u32 eq_seen = (u32)(before >> 32);
  u32 o = (u32)before + (eq_seen < st.q ? eq_seen : st.q);
  u32* out = words + (size_t)m * K;
  u32* zero_row = zero ? reinterpret_cast<u32*>(zero + (size_t)m * N) - a : nullptr;
  const u32 first = a ? 1u : 0u;
  const u32 last = (u32)(vend / kWaveTile);
  TileRegs nxt;
  if (t0 >= first && t0 < last) load_filter_tile<true>(rowv, a, vend, t0, lane, nxt);
  else load_filter_tile<false>(rowv, a, vend, t0, lane, nxt);
  for (u32 tile = t0; tile < t1; ++tile) {
    const TileRegs r = nxt;
    if (tile + 1 < t1) {
      if (tile + 1 >= first && tile + 1 < last) load_filter_tile<true>(rowv, a, vend, tile + 1, lane, nxt);
      else load_filter_tile<false>(rowv, a, vend, tile + 1, lane, nxt);
    }
    if (tile >= first && tile < last) emit_range_tile<true>(r, a, tile, lane, st.T, st.q, o, eq_seen, out, K, zero_row);
    else emit_range_tile<false>(r, a, tile, lane, st.T, st.q, o, eq_seen, out, K, zero_row);
  }
}

// counts[m] and the pad words of rows that selected zeros.
__global__ void k_finish_rows(const RowState* __restrict__ rs, u64 K, u32* __restrict__ words, u32* __restrict__ counts,
                              u32* __restrict__ status, u32* __restrict__ nan_flag) {
  const u32 m = blockIdx.y;
  const RowState st = rs[m];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (nan_flag && m == 0) *nan_flag = status[0] ? 1u : 0u;  // every kernel that raises it has run
    counts[m] = st.count;
    if (st.mode == kModeGeneral && !st.row_emit) atomicAdd(&status[1], 1u);
    if (st.mode == kModeCandWide) atomicAdd(&status[4], 1u);
    if (st.mode == kModeGeneral && st.row_emit) atomicAdd(&status[5], 1u);
    if (st.mode == kModeRangeEmit) atomicAdd(&status[6], 1u);
  }
  u32* out = words + (size_t)m * K;
  for (u64 i = (u64)st.count + blockIdx.x * blockDim.x + threadIdx.x; i < K; i += (u64)gridDim.x * blockDim.x)
    out[i] = S3GD_PAD;
}

__global__ void k_zero_counts(u32* counts, u32 M, u32* nan_flag) {
  const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < M) counts[i] = 0;
  if (i == 0 && nan_flag) *nan_flag = 0;  // K = 0 looks at no entry
}

// ------------------------------------------------------------------------------------------------
// Streaming launches use one round of resident blocks, split evenly over the rows.
static u32 blocks_per_row(u32 M, u32 n_tiles, u32 stream_blocks) {
  u32 gx = stream_blocks / M;
  if (gx > n_tiles) gx = n_tiles;
  return gx < 1 ? 1 : gx;
}

u32 resident_stream_blocks(int device, bool with_memory) {
  int cus = 0, per_cu = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0) cus = 256;
  const hipError_t e = with_memory ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_filter_chunks<false>, kBlock, 0)
                                   : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_filter<false>, kBlock, 0);
  if (e != hipSuccess || per_cu <= 0) per_cu = 4;
  const u32 n = (u32)cus * (u32)per_cu;
  return n > kMaxStreamBlocks ? kMaxStreamBlocks : n;
}

hipError_t launch_plain_read(const Workspace& ws, const float* buf, u64 n, hipStream_t s) {
  const u32 n_wtiles = (u32)(n / kWaveTile);  // whole tiles only: a calibration, not a reduction
  if (n_wtiles == 0) return hipSuccess;
  u32 gx = ws.stream_blocks;
  if (gx > (n_wtiles + kWaves - 1) / kWaves) gx = (n_wtiles + kWaves - 1) / kWaves;
  const u32 tiles_per_wave = (n_wtiles + gx * kWaves - 1) / (gx * kWaves);
  ws.prof->begin(KID_PLAIN_READ, s);
  k_plain_read<<<gx, kBlock, 0, s>>>(buf, n_wtiles, tiles_per_wave, ws.status + 7);
  ws.prof->end(s);
  return hipGetLastError();
}

// Upper estimate of the candidates per row when the sample rank is r and the sample fraction f:
// the count of keys above the r-th largest sample key is about r / f with deviation sqrt(r) / f.
static double candidate_bound(double r, double f) { return 1.25 * (r + 6.0 * sqrt(r) + 8.0) / f; }

EncodePlan plan_encode(u32 M, u64 N, u64 K, u64 cand_pool, u32 stream_blocks, bool chunks) {
  EncodePlan p{};
  p.n_tiles = encode_tiles(N);
  p.gx = blocks_per_row(M, p.n_tiles, stream_blocks);
  p.candidates = false;
  if (K == 0 || N < (1ull << 17)) return p;
  // Dense K: keeping every entry at or above L would take a pool as large as the row.  The filter
  // pass then keeps only the entries inside the bins above L (a bracket around the K-th key), counts
  // the ones above, and the words come from a second pass over the row once the threshold is known:
  // two reads instead of the general route's five.  With a memory (the chunked pass fills no bins) the
  // radix select runs over the bracket's candidates and the row passes count and emit: three reads.
  p.bracket = K * 16 > N;
  // sample size: about 256 sampled entries above the K-th magnitude, between 2^15 and 2^18,
  // and never more than a quarter of the row
  // (with a bracket the largest sample: the K-th key has to fall inside the bins above L)
  u64 s = 1ull << 15;
  while (s < (1ull << 18) && s * 8 <= N && (p.bracket || (double)s * (double)K < 256.0 * (double)N)) s <<= 1;
  const double f = (double)s / (double)N, kf = (double)K * f;
  const double r = ceil(kf + 6.0 * sqrt(kf) + 8.0);
  if (r >= (double)s) return p;
  p.n_wtiles = (u32)((N + 3 + kWaveTile - 1) / kWaveTile);
  p.tiles_per_wave = (p.n_wtiles + p.gx * kWaves - 1) / (p.gx * kWaves);
  p.bound = candidate_bound(r, f);
  // slab: the power of two at or above the candidates expected per wave of the filter pass
  const double per_wave = p.bound / ((double)p.gx * kWaves);
  p.slab = kSlabMin;
  while (p.slab < kSlabMax && (double)p.slab < per_wave) p.slab <<= 1;
  // a row needs room for its candidates, for the first slab of every wave, for the unused part of the
  // later (doubling) slabs of waves that overflowed (at most what they hold), and a tile of slack
  double need = 2.0 * p.bound + (double)p.gx * kWaves * p.slab + kWaveTile;
  if (p.bracket) {
    // how many entries fall inside the bracket depends on the distribution: the row takes its share of
    // the pool, half of it as first slabs; a row that needs more falls back to the general route
    need = floor((double)cand_pool / M);
    if (need > (double)N + 2.0 * kWaveTile) need = (double)N + 2.0 * kWaveTile;
    p.slab = kSlabMin;
    while (p.slab < kSlabMax && (double)p.slab * 2.0 * p.gx * kWaves < need / 2.0) p.slab <<= 1;
    if ((double)p.gx * kWaves * p.slab + kWaveTile > need) return p;
  }
  if (chunks) {  // blocks reserve exactly what they found: no slabs
    if (!p.bracket) need = 2.0 * p.bound + kWaveTile;
    p.n_chunks = chunk_count(N);
    p.n_lists = chunk_lists(N);
  }
  if (need * M > (double)cand_pool || need > 4.0e9) return p;
  p.candidates = true;
  p.chunks = chunks;
  p.n_units = (u32)(s / kSampleUnit);
  p.unit_stride = N / p.n_units;
  p.sample_rank = (u32)r;
  p.cand_stride = (u32)need;
  return p;
}

u64 candidate_pool_entries(u32 M_max, u64 N_max, u64 K_max) {
  double best = 0;
  // the bound is not monotone in K (the sample size changes in powers of two): take the largest
  // over K_max and the sparsities below it down to 1e-5
  for (double k = (double)(K_max < N_max / 16 ? K_max : N_max / 16); k >= 1.0 && k >= 1e-5 * (double)N_max; k /= 2.0) {
    const EncodePlan p = plan_encode(1, N_max, (u64)k, ~0ull, 1, false);
    if (p.candidates && p.bound > best) best = p.bound;
  }
  if (best == 0) return 0;
  // per row: twice the bound, as much again (at most twice the bound) in first slabs, one tile of
  // slack; once: a smallest slab per wave of a streaming launch
  u64 pool = (u64)M_max * (4 * (u64)best + kWaveTile) + (u64)(kMaxStreamBlocks + M_max) * kWaves * kSlabMin;
  // dense K (bracket): an eighth of the row, 25 % of the gradients' bytes
  if (K_max * 16 > N_max && pool < (u64)M_max * (N_max / 8)) pool = (u64)M_max * (N_max / 8);
  return pool;
}

// `err` NULL: the rows of `grads` are compressed as they are.  Otherwise the rows are
// g = grads + eta * err, and on return err holds the new memory g - TopK(g).
hipError_t launch_encode(const Workspace& ws, const float* grads, float* err, float eta, u32 M, u64 N, u64 K, u32* words,
                         u32* counts, hipStream_t s, u32* nan_flag) {
  Profiler& P = *ws.prof;
#define S3GD_LAUNCH(KID, ...) do { P.begin(KID, s); __VA_ARGS__; P.end(s); } while (0)
  // With a memory the filter pass reads two rows and writes one: that mix runs fastest as blocks in index order.
  // `grads` NULL with `err`: the caller has already formed g in the memory buffer (accumulated into it); the row is
  // then read like plain gradients, and only the zeros over the sent entries distinguish the call.
  const bool formed = err && !grads;
  if (formed) grads = err;
  float* mem = formed ? nullptr : err;  // the memory to add in, if any
  const EncodePlan p = plan_encode(M, N, K, ws.cand_pool, mem ? ws.stream_blocks_mem : ws.stream_blocks, mem != nullptr);
  if (mem && !(K > 0 && p.candidates)) {  // no filter pass will run: form g in the memory buffer first
    const u64 total = (u64)M * N;
    const u32 head = (u32)((4 - ((reinterpret_cast<uintptr_t>(err) >> 2) & 3u)) & 3u);
    u64 blocks = (total / 4 + kBlock - 1) / kBlock;
    if (blocks > ws.stream_blocks_mem) blocks = ws.stream_blocks_mem;
    if (blocks < 1) blocks = 1;
    S3GD_LAUNCH(KID_COMPENSATE, (k_compensate<<<(u32)blocks, kBlock, 0, s>>>(grads, err, eta, total, head)));
  }
  if (K == 0) {
    k_zero_counts<<<(M + 255) / 256, 256, 0, s>>>(counts, M, nan_flag);
    return hipGetLastError();
  }
  const float* src = err ? err : grads;  // what the general route reads: with a memory, g sits in err by then
  const u32 n_tiles = p.n_tiles;
  const u32 stride = tile_stride(N);
  const dim3 grid(p.gx, M);
  const u32 k32 = (u32)K;
  const bool all = K == N;  // signSGD with majority vote: every non-zero entry is sent, nothing to select
  S3GD_LAUNCH(KID_ENCODE_INIT, (k_encode_init<<<dim3(2, M), 256, 0, s>>>(ws.rs, ws.hist, ws.status, M, p.candidates ? p.sample_rank : k32,
                                                                         p.candidates ? kModeCandidates : kModeGeneral,
                                                                         p.candidates && !p.chunks ? p.gx * (u32)kWaves * p.slab : 0u,
                                                                         p.candidates && p.bracket ? 1u : 0u, all ? 1u : 0u)));
  const u32 n_waves = !p.candidates ? 0u : (p.chunks ? p.n_lists : p.gx * (u32)kWaves);  // segment lists per row
  const u32 wstride = p.chunks ? p.n_lists + 4 : wave_stride(p.gx);
  if (p.candidates) {
    const u32 n_wt = p.n_wtiles;
    const dim3 sgrid((p.n_units * kSampleUnit + kSamplePerBlock - 1) / kSamplePerBlock, M);
    // sampled entries at or above L that stand for a row's whole share of the pool (a bracket keeps only part of them)
    const double cap = (double)p.cand_stride * ((double)p.n_units * kSampleUnit / (double)N);
    const u32 sample_cap = p.bracket ? 0u : (cap < 1.0 ? 1u : (cap > 4.0e9 ? 0u : (u32)cap));
    S3GD_LAUNCH(KID_SAMPLE, (k_sample_hist<0><<<sgrid, kBlock, 0, s>>>(grads, mem, eta, N, ws.rs, ws.hist, p.n_units, p.unit_stride)));
    S3GD_LAUNCH(KID_RESOLVE, (k_resolve<0, kResolveSample><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, k32, 1u, 0u, ws.status)));
    S3GD_LAUNCH(KID_SAMPLE, (k_sample_hist<1><<<sgrid, kBlock, 0, s>>>(grads, mem, eta, N, ws.rs, ws.hist, p.n_units, p.unit_stride)));
    S3GD_LAUNCH(KID_RESOLVE, (k_resolve<1, kResolveSample><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, k32, p.chunks ? 0u : 1u, sample_cap, ws.status)));
    if (p.chunks && p.bracket)
      S3GD_LAUNCH(KID_FILTER_MEM, (k_filter_chunks<true><<<dim3(p.n_chunks, M), kBlock, 0, s>>>(grads, err, eta, N, ws.rs, ws.cand, p.cand_stride,
                                                                                               ws.wave_seg, ws.wave_nseg, wstride,
                                                                                               p.n_chunks, ws.status)));
    else if (p.chunks)
      S3GD_LAUNCH(KID_FILTER_MEM, (k_filter_chunks<false><<<dim3(p.n_chunks, M), kBlock, 0, s>>>(grads, err, eta, N, ws.rs, ws.cand, p.cand_stride,
                                                                                                ws.wave_seg, ws.wave_nseg, wstride,
                                                                                                p.n_chunks, ws.status)));
    else if (p.bracket)
      S3GD_LAUNCH(KID_FILTER, (k_filter<true><<<grid, kBlock, 0, s>>>(grads, N, ws.rs, ws.hist, ws.cand, p.cand_stride, ws.wave_seg,
                                                                     ws.wave_nseg, wstride, n_wt, p.tiles_per_wave, p.slab, ws.status, ws.wave_sure)));
    else
      S3GD_LAUNCH(KID_FILTER, (k_filter<false><<<grid, kBlock, 0, s>>>(grads, N, ws.rs, ws.hist, ws.cand, p.cand_stride, ws.wave_seg,
                                                                      ws.wave_nseg, wstride, n_wt, p.tiles_per_wave, p.slab, ws.status,
                                                                      ws.wave_sure)));
    S3GD_LAUNCH(KID_RESOLVE, (k_resolve<0, kResolveFilter><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, k32, p.chunks ? 0u : 1u, 0u, ws.status)));
  }
  // Radix select: over the row for general rows, over the candidates for the others (the last level
  // only, unless the filter's bins could not place the K-th key).
  // launches that walk segment lists: a wave per list, up to four rounds of resident blocks
  u32 lx = (n_waves + kWaves - 1) / kWaves;
  if (lx > 4 * p.gx) lx = 4 * p.gx;
  if (lx < p.gx) lx = p.gx;
  const dim3 lgrid(lx, M);
  const dim3 hgrid(p.candidates ? 4 * p.gx : p.gx, M);  // histogram launches
  // where the candidates' order does not matter a list is shared by as many waves as that grid has for it
  u32 parts = n_waves ? hgrid.x * (u32)kWaves / n_waves : 1u;
  parts = parts < 1 ? 1u : (parts > 4 ? 4u : parts);
#define S3GD_HIST_ARGS src, N, ws.rs, ws.hist, n_tiles, ws.status, ws.cand, p.cand_stride, ws.wave_seg, ws.wave_nseg, wstride, n_waves, parts
  if (!all) {
    S3GD_LAUNCH(KID_HIST0, (k_hist_rows<0><<<hgrid, kBlock, 0, s>>>(S3GD_HIST_ARGS)));
    S3GD_LAUNCH(KID_RESOLVE, (k_resolve<0, kResolveRadix><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, k32, 1u, 0u, ws.status)));
    S3GD_LAUNCH(KID_HIST1, (k_hist_rows<1><<<hgrid, kBlock, 0, s>>>(S3GD_HIST_ARGS)));
    S3GD_LAUNCH(KID_RESOLVE, (k_resolve<1, kResolveRadix><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, k32, 1u, 0u, ws.status)));
    S3GD_LAUNCH(KID_HIST2, (k_hist_rows<2><<<hgrid, kBlock, 0, s>>>(S3GD_HIST_ARGS)));
    S3GD_LAUNCH(KID_RESOLVE, (k_resolve<2, kResolveRadix><<<M, kBlock, 0, s>>>(ws.rs, ws.hist, k32, 1u, 0u, ws.status)));
  }
#undef S3GD_HIST_ARGS
  if (p.candidates) {  // one wave per segment list
    S3GD_LAUNCH(KID_CAND_SELECT, (k_cand_count<<<lgrid, kBlock, 0, s>>>(ws.rs, ws.cand, p.cand_stride, ws.wave_seg, ws.wave_nseg, wstride,
                                                                      n_waves, ws.wave_sum, ws.wave_sure)));
    S3GD_LAUNCH(KID_SCAN_TILES, (k_scan_tiles<<<M, kScanBlock, 0, s>>>(ws.wave_sum, n_waves, wstride, ws.rs, 1u)));
    S3GD_LAUNCH(KID_CAND_EMIT, (k_cand_emit<<<lgrid, kBlock, 0, s>>>(ws.rs, ws.cand, p.cand_stride, ws.wave_seg, ws.wave_nseg, wstride,
                                                                   n_waves, ws.wave_sum, K, words, err, N)));
    if (p.bracket && !p.chunks)
      S3GD_LAUNCH(KID_RANGE_EMIT, (k_range_emit<<<grid, kBlock, 0, s>>>(grads, N, K, ws.rs, ws.wave_sum, wstride, p.n_wtiles, p.tiles_per_wave,
                                                                 words, err)));
  }
  // General rows: per-tile counts and the emit pass (both return at once for the other rows).
  S3GD_LAUNCH(KID_TILE_COUNT, (k_tile_count<<<grid, kBlock, 0, s>>>(src, N, ws.rs, ws.tile_cnt, n_tiles, stride, ws.status)));
  S3GD_LAUNCH(KID_SCAN_TILES, (k_scan_tiles<<<M, kScanBlock, 0, s>>>(ws.tile_cnt, n_tiles, stride, ws.rs, 0u)));
  S3GD_LAUNCH(KID_EMIT, (k_emit_rows<<<grid, kBlock, 0, s>>>(src, N, K, ws.rs, ws.tile_cnt, n_tiles, stride, words, err)));
  u32 fx = (u32)((K + 4095) / 4096);
  if (fx > 64) fx = 64;
  S3GD_LAUNCH(KID_FINISH, (k_finish_rows<<<dim3(fx, M), 256, 0, s>>>(ws.rs, K, words, counts, ws.status, nan_flag)));
#undef S3GD_LAUNCH
  return hipGetLastError();
}

}  // namespace s3gd
