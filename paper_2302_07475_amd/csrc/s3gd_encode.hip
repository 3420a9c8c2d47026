// Worker side of Algorithm 1: batched top-K magnitude selection and sign encoding.
//
// The magnitude order of fp32 values equals the unsigned order of key = bits & 0x7FFFFFFF
// (true for denormals, +-0 and +-Inf).  The K-th largest key T of each row is found by radix
// select over the key's digits; the row then emits, in ascending index, every entry with
// key > T and the first q = K - #{key > T} entries with key == T (Section 2.1 eq. "topk": the
// threshold lies between the K-th and (K+1)-th magnitude; ties go to the lowest index).
//
// Two routes reach the same T, q and words:
//   candidate route  a strided sample of the row gives two bounds L < U with, very likely,
//                    #{key >= U} <= K <= #{key >= L}.  ONE pass over the row writes the message word
//                    of every candidate (key >= L), in ascending index, into per-wave segments of a
//                    pool; the candidates inside the bracket [L, U) also leave a record (position,
//                    bits) and are histogrammed.  T is then resolved among the bracket's records,
//                    and the emit pass copies the candidate words minus the bracket's losers.  The
//                    entries at or above U are selected whatever T turns out to be, so nothing but
//                    their words is ever kept: at K = N/10 the row is read once and a tenth of it is
//                    written, read and written again, instead of the row being read twice.
//                    If the bracket is wider than the pass's 2048 bins the radix select simply runs
//                    over its records.  K = N selects nothing: count and emit (two reads).
//   general route    three histogram passes over the row (11 + 10 + 10 key bits), a per-tile count
//                    pass and an emit pass.  Any row for which the candidate route's checks fail
//                    (too few or too many candidates, tiny rows, K above N/2) takes it; the choice is
//                    made on the device, per row, with no host synchronisation.
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
__device__ __forceinline__ void store_stream8(u64* p, u64 v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void store_stream4(u32* p, u32 v) { __builtin_nontemporal_store(v, p); }

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
// The candidates of a row, as the filter pass left them: a table of segment lists, each of at most
// kChain segments.  A segment is a run of candidate words (the message words of entries with key >= L,
// in ascending index) in the row's word pool, and a run of bracket records in the row's record pool:
// one record (position of the candidate inside its segment, fp32 bits) for every candidate of the
// segment with key < U, in the same order.  Lists in order and segments in order enumerate the
// candidates in ascending index.  A walk numbers the entries of one list 0 .. total-1 across its
// segments, so that a wave takes them 64 (or more) at a time whatever the segment lengths are.
struct RecordWalk {  // the bracket records of a list
  u32 first[kChain], count[kChain], slot[kChain];  // flat number of a segment's first record, its length, its first slot
  u32 total;        // records in the list
  u32 words_total;  // candidate words in the list
  bool single;      // at most one segment (the usual case: the wave's first slab sufficed); wave-uniform
  const uint2* pool;
  __device__ RecordWalk(const u64* __restrict__ wave_seg, const u64* __restrict__ wave_segb, const u32* __restrict__ wave_nseg,
                        u32 wave_stride, const uint2* recs, u32 brk_stride, u32 m, u32 g)
      : total(0), words_total(0), pool(recs + (size_t)m * brk_stride) {
    const u64* segs = wave_segb + ((size_t)m * wave_stride + g) * kChain;
    const u64* wsegs = wave_seg + ((size_t)m * wave_stride + g) * kChain;
    const u32 n_seg = wave_nseg[(size_t)m * wave_stride + g];
#pragma unroll
    for (int c = 0; c < kChain; ++c) {
      const u64 sg = segs[c], wg = wsegs[c];  // the whole lines are loaded; entries past n_seg are stale
      // (the same in every lane: said so, they live in scalar registers)
      slot[c] = __builtin_amdgcn_readfirstlane((u32)(sg >> 32));
      count[c] = __builtin_amdgcn_readfirstlane((u32)c < n_seg ? (u32)sg : 0u);
      first[c] = total;
      total += count[c];
      words_total += __builtin_amdgcn_readfirstlane((u32)c < n_seg ? (u32)wg : 0u);
    }
    single = __builtin_amdgcn_readfirstlane(n_seg <= 1u ? 1 : 0) != 0;
  }
  // pool slot of record j < total
  __device__ __forceinline__ u32 locate(u32 j) const {
    if (single) return slot[0] + j;
    u32 at = 0;
#pragma unroll
    for (int c = 0; c < kChain; ++c) {
      const u32 d = j - first[c];  // wraps to a huge value for records of earlier segments
      if (d < count[c]) at = slot[c] + d;
    }
    return at;
  }
  // the segment record j < total belongs to
  __device__ __forceinline__ u32 segment_of(u32 j) const {
    u32 sg = 0;
#pragma unroll
    for (int c = 1; c < kChain; ++c)
      if (j >= first[c] && count[c]) sg = (u32)c;
    return sg;
  }
};

struct WordWalk {  // the candidate words of a list
  u32 first[kChain], count[kChain], slot[kChain];
  u32 total;
  bool single;
  const u32* pool;
  __device__ WordWalk(const u64* __restrict__ wave_seg, const u32* __restrict__ wave_nseg, u32 wave_stride, const u32* words,
                      u32 cand_stride, u32 m, u32 g)
      : total(0), pool(words + (size_t)m * cand_stride) {
    const u64* segs = wave_seg + ((size_t)m * wave_stride + g) * kChain;
    const u32 n_seg = wave_nseg[(size_t)m * wave_stride + g];
#pragma unroll
    for (int c = 0; c < kChain; ++c) {
      const u64 sg = segs[c];
      slot[c] = __builtin_amdgcn_readfirstlane((u32)(sg >> 32));
      count[c] = __builtin_amdgcn_readfirstlane((u32)c < n_seg ? (u32)sg : 0u);
      first[c] = total;
      total += count[c];
    }
    single = __builtin_amdgcn_readfirstlane(n_seg <= 1u ? 1 : 0) != 0;
  }
  __device__ __forceinline__ u32 locate(u32 j) const {
    if (single) return slot[0] + j;
    u32 at = 0;
#pragma unroll
    for (int c = 0; c < kChain; ++c) {
      const u32 d = j - first[c];
      if (d < count[c]) at = slot[c] + d;
    }
    return at;
  }
};
constexpr int kWalk = 4;  // entries a lane has in flight where their order does not matter

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

// ------------------------------------------------------------------------------------------------
// Resolve steps.  A histogram filled by one kernel is read by the NEXT kernel: every block of that
// kernel picks the bin that holds the sought rank (a block-wide scan over the row's bins, thread 0
// owning the highest), all blocks arriving at the same state, and the first block of the row writes
// the state to the buffer the kernel after reads.  This takes the place of a one-block-per-row
// kernel between every two passes: a launch costs about as much as such a kernel runs (4 to 5 us),
// and a step over a few hundred MB is a dozen of them.

// Among `PER` consecutive bins of this thread (c[0] the highest), with `above` entries in the bins
// above them: the bin that holds rank k (1-based from the largest), if it is one of them.
template <int PER>
__device__ __forceinline__ bool find_rank(const u32 (&c)[PER], u32 above, u32 k, int top, u32* digit, u32* rank_inside, u32* upto) {
  u32 acc = above;
  bool found = false;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    if (k >= 1 && acc < k && k <= acc + c[i]) {
      *digit = (u32)(top - i);
      *rank_inside = k - acc;
      *upto = acc + c[i];
      found = true;
    }
    acc += c[i];
  }
  return found;
}

struct Found {
  u32 hit;        // the rank lies inside the histogram
  u32 digit;      // the bin that holds it
  u32 inside;     // its rank among the entries of that bin
  u32 upto;       // entries in that bin and the bins above it
};

// Looks up two ranks (k2 may be 0: none) in the NB bins at h.  Called by every thread of the block;
// every thread receives the same answers.  *total = entries in all bins, *top_count = entries in the
// highest bin.  `lds`: kWaves + 10 words.
template <int NB>
__device__ __forceinline__ void find_in_bins(const u32* __restrict__ h, u32 k1, u32 k2, u32* lds, Found* f1, Found* f2, u32* total,
                                             u32* top_count) {
  constexpr int PER = NB / kBlock;
  const int top = NB - 1 - (int)threadIdx.x * PER;
  u32 c[PER];
  u32 s = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) { c[i] = h[top - i]; s += c[i]; }
  const u32 above = block_excl_scan<u32>(s, total, lds);
  u32* r = lds + kWaves;
  if (threadIdx.x == 0) { r[0] = 0; r[4] = 0; r[8] = c[0]; }
  __syncthreads();
  u32 digit, inside, upto;
  if (find_rank<PER>(c, above, k1, top, &digit, &inside, &upto)) { r[0] = 1; r[1] = digit; r[2] = inside; r[3] = upto; }
  if (find_rank<PER>(c, above, k2, top, &digit, &inside, &upto)) { r[4] = 1; r[5] = digit; r[6] = inside; r[7] = upto; }
  __syncthreads();
  *f1 = Found{r[0], r[1], r[2], r[3]};
  *f2 = Found{r[4], r[5], r[6], r[7]};
  *top_count = r[8];
  __syncthreads();  // r is free again
}

constexpr int kResolveLds = kWaves + 10;

// The sample, first level (key bits [30:20]): the bins that hold the sample ranks of L and of U.
// Until U is there its prefix and its rank travel in the fields T and q.
__device__ __forceinline__ RowState advance_sample0(RowState st, const u32* __restrict__ h, u32* lds) {
  if (st.mode != kModeCandidates) return st;  // block-uniform
  Found lo, hi;
  u32 total, top_count;
  find_in_bins<kHistBins>(h, st.k_rem, st.q, lds, &lo, &hi, &total, &top_count);
  if (lo.hit) { st.prefix = lo.digit; st.k_rem = lo.inside; }
  if (hi.hit) { st.T = hi.digit; st.q = hi.inside; }
  return st;
}

// The sample, second level (key bits [19:10]): bins 0..1023 hold the keys under L's prefix, bins
// 1024..2047 those under U's.  Ends with L = the 21-bit prefix of the sample key of rank `rank_lo`,
// U = one past the 21-bit prefix of the sample key of the upper rank (both shifted back to key
// units), so that at least rank_lo sampled keys are >= L and fewer than the upper rank are >= U.
// `have_bins` is 0 when the filter pass is the chunked one (with a memory): that pass must run over
// every row to form g, so no row leaves the candidate route before it.
__device__ __forceinline__ RowState advance_sample1(RowState st, const u32* __restrict__ h, u32 K, u32 rank_lo, u32 have_bins,
                                                    u32 sample_cap, u32* lds, bool* diverted) {
  *diverted = false;
  if (st.mode != kModeCandidates) return st;  // block-uniform
  Found lo, hi, none;
  u32 total, top_count;
  find_in_bins<1024>(h, st.k_rem, 0u, lds, &lo, &none, &total, &top_count);
  find_in_bins<1024>(h + 1024, st.q, 0u, lds, &hi, &none, &total, &top_count);
  if (lo.hit) {
    st.L = ((st.prefix << 10) | lo.digit) << 10;
    // L = 0: the sample holds fewer than its share of non-zero entries (a mostly-zero row with K
    // above its non-zeros), every entry would be a candidate.  The row goes to the general route
    // before the filter pass instead of after it, unless that pass must still form g in the memory.
    if (st.L == 0 && have_bins) st.mode = kModeGeneral;
    // Likewise a row with so many entries at or above L that they cannot fit its share of the
    // pool (all entries equal, heavy ties at the threshold): `sample_cap` is the number of
    // sampled entries that stands for a full pool (0: no such check).
    if (sample_cap && have_bins && (rank_lo - st.k_rem) + lo.upto > sample_cap) st.mode = kModeGeneral;
    *diverted = st.mode == kModeGeneral;
  }
  st.U = kNoUpper;
  if (hi.hit) st.U = (((st.T << 10) | hi.digit) + 1u) << 10;  // the prefix is below 2^21: at most 2^31 = kNoUpper
  st.prefix = 0;
  st.k_rem = K;
  st.T = 0;
  st.q = 0;
  return st;
}

// After the filter pass: does the candidate route stand, and where does the radix select start.
// The filter pass histogrammed the bracket's records into 2048 bins of (key - L) >> 10, the last one
// open-ended (a pass in chunks fills no bins: `have_bins` 0).  With n_sure = candidates outside the
// bracket (all of them selected), the K-th key overall is the (K - n_sure)-th of the bracket.
__device__ __forceinline__ RowState advance_filter(RowState st, const u32* __restrict__ h, const RowCounters& rc, u32 K, u32 have_bins,
                                                   u32* lds) {
  if (st.mode != kModeCandidates) return st;  // block-uniform
  st.n_cand = have_bins ? rc.n_cand : rc.n_alloc;  // a pass in chunks: what its blocks reserved
  st.n_brk = have_bins ? rc.n_brk : rc.n_alloc_b;
  const u32 n_sure = st.n_cand - st.n_brk;
  const u32 k = K >= n_sure ? K - n_sure : 0u;
  Found f, none;
  u32 total, top_count;
  find_in_bins<kHistBins>(h, k, 0u, lds, &f, &none, &total, &top_count);
  // The route stands only if no wave ran out of room, no more than K entries were taken for sure and
  // the K-th largest key is among the bracket's records (or is the smallest sure one: k = 0).
  const bool usable = !rc.overflow && n_sure <= K && st.n_brk >= k && (!have_bins || total == st.n_brk);
  st.prefix = 0;
  if (!usable) {
    st.mode = kModeGeneral;
    st.k_rem = K;
  } else if (k == 0) {  // every selected entry is a sure one: the threshold is the bracket's upper end
    st.mode = kModeCandDone;
    st.T = st.U - 1u;
    st.q = 0;
    st.c_gt = K;
    st.count = K;
  } else if (have_bins && top_count < k && f.hit) {  // the bins place the K-th key: its upper 21 bits are fixed
    st.prefix = (st.L >> 10) + f.digit;
    st.k_rem = f.inside;
  } else {  // it sits in the open top bin (or there are no bins): the radix select starts over, among the records
    st.mode = kModeCandWide;
    st.k_rem = k;
  }
  return st;
}

// One level of the radix select (11 + 10 + 10 key bits).
template <int LEVEL>
__device__ __forceinline__ RowState advance_radix(RowState st, const u32* __restrict__ h, u32 K, u32* lds) {
  constexpr int NB = 1 << digit_bits(LEVEL);
  Found f, none;
  u32 total, top_count;
  find_in_bins<NB>(h, st.k_rem, 0u, lds, &f, &none, &total, &top_count);
  if (f.hit) {
    st.prefix = (st.prefix << digit_bits(LEVEL)) | f.digit;
    st.k_rem = f.inside;
    if (LEVEL == 2) {
      st.T = st.prefix;
      st.q = st.T == 0 ? 0u : st.k_rem;
      st.c_gt = K - st.k_rem;
      st.count = st.c_gt + st.q;
    }
  }
  return st;
}

// Which rows a level of the radix select is still open for when its histogram has been filled.
__device__ __forceinline__ bool radix_open(const RowState& st, int level) {
  if (st.mode == kModeGeneral) return st.row_emit == 0;
  if (st.mode == kModeCandWide) return true;
  return st.mode == kModeCandidates && level == 2;  // the filter's bins fixed the upper 21 bits
}

__device__ __forceinline__ u32* stage_hist(u32* hist, int stage, u32 M, u32 m) { return hist + ((size_t)stage * M + m) * kHistBins; }
enum { kStageSample0 = 0, kStageSample1 = 1, kStageFilter = 2, kStageRadix0 = 3 };  // radix level l: kStageRadix0 + l

// The tables the filter pass leaves for the kernels after it.
struct CandTables {
  u32* cand;       // [M][cand_stride] candidate words
  uint2* recs;     // [M][brk_stride]  bracket records
  u32* kept;       // [M][cand_stride] the fp32 bits of every candidate, slot for slot with its word (only the
                   // pass with a memory keeps them: it stores +0.0 over entries it takes for sure); else NULL
  u32 cand_stride, brk_stride, brk_shift;
  u64* wave_seg;   // [M][wave_stride][kChain]
  u64* wave_segb;  // [M][wave_stride][kChain]
  u32* wave_nseg;  // [M][wave_stride]
  u32 wave_stride, n_lists;
};

// ------------------------------------------------------------------------------------------------
// state reset for calls that take no sample (tiny rows, K = N): a kernel rather than a memset so that
// callers may capture the call into a graph.  Calls that do take one reset the state in its first kernel.
__device__ __forceinline__ void init_row(RowState* rs, RowCounters* rc, u32* status, u32 m, u32 M, u32 first_rank, u32 upper_rank, u32 mode,
                                         u32 first_alloc, u32 all_selected) {
  RowState s{};
  s.k_rem = first_rank;  // K on the general route, the sample rank of L on the candidate route
  s.q = upper_rank;      // candidate route: the sample rank of U (0: no entry is sure); cleared once U is there
  s.mode = mode;
  s.U = kNoUpper;
  s.row_emit = all_selected ? 2u : 0u;  // K = N: threshold 0, no tie slots (the zero-filled T and q), count from the scan
  rs[m] = s;
  RowCounters c{};
  c.n_alloc = first_alloc;  // candidate slots already handed out: the first slab of every wave of the filter pass
  rc[m] = c;
  if (m == 0) { status[0] = 0; status[1] = 0; status[2] = M; status[4] = 0; status[5] = 0; status[6] = 0; status[7] = 0; }
}

__global__ void k_encode_init(RowState* rs, RowCounters* rc, u32* status, u32 M, u32 K, u32 all_selected) {
  const u32 m = blockIdx.x * blockDim.x + threadIdx.x;
  if (m < M) init_row(rs, rc, status, m, M, K, 0u, kModeGeneral, 0u, all_selected);
}

// Zeroes the histograms of a call whose scratch may hold anything (scratch shared between shapes).
__global__ void k_clear_hist(u32* hist, u64 n) {
  for (u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (u64)gridDim.x * blockDim.x) hist[i] = 0;
}

// Histogram pass of one radix level (11 + 10 + 10 key bits, most significant first).
//   general rows            over the whole row
//   wide candidate rows     over the row's bracket records, every level
//   other candidate rows    over the bracket records at the last level only: the filter pass has
//                           already fixed the upper 21 bits
// Before that, every block takes the resolve step that has become possible: level 0 the verdict on
// the filter pass, the other levels the level before.
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void k_hist_rows(const float* __restrict__ grads, u64 N, u32 K, const RowState* __restrict__ rs_in,
                                                      RowState* __restrict__ rs_out, const RowCounters* __restrict__ rc,
                                                      u32* __restrict__ hist, u32 n_tiles, u32* __restrict__ status, CandTables t,
                                                      u32 parts, u32 have_bins) {
  constexpr int NB = 1 << digit_bits(LEVEL);
  constexpr int SH = digit_shift(LEVEL);
  const u32 m = blockIdx.y, M = gridDim.y;
  __shared__ u32 h[NB];
  __shared__ u32 lds[kResolveLds];
  RowState st = rs_in[m];
  if (LEVEL == 0) {
    if (st.mode == kModeCandidates) st = advance_filter(st, stage_hist(hist, kStageFilter, M, m), rc[m], K, have_bins, lds);
  } else if (radix_open(st, LEVEL - 1)) {
    if (LEVEL == 1) st = advance_radix<0>(st, stage_hist(hist, kStageRadix0, M, m), K, lds);
    else st = advance_radix<1>(st, stage_hist(hist, kStageRadix0 + 1, M, m), K, lds);
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) rs_out[m] = st;
  if (!radix_open(st, LEVEL)) return;  // block-uniform
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
  } else {  // `parts` waves per segment list, each with a share of its records (their order does not matter here)
    const u32 lane = lane_id();
    for (u32 w = blockIdx.x * kWaves + (threadIdx.x >> 6); w < t.n_lists * parts; w += gridDim.x * kWaves) {
      const u32 g = w / parts, part = w - g * parts;
      const RecordWalk lw(t.wave_seg, t.wave_segb, t.wave_nseg, t.wave_stride, t.recs, t.brk_stride, m, g);
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
  u32* out = stage_hist(hist, kStageRadix0 + LEVEL, M, m);
  for (int i = threadIdx.x; i < NB; i += kBlock) {
    const u32 c = h[i];
    if (c) atomicAdd(&out[i], c);
  }
  if (LEVEL == 0 && nan) status[0] = 1;
}

// Per tile: entries above the threshold and entries equal to it, packed as (eq << 32) | gt.
// Every block first takes the last resolve step of the rows the radix select ran over the whole row for.
__global__ __launch_bounds__(kBlock) void k_tile_count(const float* __restrict__ grads, u64 N, u32 K, const RowState* __restrict__ rs_in,
                                                       RowState* __restrict__ rs_out, u32* __restrict__ hist,
                                                       u64* __restrict__ tile_cnt, u32 n_tiles, u32 tile_stride,
                                                       u32* __restrict__ status) {
  const u32 m = blockIdx.y, M = gridDim.y;
  __shared__ u32 lds[2 * kWaves > kResolveLds ? 2 * kWaves : kResolveLds];
  RowState st = rs_in[m];
  if (st.mode == kModeGeneral && st.row_emit == 0) st = advance_radix<2>(st, stage_hist(hist, kStageRadix0 + 2, M, m), K, lds);
  if (blockIdx.x == 0 && threadIdx.x == 0) rs_out[m] = st;
  if (st.mode != kModeGeneral) return;
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
                                                           RowState* __restrict__ rs) {
  if (rs[blockIdx.x].mode != kModeGeneral) return;
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
    if (rs[blockIdx.x].row_emit == 2u) {  // K = N: every non-zero entry is sent
      rs[blockIdx.x].c_gt = (u32)carry;
      rs[blockIdx.x].count = (u32)carry;
    }
  }
}

// Emits the words of every tile at its scanned offset, in ascending index.
// With a memory (`err` non-NULL) `grads` IS the memory buffer holding g, and every entry whose sign
// is sent is overwritten with +0.0; a tile is read and rewritten by the same block only.
// As the last kernel of a call it also ends the call for every row, whatever its route: counts[m],
// the pad words of rows that selected zeros, the route counters, the NaN flag, the histograms back to
// zero for the next call, and the rows' final state in the first state buffer.
__global__ __launch_bounds__(kBlock) void k_emit_rows(const float* grads, u64 N, u64 K, const RowState* __restrict__ rs,
                                                      RowState* __restrict__ rs_copy, const u64* __restrict__ tile_cnt, u32 n_tiles,
                                                      u32 tile_stride, u32* __restrict__ words, float* err, u32* __restrict__ counts,
                                                      u32* __restrict__ status, u32* __restrict__ nan_flag, u32* __restrict__ hist) {
  const u32 m = blockIdx.y, M = gridDim.y;
  const RowState st = rs[m];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (nan_flag && m == 0) *nan_flag = status[0] ? 1u : 0u;  // every kernel that raises it has run
    counts[m] = st.count;
    if (st.mode == kModeGeneral && !st.row_emit) atomicAdd(&status[1], 1u);
    if (st.mode == kModeCandWide) atomicAdd(&status[4], 1u);
    if (st.mode == kModeGeneral && st.row_emit) atomicAdd(&status[5], 1u);
    if (rs_copy) rs_copy[m] = st;
  }
  for (u64 i = (u64)st.count + blockIdx.x * blockDim.x + threadIdx.x; i < K; i += (u64)gridDim.x * blockDim.x)
    words[(size_t)m * K + i] = S3GD_PAD;
  for (int stage = 0; stage < kHistStages; ++stage) {
    u32* h = stage_hist(hist, stage, M, m);
    for (u32 i = blockIdx.x * blockDim.x + threadIdx.x; i < (u32)kHistBins; i += gridDim.x * blockDim.x) h[i] = 0;
  }
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
// Level 0: key bits [30:20] into 2048 bins; its first block per row also resets the row's state and
// counters for the call.  Level 1: every block first resolves level 0, then key bits [19:10] of the
// keys under L's prefix go into bins 0..1023 and of the keys under U's prefix into bins 1024..2047.
// With a memory (`err` non-NULL) the sampled value is g~ + eta * e.
template <int LEVEL>
__global__ __launch_bounds__(kBlock) void k_sample_hist(const float* __restrict__ grads, const float* __restrict__ err, float eta, u64 N,
                                                        const RowState* __restrict__ rs_in, RowState* __restrict__ rs_out,
                                                        RowCounters* __restrict__ rc, u32* __restrict__ status, u32* __restrict__ hist,
                                                        u32 n_units, u64 unit_stride, u32 rank_lo, u32 rank_hi, u32 first_alloc) {
  const u32 m = blockIdx.y, M = gridDim.y;
  __shared__ u32 h[kHistBins];
  __shared__ u32 lds[kResolveLds];
  RowState st{};
  if (LEVEL == 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) init_row(rs_out, rc, status, m, M, rank_lo, rank_hi, kModeCandidates, first_alloc, 0u);
  } else {
    st = advance_sample0(rs_in[m], stage_hist(hist, kStageSample0, M, m), lds);
    if (blockIdx.x == 0 && threadIdx.x == 0) rs_out[m] = st;
  }
  for (int i = threadIdx.x; i < kHistBins; i += kBlock) h[i] = 0;
  __syncthreads();
  const u32* row = reinterpret_cast<const u32*>(grads + (size_t)m * N);
  const u32* erow = err ? reinterpret_cast<const u32*>(err + (size_t)m * N) : nullptr;
  const u32 n_samples = n_units * kSampleUnit;
  const bool upper = st.q != 0;  // a rank is sought for U as well
#pragma unroll 4
  for (u32 i = blockIdx.x * kSamplePerBlock + threadIdx.x; i < (blockIdx.x + 1) * kSamplePerBlock && i < n_samples; i += kBlock) {
    const u32 u = i / kSampleUnit, e = i % kSampleUnit;
    const u64 pos = sample_unit_start(u, unit_stride) + e;
    u32 bits = row[pos];
    if (erow) bits = compensate_bits(bits, erow[pos], eta);
    const u32 key = bits & 0x7FFFFFFFu;
    if (LEVEL == 0) {
      atomicAdd(&h[key >> 20], 1u);
    } else {
      const u32 d = (key >> 10) & 1023u;
      if ((key >> 20) == st.prefix) atomicAdd(&h[d], 1u);
      if (upper && (key >> 20) == st.T) atomicAdd(&h[1024u + d], 1u);
    }
  }
  __syncthreads();
  u32* out = stage_hist(hist, LEVEL == 0 ? kStageSample0 : kStageSample1, M, m);
  for (int i = threadIdx.x; i < kHistBins; i += kBlock) {
    const u32 c = h[i];
    if (c) atomicAdd(&out[i], c);
  }
}

// The one pass over the gradients.  Every entry with key >= L is a candidate: its message word
// (n << 1) | (g < 0) is kept; if its key is below U it also leaves a bracket record (its position
// among the words of its segment, its fp32 bits).
// Waves work independently (no block barrier inside the loop): a wave owns a contiguous run of
// wave tiles (1024 entries each) and appends its candidates, in ascending index, to slabs of the
// row's pools.  What a wave leaves behind is its SEGMENT LIST: up to kChain segments (first word
// slot, words; first record slot, records), written once when the wave ends.  Waves in order, and
// each wave's segments in order, list the row's candidates in ascending index; the kernels after
// the pass walk them that way, one wave per list.  The block also histograms (key - L) >> 10 of the
// bracket's records into 2048 bins, the last of which is open-ended.
//
// Slabs.  A slab of n word slots comes with n >> brk_shift record slots (record slot = word slot >>
// brk_shift, so one reservation serves both).  Every wave starts with a slab of its own, assigned by
// position (no atomic), sized to about twice the candidates a wave expects; only a wave that fills
// it (skewed rows) reserves another, twice as large each time, with a returning atomic on the row's
// counter.  A wave that would need more than kChain segments (more than a hundred times its share)
// marks the row for the general route.  Those atomics are what must stay rare:
// all waves of a row hit ONE address, a few thousand of them per millisecond queue up behind each
// other, and a wave waiting for its atomic also waits for its prefetched tile (measured with
// 256-entry slabs reserved on demand: 26 000 atomics cost 0.4 ms of a 3.2 ms pass).
//
// Stores are rare and non-temporal: on this memory system ANY store traffic mixed into the read
// stream costs several per cent of read bandwidth, whatever its volume (measured: one 8-byte store
// per 4 KB read, or one 512-byte store per 256 KB read, both cost 9 %; non-temporal stores issued
// every 2 MB read cost 2.5 %).  So candidates are staged in LDS, as (index, bits), and leave it about
// thirteen hundred at a time; only then is a candidate turned into its word and, inside the bracket,
// its record, binned and tested for NaN: a candidate per lane instead of a lane or two at a time
// under the per-tile code's branches.
// (the stage is as large as three blocks per CU allow, 11 KB per wave: what the stores cost follows how
// often a wave issues them, and 1408 entries instead of 1024 took 3.6 % off the pass at K/N = 0.01)
constexpr int kStage = 1408;       // staged candidates per wave (at least a tile's 1024)
constexpr int kStageFlush = 1280;  // flush once this many are staged

struct FilterWave {
  u32 cur, end, total;  // word slab cursor, slab end, candidates so far (wave-uniform)
  u32 fill;             // candidates staged in LDS; they belong to word slots [cur - fill, cur)
  u32 seg_base, n_seg;  // first word slot of the segment being filled; segments already closed
  u32 nb, nb_total;     // bracket records written for the segment being filled / by the wave so far
  u32 pend;             // upper bound on the records the staged candidates will leave
  u32 brk_cap;          // bracket records the segment being filled has room for
  u64* segs;            // the wave's segment list in global memory, kChain entries: words ...
  u64* segsb;           // ... and records
  bool overflow, nan;
};

// Ends the segment being filled: its runs go to the wave's list.
__device__ __forceinline__ void close_segment(FilterWave& w, u32 lane, u32 brk_shift) {
  const u32 count = w.cur - w.seg_base;
  if (count == 0) return;  // wave-uniform
  if (w.n_seg < (u32)kChain) {
    if (lane == 0) {
      w.segs[w.n_seg] = ((u64)w.seg_base << 32) | count;
      w.segsb[w.n_seg] = ((u64)(w.seg_base >> brk_shift) << 32) | w.nb;
    }
    ++w.n_seg;
  } else {
    w.overflow = true;
  }
  w.nb_total += w.nb;
  w.nb = 0;
}

// Turns the staged candidates into words and records, written to the wave's slab, and enters the
// records into the block's bins.
__device__ __forceinline__ void flush_stage(FilterWave& w, const u64* stage, u32* __restrict__ out, uint2* __restrict__ outb, u32 lane,
                                            u32 L, u32 U, u32 brk_shift, u32* h) {
  __builtin_amdgcn_wave_barrier();
  const u32 first = w.cur - w.fill;
  u32* dst = out + first;
  u64* dstb = reinterpret_cast<u64*>(outb) + (w.seg_base >> brk_shift);
  const u32 Lq = L >> 10;
  for (u32 i0 = 0; i0 < w.fill; i0 += 64) {  // wave-uniform
    const u32 i = i0 + lane;
    const bool ok = i < w.fill;
    const u64 cd = ok ? stage[i] : 0ull;
    const u32 bits = (u32)(cd >> 32), key = bits & 0x7FFFFFFFu;
    if (ok) store_stream4(dst + i, ((u32)cd << 1) | (bits >> 31));
    w.nan |= ok && key > 0x7F800000u;
    const bool brk = ok && key < U;
    const u64 bm = ballot(brk);
    if (brk) {
      store_stream8(dstb + w.nb + ballot_rank(bm), ((u64)bits << 32) | (first + i - w.seg_base));
      const u32 bin = (key >> 10) - Lq;
      // the open top bin takes most records of a row whose bracket is far wider than the bins: one add per wave for those
      const bool top = bin >= (u32)kHistBins - 1;
      const u64 tm = ballot(top);
      if (!top) atomicAdd(&h[bin], 1u);
      else if (ballot_rank(tm) == 0) atomicAdd(&h[kHistBins - 1], (u32)__popcll(tm));
    }
    w.nb += (u32)__popcll(bm);
  }
  __builtin_amdgcn_wave_barrier();
  w.fill = 0;
  w.pend = 0;
}

// Writes the candidates of one tile, in ascending index, to the LDS stage.
__device__ __forceinline__ void place_candidates(const TileRegs& r, const bool (&pr)[kLoads * 4], const u64 (&mk)[kLoads * 4],
                                                 const u32 (&tot)[kLoads], u32 first_slot, u64 v0, u64* dst_stage) {
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
        dst_stage[o] = ((u64)r.b[i] << 32) | (u32)(v0 + (u64)j * 256 + e);
        ++o;
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

// The same for the pass with a memory: entries whose key is at or above `sure_from` are stored as +0.0.
// CHANGED_ONLY (the row is rewritten in place): a 64-byte run, the 16 bytes of four neighbouring lanes, is
// stored only if it holds such an entry.
template <bool INTERIOR, bool CHANGED_ONLY = false>
__device__ __forceinline__ void store_chunk_tile(u32* __restrict__ rowv, u32 tile, u32 lane, const TileRegs& r, u32 sure_from) {
  const u64 vbase = (u64)tile * kWaveTile;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    u32* p = rowv + vbase + (u64)j * 256 + (u64)lane * 4;
    u32 v[4];
    bool any = false;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool sure = (r.b[4 * j + e] & 0x7FFFFFFFu) >= sure_from && (INTERIOR || ((r.valid >> (4 * j + e)) & 1u));
      v[e] = sure ? 0u : r.b[4 * j + e];
      any |= sure;
    }
    if (CHANGED_ONLY && ((ballot(any) >> (lane & ~3u)) & 0xFull) == 0) continue;
    if (INTERIOR || ((r.valid >> (4 * j)) & 0xFu) == 0xFu) {
      store_stream16(p, v[0], v[1], v[2], v[3]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if ((r.valid >> (4 * j + e)) & 1u) p[e] = v[e];
    }
  }
}

template <bool INTERIOR>
__device__ __forceinline__ void filter_tile(const TileRegs& r, u32 a, u32 tile, u32 lane, u32 L, u32 U, u32* h, u64* stage, u32* n_alloc,
                                            u32* __restrict__ out, uint2* __restrict__ outb, u32 cand_stride, u32 slab, u32 brk_shift,
                                            FilterWave& w) {
  // One compare per entry; its lane mask doubles as the wave ballot, so counting and ranking the
  // candidates below is scalar work plus a few mbcnt.
  bool pr[kLoads * 4];
  u64 mk[kLoads * 4];
  u64 any = 0;
#pragma unroll
  for (int i = 0; i < kLoads * 4; ++i) {
    const u32 key = r.b[i] & 0x7FFFFFFFu;
    pr[i] = key >= L;
    if (!INTERIOR) pr[i] = pr[i] && ((r.valid >> i) & 1u);
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
  // Room for the tile's words and for its records.  Which candidates lie inside the bracket is only
  // looked at when they leave the stage; until the records could run out every candidate counts as one.
  bool full = w.cur + total > w.end;
  u32 recs_here = total;
  if (!full && w.nb + w.pend + total > w.brk_cap) {
    recs_here = 0;  // the tile's records, counted
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) recs_here += (u32)__popcll(ballot(pr[i] && (r.b[i] & 0x7FFFFFFFu) < U));
    if (w.nb + w.pend + recs_here > w.brk_cap) {
      flush_stage(w, stage, out, outb, lane, L, U, brk_shift, h);  // now the segment's record count is exact
      full = w.nb + recs_here > w.brk_cap;
    }
  }
  if (full) {
    flush_stage(w, stage, out, outb, lane, L, U, brk_shift, h);  // staged candidates belong to the old slab
    close_segment(w, lane, brk_shift);
    // the next slab: twice the previous one (slab, slab, 2 slab, 4 slab, ...), and at least what the tile needs
    const u32 grown = slab << (w.n_seg > 1 ? w.n_seg - 1 : 0);
    const u32 room = total > (recs_here << brk_shift) ? total : (recs_here << brk_shift);
    const u32 fit = (room + slab - 1) / slab * slab;
    const u32 need = grown > fit ? grown : fit;
    u32 b = 0;
    if (lane == 0) b = atomicAdd(n_alloc, need);
    w.cur = __builtin_amdgcn_readfirstlane(b);
    w.end = w.cur + need;
    w.seg_base = w.cur;
    w.brk_cap = need >> brk_shift;
    if (w.end > cand_stride || w.end < w.cur) {  // pool exhausted (or the counter wrapped): nothing more is written
      w.overflow = true;
      w.end = w.cur;
      w.seg_base = w.cur;
    }
  }
  if (w.overflow) return;
  if (w.fill + total > (u32)kStage) flush_stage(w, stage, out, outb, lane, L, U, brk_shift, h);
  const u64 v0 = (u64)tile * kWaveTile + (u64)lane * 4 - a;
  place_candidates(r, pr, mk, tot, w.fill, v0, stage);
  w.fill += total;
  w.pend += recs_here;
  w.cur += total;
  w.total += total;
  if (w.fill >= (u32)kStageFlush) flush_stage(w, stage, out, outb, lane, L, U, brk_shift, h);
}

// The filter pass over rows that are read only: persistent waves, each with a range of its own.
// Every block first resolves the second level of the sample: the bounds L and U of its row.
__global__ __launch_bounds__(kBlock) void k_filter(const float* __restrict__ grads, u64 N, u32 K, const RowState* __restrict__ rs_in,
                                                   RowState* __restrict__ rs_out, RowCounters* __restrict__ rc, u32* __restrict__ hist,
                                                   CandTables t, u32 n_wtiles, u32 tiles_per_wave, u32 slab, u32 rank_lo, u32 sample_cap,
                                                   u32* __restrict__ status) {
  const u32 m = blockIdx.y, M = gridDim.y;
  // A little over 40 KB of LDS: three blocks share a compute unit.  (With the resolve scratch taken from
  // the stage area four fit, and the pass is 1 % to 6 % slower: more waves in flight help a stream of
  // reads no further, and the stores of four blocks disturb it more than those of three.)
  __shared__ u32 h[kHistBins];
  __shared__ u64 stage_all[kWaves][kStage];
  __shared__ u32 lds[kResolveLds];
  bool diverted;
  const RowState st = advance_sample1(rs_in[m], stage_hist(hist, kStageSample1, M, m), K, rank_lo, 1u, sample_cap, lds, &diverted);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    rs_out[m] = st;
    if (diverted) atomicAdd(&status[7], 1u);
  }
  if (st.mode != kModeCandidates) return;  // block-uniform
  for (int i = threadIdx.x; i < kHistBins; i += kBlock) h[i] = 0;
  __syncthreads();
  const float* row = grads + (size_t)m * N;
  const u32 a = (u32)((reinterpret_cast<uintptr_t>(row) >> 2) & 3u);
  const u32* rowv = reinterpret_cast<const u32*>(row) - a;
  const u64 vend = N + a;
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  u32* out = t.cand + (size_t)m * t.cand_stride;
  uint2* outb = t.recs + (size_t)m * t.brk_stride;
  u64* stage = stage_all[wave];
  const u32 g = blockIdx.x * kWaves + wave;  // the wave's position among the waves of its row
  FilterWave w{};
  w.cur = g * slab;  // the wave's first slab; the row's slot counter starts past all of them
  w.end = w.cur + slab;
  w.seg_base = w.cur;
  w.brk_cap = slab >> t.brk_shift;
  w.segs = t.wave_seg + ((size_t)m * t.wave_stride + g) * kChain;
  w.segsb = t.wave_segb + ((size_t)m * t.wave_stride + g) * kChain;
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
    if (tile >= first && tile < last)
      filter_tile<true>(r, a, tile, lane, st.L, st.U, h, stage, &rc[m].n_alloc, out, outb, t.cand_stride, slab, t.brk_shift, w);
    else
      filter_tile<false>(r, a, tile, lane, st.L, st.U, h, stage, &rc[m].n_alloc, out, outb, t.cand_stride, slab, t.brk_shift, w);
  }
  if (!w.overflow) {
    flush_stage(w, stage, out, outb, lane, st.L, st.U, t.brk_shift, h);
    close_segment(w, lane, t.brk_shift);
  }
  if (lane == 0) {
    t.wave_nseg[(size_t)m * t.wave_stride + g] = w.overflow ? 0u : w.n_seg;
    if (w.overflow) rc[m].overflow = 1;
  }
  if (w.nan) status[0] = 1;
  __syncthreads();  // every wave is done with its stage
  if (lane == 0) { lds[2 * wave] = w.total; lds[2 * wave + 1] = w.nb_total; }
  __syncthreads();
  // one addition per block for both counts: every wave of the row ends at about the same time, and
  // additions to one address complete one after the other
  if (threadIdx.x == 0) {
    u32 block_cand = 0, block_brk = 0;
    for (int i = 0; i < kWaves; ++i) { block_cand += lds[2 * i]; block_brk += lds[2 * i + 1]; }
    if (block_cand) atomicAdd(reinterpret_cast<unsigned long long*>(&rc[m].n_cand), ((unsigned long long)block_brk << 32) | block_cand);
  }
  u32* bins = stage_hist(hist, kStageFilter, M, m);
  for (int i = threadIdx.x; i < kHistBins; i += kBlock) {
    const u32 c = h[i];
    if (c) atomicAdd(&bins[i], c);
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

// The chunked pass with a memory, bare: a block per 8192 consecutive entries, launched in index order,
// reads its part of `a` and of `b` and writes a + b over b (the loads, the stores and the rounding of
// k_filter_chunks with eta = 1, none of its counting, reserving or placing).
__global__ __launch_bounds__(kBlock) void k_plain_rmw(const float* __restrict__ a, float* __restrict__ b) {
  const u32* av = reinterpret_cast<const u32*>(a);
  u32* bv = reinterpret_cast<u32*>(b);
  const u32 lane = lane_id(), wave = threadIdx.x >> 6;
  const u32 t0 = (blockIdx.x * kWaves + wave) * kChunkTiles;
  TileRegs r[kChunkTiles], e[kChunkTiles];
#pragma unroll
  for (int k = 0; k < kChunkTiles; ++k) {
    load_filter_tile<true>(av, 0, 0, t0 + k, lane, r[k]);
    load_filter_tile<true>(bv, 0, 0, t0 + k, lane, e[k]);
  }
#pragma unroll
  for (int k = 0; k < kChunkTiles; ++k) {
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) r[k].b[i] = compensate_bits(r[k].b[i], e[k].b[i], 1.0f);
    store_filter_tile<true>(bv, t0 + k, lane, r[k]);
  }
}

// Six waves per SIMD (80 registers, seven of them spilled) measured 2 % faster than the five the kernel takes
// by itself (85 registers); so did it against a variant that reaches six without spilling (its block sums
// and wave number kept in scalar registers: 79 registers, 3 % slower on the same machine).  The form that
// stores zeros over the sure entries needs 100 registers (the stored values are new 16-byte tuples beside
// the tile's own): at six waves it spills 54 and is 10 % slower, at five it spills two and is 3 % slower
// than the plain form, so it runs at five and only where the zeros it saves the emit pass outweigh that.
constexpr int kChunkWavesPerSimd = 6;
constexpr int kChunkWavesPerSimdZero = 5;

// ---- the filter pass with a memory, in chunks --------------------------------------------------
// The row is g = grads + eta * err, and g is written over err as it is filtered (grads and err rows
// start at the same 16-byte phase, checked by the caller).  One block per chunk of 8192 consecutive
// entries, launched in index order; a wave holds its kChunkTiles consecutive wave tiles in
// registers.  The block counts its candidates and its bracket records, reserves exactly that many
// slots of the row's two pools with one atomic each, and its waves write them there in ascending
// index.  Chunk c leaves its two runs as entry c of the row's segment tables, so that list g of the
// tables (kChain entries) is chunks g*kChain .. g*kChain + kChain - 1 in order.  No bins are filled:
// the radix select then runs over the records at every level.
//
// Why not persistent waves as in k_filter: this pass reads two rows and writes one, and blocks
// dispatched in index order keep the running blocks inside a compact window of the three streams,
// which the memory system rewards (a bare read-modify-write stream: 5.9 TB/s against 5.2 TB/s for
// waves that each stream a far-apart range).  A read-only pass gains nothing from it, and the
// returning atomics per block, harmless next to 96 KB of traffic, would bound it: atomics on one
// counter (or on the neighbouring counters of a few rows) complete at about 86 per microsecond.
template <bool INTERIOR>
__device__ __forceinline__ void count_chunk_tile(const TileRegs& r, u32 L, u32 U, u32& cand, u32& brk, bool& nan) {
#pragma unroll
  for (int i = 0; i < kLoads * 4; ++i) {
    const u32 key = r.b[i] & 0x7FFFFFFFu;
    bool p = key >= L;
    if (!INTERIOR) p = p && ((r.valid >> i) & 1u);
    nan |= p && key > 0x7F800000u;
    cand += (u32)__popcll(ballot(p));
    brk += (u32)__popcll(ballot(p && key < U));
  }
}

// Writes the words and the records of one tile at their exact slots.  `first_word`, `first_rec`: the
// tile's first slots; `seg_word`: the first word slot of the chunk (records hold positions relative to it).
template <bool INTERIOR>
__device__ __forceinline__ void place_chunk_tile(const TileRegs& r, u32 a, u32 tile, u32 lane, u32 L, u32 U, u32 first_word, u32 first_rec,
                                                 u32 seg_word, u32* __restrict__ out, uint2* __restrict__ outb, u32* __restrict__ kept) {
  const u64 v0 = (u64)tile * kWaveTile + (u64)lane * 4 - a;
  u32 run = first_word, runb = first_rec;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) {
    bool pr[4], br[4];
    u64 mk[4], bk[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const u32 key = r.b[4 * j + e] & 0x7FFFFFFFu;
      pr[e] = key >= L;
      if (!INTERIOR) pr[e] = pr[e] && ((r.valid >> (4 * j + e)) & 1u);
      br[e] = pr[e] && key < U;
      mk[e] = ballot(pr[e]);
      bk[e] = ballot(br[e]);
    }
    if ((mk[0] | mk[1] | mk[2] | mk[3]) == 0) continue;  // wave-uniform
    u32 o = run + ballot_rank(mk[0]) + ballot_rank(mk[1]) + ballot_rank(mk[2]) + ballot_rank(mk[3]);
    u32 ob = runb + ballot_rank(bk[0]) + ballot_rank(bk[1]) + ballot_rank(bk[2]) + ballot_rank(bk[3]);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (pr[e]) {
        const u32 bits = r.b[4 * j + e];
        out[o] = ((u32)(v0 + (u64)j * 256 + e) << 1) | (bits >> 31);
        if (kept) kept[o] = bits;  // (uniform)
        if (br[e]) { outb[ob] = make_uint2(o - seg_word, bits); ++ob; }
        ++o;
      }
    }
    run += (u32)__popcll(mk[0]) + (u32)__popcll(mk[1]) + (u32)__popcll(mk[2]) + (u32)__popcll(mk[3]);
    runb += (u32)__popcll(bk[0]) + (u32)__popcll(bk[1]) + (u32)__popcll(bk[2]) + (u32)__popcll(bk[3]);
  }
}

// FORMED: the memory buffer already holds g (the caller accumulated the gradients into it): the pass reads the one
// row and rewrites it with the zeros, which from K = N/32 on costs less than the read-only pass followed by a
// scattered store per sent entry.
template <bool ZERO_SURE, bool FORMED>
__global__ __launch_bounds__(kBlock, ZERO_SURE ? kChunkWavesPerSimdZero : kChunkWavesPerSimd) void k_filter_chunks(const float* __restrict__ grads, float* __restrict__ err, float eta, u64 N,
                                                          const RowState* __restrict__ rs_in, RowState* __restrict__ rs_out,
                                                          RowCounters* __restrict__ rc, CandTables t, u32 n_chunks,
                                                          u32* __restrict__ status) {
  static_assert(kChunkTiles == 2, "the two wave tiles of a chunk are held in named registers");
  static_assert(ZERO_SURE || !FORMED, "a formed row is only rewritten for the zeros");
  const u32 m = blockIdx.y;
  __shared__ u32 wsum[kWaves], wsumb[kWaves];
  __shared__ u32 sbase, sbaseb;
  // (the bounds L and U were resolved by a kernel of their own: this one has a block per 32 KB of the row)
  const RowState st = rs_in[m];
  if (blockIdx.x == 0 && threadIdx.x == 0) rs_out[m] = st;
  if (st.mode != kModeCandidates) return;  // block-uniform
  u32* const cand = t.cand;
  uint2* const recs = t.recs;
  const u32 cand_stride = t.cand_stride, brk_stride = t.brk_stride, list_stride = t.wave_stride;
  u64* const list_seg = t.wave_seg;
  u64* const list_segb = t.wave_segb;
  u32* const list_nseg = t.wave_nseg;
  const float* row = (FORMED ? err : grads) + (size_t)m * N;
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
  TileRegs r0, r1;
  if (FORMED) {
    const u32 sure_from = st.U;
    if (in0) load_filter_tile<true>(rowv, a, vend, t0, lane, r0); else load_filter_tile<false>(rowv, a, vend, t0, lane, r0);
    if (in1) load_filter_tile<true>(rowv, a, vend, t1, lane, r1); else load_filter_tile<false>(rowv, a, vend, t1, lane, r1);
    if (in0) store_chunk_tile<true, true>(errv, t0, lane, r0, sure_from); else store_chunk_tile<false, true>(errv, t0, lane, r0, sure_from);
    if (in1) store_chunk_tile<true, true>(errv, t1, lane, r1, sure_from); else store_chunk_tile<false, true>(errv, t1, lane, r1, sure_from);
  } else {
    TileRegs e0, e1;
    if (in0) { load_filter_tile<true>(rowv, a, vend, t0, lane, r0); load_filter_tile<true>(errv, a, vend, t0, lane, e0); }
    else { load_filter_tile<false>(rowv, a, vend, t0, lane, r0); load_filter_tile<false>(errv, a, vend, t0, lane, e0); }
    if (in1) { load_filter_tile<true>(rowv, a, vend, t1, lane, r1); load_filter_tile<true>(errv, a, vend, t1, lane, e1); }
    else { load_filter_tile<false>(rowv, a, vend, t1, lane, r1); load_filter_tile<false>(errv, a, vend, t1, lane, e1); }
    // g = grads + eta * err goes over err right away: the stores are under way while the candidates are counted.
    // ZERO_SURE: the entries at or above U go as +0.0: they are selected whatever the threshold turns out to
    // be, and the emit pass is spared a scattered 4-byte store per sent entry.  Their magnitudes stay in
    // `kept`, beside their words, for the rare row that is handed to the general route after all (k_restore_kept).
    const u32 sure_from = ZERO_SURE ? st.U : kNoUpper;
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) r0.b[i] = compensate_bits(r0.b[i], e0.b[i], eta);
    if (ZERO_SURE) { if (in0) store_chunk_tile<true>(errv, t0, lane, r0, sure_from); else store_chunk_tile<false>(errv, t0, lane, r0, sure_from); }
    else { if (in0) store_filter_tile<true>(errv, t0, lane, r0); else store_filter_tile<false>(errv, t0, lane, r0); }
#pragma unroll
    for (int i = 0; i < kLoads * 4; ++i) r1.b[i] = compensate_bits(r1.b[i], e1.b[i], eta);
    if (ZERO_SURE) { if (in1) store_chunk_tile<true>(errv, t1, lane, r1, sure_from); else store_chunk_tile<false>(errv, t1, lane, r1, sure_from); }
    else { if (in1) store_filter_tile<true>(errv, t1, lane, r1); else store_filter_tile<false>(errv, t1, lane, r1); }
  }
  u32 c0 = 0, b0 = 0, c1 = 0, b1 = 0;
  bool nan = false;
  if (in0) count_chunk_tile<true>(r0, st.L, st.U, c0, b0, nan); else count_chunk_tile<false>(r0, st.L, st.U, c0, b0, nan);
  if (in1) count_chunk_tile<true>(r1, st.L, st.U, c1, b1, nan); else count_chunk_tile<false>(r1, st.L, st.U, c1, b1, nan);
  if (lane == 0) { wsum[wave] = c0 + c1; wsumb[wave] = b0 + b1; }
  if (nan) status[0] = 1;
  __syncthreads();
  u32 before = 0, total = 0, beforeb = 0, totalb = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const u32 c = wsum[w], b = wsumb[w];
    if ((u32)w < wave) { before += c; beforeb += b; }
    total += c;
    totalb += b;
  }
  if (threadIdx.x == 0) {
    u32 base = 0, baseb = 0;
    bool fits = true;
    if (total) {
      // one returning addition serves both pools (the two counters are one aligned 64-bit word): such
      // additions complete one after the other, about 86 per microsecond, and every block makes one
      const unsigned long long both = atomicAdd(reinterpret_cast<unsigned long long*>(&rc[m].n_alloc),
                                                ((unsigned long long)totalb << 32) | total);
      base = (u32)both;
      baseb = (u32)(both >> 32);
      fits = base + total <= cand_stride && base + total >= base && baseb + totalb <= brk_stride && baseb + totalb >= baseb;
      if (!fits) rc[m].overflow = 1;
    }
    sbase = fits ? base : 0xFFFFFFFFu;
    sbaseb = baseb;
    list_seg[(size_t)m * list_stride * kChain + chunk] = fits ? (((u64)base << 32) | total) : 0ull;
    list_segb[(size_t)m * list_stride * kChain + chunk] = fits ? (((u64)baseb << 32) | totalb) : 0ull;
    if (chunk % kChain == 0) {
      const u32 left = n_chunks - chunk;
      list_nseg[(size_t)m * list_stride + chunk / kChain] = left < (u32)kChain ? left : (u32)kChain;
    }
  }
  __syncthreads();
  const u32 base = sbase, baseb = sbaseb;
  if (ZERO_SURE && total != 0 && base == 0xFFFFFFFFu) {  // no room: nothing of this chunk is kept, so its part of g goes back whole
    if (in0) store_chunk_tile<true>(errv, t0, lane, r0, kNoUpper); else store_chunk_tile<false>(errv, t0, lane, r0, kNoUpper);
    if (in1) store_chunk_tile<true>(errv, t1, lane, r1, kNoUpper); else store_chunk_tile<false>(errv, t1, lane, r1, kNoUpper);
  }
  if (total == 0 || base == 0xFFFFFFFFu) return;
  u32* out = cand + (size_t)m * cand_stride;
  u32* kept = ZERO_SURE ? t.kept + (size_t)m * cand_stride : nullptr;
  uint2* outb = recs + (size_t)m * brk_stride;
  if (c0) {
    if (in0) place_chunk_tile<true>(r0, a, t0, lane, st.L, st.U, base + before, baseb + beforeb, base, out, outb, kept);
    else place_chunk_tile<false>(r0, a, t0, lane, st.L, st.U, base + before, baseb + beforeb, base, out, outb, kept);
  }
  if (c1) {
    if (in1) place_chunk_tile<true>(r1, a, t1, lane, st.L, st.U, base + before + c0, baseb + beforeb + b0, base, out, outb, kept);
    else place_chunk_tile<false>(r1, a, t1, lane, st.L, st.U, base + before + c0, baseb + beforeb + b0, base, out, outb, kept);
  }
}

// ---- the count and emit passes of the candidate route ---------------------------------------------
// k_cand_count, a wave per segment list: takes the last resolve step (the threshold T and the tie
// quota q) and leaves (records equal to T << 32) | (candidates that are selected without being ties:
// the records above T and every candidate outside the bracket) of each list.
// k_cand_emit, a block per segment list: adds up the counts of the lists before its own (every block
// for itself, with all loads in flight at once: a row has at most a few thousand lists; beyond that a
// scan kernel runs in between and the block reads its sum), which gives the slot of its first word
// and the ties already served, then copies its candidate words minus the bracket's losers (records
// below T, and the ties beyond the quota, which is applied in index order) to the row's message, in
// ascending index.  The losers of kDropRound candidates at a time are marked in an LDS bit map by the
// waves' walks over their records (a quarter of the list's records per wave); a wave then copies its
// quarter of the round's words past the marks, its first slot following from the marks before its
// quarter.  With a memory (`err` non-NULL), +0.0 goes over every entry whose sign is sent.
// A list is the candidates of one wave of the filter pass (a few hundred to tens of thousands), and
// every step of a walk over it is a round trip to memory: four waves per list, each with four groups
// of 64 entries in flight, keep those chains short.
constexpr u32 kDropRound = 65536;
constexpr u32 kSumDirect = 2048;  // lists per row up to which an emit block adds up its predecessors' counts itself

// One group of kWalk * 64 entries of a walk, all loads issued together.
template <typename Walk, typename T>
__device__ __forceinline__ void load_group(const Walk& w, u32 j0, u32 end, u32 lane, T (&buf)[kWalk]) {
#pragma unroll
  for (int u = 0; u < kWalk; ++u) {
    const u32 j = j0 + (u32)u * 64u + lane;
    buf[u] = j < end ? w.pool[w.locate(j)] : T{};
  }
}

// The share of wave `wave` when `n` entries starting at `first` are dealt out to the block's waves in
// runs of whole 64s.
__device__ __forceinline__ void wave_share(u32 first, u32 n, u32 wave, u32 n_waves, u32* lo, u32* hi) {
  const u32 each = (((n + n_waves - 1) / n_waves) + 63u) & ~63u;
  const u32 a = wave * each < n ? wave * each : n;
  const u32 b = a + each < n ? a + each : n;
  *lo = first + a;
  *hi = first + b;
}

__global__ __launch_bounds__(kBlock) void k_cand_count(const RowState* __restrict__ rs_in, RowState* __restrict__ rs_out,
                                                       u32* __restrict__ hist, CandTables t, u32 K, u64* __restrict__ list_counts,
                                                       u32 resolved) {
  const u32 m = blockIdx.y, M = gridDim.y;
  __shared__ u32 lds[kResolveLds];
  RowState st = rs_in[m];
  if (st.mode == kModeGeneral) {  // block-uniform
    if (blockIdx.x == 0 && threadIdx.x == 0) rs_out[m] = st;
    return;
  }
  const u32 lane = lane_id();
  const u32 g = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const bool mine = g < t.n_lists;  // wave-uniform
  // the list's table and its first records are requested before the threshold is resolved
  const RecordWalk rw(t.wave_seg, t.wave_segb, t.wave_nseg, t.wave_stride, t.recs, t.brk_stride, m, mine ? g : 0u);
  uint2 rbuf[kWalk];
  load_group(rw, 0u, mine ? rw.total : 0u, lane, rbuf);
  if (!resolved && (st.mode == kModeCandidates || st.mode == kModeCandWide))
    st = advance_radix<2>(st, stage_hist(hist, kStageRadix0 + 2, M, m), K, lds);
  if (blockIdx.x == 0 && threadIdx.x == 0) rs_out[m] = st;
  if (!mine) return;  // whole waves leave; nothing below synchronises across waves
  u32 gt = 0, eq = 0;
  for (u32 i0 = 0; i0 < rw.total; i0 += 64 * kWalk) {  // wave-uniform
    uint2 rec[kWalk];
    if (i0 == 0) {
#pragma unroll
      for (int u = 0; u < kWalk; ++u) rec[u] = rbuf[u];
    } else {
      load_group(rw, i0, rw.total, lane, rec);
    }
#pragma unroll
    for (int u = 0; u < kWalk; ++u) {
      const bool ok = i0 + (u32)u * 64u + lane < rw.total;
      const u32 key = rec[u].y & 0x7FFFFFFFu;
      gt += ok && key > st.T;
      eq += ok && key == st.T;
    }
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) { gt += __shfl_xor(gt, d, 64); eq += __shfl_xor(eq, d, 64); }
  gt += rw.words_total - rw.total;  // outside the bracket: all greater than T
  if (lane == 0) list_counts[(size_t)m * t.wave_stride + g] = ((u64)eq << 32) | gt;
}

// In-place exclusive scan of the lists' counts of every row (rows with more than kSumDirect lists).
__global__ __launch_bounds__(kScanBlock) void k_scan_lists(u64* __restrict__ list_counts, u32 n_lists, u32 stride,
                                                           const RowState* __restrict__ rs) {
  if (rs[blockIdx.x].mode == kModeGeneral) return;
  __shared__ u64 lds[kScanBlock / 64];
  u64* t = list_counts + (size_t)blockIdx.x * stride;
  u64 carry = 0;
  for (u32 base = 0; base < n_lists; base += kScanBlock * 4) {
    const u32 i0 = base + threadIdx.x * 4;
    u64 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = (i0 + k < n_lists) ? t[i0 + k] : 0;
    const u64 s = v[0] + v[1] + v[2] + v[3];
    u64 total;
    u64 ex = carry + block_excl_scan<u64>(s, &total, lds);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (i0 + k < n_lists) t[i0 + k] = ex;
      ex += v[k];
    }
    carry += total;
  }
}

// The tables of one list in LDS (the emit pass: a block per list).
struct ListTable {
  u32 wslot[kChain], wcount[kChain], wfirst[kChain];  // words: first slot, length, flat number of the first word of each segment
  u32 rslot[kChain], rcount[kChain], rfirst[kChain];  // records: the same
  u32 wtotal, rtotal, nseg;
};
__device__ __forceinline__ u32 locate_word(const ListTable& lt, u32 j) {
  if (lt.nseg <= 1u) return lt.wslot[0] + j;  // block-uniform
  u32 at = 0;
#pragma unroll
  for (int c = 0; c < kChain; ++c) {
    const u32 d = j - lt.wfirst[c];  // wraps to a huge value for words of earlier segments
    if (d < lt.wcount[c]) at = lt.wslot[c] + d;
  }
  return at;
}
// slot of record j, and the flat number of the first word of its segment
__device__ __forceinline__ u32 locate_record(const ListTable& lt, u32 j, u32* seg_word) {
  if (lt.nseg <= 1u) { *seg_word = 0; return lt.rslot[0] + j; }  // block-uniform
  u32 at = 0, sw = 0;
#pragma unroll
  for (int c = 0; c < kChain; ++c) {
    const u32 d = j - lt.rfirst[c];
    if (d < lt.rcount[c]) { at = lt.rslot[c] + d; sw = lt.wfirst[c]; }
  }
  *seg_word = sw;
  return at;
}
__device__ __forceinline__ void load_words(const ListTable& lt, const u32* pool, u32 j0, u32 end, u32 lane, u32 (&buf)[kWalk]) {
#pragma unroll
  for (int u = 0; u < kWalk; ++u) {
    const u32 j = j0 + (u32)u * 64u + lane;
    buf[u] = j < end ? pool[locate_word(lt, j)] : 0u;
  }
}
// records with the flat number of their candidate in .x
__device__ __forceinline__ void load_records(const ListTable& lt, const uint2* pool, u32 j0, u32 end, u32 lane, uint2 (&buf)[kWalk]) {
#pragma unroll
  for (int u = 0; u < kWalk; ++u) {
    const u32 j = j0 + (u32)u * 64u + lane;
    u32 seg_word = 0;
    buf[u] = j < end ? pool[locate_record(lt, j, &seg_word)] : make_uint2(0, 0);
    buf[u].x += seg_word;
  }
}

// WINNERS: the filter pass has already stored +0.0 over the sure entries (t.kept is set), so only the bracket's
// winners are still to be zeroed in the memory: they get a bit map of their own.
template <bool WINNERS>
__global__ __launch_bounds__(kBlock) void k_cand_emit(const RowState* __restrict__ rs, CandTables t, u64 K, const u64* __restrict__ list_counts,
                                                      u32 scanned, u32* __restrict__ words, float* __restrict__ err, u64 N) {
  const u32 m = blockIdx.y;
  __shared__ u32 drop[kDropRound / 32];
  __shared__ u32 won[WINNERS ? kDropRound / 32 : 1];
  __shared__ u32 part_eq[kWaves];
  __shared__ u64 lists_before;
  __shared__ ListTable lt;
  const RowState st = rs[m];
  if (st.mode == kModeGeneral) return;  // block-uniform
  const u32 lane = lane_id(), wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;  // one, two or four waves per list
  const u32 g = blockIdx.x;
  const u64* counts = list_counts + (size_t)m * t.wave_stride;
  // the counts of the lists before this one: the last wave adds them up, all loads in flight at once
  u64 mine = 0;
  if (wave == n_waves - 1) {
    if (scanned) {
      mine = lane == 0 ? counts[g] : 0ull;
    } else {
      for (u32 i = lane; i < g; i += 64) mine += counts[i];
    }
  }
  // the list's tables, by the first lanes of the first wave
  if (threadIdx.x < (u32)kChain) {
    const u32 c = threadIdx.x;
    const u32 n_seg = t.wave_nseg[(size_t)m * t.wave_stride + g];
    const u64 wg = t.wave_seg[((size_t)m * t.wave_stride + g) * kChain + c];
    const u64 rg = t.wave_segb[((size_t)m * t.wave_stride + g) * kChain + c];
    const u32 wc = c < n_seg ? (u32)wg : 0u, rcnt = c < n_seg ? (u32)rg : 0u;
    lt.wslot[c] = (u32)(wg >> 32);
    lt.rslot[c] = (u32)(rg >> 32);
    lt.wcount[c] = wc;
    lt.rcount[c] = rcnt;
    u32 wf = 0, rf = 0, wt = 0, rt = 0;  // the eight lanes scan their counts
#pragma unroll
    for (int d = 0; d < kChain; ++d) {
      const u32 wo = __shfl(wc, d, 64), ro = __shfl(rcnt, d, 64);
      if ((u32)d < c) { wf += wo; rf += ro; }
      wt += wo;
      rt += ro;
    }
    lt.wfirst[c] = wf;
    lt.rfirst[c] = rf;
    if (c == 0) { lt.wtotal = wt; lt.rtotal = rt; lt.nseg = n_seg; }
  }
  __syncthreads();
  if (lt.wtotal == 0) return;  // block-uniform
  const u32* wpool = t.cand + (size_t)m * t.cand_stride;
  const uint2* rpool = t.recs + (size_t)m * t.brk_stride;
  u32 rlo, rhi;  // this wave's records
  wave_share(0u, lt.rtotal, wave, n_waves, &rlo, &rhi);
  u32 wlo, whi;  // this wave's words of the first round
  wave_share(0u, lt.wtotal < kDropRound ? lt.wtotal : kDropRound, wave, n_waves, &wlo, &whi);
  uint2 rbuf[kWalk];
  u32 wbuf[kWalk];
  load_records(lt, rpool, rlo, rhi, lane, rbuf);
  load_words(lt, wpool, wlo, whi, lane, wbuf);
  float* erow = err ? err + (size_t)m * N : nullptr;
  u32* out = words + (size_t)m * K;
  // the ties among this wave's records (the waves after it must know)
  u32 eq = 0;
  for (u32 i0 = rlo; i0 < rhi; i0 += 64 * kWalk) {  // wave-uniform
    uint2 rec[kWalk];
    if (i0 == rlo) {
#pragma unroll
      for (int u = 0; u < kWalk; ++u) rec[u] = rbuf[u];
    } else {
      load_records(lt, rpool, i0, rhi, lane, rec);
    }
#pragma unroll
    for (int u = 0; u < kWalk; ++u) eq += i0 + (u32)u * 64u + lane < rhi && (rec[u].y & 0x7FFFFFFFu) == st.T;
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) eq += __shfl_xor(eq, d, 64);
  if (wave == n_waves - 1) {
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) mine += __shfl_xor(mine, d, 64);
    if (lane == 0) lists_before = mine;
  }
  if (lane == 0) part_eq[wave] = eq;
  if (threadIdx.x + n_waves < (u32)kWaves) part_eq[threadIdx.x + n_waves] = 0;  // the waves the block does not have
  __syncthreads();
  const u64 before = lists_before;  // (ties << 32) | selected without ties, over the lists before this one
  u32 eq_first = (u32)(before >> 32);  // ties before this wave's first record
#pragma unroll
  for (int w = 0; w < kWaves; ++w)
    if ((u32)w < wave) eq_first += part_eq[w];
  u32 o_round = (u32)before + ((u32)(before >> 32) < st.q ? (u32)(before >> 32) : st.q);
  const u32 wtotal = lt.wtotal;

  for (u32 a0 = 0; a0 < wtotal; a0 += kDropRound) {  // block-uniform
    const u32 a1 = a0 + kDropRound < wtotal ? a0 + kDropRound : wtotal;
    for (u32 i = threadIdx.x; i < (a1 - a0 + 31) / 32; i += blockDim.x) {
      drop[i] = 0;
      if (WINNERS) won[i] = 0;
    }
    __syncthreads();
    // this wave's records, in order: those of candidates before the round only count as ties seen, those
    // of the round are marked if they lose, and the walk ends at the first one beyond the round
    u32 eq_seen = eq_first;
    for (u32 i0 = rlo; i0 < rhi; i0 += 64 * kWalk) {  // wave-uniform
      uint2 rec[kWalk];
      if (i0 == rlo) {
#pragma unroll
        for (int u = 0; u < kWalk; ++u) rec[u] = rbuf[u];
      } else {
        load_records(lt, rpool, i0, rhi, lane, rec);
      }
      bool beyond = false;
#pragma unroll
      for (int u = 0; u < kWalk; ++u) {
        const bool ok = i0 + (u32)u * 64u + lane < rhi;
        const u32 at = rec[u].x;  // number of the record's candidate in the list
        const bool upto = ok && at < a1;  // the records ascend: these lanes are the low ones
        const u32 key = rec[u].y & 0x7FFFFFFFu;
        const bool is_eq = upto && key == st.T;
        const u64 eqm = ballot(is_eq);
        const bool sel = key > st.T || (is_eq && eq_seen + ballot_rank(eqm) < st.q);
        if (upto && at >= a0 && !sel) atomicOr(&drop[(at - a0) >> 5], 1u << ((at - a0) & 31u));
        if (WINNERS && upto && at >= a0 && sel) atomicOr(&won[(at - a0) >> 5], 1u << ((at - a0) & 31u));
        eq_seen += (u32)__popcll(eqm);
        beyond = beyond || ballot(ok && !upto) != 0;
      }
      if (beyond) break;  // wave-uniform
    }
    __syncthreads();
    // this wave's quarter of the round's words: its first slot follows from the marks before it
    if (a0 != 0) wave_share(a0, a1 - a0, wave, n_waves, &wlo, &whi);
    u32 marked = 0, marked_all = 0;
    for (u32 i = lane; i < (a1 - a0 + 31) / 32; i += 64) {
      const u32 c = (u32)__popc(drop[i]);
      marked_all += c;
      if (i * 32 < wlo - a0) marked += c;  // wlo - a0 is a multiple of 64: whole words
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) { marked += __shfl_xor(marked, d, 64); marked_all += __shfl_xor(marked_all, d, 64); }
    u32 o = o_round + (wlo - a0) - marked;
    u32 wd[kWalk];
    if (a0 == 0) {
#pragma unroll
      for (int u = 0; u < kWalk; ++u) wd[u] = wbuf[u];
    } else {
      load_words(lt, wpool, wlo, whi, lane, wd);
    }
    for (u32 i0 = wlo; i0 < whi; i0 += 64 * kWalk) {  // wave-uniform trip count
      u32 nx[kWalk];  // the next group is requested before this one is placed
      load_words(lt, wpool, i0 + 64 * kWalk, whi, lane, nx);
#pragma unroll
      for (int u = 0; u < kWalk; ++u) {
        if (i0 + (u32)u * 64u >= whi) break;  // wave-uniform
        const u32 j = i0 + (u32)u * 64u + lane;
        const bool sel = j < whi && !((drop[(j - a0) >> 5] >> ((j - a0) & 31u)) & 1u);
        const u64 sel_mask = ballot(sel);
        if (sel) {
          const u32 pos = o + ballot_rank(sel_mask);
          if (pos < K) {  // pos < K by construction
            out[pos] = wd[u];
            if (erow && (!WINNERS || ((won[(j - a0) >> 5] >> ((j - a0) & 31u)) & 1u))) erow[wd[u] >> 1] = 0.0f;
          }
        }
        o += (u32)__popcll(sel_mask);
      }
#pragma unroll
      for (int u = 0; u < kWalk; ++u) wd[u] = nx[u];
    }
    o_round += (a1 - a0) - marked_all;
    __syncthreads();  // the marks are cleared for the next round
  }
}

// A resolve step as a kernel of its own (one block per row), for the consumers whose grids are too
// large to repeat it in every block.
enum { kStepSample1 = 0, kStepRadix2Cand = 1, kStepFilter = 2 };
template <int STEP>
__global__ __launch_bounds__(kBlock) void k_advance(const RowState* __restrict__ rs_in, RowState* __restrict__ rs_out, u32* __restrict__ hist,
                                                    u32 K, u32 rank_lo, u32 have_bins, u32 sample_cap, u32* __restrict__ status,
                                                    const RowCounters* __restrict__ rcs) {
  const u32 m = blockIdx.x, M = gridDim.x;
  const RowCounters* rc = rcs + m;
  __shared__ u32 lds[kResolveLds];
  RowState st = rs_in[m];
  if (STEP == kStepSample1) {
    bool diverted;
    st = advance_sample1(st, stage_hist(hist, kStageSample1, M, m), K, rank_lo, have_bins, sample_cap, lds, &diverted);
    if (threadIdx.x == 0 && diverted) atomicAdd(&status[7], 1u);
  } else if (STEP == kStepFilter) {  // the row leaves kModeCandidates here when there are no bins, so the histogram pass does not repeat the step
    if (st.mode == kModeCandidates) st = advance_filter(st, stage_hist(hist, kStageFilter, M, m), *rc, K, have_bins, lds);
  } else if (st.mode == kModeCandidates || st.mode == kModeCandWide) {
    st = advance_radix<2>(st, stage_hist(hist, kStageRadix0 + 2, M, m), K, lds);
  }
  if (threadIdx.x == 0) rs_out[m] = st;
}

// The pass with a memory stored +0.0 over the entries it took for sure.  A row that is handed to the general
// route after that pass (its pool ran out, or more than K entries were at or above U) gets them back: every
// candidate that found room has its bits in `kept`, slot for slot with its word (for the candidates inside
// the bracket this rewrites what is there).  A wave per chunk of the pass; chunks without room kept nothing
// and zeroed nothing (their table entry is empty).
__global__ __launch_bounds__(kBlock) void k_restore_kept(const RowState* __restrict__ rs, CandTables t, u32 n_chunks, float* __restrict__ err, u64 N) {
  const u32 m = blockIdx.y;
  if (rs[m].mode != kModeGeneral) return;  // block-uniform
  const u32 lane = lane_id();
  const u32* words = t.cand + (size_t)m * t.cand_stride;
  const u32* kept = t.kept + (size_t)m * t.cand_stride;
  u32* row = reinterpret_cast<u32*>(err + (size_t)m * N);
  for (u32 c = blockIdx.x * kWaves + (threadIdx.x >> 6); c < n_chunks; c += gridDim.x * kWaves) {
    const u64 sg = t.wave_seg[(size_t)m * t.wave_stride * kChain + c];
    const u32 base = (u32)(sg >> 32), count = (u32)sg;
    for (u32 j = lane; j < count; j += 64) row[words[base + j] >> 1] = kept[base + j];
  }
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
  const hipError_t e = with_memory ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (k_filter_chunks<false, false>), kBlock, 0)
                                   : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_filter, kBlock, 0);
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

hipError_t launch_plain_rmw(const Workspace& ws, const float* a, float* b, u64 n, hipStream_t s) {
  const u64 n_chunks = n / ((u64)kWaveTile * kChunkTiles * kWaves);  // whole chunks only
  if (n_chunks == 0) return hipSuccess;
  if (n_chunks > 0x7FFFFFFFull) return hipErrorInvalidValue;
  ws.prof->begin(KID_PLAIN_RMW, s);
  k_plain_rmw<<<(u32)n_chunks, kBlock, 0, s>>>(a, b);
  ws.prof->end(s);
  return hipGetLastError();
}

// Upper estimate of the candidates per row when the sample rank is r and the sample fraction f:
// the count of keys above the r-th largest sample key is about r / f with deviation sqrt(r) / f.
static double candidate_bound(double r, double f) { return 1.25 * (r + 6.0 * sqrt(r) + 8.0) / f; }

// Word slots a row needs beyond the first slabs of its waves: what waves of skewed rows reserve on
// top (the bound is a quarter above the candidates expected, so this is nearly twice the row's
// candidates: all of them in later slabs, and most of that again lost to the doubling); at dense K,
// where the bound itself is a large part of the row and the candidates cannot crowd into a few
// waves' ranges, a sixteenth of the row and a quarter of the bound.
static double extra_slots(double bound, u64 N) {
  const double a = 1.5 * bound, b = 0.25 * bound + (double)N / 16.0;
  return a < b ? a : b;
}
static double first_slab_factor(double bound, u64 N) { return bound > (double)N / 16.0 ? 1.1 : 1.25; }

// The sample: how many entries, the ranks of the two bounds, the candidates to expect.
struct SamplePlan {
  u64 s;          // sampled entries per row (a power of two)
  double r, r_hi; // sample ranks of L and of U (r_hi 0: no entry is sure)
  double bound;   // upper estimate of the candidates per row
  u32 brk_shift;  // a segment of n word slots gets n >> brk_shift record slots
  bool ok;
};
static SamplePlan plan_sample(u64 N, u64 K) {
  SamplePlan sp{};
  // about 1024 sampled entries above the K-th magnitude, between 2^15 and 2^18 and never more than an
  // eighth of the row; at dense K (where every candidate kept costs a word written, read and written
  // again) the largest sample, for the tightest bounds
  const bool dense = K * 64 > N;
  u64 s = 1ull << 15;
  while (s < (1ull << 18) && s * 8 <= N && (dense || (double)s * (double)K < 1024.0 * (double)N)) s <<= 1;
  const double f = (double)s / (double)N, kf = (double)K * f;
  sp.s = s;
  sp.r = ceil(kf + 6.0 * sqrt(kf) + 8.0);
  sp.r_hi = floor(kf - 6.0 * sqrt(kf) - 8.0);
  if (sp.r_hi < 1.0) sp.r_hi = 0.0;
  sp.bound = candidate_bound(sp.r, f);
  // the share of the candidates that lies inside the bracket, with the same slack as the bound
  const double phi = (sp.r - sp.r_hi + 12.0 * sqrt(sp.r)) / sp.r;
  sp.brk_shift = phi > 0.2 ? 0u : (phi > 0.1 ? 1u : (phi > 0.05 ? 2u : 3u));
  sp.ok = sp.r < (double)s && sp.bound <= 0.75 * (double)N;
  return sp;
}

EncodePlan plan_encode(u32 M, u64 N, u64 K, u64 pool_bytes, u32 stream_blocks, bool chunks) {
  EncodePlan p{};
  p.n_tiles = encode_tiles(N);
  p.gx = blocks_per_row(M, p.n_tiles, stream_blocks);
  p.candidates = false;
  if (K == 0 || K == N || N < (1ull << 17)) return p;  // K = N selects nothing: count and emit
  const SamplePlan sp = plan_sample(N, K);
  if (!sp.ok) return p;  // K above about N/2: the candidates would be most of the row
  p.n_wtiles = (u32)((N + 3 + kWaveTile - 1) / kWaveTile);
  p.tiles_per_wave = (p.n_wtiles + p.gx * kWaves - 1) / (p.gx * kWaves);
  p.bound = sp.bound;
  p.brk_shift = sp.brk_shift;
  // slab: somewhat above the candidates expected per wave of the filter pass, a multiple of 256
  const double per_wave = first_slab_factor(sp.bound, N) * sp.bound / ((double)p.gx * kWaves);
  double slab = ceil(per_wave / kSlabMin) * kSlabMin;
  if (slab < kSlabMin) slab = kSlabMin;
  if (slab > kSlabMax) slab = kSlabMax;
  p.slab = (u32)slab;
  // a row needs room for the first slab of every wave and for what waves of skewed rows reserve on top
  double need = extra_slots(sp.bound, N) + (double)p.gx * kWaves * p.slab + kWaveTile;
  if (chunks) {  // blocks reserve exactly what they found: no slabs
    need = sp.bound + kWaveTile;
    p.n_chunks = chunk_count(N);
    p.n_lists = chunk_lists(N);
  }
  if (need > 4.0e9) return p;
  p.cand_stride = ((u32)need + 3u) & ~3u;
  p.brk_stride = (((p.cand_stride >> p.brk_shift) + 64u) + 1u) & ~1u;
  // with a memory, from K = N/512 on, the pass stores zeros over the entries it takes for sure and keeps their bits
  // beside their words (below that the scattered zeros of the emit pass cost less than the slower pass)
  p.zero_sure = chunks && K * 512 >= N;
  if ((double)M * ((p.zero_sure ? 8.0 : 4.0) * p.cand_stride + 8.0 * p.brk_stride) + 16.0 > (double)pool_bytes) return p;
  p.candidates = true;
  p.chunks = chunks;
  p.n_units = (u32)(sp.s / kSampleUnit);
  p.unit_stride = N / p.n_units;
  p.sample_rank = (u32)sp.r;
  p.sample_rank_hi = (u32)sp.r_hi;
  return p;
}

u64 candidate_pool_bytes(u32 M_max, u64 N_max, u64 K_max) {
  // the need is not monotone in K (the sample size changes in powers of two, the record share in
  // steps): take the largest over K_max and the sparsities below it down to 1e-5
  double best = 0;
  for (double k = (double)K_max; k >= 1.0 && k >= 1e-5 * (double)N_max; k /= 2.0) {
    if ((u64)k >= N_max || N_max < (1ull << 17)) continue;
    const SamplePlan sp = plan_sample(N_max, (u64)k);
    if (!sp.ok) continue;
    // per row: what skewed waves reserve on top, the first slabs (rounded up to whole slabs below), two tiles of slack
    const double slots = extra_slots(sp.bound, N_max) + first_slab_factor(sp.bound, N_max) * sp.bound + 2.0 * kWaveTile;
    const double bytes = 4.0 * (slots + 4.0) + 8.0 * (slots / (double)(1u << sp.brk_shift) + 66.0);
    if (bytes > best) best = bytes;
    // the pass with a memory: exactly the candidates found, and their bits kept beside their words
    const double slots_c = sp.bound + 2.0 * kWaveTile;
    const double bytes_c = 8.0 * (slots_c + 4.0) + 8.0 * (slots_c / (double)(1u << sp.brk_shift) + 66.0);
    if (bytes_c > best) best = bytes_c;
  }
  if (best == 0) return 0;
  // once: the rounding of every wave's first slab to a whole smallest slab, words and records
  const u64 rounding = (u64)(kMaxStreamBlocks + M_max) * kWaves * kSlabMin * 12ull;
  return (u64)M_max * (u64)best + rounding;
}

// `err` NULL: the rows of `grads` are compressed as they are.  Otherwise the rows are
// g = grads + eta * err, and on return err holds the new memory g - TopK(g).
//
// A call on the candidate route is eleven launches (sample x 2, filter, radix histograms x 3, count,
// emit, and the three kernels of the general route, which return at once unless a row needs them):
// every resolve step between two passes is taken by the blocks of the later pass.
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
  // a formed row takes the pass in chunks too once K reaches N/32: rewriting the row with the zeros in it then
  // costs less than the read-only pass followed by a scattered store per sent entry (M = 8, N = 1.24e8:
  // 1.73 ms against 1.47 ms at K = N/50, 1.89 ms against 2.8 ms at K = N/20)
  const bool rewrite = formed && K * 32 >= N;
  EncodePlan p = plan_encode(M, N, K, ws.pool_bytes, (mem || rewrite) ? ws.stream_blocks_mem : ws.stream_blocks, mem != nullptr || rewrite);
  if (rewrite && !p.candidates) p = plan_encode(M, N, K, ws.pool_bytes, ws.stream_blocks, false);
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
  if (ws.hist_dirty) {
    const u64 n = (u64)kHistStages * M * kHistBins;
    S3GD_LAUNCH(KID_ENCODE_INIT, (k_clear_hist<<<(u32)((n + 1023) / 1024 < 256 ? (n + 1023) / 1024 : 256), 256, 0, s>>>(ws.hist, n)));
  }
  // the two state buffers: every kernel reads `cur` and writes `nxt`
  RowState* cur = ws.rs;
  RowState* nxt = ws.rs + ws.M_max;
#define S3GD_SWAP do { RowState* t_ = cur; cur = nxt; nxt = t_; } while (0)
  CandTables t{};
  t.wave_seg = ws.wave_seg;
  t.wave_segb = ws.wave_segb;
  t.wave_nseg = ws.wave_nseg;
  u32 have_bins = 1;
  if (p.candidates) {
    t.n_lists = p.chunks ? p.n_lists : p.gx * (u32)kWaves;  // segment lists per row
    t.wave_stride = p.chunks ? p.n_lists + 4 : wave_stride(p.gx);
    // the pool: the candidate words of every row, then their bracket records
    t.cand = reinterpret_cast<u32*>(ws.pool);
    t.recs = reinterpret_cast<uint2*>(ws.pool + (((size_t)M * p.cand_stride * 4 + 15) & ~(size_t)15));
    t.kept = p.zero_sure ? reinterpret_cast<u32*>(ws.pool + ((((size_t)M * p.cand_stride * 4 + 15) & ~(size_t)15) + (size_t)M * p.brk_stride * 8))
                      : nullptr;
    t.cand_stride = p.cand_stride;
    t.brk_stride = p.brk_stride;
    t.brk_shift = p.brk_shift;
    have_bins = p.chunks ? 0u : 1u;
    const dim3 sgrid((p.n_units * kSampleUnit + kSamplePerBlock - 1) / kSamplePerBlock, M);
    // sampled entries at or above L that stand for a row's whole share of the pool
    const double cap = (double)p.cand_stride * ((double)p.n_units * kSampleUnit / (double)N);
    const u32 sample_cap = cap < 1.0 ? 1u : (cap > 4.0e9 ? 0u : (u32)cap);
    const u32 first_alloc = p.chunks ? 0u : p.gx * (u32)kWaves * p.slab;
    S3GD_LAUNCH(KID_SAMPLE, (k_sample_hist<0><<<sgrid, kBlock, 0, s>>>(grads, mem, eta, N, cur, cur, ws.rc, ws.status, ws.hist, p.n_units,
                                                                       p.unit_stride, p.sample_rank, p.sample_rank_hi, first_alloc)));
    S3GD_LAUNCH(KID_SAMPLE, (k_sample_hist<1><<<sgrid, kBlock, 0, s>>>(grads, mem, eta, N, cur, nxt, ws.rc, ws.status, ws.hist, p.n_units,
                                                                       p.unit_stride, p.sample_rank, p.sample_rank_hi, first_alloc)));
    S3GD_SWAP;
    if (p.chunks) {
      S3GD_LAUNCH(KID_RESOLVE, (k_advance<kStepSample1><<<M, kBlock, 0, s>>>(cur, nxt, ws.hist, k32, p.sample_rank, 0u, 0u, ws.status, ws.rc)));
      S3GD_SWAP;
      if (p.zero_sure) {
        if (formed)
          S3GD_LAUNCH(KID_FILTER_MEM, (k_filter_chunks<true, true><<<dim3(p.n_chunks, M), kBlock, 0, s>>>(grads, err, eta, N, cur, nxt, ws.rc, t,
                                                                                                         p.n_chunks, ws.status)));
        else
          S3GD_LAUNCH(KID_FILTER_MEM, (k_filter_chunks<true, false><<<dim3(p.n_chunks, M), kBlock, 0, s>>>(grads, err, eta, N, cur, nxt, ws.rc, t,
                                                                                                          p.n_chunks, ws.status)));
        S3GD_SWAP;
        // the verdict on the pass, and for a row it sends to the general route the entries back that the pass stored as zeros
        S3GD_LAUNCH(KID_RESOLVE, (k_advance<kStepFilter><<<M, kBlock, 0, s>>>(cur, nxt, ws.hist, k32, 0u, 0u, 0u, ws.status, ws.rc)));
        S3GD_SWAP;
        const u32 rx = (p.n_chunks + kWaves - 1) / kWaves;
        S3GD_LAUNCH(KID_RESOLVE, (k_restore_kept<<<dim3(rx < 1024u ? rx : 1024u, M), kBlock, 0, s>>>(cur, t, p.n_chunks, err, N)));
      } else {
        S3GD_LAUNCH(KID_FILTER_MEM, (k_filter_chunks<false, false><<<dim3(p.n_chunks, M), kBlock, 0, s>>>(grads, err, eta, N, cur, nxt, ws.rc, t,
                                                                                                         p.n_chunks, ws.status)));
        S3GD_SWAP;
      }
    } else {
      S3GD_LAUNCH(KID_FILTER, (k_filter<<<grid, kBlock, 0, s>>>(grads, N, k32, cur, nxt, ws.rc, ws.hist, t, p.n_wtiles, p.tiles_per_wave, p.slab,
                                                               p.sample_rank, sample_cap, ws.status)));
      S3GD_SWAP;
    }
  } else {
    S3GD_LAUNCH(KID_ENCODE_INIT, (k_encode_init<<<(M + 255) / 256, 256, 0, s>>>(cur, ws.rc, ws.status, M, k32, all ? 1u : 0u)));
  }
  // Radix select: over the row for general rows, over the bracket's records for the others (the last
  // level only, unless the filter's bins could not place the K-th key).
  const dim3 hgrid(p.candidates ? 4 * p.gx : p.gx, M);  // histogram launches
  // where the records' order does not matter a list is shared by as many waves as that grid has for it
  u32 parts = t.n_lists ? hgrid.x * (u32)kWaves / t.n_lists : 1u;
  parts = parts < 1 ? 1u : (parts > 4 ? 4u : parts);
  if (!all) {
    S3GD_LAUNCH(KID_HIST0, (k_hist_rows<0><<<hgrid, kBlock, 0, s>>>(src, N, k32, cur, nxt, ws.rc, ws.hist, n_tiles, ws.status, t, parts, have_bins)));
    S3GD_SWAP;
    S3GD_LAUNCH(KID_HIST1, (k_hist_rows<1><<<hgrid, kBlock, 0, s>>>(src, N, k32, cur, nxt, ws.rc, ws.hist, n_tiles, ws.status, t, parts, have_bins)));
    S3GD_SWAP;
    S3GD_LAUNCH(KID_HIST2, (k_hist_rows<2><<<hgrid, kBlock, 0, s>>>(src, N, k32, cur, nxt, ws.rc, ws.hist, n_tiles, ws.status, t, parts, have_bins)));
    S3GD_SWAP;
  }
  if (p.candidates) {
    const u32 cx = (t.n_lists + kWaves - 1) / kWaves;  // count: a wave per segment list
    const u32 pre = cx > 2048 ? 1u : 0u;  // too many blocks to repeat the last resolve step in each
    if (pre) {
      S3GD_LAUNCH(KID_RESOLVE, (k_advance<kStepRadix2Cand><<<M, kBlock, 0, s>>>(cur, nxt, ws.hist, k32, 0u, 0u, 0u, ws.status, ws.rc)));
      S3GD_SWAP;
    }
    S3GD_LAUNCH(KID_CAND_SELECT, (k_cand_count<<<dim3(cx, M), kBlock, 0, s>>>(cur, nxt, ws.hist, t, k32, ws.wave_sum, pre)));
    S3GD_SWAP;
    const u32 scanned = t.n_lists > kSumDirect ? 1u : 0u;
    if (scanned) S3GD_LAUNCH(KID_SCAN_TILES, (k_scan_lists<<<M, kScanBlock, 0, s>>>(ws.wave_sum, t.n_lists, t.wave_stride, cur)));
    // a block per list, of two or four waves by the length of the lists: every block is a chain of round
    // trips to memory, and smaller blocks leave room for more of them at a time (measured with one, two
    // and four waves on lists of 300 to 5000 candidates: two waves best throughout)
    const double per_list = p.bound / (double)t.n_lists;
    const u32 ew = per_list < 6144.0 ? 128u : (u32)kBlock;
    if (err && t.kept) S3GD_LAUNCH(KID_CAND_EMIT, (k_cand_emit<true><<<dim3(t.n_lists, M), ew, 0, s>>>(cur, t, K, ws.wave_sum, scanned, words, err, N)));
    else S3GD_LAUNCH(KID_CAND_EMIT, (k_cand_emit<false><<<dim3(t.n_lists, M), ew, 0, s>>>(cur, t, K, ws.wave_sum, scanned, words, err, N)));
  }
  // General rows: per-tile counts and the emit pass (both return at once for the other rows); the emit
  // kernel also ends the call for every row.
  S3GD_LAUNCH(KID_TILE_COUNT, (k_tile_count<<<grid, kBlock, 0, s>>>(src, N, k32, cur, nxt, ws.hist, ws.tile_cnt, n_tiles, stride, ws.status)));
  S3GD_SWAP;
  S3GD_LAUNCH(KID_SCAN_TILES, (k_scan_tiles<<<M, kScanBlock, 0, s>>>(ws.tile_cnt, n_tiles, stride, cur)));
  S3GD_LAUNCH(KID_EMIT, (k_emit_rows<<<grid, kBlock, 0, s>>>(src, N, K, cur, cur == ws.rs ? nullptr : ws.rs, ws.tile_cnt, n_tiles, stride, words, err,
                                                            counts, ws.status, nan_flag, ws.hist)));
#undef S3GD_SWAP
#undef S3GD_LAUNCH
  return hipGetLastError();
}

}  // namespace s3gd
