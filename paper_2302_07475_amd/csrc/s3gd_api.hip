// C ABI of the library: argument checks, scratch ownership, stage sequencing.
#include <math.h>
#include <mutex>
#include <new>

#include "s3gd_common.h"
#include "s3gd_kernels.h"

using namespace s3gd;

static_assert(KID_COUNT == S3GD_PROFILE_KERNELS, "header and kernel id list disagree");

struct s3gd_ctx {
  int device;
  u32 M_max;
  u64 N_max, K_max;
  void* base;
  size_t bytes;
  Workspace ws;
  Profiler prof;
  int last_hip;
};

namespace {

constexpr u32 kMaxRows = S3GD_M_LIMIT;  // rows map to gridDim.y

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Layout {
  size_t rs, rc, status, hist, tile_cnt, seg, blk_sum, wave_seg, wave_segb, wave_nseg, wave_sum, pool, total;
  u64 pool_bytes;
};

Layout layout(u32 M, u64 N, u64 K) {
  Layout l{};
  size_t off = 0;
  l.rs = off;       off = align_up(off + 2 * sizeof(RowState) * (size_t)M, 256);
  l.rc = off;       off = align_up(off + sizeof(RowCounters) * (size_t)M, 256);
  l.status = off;   off = align_up(off + sizeof(u32) * 8, 256);
  l.hist = off;     off = align_up(off + sizeof(u32) * (size_t)kHistStages * M * kHistBins, 256);
  l.tile_cnt = off; off = align_up(off + sizeof(u64) * (size_t)M * tile_stride(N), 256);
  l.seg = off;      off = align_up(off + sizeof(u32) * (size_t)M * seg_row_entries(N), 256);
  l.wave_seg = off; off = align_up(off + sizeof(u64) * wave_table_entries(M, N) * kChain, 256);
  l.wave_nseg = off; off = align_up(off + sizeof(u32) * wave_table_entries(M, N), 256);
  l.wave_sum = off; off = align_up(off + sizeof(u64) * wave_table_entries(M, N), 256);
  l.wave_segb = off; off = align_up(off + sizeof(u64) * wave_table_entries(M, N) * kChain, 256);
  l.blk_sum = off;  off = align_up(off + sizeof(u64) * (size_t)M * blk_stride(N), 256);
  l.pool_bytes = candidate_pool_bytes(M, N, K);
  l.pool = off;     off = align_up(off + (size_t)l.pool_bytes, 256);
  l.total = off;
  return l;
}

// Points the views of a workspace at a block of device memory laid out by `l`.
void bind_workspace(Workspace& ws, char* b, const Layout& l) {
  ws.rs = reinterpret_cast<RowState*>(b + l.rs);
  ws.rc = reinterpret_cast<RowCounters*>(b + l.rc);
  ws.status = reinterpret_cast<u32*>(b + l.status);
  ws.hist = reinterpret_cast<u32*>(b + l.hist);
  ws.tile_cnt = reinterpret_cast<u64*>(b + l.tile_cnt);
  ws.seg = reinterpret_cast<u32*>(b + l.seg);
  ws.wave_seg = reinterpret_cast<u64*>(b + l.wave_seg);
  ws.wave_nseg = reinterpret_cast<u32*>(b + l.wave_nseg);
  ws.wave_sum = reinterpret_cast<u64*>(b + l.wave_sum);
  ws.wave_segb = reinterpret_cast<u64*>(b + l.wave_segb);
  ws.blk_sum = reinterpret_cast<u64*>(b + l.blk_sum);
  ws.pool = b + l.pool;
  ws.pool_bytes = l.pool_bytes;
}

// Makes the context's device current for the duration of a call.
struct DeviceGuard {
  int prev = -1;
  bool switched = false;
  hipError_t err = hipSuccess;
  explicit DeviceGuard(int dev) {
    err = hipGetDevice(&prev);
    if (err == hipSuccess && prev != dev) {
      err = hipSetDevice(dev);
      switched = err == hipSuccess;
    }
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_shape(const s3gd_ctx* c, u32 M, u64 N, u64 K) {
  if (!c) return S3GD_E_INVAL;
  if (M == 0 || N == 0) return S3GD_E_INVAL;
  if (N > S3GD_N_LIMIT) return S3GD_E_RANGE;
  if (K > N) return S3GD_E_INVAL;
  if (M > c->M_max || N > c->N_max || K > c->K_max) return S3GD_E_INVAL;
  return S3GD_OK;
}

int hip_fail(s3gd_ctx* c, hipError_t e) {
  c->last_hip = (int)e;
  return S3GD_E_HIP;
}

}  // namespace

extern "C" {

S3GD_API size_t s3gd_workspace_bytes(uint32_t M_max, uint64_t N_max, uint64_t K_max) {
  if (M_max == 0 || N_max == 0 || N_max > S3GD_N_LIMIT) return 0;
  return layout(M_max, N_max, K_max).total;
}

S3GD_API int s3gd_create(s3gd_ctx** out, int device, uint32_t M_max, uint64_t N_max, uint64_t K_max) {
  if (!out) return S3GD_E_INVAL;
  *out = nullptr;
  if (M_max == 0 || M_max > kMaxRows || N_max == 0 || device < 0) return S3GD_E_INVAL;
  if (N_max > S3GD_N_LIMIT) return S3GD_E_RANGE;
  if (K_max > N_max) K_max = N_max;
  s3gd_ctx* c = new (std::nothrow) s3gd_ctx{};
  if (!c) return S3GD_E_NOMEM;
  c->device = device;
  c->M_max = M_max;
  c->N_max = N_max;
  c->K_max = K_max;
  DeviceGuard g(device);
  if (g.err != hipSuccess) { delete c; return S3GD_E_HIP; }
  const Layout l = layout(M_max, N_max, K_max);
  const hipError_t e = hipMalloc(&c->base, l.total);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return e == hipErrorOutOfMemory ? S3GD_E_NOMEM : S3GD_E_HIP;
  }
  c->bytes = l.total;
  char* b = static_cast<char*>(c->base);
  // the status words start clear: each call resets only the flags it can raise itself
  // ... and the histograms start all zero: every call leaves them that way
  if (hipMemset(b + l.status, 0, sizeof(u32) * 8) != hipSuccess ||
      hipMemset(b + l.hist, 0, sizeof(u32) * (size_t)kHistStages * M_max * kHistBins) != hipSuccess ||
      hipDeviceSynchronize() != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(c->base);
    delete c;
    return S3GD_E_HIP;
  }
  bind_workspace(c->ws, b, l);
  c->ws.M_max = M_max;
  c->ws.hist_dirty = false;
  c->ws.stream_blocks = resident_stream_blocks(device, false);
  c->ws.stream_blocks_mem = resident_stream_blocks(device, true);
  c->ws.prof = &c->prof;
  *out = c;
  return S3GD_OK;
}

S3GD_API int s3gd_destroy(s3gd_ctx* ctx) {
  if (!ctx) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (ctx->prof.ev) {
    for (int i = 0; i < 2 * Profiler::kPairs; ++i) (void)hipEventDestroy(ctx->prof.ev[i]);
    delete[] ctx->prof.ev;
  }
  const hipError_t e = hipFree(ctx->base);
  delete ctx;
  return e == hipSuccess ? S3GD_OK : S3GD_E_HIP;
}

S3GD_API int s3gd_topk_sign_encode(s3gd_ctx* ctx, const float* grads, uint32_t M, uint64_t N, uint64_t K, uint32_t* words,
                          uint32_t* counts, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!grads || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!aligned(grads, 4) || !aligned(words, 4) || !aligned(counts, 4)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_encode(ctx->ws, grads, nullptr, 0.0f, M, N, K, words, counts, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_majority_vote(s3gd_ctx* ctx, const uint32_t* words, const uint32_t* counts, uint32_t M, uint64_t N, uint64_t K,
                       int32_t* tally, int8_t* votes, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!counts || (K > 0 && !words) || (!tally && !votes)) return S3GD_E_INVAL;
  if (!aligned(words, 4) || !aligned(counts, 4) || !aligned(tally, 16) || !aligned(votes, 16)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_vote(ctx->ws, words, counts, M, N, K, tally, votes, nullptr, 0.0f, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

// A step size or momentum factor: finite and >= 0.  Negative zero is refused as well: with it
// lr * 0 is -0.0 and x - (-0.0) turns a parameter of -0.0 into +0.0, so "a coordinate without a
// vote and without momentum keeps its bits" would no longer hold.
static bool step_size_ok(float a) { return a >= 0.0f && !std::isinf(a) && !std::signbit(a); }

S3GD_API int s3gd_apply_update(s3gd_ctx* ctx, float* x, const int8_t* votes, float lr, uint64_t N, s3gd_stream_t stream) {
  if (!ctx || !x || !votes || N == 0) return S3GD_E_INVAL;
  if (N > S3GD_N_LIMIT) return S3GD_E_RANGE;
  if (N > ctx->N_max) return S3GD_E_INVAL;
  if (!step_size_ok(lr)) return S3GD_E_INVAL;
  if (!aligned(x, 16) || !aligned(votes, 16)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_update(ctx->ws, x, votes, lr, N, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_step(s3gd_ctx* ctx, const float* grads, uint32_t M, uint64_t N, uint64_t K, float* x, float lr, uint32_t* words,
              uint32_t* counts, int32_t* tally, int8_t* votes, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!grads || !x || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!step_size_ok(lr)) return S3GD_E_INVAL;
  if (!aligned(grads, 4) || !aligned(words, 4) || !aligned(counts, 4) || !aligned(x, 16) || !aligned(tally, 16) ||
      !aligned(votes, 16))
    return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_encode(ctx->ws, grads, nullptr, 0.0f, M, N, K, words, counts, s);
  if (e != hipSuccess) return hip_fail(ctx, e);
  if (K == 0 && !tally && !votes) return S3GD_OK;  // nobody votes, nothing moves
  e = launch_vote(ctx->ws, words, counts, M, N, K, tally, votes, x, lr, s);
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

// ---- the step on a static scratch array ----------------------------------------------------------
// For callers that cannot allocate.  `scratch` is a host-side stand-in for the array, not a device
// address: its address on each device comes from hipGetSymbolAddress, once per device, and only that
// pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[S3GD_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
struct StaticScratch {
  bool ready = false;
  char* ptr = nullptr;  // this device's copy of `scratch`
  u32 stream_blocks = 0, stream_blocks_mem = 0;
  Profiler prof;        // never enabled: the launch functions expect one
};
StaticScratch g_static[kMaxDevices];
std::mutex g_static_mutex;

// Looks up the array's address on `device` (which is current) the first time the device is used.
hipError_t static_scratch(int device, StaticScratch** out) {
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticScratch& st = g_static[device];
  if (!st.ready) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    st.ptr = static_cast<char*>(p);
    st.stream_blocks = resident_stream_blocks(device, false);
    st.stream_blocks_mem = resident_stream_blocks(device, true);
    st.ready = true;
  }
  *out = &st;
  return hipSuccess;
}
}  // namespace

S3GD_API int s3gd_step_static(int device, const float* grads, uint32_t M, uint64_t N, uint64_t K, float* x, float lr, uint32_t* words,
                     uint32_t* counts, int32_t* tally, int8_t* votes, uint32_t* nan_flag, s3gd_stream_t stream) {
  if (device < 0 || device >= kMaxDevices) return S3GD_E_INVAL;
  if (M == 0 || M > kMaxRows || N == 0) return S3GD_E_INVAL;
  if (N > S3GD_N_LIMIT) return S3GD_E_RANGE;
  if (K > N) return S3GD_E_INVAL;
  if (!grads || !x || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!step_size_ok(lr)) return S3GD_E_INVAL;
  if (!aligned(grads, 4) || !aligned(words, 4) || !aligned(counts, 4) || !aligned(x, 16) || !aligned(tally, 16) ||
      !aligned(votes, 16) || !aligned(nan_flag, 4))
    return S3GD_E_INVAL;
  const Layout l = layout(M, N, K);
  if (l.total > S3GD_STATIC_SCRATCH_BYTES) return S3GD_E_TOOBIG;
  DeviceGuard g(device);
  if (g.err != hipSuccess) return S3GD_E_HIP;
  StaticScratch* st = nullptr;
  if (static_scratch(device, &st) != hipSuccess) {
    (void)hipGetLastError();
    return S3GD_E_HIP;
  }
  Workspace ws{};
  bind_workspace(ws, st->ptr, l);
  ws.M_max = M;
  ws.hist_dirty = true;  // the array is laid out anew for every shape: what lies under the histograms is anybody's
  ws.stream_blocks = st->stream_blocks;
  ws.stream_blocks_mem = st->stream_blocks_mem;
  ws.prof = &st->prof;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (launch_encode(ws, grads, nullptr, 0.0f, M, N, K, words, counts, s, nan_flag) != hipSuccess) return S3GD_E_HIP;
  if (K == 0 && !tally && !votes) return S3GD_OK;  // nobody votes, nothing moves
  return launch_vote(ws, words, counts, M, N, K, tally, votes, x, lr, s) == hipSuccess ? S3GD_OK : S3GD_E_HIP;
}

namespace {
int check_memory_args(const float* grads, const float* err, float eta, u32 M, u64 N) {
  if (!grads || !err) return S3GD_E_INVAL;
  if (!(eta >= 0.0f) || isinf(eta)) return S3GD_E_INVAL;
  const uintptr_t g = reinterpret_cast<uintptr_t>(grads), e = reinterpret_cast<uintptr_t>(err);
  if ((g & 3) || (e & 3) || ((g ^ e) & 15)) return S3GD_E_INVAL;
  const uintptr_t bytes = (uintptr_t)M * N * 4;
  if (g < e + bytes && e < g + bytes) return S3GD_E_INVAL;  // overlap
  return S3GD_OK;
}
}  // namespace

S3GD_API int s3gd_topk_sign_encode_ec(s3gd_ctx* ctx, const float* grads, float* err, float eta, uint32_t M, uint64_t N, uint64_t K,
                             uint32_t* words, uint32_t* counts, s3gd_stream_t stream) {
  int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if ((rc = check_memory_args(grads, err, eta, M, N))) return rc;
  if (!counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!aligned(words, 4) || !aligned(counts, 4)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_encode(ctx->ws, grads, err, eta, M, N, K, words, counts, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_step_ec(s3gd_ctx* ctx, const float* grads, float* err, float eta, uint32_t M, uint64_t N, uint64_t K, float* x,
                 float lr, uint32_t* words, uint32_t* counts, int32_t* tally, int8_t* votes, s3gd_stream_t stream) {
  int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if ((rc = check_memory_args(grads, err, eta, M, N))) return rc;
  if (!x || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!step_size_ok(lr)) return S3GD_E_INVAL;
  if (!aligned(words, 4) || !aligned(counts, 4) || !aligned(x, 16) || !aligned(tally, 16) || !aligned(votes, 16)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_encode(ctx->ws, grads, err, eta, M, N, K, words, counts, s);
  if (e != hipSuccess) return hip_fail(ctx, e);
  if (K == 0 && !tally && !votes) return S3GD_OK;  // nobody votes, nothing moves
  e = launch_vote(ctx->ws, words, counts, M, N, K, tally, votes, x, lr, s);
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_topk_sign_encode_acc(s3gd_ctx* ctx, float* acc, uint32_t M, uint64_t N, uint64_t K, uint32_t* words,
                              uint32_t* counts, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!acc || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!aligned(acc, 4) || !aligned(words, 4) || !aligned(counts, 4)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_encode(ctx->ws, nullptr, acc, 0.0f, M, N, K, words, counts, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_step_acc(s3gd_ctx* ctx, float* acc, uint32_t M, uint64_t N, uint64_t K, float* x, float lr, uint32_t* words,
                  uint32_t* counts, int32_t* tally, int8_t* votes, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!acc || !x || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!step_size_ok(lr)) return S3GD_E_INVAL;
  if (!aligned(acc, 4) || !aligned(words, 4) || !aligned(counts, 4) || !aligned(x, 16) || !aligned(tally, 16) || !aligned(votes, 16))
    return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_encode(ctx->ws, nullptr, acc, 0.0f, M, N, K, words, counts, s);
  if (e != hipSuccess) return hip_fail(ctx, e);
  if (K == 0 && !tally && !votes) return S3GD_OK;  // nobody votes, nothing moves
  e = launch_vote(ctx->ws, words, counts, M, N, K, tally, votes, x, lr, s);
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_apply_update_momentum(s3gd_ctx* ctx, float* x, float* v, const int8_t* votes, float lr, float mu, uint64_t N,
                               s3gd_stream_t stream) {
  if (!ctx || !x || !v || !votes || N == 0) return S3GD_E_INVAL;
  if (N > S3GD_N_LIMIT) return S3GD_E_RANGE;
  if (N > ctx->N_max) return S3GD_E_INVAL;
  if (!step_size_ok(lr) || !step_size_ok(mu)) return S3GD_E_INVAL;
  if (!aligned(x, 16) || !aligned(v, 16) || !aligned(votes, 16)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_update_momentum(ctx->ws, x, v, votes, lr, mu, N, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_step_momentum(s3gd_ctx* ctx, const float* grads, float* err, float eta, uint32_t M, uint64_t N, uint64_t K,
                       float* x, float* v, float lr, float mu, uint32_t* words, uint32_t* counts, s3gd_stream_t stream) {
  int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (err && !grads) {  // the memory already holds the compensated gradients (as in s3gd_step_acc)
    if (!aligned(err, 4)) return S3GD_E_INVAL;
  } else if (err) {
    if ((rc = check_memory_args(grads, err, eta, M, N))) return rc;
  } else if (!grads || !aligned(grads, 4)) {
    return S3GD_E_INVAL;
  }
  if (!x || !v || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!step_size_ok(lr) || !step_size_ok(mu)) return S3GD_E_INVAL;
  if (!aligned(words, 4) || !aligned(counts, 4) || !aligned(x, 16) || !aligned(v, 16)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_encode(ctx->ws, grads, err, err ? eta : 0.0f, M, N, K, words, counts, s);
  if (e != hipSuccess) return hip_fail(ctx, e);
  e = launch_vote_momentum(ctx->ws, words, counts, M, N, K, x, v, lr, mu, s);  // also with K == 0: the momentum still moves x
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_randk_sign_encode(s3gd_ctx* ctx, const float* grads, uint32_t M, uint64_t N, uint64_t K, uint64_t seed, uint32_t t,
                           uint32_t* words, uint32_t* counts, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!grads || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!aligned(grads, 4) || !aligned(words, 4) || !aligned(counts, 4)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_randk_encode(ctx->ws, grads, M, N, K, seed, t, words, counts, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_step_randk(s3gd_ctx* ctx, const float* grads, uint32_t M, uint64_t N, uint64_t K, uint64_t seed, uint32_t t,
                    float* x, float lr, uint32_t* words, uint32_t* counts, int32_t* tally, int8_t* votes,
                    s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!grads || !x || !counts || (K > 0 && !words)) return S3GD_E_INVAL;
  if (!step_size_ok(lr)) return S3GD_E_INVAL;
  if (!aligned(grads, 4) || !aligned(words, 4) || !aligned(counts, 4) || !aligned(x, 16) || !aligned(tally, 16) ||
      !aligned(votes, 16))
    return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_randk_encode(ctx->ws, grads, M, N, K, seed, t, words, counts, s);
  if (e != hipSuccess) return hip_fail(ctx, e);
  if (K == 0 && !tally && !votes) return S3GD_OK;
  e = launch_vote(ctx->ws, words, counts, M, N, K, tally, votes, x, lr, s);
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_vote_update(s3gd_ctx* ctx, const uint32_t* words, const uint32_t* counts, uint32_t M, uint64_t N, uint64_t K,
                     float* x, float lr, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!counts || (K > 0 && !words) || !x) return S3GD_E_INVAL;
  if (!step_size_ok(lr)) return S3GD_E_INVAL;
  if (!aligned(words, 4) || !aligned(counts, 4) || !aligned(x, 16)) return S3GD_E_INVAL;
  if (K == 0) return S3GD_OK;  // nobody votes, nothing moves
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_vote(ctx->ws, words, counts, M, N, K, nullptr, nullptr, x, lr, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API uint64_t s3gd_packed_row_words(uint64_t N, uint64_t K) {
  if (N == 0 || N > S3GD_N_LIMIT) return 0;
  return packed_row_capacity(N, K);
}

S3GD_API int s3gd_pack_messages(s3gd_ctx* ctx, const uint32_t* words, const uint32_t* counts, uint32_t M, uint64_t N, uint64_t K,
                       uint32_t* packed, uint64_t row_words, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!counts || (K > 0 && !words) || !packed) return S3GD_E_INVAL;
  if (!aligned(words, 4) || !aligned(counts, 4) || !aligned(packed, 8)) return S3GD_E_INVAL;
  if ((row_words & 1) || row_words < packed_row_capacity(N, K)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_pack(ctx->ws, words, counts, M, N, K, packed, row_words, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_unpack_messages(s3gd_ctx* ctx, const uint32_t* packed, uint64_t row_words, uint32_t M, uint64_t N, uint64_t K,
                         uint32_t* words, uint32_t* counts, s3gd_stream_t stream) {
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  if (!counts || (K > 0 && !words) || !packed) return S3GD_E_INVAL;
  if (!aligned(words, 4) || !aligned(counts, 4) || !aligned(packed, 8)) return S3GD_E_INVAL;
  if ((row_words & 1) || row_words < 2) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_unpack(ctx->ws, packed, row_words, M, N, K, words, counts, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_votes_to_message(s3gd_ctx* ctx, const int8_t* votes, uint64_t N, uint64_t capacity, uint32_t* words,
                          uint32_t* count, s3gd_stream_t stream) {
  if (!ctx || !votes || !count || (capacity > 0 && !words) || N == 0) return S3GD_E_INVAL;
  if (N > S3GD_N_LIMIT) return S3GD_E_RANGE;
  if (N > ctx->N_max) return S3GD_E_INVAL;
  if (!aligned(votes, 16) || !aligned(words, 4) || !aligned(count, 4)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_votes_to_message(ctx->ws, votes, N, capacity, words, count, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_last_async_status(s3gd_ctx* ctx, s3gd_stream_t stream) {
  if (!ctx) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  u32 st[4] = {0, 0, 0, 0};
  hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
  if (e == hipSuccess) e = hipMemcpy(st, ctx->ws.status, sizeof(st), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(ctx, e);
  if (st[0]) return S3GD_E_NAN;
  if (st[3] & kCodingFormat) return S3GD_E_FORMAT;
  if (st[3] & kCodingCapacity) return S3GD_E_CAPACITY;
  return S3GD_OK;
}

S3GD_API int s3gd_last_encode_info(s3gd_ctx* ctx, s3gd_stream_t stream, uint32_t* out) {
  if (!ctx || !out) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  u32 st[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
  if (e == hipSuccess) e = hipMemcpy(st, ctx->ws.status, sizeof(st), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(ctx, e);
  out[0] = st[2];
  out[1] = st[1];
  out[2] = st[4];
  out[3] = st[5];
  out[4] = st[7];
  return S3GD_OK;
}

S3GD_API int s3gd_last_row_state(s3gd_ctx* ctx, s3gd_stream_t stream, uint32_t m, uint32_t* out) {
  if (!ctx || !out || m >= ctx->M_max) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
  if (e == hipSuccess) e = hipMemcpy(out, ctx->ws.rs + m, sizeof(RowState), hipMemcpyDeviceToHost);
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_encode_plan_info(const s3gd_ctx* ctx, uint32_t M, uint64_t N, uint64_t K, int with_memory, uint64_t* out) {
  if (!out) return S3GD_E_INVAL;
  const int rc = check_shape(ctx, M, N, K);
  if (rc) return rc;
  const EncodePlan p = plan_encode(M, N, K, ctx->ws.pool_bytes, with_memory ? ctx->ws.stream_blocks_mem : ctx->ws.stream_blocks,
                                   with_memory != 0);
  out[0] = p.candidates;
  out[1] = (p.chunks ? 1u : 0u) | (p.zero_sure ? 2u : 0u);
  out[2] = p.brk_shift;
  out[3] = p.gx;
  out[4] = p.tiles_per_wave;
  out[5] = p.slab;
  out[6] = p.cand_stride;
  out[7] = p.n_units;
  out[8] = p.unit_stride;
  out[9] = p.sample_rank;
  out[10] = kChain;
  out[11] = kSampleUnit;
  return S3GD_OK;
}

S3GD_API uint64_t s3gd_encode_sample_unit_start(uint32_t u, uint64_t unit_stride) {
  return unit_stride >= (uint64_t)kSampleUnit ? sample_unit_position(u, unit_stride) : 0;
}

S3GD_API int s3gd_profile_enable(s3gd_ctx* ctx, int on) {
  if (!ctx) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (on && !ctx->prof.ev) {
    ctx->prof.ev = new (std::nothrow) hipEvent_t[2 * Profiler::kPairs];
    if (!ctx->prof.ev) return S3GD_E_NOMEM;
    for (int i = 0; i < 2 * Profiler::kPairs; ++i) {
      // timing only (read after the stream has been synchronised): no system-scope fence, whose cache write-back and
      // invalidation would idle the stream around every timed kernel
      const hipError_t e = hipEventCreateWithFlags(&ctx->prof.ev[i], hipEventDisableSystemFence);
      if (e != hipSuccess) {  // leave no half-made event array behind
        for (int j = 0; j < i; ++j) (void)hipEventDestroy(ctx->prof.ev[j]);
        delete[] ctx->prof.ev;
        ctx->prof.ev = nullptr;
        ctx->prof.mode = 0;
        return hip_fail(ctx, e);
      }
    }
  }
  ctx->prof.mode = on == 2 ? 2 : (on != 0 ? 1 : 0);
  ctx->prof.used = 0;
  return S3GD_OK;
}

S3GD_API int s3gd_profile_read(s3gd_ctx* ctx, s3gd_stream_t stream, float* ms_sum, uint32_t* launches, int n) {
  if (!ctx || !ms_sum || !launches || n < S3GD_PROFILE_KERNELS) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  for (int i = 0; i < n; ++i) { ms_sum[i] = 0.0f; launches[i] = 0; }
  const hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(ctx, e);
  for (int i = 0; i < ctx->prof.used; ++i) {
    float ms = 0.0f;
    const hipError_t e2 = hipEventElapsedTime(&ms, ctx->prof.ev[2 * i], ctx->prof.ev[2 * i + 1]);
    if (e2 != hipSuccess) return hip_fail(ctx, e2);
    ms_sum[ctx->prof.kid[i]] += ms;
    launches[ctx->prof.kid[i]] += 1;
  }
  ctx->prof.used = 0;
  return S3GD_OK;
}

S3GD_API const char* s3gd_profile_kernel_name(int id) {
  static const char* names[KID_COUNT] = {
      "encode_init", "hist_rows_0", "hist_rows_1", "hist_rows_2", "resolve", "tile_count", "scan_tiles", "emit_rows",
      "sample", "filter", "cand_select", "cand_emit", "seg_bounds", "vote_dense", "vote_sparse",
      "apply_update", "compensate", "filter_mem", "vote_momentum", "apply_momentum", "pack", "unpack",
      "votes_to_message", "randk", "plain_read", "plain_rmw"};
  return (id >= 0 && id < KID_COUNT) ? names[id] : nullptr;
}

S3GD_API int s3gd_calibrate_read(s3gd_ctx* ctx, const float* buf, uint64_t n, s3gd_stream_t stream) {
  if (!ctx || !buf || !aligned(buf, 16)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_plain_read(ctx->ws, buf, n, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_calibrate_rmw(s3gd_ctx* ctx, const float* a, float* b, uint64_t n, s3gd_stream_t stream) {
  if (!ctx || !a || !b || !aligned(a, 16) || !aligned(b, 16)) return S3GD_E_INVAL;
  DeviceGuard g(ctx->device);
  if (g.err != hipSuccess) return hip_fail(ctx, g.err);
  const hipError_t e = launch_plain_rmw(ctx->ws, a, b, n, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? S3GD_OK : hip_fail(ctx, e);
}

S3GD_API int s3gd_last_hip_error(const s3gd_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

S3GD_API const char* s3gd_strerror(int code) {
  switch (code) {
    case S3GD_OK: return "ok";
    case S3GD_E_INVAL: return "invalid argument";
    case S3GD_E_RANGE: return "N exceeds 2^31 - 2";
    case S3GD_E_HIP: return "HIP runtime error";
    case S3GD_E_NOMEM: return "out of device memory";
    case S3GD_E_NAN: return "NaN in gradients";
    case S3GD_E_FORMAT: return "packed vector does not decode";
    case S3GD_E_CAPACITY: return "output buffer too small";
    case S3GD_E_TOOBIG: return "shape needs more scratch than the static array holds";
    default: return "unknown error";
  }
}

}  // extern "C"
