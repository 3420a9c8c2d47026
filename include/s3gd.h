/*
 * s3gd.h - C ABI of the S3GD-MV step library for AMD MI355X (gfx950).
 *
 * One step of sparse sign SGD with majority vote (Algorithm 1 of the paper, the
 * lines after the local gradient exists):
 *
 *   1. every worker m keeps the K largest-magnitude entries of its gradient
 *      g_m in R^N and sends only their signs, TopKSign(g_m)   (Section 2.1,
 *      eqs. "topk" and "topksign"; Section 2.2 "Gradient compression");
 *   2. the server sums the ternary messages per coordinate and takes the sign
 *      of the sum, with sgn(0) = 0                            (Section 2.2
 *      "Majority vote");
 *   3. the model moves by x <- x - delta * vote               (eq. "s3gd").
 *
 * All M workers are held as one row-major [M, N] fp32 tensor on one GPU.
 *
 * Conventions
 *   - Every pointer marked "dev" is DEVICE memory owned by the CALLER; the
 *     library never frees, reallocates or keeps it after the call's work has
 *     run.  Pointers marked "host" are ordinary host memory.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and return without synchronising the host.  Outputs are
 *     valid once the stream has reached that point.
 *   - Return value: 0 on success, a negative S3GD_E_* code otherwise.  Argument
 *     checks are done on the host before anything is enqueued; a failed call
 *     enqueues nothing.  No exceptions, no abort, nothing printed.
 *   - A context owns only scratch memory.  It is bound to one device and must
 *     not be used from two host threads or two streams at the same time.
 *   - Results are deterministic: the same inputs give bit-identical outputs.
 *
 * Message format (one 32-bit word per selected non-zero entry)
 *     word = (n << 1) | (g_{m,n} < 0)
 *   Words of a row are in ascending n.  A row has K slots; slots beyond
 *   counts[m] hold S3GD_PAD.  counts[m] == K unless fewer than K entries of the
 *   row are non-zero: a selected entry that is +0 or -0 has sgn = 0, sends
 *   nothing and is not in the support set N_m of Section 2.2.
 *
 * Selection rule.  Exactly K indices are selected per row.  The paper places
 *   the threshold between the K-th and (K+1)-th largest magnitude and says
 *   nothing about equal magnitudes; here the order is (|g| descending, index
 *   ascending), i.e. among equal magnitudes the lowest index wins.
 */
#ifndef S3GD_H
#define S3GD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define S3GD_API __attribute__((visibility("default")))
#else
#define S3GD_API
#endif

#define S3GD_OK 0
#define S3GD_E_INVAL (-1) /* NULL pointer, M == 0, N == 0, K > N, size above the context's maxima,  */
                          /* M_max > S3GD_M_LIMIT, misaligned buffer, lr or eta negative or not     */
                          /* finite, both vote outputs NULL, memory buffer at another 16-byte phase */
                          /* than the gradients                                                     */
#define S3GD_E_RANGE (-2) /* N > S3GD_N_LIMIT: index, sign bit and pad word must fit 32 bits         */
#define S3GD_E_HIP (-3)   /* a HIP runtime call failed; s3gd_last_hip_error() has its code           */
#define S3GD_E_NOMEM (-4) /* scratch allocation failed                                               */
#define S3GD_E_NAN (-5)   /* reported by s3gd_last_async_status(): a NaN was seen in grads           */
#define S3GD_E_FORMAT (-6)   /* reported by s3gd_last_async_status(): a packed vector did not decode */
#define S3GD_E_CAPACITY (-7) /* reported by s3gd_last_async_status(): an output buffer of the coding */
                             /* calls was too small for the vector it had to hold                    */

#define S3GD_E_TOOBIG (-8)   /* s3gd_step_static: the shape needs more scratch than the static array holds */

#define S3GD_PAD 0xFFFFFFFFu
#define S3GD_N_LIMIT 2147483646ull /* 2^31 - 2 */
#define S3GD_M_LIMIT 65535u        /* workers per context: rows are the second grid dimension of a launch */

typedef struct s3gd_ctx s3gd_ctx; /* opaque */
typedef void* s3gd_stream_t;      /* hipStream_t */

/* Bytes of device scratch a context created for these maxima allocates.  Pure host function. */
S3GD_API size_t s3gd_workspace_bytes(uint32_t M_max, uint64_t N_max, uint64_t K_max);

/* Creates a context on `device` and allocates its scratch once (hipMalloc).  Calls with
 * M <= M_max, N <= N_max, K <= K_max never allocate.  `out` is host memory.
 * M_max above S3GD_M_LIMIT or N_max == 0 is S3GD_E_INVAL; N_max above S3GD_N_LIMIT is S3GD_E_RANGE;
 * K_max above N_max is taken as N_max. */
S3GD_API int s3gd_create(s3gd_ctx** out, int device, uint32_t M_max, uint64_t N_max, uint64_t K_max);

/* Frees the scratch.  The caller must have synchronised every stream that used the context. */
S3GD_API int s3gd_destroy(s3gd_ctx* ctx);

/*
 * Worker side of Algorithm 1: words[m, :] = TopKSign(g_m) in the message format above
 * (Section 2.1 eqs. "topk", "topksign"; Section 2.2 "Gradient compression").
 *
 *   grads   dev, const  [M, N] fp32, row stride N, 4-byte aligned.  Never modified.  +-Inf is
 *                       legal; NaN is outside the contract (it is detected and reported through
 *                       s3gd_last_async_status, the outputs are then unspecified but in bounds).
 *   words   dev, out    [M, K] uint32, 4-byte aligned.  Every slot is written.
 *   counts  dev, out    [M] uint32.
 *   K       0 <= K <= N.  K == 0 writes counts = 0 only.  K == N sends every non-zero sign
 *           (signSGD with majority vote).
 * Outputs must not overlap inputs.
 */
S3GD_API int s3gd_topk_sign_encode(s3gd_ctx* ctx, const float* grads, uint32_t M, uint64_t N, uint64_t K,
                          uint32_t* words, uint32_t* counts, s3gd_stream_t stream);

/*
 * Server side: tally[n] = sum_m TopKSign(g_m)_n, votes[n] = sgn(tally[n]) with sgn(0) = 0
 * (Section 2.2 "Majority vote"; Algorithm 1, the "receive" line).
 *
 *   words, counts  dev, const  as written by s3gd_topk_sign_encode: ascending indices < N per row,
 *                              counts[m] <= K.  Rows with counts[m] == 0 cast no vote.
 *   tally   dev, out, nullable [N] int32, 16-byte aligned.
 *   votes   dev, out, nullable [N] int8,  16-byte aligned.  Not both NULL.
 * Every element of each non-NULL output is written (0 outside the union of supports).
 */
S3GD_API int s3gd_majority_vote(s3gd_ctx* ctx, const uint32_t* words, const uint32_t* counts, uint32_t M,
                       uint64_t N, uint64_t K, int32_t* tally, int8_t* votes, s3gd_stream_t stream);

/*
 * Model update, eq. "s3gd": x[n] <- fp32(x[n] - lr * votes[n]), one rounding; x[n] is left
 * bit-identical where votes[n] == 0.
 *
 *   x      dev, in/out  [N] fp32, 16-byte aligned.
 *   votes  dev, const   [N] int8 in {-1, 0, +1}, 16-byte aligned.
 *   lr     step size delta >= 0, finite (negative zero is refused).
 */
S3GD_API int s3gd_apply_update(s3gd_ctx* ctx, float* x, const int8_t* votes, float lr, uint64_t N,
                      s3gd_stream_t stream);

/*
 * The three calls above fused into one enqueue, same results.  tally and votes may both be
 * NULL; then the vote is applied to x without being materialised and only the cache lines of
 * x that hold a voted coordinate are touched.
 */
S3GD_API int s3gd_step(s3gd_ctx* ctx, const float* grads, uint32_t M, uint64_t N, uint64_t K, float* x,
              float lr, uint32_t* words, uint32_t* counts, int32_t* tally, int8_t* votes,
              s3gd_stream_t stream);

/*
 * s3gd_step for callers that cannot allocate device memory or hold a context: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit for bit the same outputs as s3gd_step, but the scratch (row states, histograms, candidate
 * pool, segment tables) lives in a static device array of S3GD_STATIC_SCRATCH_BYTES that every GPU
 * the library runs on holds until the process ends.  The call allocates and frees nothing.
 *
 *   device    the GPU that holds every buffer of the call; made current for the call.
 *   nan_flag  dev, out, nullable  [1] uint32: 1 if a NaN was seen in grads (outputs then unspecified
 *             but in bounds), else 0; valid once the stream has reached this point.  It stands in
 *             for s3gd_last_async_status, which needs a context.
 *   Shapes with s3gd_workspace_bytes(M, N, K) > S3GD_STATIC_SCRATCH_BYTES are refused with
 *   S3GD_E_TOOBIG before anything is enqueued; M above S3GD_M_LIMIT is S3GD_E_INVAL.
 *
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's contents (each
 * call resets what it needs): calls that overlap in time on one GPU, from any stream or thread, race
 * and must be ordered by the caller.  The first call on a device looks up the array's address; make
 * one call outside a capture before capturing others.
 */
#define S3GD_STATIC_SCRATCH_BYTES (128ull << 20)
S3GD_API int s3gd_step_static(int device, const float* grads, uint32_t M, uint64_t N, uint64_t K, float* x, float lr,
                     uint32_t* words, uint32_t* counts, int32_t* tally, int8_t* votes, uint32_t* nan_flag,
                     s3gd_stream_t stream);

/*
 * Worker side of Algorithm 1 WITH the error-compensation memory (Section 2.2 "Gradient update with
 * sparsification error compensation", eq. "gradupdate" and the unlabelled memory equation that
 * follows it; Algorithm 1, the two lines before "send"):
 *
 *     g_m   = g~_m + eta * e_m          evaluated in fp32 as written: a rounded product, then a
 *                                       rounded sum (eta = 1, the paper's setting, makes it one sum)
 *     words = TopKSign(g_m)             exactly as s3gd_topk_sign_encode would encode g_m
 *     e_m  <- g_m - TopK(g_m)           g_m off the selected set; +0.0 where a sign was sent; a
 *                                       selected entry that is +-0 sends nothing and keeps its bits
 *
 *   grads   dev, const   [M, N] fp32: the fresh stochastic gradients g~.  Never modified.
 *   err     dev, in/out  [M, N] fp32: e_m on entry, the new memory on return.  Must start at the same
 *                        16-byte phase as grads ((grads - err) a multiple of 16 bytes) and must not
 *                        overlap it.  Zero-fill it before the first iteration (e^0 = 0).
 *   eta     weight of the memory, finite and >= 0.
 *   words, counts, K     as in s3gd_topk_sign_encode.  K == 0 still folds the gradient into the
 *                        memory (err <- g~ + eta * err).
 * NaN in g (from the inputs, or from Inf - Inf) is reported through s3gd_last_async_status.
 */
S3GD_API int s3gd_topk_sign_encode_ec(s3gd_ctx* ctx, const float* grads, float* err, float eta, uint32_t M, uint64_t N,
                             uint64_t K, uint32_t* words, uint32_t* counts, s3gd_stream_t stream);

/* One whole iteration of Algorithm 1 for all workers: s3gd_topk_sign_encode_ec, then the vote and
 * the update as in s3gd_step (tally and votes nullable in the same way). */
S3GD_API int s3gd_step_ec(s3gd_ctx* ctx, const float* grads, float* err, float eta, uint32_t M, uint64_t N, uint64_t K,
                 float* x, float lr, uint32_t* words, uint32_t* counts, int32_t* tally, int8_t* votes,
                 s3gd_stream_t stream);

/*
 * The same iteration when the caller has already formed g_m in the memory buffer (Section 2.2, the same
 * two equations): a backward pass that accumulates its gradients into the buffer leaves
 * g_m = g~_m + e_m there (eta = 1), and any other eta is a scaling the caller applies before
 * accumulating.  The encode then reads one tensor instead of two and leaves only the zeros in it:
 *
 *     words = TopKSign(acc_m),   acc_m <- acc_m - TopK(acc_m)      (+0.0 where a sign was sent)
 *
 *   acc    dev, in/out  [M, N] fp32, row stride N, 4-byte aligned: g_m on entry, the new memory on
 *                       return.  Only the sent entries differ on return; while the call runs, other
 *                       entries may be stored again with their own value (from K = N/32 on the row is
 *                       rewritten in 64-byte runs) or hold +0.0 for a time, so nothing else may read
 *                       the buffer before the call has finished on `stream`.
 *   words, counts, x, lr, tally, votes   as in s3gd_topk_sign_encode / s3gd_step.
 *
 * Bit for bit the result of s3gd_topk_sign_encode_ec / s3gd_step_ec called with gradients and memory
 * whose fp32 sum is acc (for eta = 1).
 */
S3GD_API int s3gd_topk_sign_encode_acc(s3gd_ctx* ctx, float* acc, uint32_t M, uint64_t N, uint64_t K, uint32_t* words,
                              uint32_t* counts, s3gd_stream_t stream);
S3GD_API int s3gd_step_acc(s3gd_ctx* ctx, float* acc, uint32_t M, uint64_t N, uint64_t K, float* x, float lr, uint32_t* words,
                  uint32_t* counts, int32_t* tally, int8_t* votes, s3gd_stream_t stream);

/*
 * Momentum form of the update (Section 4 "Effects of optimization hyper-parameters"):
 *     v[n] <- fp32(fp32(mu * v[n]) + votes[n]),   x[n] <- fp32(x[n] - fp32(lr * v[n]))
 * with the new v in the second formula; every operation is rounded once.  mu == 0 gives the same x
 * as s3gd_apply_update, bit for bit.
 *
 *   x, v   dev, in/out  [N] fp32, 16-byte aligned.  v is the momentum state; zero-fill it before
 *                       the first iteration.
 *   votes  dev, const   [N] int8 in {-1, 0, +1}, 16-byte aligned.
 *   lr, mu finite and >= 0 (negative zero is refused).
 */
S3GD_API int s3gd_apply_update_momentum(s3gd_ctx* ctx, float* x, float* v, const int8_t* votes, float lr, float mu,
                               uint64_t N, s3gd_stream_t stream);

/*
 * One whole iteration with the momentum form of the update: encode (with the error-compensation
 * memory when err is non-NULL, exactly as s3gd_topk_sign_encode_ec; err == NULL ignores eta and
 * encodes grads as they are; grads == NULL with err non-NULL treats err as a memory that already
 * holds the compensated gradients, exactly as s3gd_topk_sign_encode_acc), majority vote, momentum
 * update.  The vote is not materialised.
 */
S3GD_API int s3gd_step_momentum(s3gd_ctx* ctx, const float* grads, float* err, float eta, uint32_t M, uint64_t N,
                       uint64_t K, float* x, float* v, float lr, float mu, uint32_t* words, uint32_t* counts,
                       s3gd_stream_t stream);

/*
 * Worker side of Algorithm 2 (Section 3.4 "Effect of the random-K sparsification"):
 * words[m, :] = RandKSign(g_m) = sgn(RandK(g_m)) in the message format above: K coordinates drawn at
 * random instead of the K largest; there is no error memory in this variant.
 *
 * The paper leaves the sampling law open.  Worker m at iteration t selects {pi(0), ..., pi(K-1)},
 * pi a pseudo-random permutation of [0, N) keyed by (seed, t, m): exactly K distinct coordinates,
 * each with probability K/N over the keys, independent across workers (what Assumption 4 and
 * Lemma 3 ask for).  pi: with b = max(2, bit length of N-1) and h = ceil(b/2), a value below 4^h is
 * split into halves of h bits and goes through 6 Feistel rounds
 * (left, right) <- (right, left ^ (F(right ^ key_r) & (2^h - 1))), where
 * F(z): z ^= z>>16; z *= 0x85EBCA6B; z ^= z>>13; z *= 0xC2B2AE35; z ^= z>>16 (mod 2^32),
 * k0 = F(lo32(seed) + 0x9E3779B9*(t+1)), k1 = F(k0 ^ hi32(seed)), k2 = F(k1 ^ 0x85EBCA77*(m+1)),
 * key_r = F(k2 + 0xC2B2AE3D*(r+1)), r = 0..5; the network is applied again while the value is >= N.
 *
 * Only the K selected entries of each row of grads are read.  Arguments as in
 * s3gd_topk_sign_encode; a selected entry that is +-0 sends nothing (counts[m] < K).
 */
S3GD_API int s3gd_randk_sign_encode(s3gd_ctx* ctx, const float* grads, uint32_t M, uint64_t N, uint64_t K, uint64_t seed,
                           uint32_t t, uint32_t* words, uint32_t* counts, s3gd_stream_t stream);

/* One whole iteration of Algorithm 2: s3gd_randk_sign_encode, then the vote and the update as in
 * s3gd_step (tally and votes nullable in the same way). */
S3GD_API int s3gd_step_randk(s3gd_ctx* ctx, const float* grads, uint32_t M, uint64_t N, uint64_t K, uint64_t seed,
                    uint32_t t, float* x, float lr, uint32_t* words, uint32_t* counts, int32_t* tally,
                    int8_t* votes, s3gd_stream_t stream);

/*
 * Server side and update in one call, from messages that are already there (for instance after
 * the workers' messages were gathered): the fused tail of s3gd_step.  Only the cache lines of x
 * that hold a voted coordinate are touched.  Arguments as in s3gd_majority_vote / s3gd_apply_update.
 */
S3GD_API int s3gd_vote_update(s3gd_ctx* ctx, const uint32_t* words, const uint32_t* counts, uint32_t M, uint64_t N,
                     uint64_t K, float* x, float lr, s3gd_stream_t stream);

/*
 * Compact wire format.  The paper prices a worker's message at about K + K*log2(N/K) bits (K signs
 * plus the support pattern; Section 2.2 "Gradient compression") and the server's answer at the
 * same expression in the size of the voted support (Section 2.2 "Model update").  These calls
 * convert between the 32-bit message words and an Elias-Fano code of the ascending index set plus
 * one sign bit per entry, n*(L+2) + ((N-1) >> L) + 1 bits for n entries with L = floor(log2(N/n)):
 * less than n*(4 + log2(N/n)).
 *
 * A packed vector is a sequence of 32-bit little-endian words:
 *     word 0        n, the number of entries
 *     word 1        L (0 when n == 0)
 *     sign section  ceil(n/64) groups of 64 bits: bit l of group g = entry 64g+l is negative
 *     low section   ceil(n/64)*L groups of 64 bits: group g*L+b holds bit b of the low L index
 *                   bits of entries 64g..64g+63, one entry per bit position
 *     high section  n + ((N-1) >> L) + 1 bits (none when n == 0), padded to a word: bit
 *                   (index_i >> L) + i is set for the i-th entry in ascending order
 * Unused bits of the sections are 0.  s3gd_packed_row_words(N, K) is an even number of words that
 * holds any vector of at most K entries; words of a row past the vector's own length are left as
 * they were.
 *
 *   words, counts  dev        message rows as written by s3gd_topk_sign_encode ([M, K], [M])
 *   packed         dev        [M, row_words] uint32, 8-byte aligned; row_words even and at least
 *                             s3gd_packed_row_words(N, K)
 * s3gd_unpack_messages writes every slot of words (S3GD_PAD past the count).  A row that does not
 * decode (header that does not fit N, K or row_words; more ones than entries; an index >= N)
 * yields S3GD_E_FORMAT from s3gd_last_async_status; such a row's count is 0 or its bad entries
 * are S3GD_PAD, and every access stays in bounds.
 */
S3GD_API uint64_t s3gd_packed_row_words(uint64_t N, uint64_t K);
S3GD_API int s3gd_pack_messages(s3gd_ctx* ctx, const uint32_t* words, const uint32_t* counts, uint32_t M, uint64_t N,
                       uint64_t K, uint32_t* packed, uint64_t row_words, s3gd_stream_t stream);
S3GD_API int s3gd_unpack_messages(s3gd_ctx* ctx, const uint32_t* packed, uint64_t row_words, uint32_t M, uint64_t N,
                         uint64_t K, uint32_t* words, uint32_t* counts, s3gd_stream_t stream);

/*
 * The server's answer as one message: a word (n << 1) | (votes[n] < 0) for every n with
 * votes[n] != 0, ascending, S3GD_PAD in the slots after them (Section 2.2: the downlink carries the
 * voted support and its signs).  It can then be packed like a worker's message (M = 1).
 *
 *   votes  dev, const  [N] int8, 16-byte aligned
 *   words  dev, out    [capacity] uint32
 *   count  dev, out    [1] uint32: the number of non-zero votes.  If it exceeds capacity only the
 *                      first `capacity` words are written and s3gd_last_async_status reports
 *                      S3GD_E_CAPACITY.
 */
S3GD_API int s3gd_votes_to_message(s3gd_ctx* ctx, const int8_t* votes, uint64_t N, uint64_t capacity, uint32_t* words,
                          uint32_t* count, s3gd_stream_t stream);

/* Synchronises `stream`, then returns 0, or S3GD_E_NAN if the last encode on this context saw a
 * NaN, or S3GD_E_FORMAT / S3GD_E_CAPACITY if the last coding call flagged its input, or
 * S3GD_E_HIP. */
S3GD_API int s3gd_last_async_status(s3gd_ctx* ctx, s3gd_stream_t stream);

/* Diagnostics of the last encode on this context, read back after synchronising `stream`:
 * out[0] = number of rows, out[1] = rows that took the general multi-pass path because the
 * single-pass candidate filter did not apply to them, out[2] = rows served by the single pass whose
 * K-th magnitude lay far above the sampled bound (their radix select ran over all three levels of
 * the candidates instead of the last), out[3] = rows whose words came from a count and an emit pass
 * over the row with a threshold known beforehand (K == N), out[4] = rows of out[1] that were
 * recognised from the sample and skipped the single pass.  `out` is host memory, 5 entries. */
S3GD_API int s3gd_last_encode_info(s3gd_ctx* ctx, s3gd_stream_t stream, uint32_t* out);

/*
 * How an encode call of this shape would be laid over the device by this context (host only, nothing
 * is enqueued): for tests and benchmarks that have to know which internal route a shape takes.
 *   out  host, 12 entries:
 *     [0] 1 if the single-pass candidate route is planned (0: the multi-pass route for every row)
 *     [1] 0: persistent waves; 1: that pass runs as one block per 8192 entries (calls with a memory);
 *         3: it also stores +0.0 over the entries that are selected whatever the threshold (K >= N/512)
 *     [2] s: a run of n candidate slots comes with room for n >> s records of candidates whose
 *         selection is still open after the pass (the others are selected whatever the threshold)
 *     [3] blocks per row of the pass, four waves each   [4] 1024-entry tiles each wave covers, in a row
 *     [5] candidate slots a wave reserves at a time     [6] candidate slots per row
 *     [7] sample units per row                          [8] row entries per sample unit window
 *     [9] rank, in the sample, of the key that becomes the lower bound of a candidate
 *     [10] segments a wave's candidate list may have    [11] consecutive entries per sample unit
 * s3gd_encode_sample_unit_start(u, out[8]) is the index of the first entry of sample unit u of a row.
 */
/* The selection state row m was left in by the last encode on this context (16 words, host memory;
 * synchronises `stream`): in order the key prefix and rank of the radix select, the threshold T, the
 * tie quota, the entries above T, the words sent, the route (0 multi-pass, 1-3 single pass), the two
 * sampled bounds, the K = N flag, candidates kept, candidates whose selection the pass left open,
 * four unused words.  For tests. */
S3GD_API int s3gd_last_row_state(s3gd_ctx* ctx, s3gd_stream_t stream, uint32_t m, uint32_t* out);
S3GD_API int s3gd_encode_plan_info(const s3gd_ctx* ctx, uint32_t M, uint64_t N, uint64_t K, int with_memory, uint64_t* out);
S3GD_API uint64_t s3gd_encode_sample_unit_start(uint32_t u, uint64_t unit_stride);

/*
 * Optional per-kernel timing for benchmarks.  When enabled (on = 1), every kernel launch made
 * through the context is bracketed by a HIP event pair recorded on the call's own stream (no host
 * synchronisation is added); on = 2 brackets only the passes over the gradients (the dominant
 * kernel of a step), two events per step.  s3gd_profile_read synchronises `stream`, adds the elapsed time of
 * every recorded pair to ms_sum[kernel id] and its launch count to launches[kernel id] (host
 * arrays of n >= S3GD_PROFILE_KERNELS entries), and clears the record.  At most 4096 launches are
 * kept between reads.  Names of the ids come from s3gd_profile_kernel_name (NULL past the end).
 */
#define S3GD_PROFILE_KERNELS 26
S3GD_API int s3gd_profile_enable(s3gd_ctx* ctx, int on);
S3GD_API int s3gd_profile_read(s3gd_ctx* ctx, s3gd_stream_t stream, float* ms_sum, uint32_t* launches, int n);
S3GD_API const char* s3gd_profile_kernel_name(int id);

/*
 * Calibration for benchmarks: a plain read of n fp32 entries of `buf` (dev, 16-byte aligned; whole
 * 1024-entry tiles only) with the launch shape and the load instructions of the selection pass and
 * none of its work.  Its duration (kernel id "plain_read" of the profile) is what this memory system
 * gives a read stream of that shape: the practical ceiling the selection pass is compared with.
 */
S3GD_API int s3gd_calibrate_read(s3gd_ctx* ctx, const float* buf, uint64_t n, s3gd_stream_t stream);

/*
 * The same for the selection pass with a memory: reads n entries of `a` and of `b` and writes a + b
 * over b (both dev, 16-byte aligned, not overlapping; whole chunks of 8192 entries only) with the
 * launch shape, loads and stores of that pass and none of its selection work (kernel id "plain_rmw").
 */
S3GD_API int s3gd_calibrate_rmw(s3gd_ctx* ctx, const float* a, float* b, uint64_t n, s3gd_stream_t stream);

/* hipError_t value of the last failed HIP call made through this context (0 if none). */
S3GD_API int s3gd_last_hip_error(const s3gd_ctx* ctx);

S3GD_API const char* s3gd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* S3GD_H */
