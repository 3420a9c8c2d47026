"""CPU oracle for one S3GD-MV step.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition of what the HIP library computes.  It
is imported by the tests, by the smoke check and by the benchmark's CPU
baseline leg, never by the product path, and it shares no code with the
kernels.  Every function cites the passage of the paper it writes out.

Readings taken where the paper is silent (the same list is kept in the design
notes):

* TopK(u) keeps the selected entries of u (it is used as a masked vector in the
  error-memory update of Algorithm 1), so TopKSign(u)_n = sgn(u_n) on the
  selected index set and 0 elsewhere (Section 2.1, eqs. "topk"/"topksign").
* Exactly K indices are selected.  Among equal magnitudes the lowest index
  wins, i.e. the order is (|u| descending, index ascending).
* A selected entry equal to +-0 has sgn = 0: it sends no sign and is not part
  of the support N_m (Section 2.2, "Majority vote").
* sgn(0) = 0 also decides vote ties and coordinates nobody voted on.
* The update is evaluated in fp32 with one rounding: x - lr * vote.
* NaN gradients are outside the input contract and are rejected.

Message format shared with the library's interface (a format, not code):
word = (index << 1) | (1 if value < 0 else 0), ascending per row, rows padded
to K words with 0xFFFFFFFF, counts[m] = number of valid words in row m.
"""
from __future__ import annotations

import numpy as np

PAD = np.uint32(0xFFFFFFFF)


def sgn(u: np.ndarray) -> np.ndarray:
    """sgn(u) = 1{u>0} - 1{u<0}, element-wise (Section 2.1, below eq. "topksign")."""
    u = np.asarray(u)
    return (u > 0).astype(np.int8) - (u < 0).astype(np.int8)


def _check_row(g: np.ndarray, K: int) -> np.ndarray:
    g = np.asarray(g)
    if g.ndim != 1 or g.dtype != np.float32:
        raise ValueError("a gradient row is a 1-d float32 array")
    if not 0 <= K <= g.shape[0]:
        raise ValueError("K must satisfy 0 <= K <= N (sparsity K/N lies in [0,1])")
    if np.isnan(g).any():
        raise ValueError("NaN in gradient: outside the input contract")
    return g


def topk_index_set(g: np.ndarray, K: int) -> np.ndarray:
    """Indices of the K largest-magnitude entries of g, ascending (TopK, eq. "topk").

    Full sort of the pairs (|g_n|, n) by magnitude descending then index
    ascending; the first K are selected.
    """
    g = _check_row(g, K)
    mag = np.abs(g)  # float comparison on |g|; -0.0 becomes +0.0
    n = np.arange(g.shape[0], dtype=np.int64)
    order = np.lexsort((n, -mag))  # last key is primary: -|g| ascending == |g| descending
    return np.sort(order[:K])


def topk_index_set_brute_force(g: np.ndarray, K: int) -> np.ndarray:
    """Same set from the rank definition, without sorting (tiny N only).

    rank(n) = #{j : |g_j| > |g_n|} + #{j < n : |g_j| == |g_n|}; n is selected
    iff rank(n) < K.
    """
    g = _check_row(g, K)
    N = g.shape[0]
    mag = [abs(float(v)) for v in g]
    sel = []
    for n in range(N):
        rank = 0
        for j in range(N):
            if mag[j] > mag[n] or (mag[j] == mag[n] and j < n):
                rank += 1
        if rank < K:
            sel.append(n)
    return np.asarray(sel, dtype=np.int64)


def rank_of(g: np.ndarray, n: int) -> int:
    """rank(n) of the definition above for one coordinate, O(N) vectorised.

    Lets a test decide membership of single coordinates at sizes where a full
    sort is too slow: n is in the top-K set iff rank_of(g, n) < K.
    """
    mag = np.abs(g)
    t = mag[n]
    return int(np.count_nonzero(mag > t)) + int(np.count_nonzero(mag[:n] == t))


def topk_sign_dense(g: np.ndarray, K: int) -> np.ndarray:
    """TopKSign(g) as the ternary vector in {-1,0,+1}^N (eq. "topksign")."""
    out = np.zeros(g.shape[0], dtype=np.int8)
    S = topk_index_set(g, K)
    out[S] = sgn(g[S])
    return out


def encode_row(g: np.ndarray, K: int) -> tuple[np.ndarray, int]:
    """The message worker m sends (Algorithm 1, "send TopKSign(g_m)"): K words, count."""
    S = topk_index_set(g, K)
    s = sgn(g[S])
    keep = s != 0  # zero entries cast no vote and are not in the support
    words = np.full(K, PAD, dtype=np.uint32)
    w = (S[keep].astype(np.uint64) << np.uint64(1)) | (s[keep] < 0).astype(np.uint64)
    words[: w.shape[0]] = w.astype(np.uint32)
    return words, int(w.shape[0])


def topk_sign_encode(G: np.ndarray, K: int) -> tuple[np.ndarray, np.ndarray]:
    """All M messages: words [M,K] uint32, counts [M] uint32 (Algorithm 1, worker loop)."""
    G = np.asarray(G)
    if G.ndim != 2 or G.dtype != np.float32:
        raise ValueError("gradients are a [M,N] float32 array")
    M = G.shape[0]
    if G.shape[1] > (1 << 31) - 2:
        raise ValueError("index + sign bit + pad word must fit 32 bits")
    words = np.empty((M, K), dtype=np.uint32)
    counts = np.empty(M, dtype=np.uint32)
    for m in range(M):
        words[m], counts[m] = encode_row(G[m], K)
    return words, counts


def majority_vote(words: np.ndarray, counts: np.ndarray, N: int) -> tuple[np.ndarray, np.ndarray]:
    """Server side (Section 2.2 "Majority vote"; Algorithm 1 "receive sgn[sum ...]").

    tally_n = sum over workers of TopKSign(g_m)_n; votes_n = sgn(tally_n).
    Coordinates outside the union of supports keep tally 0 and vote 0.
    """
    tally = np.zeros(N, dtype=np.int32)
    for m in range(words.shape[0]):
        w = words[m, : int(counts[m])]
        idx = (w >> np.uint32(1)).astype(np.int64)
        if idx.size and (idx.max() >= N):
            raise ValueError("word index out of range")
        delta = np.where((w & np.uint32(1)) == 1, np.int32(-1), np.int32(1))
        np.add.at(tally, idx, delta)  # tally[idx[i]] += delta[i] for every i, in order
    return tally, sgn(tally)


def majority_vote_loops(words, counts, N):
    """The same double loop spelled out in Python (small inputs only)."""
    tally = [0] * N
    for m in range(len(words)):
        for i in range(int(counts[m])):
            w = int(words[m][i])
            tally[w >> 1] += -1 if (w & 1) else 1
    votes = [(t > 0) - (t < 0) for t in tally]
    return np.asarray(tally, dtype=np.int32), np.asarray(votes, dtype=np.int8)


def apply_update(x: np.ndarray, votes: np.ndarray, lr) -> np.ndarray:
    """x^{t+1} = x^t - delta * vote in fp32, one rounding (eq. "s3gd")."""
    x = np.asarray(x)
    if x.dtype != np.float32:
        raise ValueError("parameters are float32")
    return (x - np.float32(lr) * votes.astype(np.float32)).astype(np.float32)


def step(G: np.ndarray, K: int, x: np.ndarray, lr) -> dict:
    """One iteration of Algorithm 1 after the gradients exist: encode, vote, update."""
    words, counts = topk_sign_encode(G, K)
    tally, votes = majority_vote(words, counts, G.shape[1])
    return dict(words=words, counts=counts, tally=tally, votes=votes, x=apply_update(x, votes, lr))


def step_dense(G: np.ndarray, K: int, x: np.ndarray, lr) -> dict:
    """Eq. "s3gd" evaluated literally on dense ternary vectors (no message format)."""
    T = np.stack([topk_sign_dense(G[m], K) for m in range(G.shape[0])]).astype(np.int32)
    tally = T.sum(axis=0, dtype=np.int32)
    votes = sgn(tally)
    return dict(tally=tally, votes=votes, x=apply_update(x, votes, lr))


# ---------------------------------------------------------------------------------------------
# Error-compensation memory (Section 2.2 "Gradient update with sparsification error compensation";
# Algorithm 1, the two lines before "send")
#
# Readings: g = g~ + eta * e is evaluated in fp32 as written (a product, then a sum: two
# roundings; eta = 1, the paper's setting, makes both exact).  TopK(g) is the masked vector
# (it is subtracted from g), so e' = g - TopK(g) keeps g off the selected set and is zero on it.
# The zero is written as +0.0 wherever a sign was sent; a selected entry that is itself +-0 sends
# nothing and keeps its bits (the literal difference would turn -0.0 into +0.0, and an infinite
# selected entry into NaN: neither changes any later selection or vote).

def compensate(G_tilde: np.ndarray, E: np.ndarray, eta) -> np.ndarray:
    """g_m = g~_m + eta * e_m (eq. "gradupdate"), fp32."""
    if G_tilde.dtype != np.float32 or E.dtype != np.float32 or G_tilde.shape != E.shape:
        raise ValueError("gradients and error memory are float32 arrays of one shape")
    prod = (np.float32(eta) * E).astype(np.float32)
    return (G_tilde + prod).astype(np.float32)


def residual(G: np.ndarray, words: np.ndarray, counts: np.ndarray) -> np.ndarray:
    """e_m' = g_m - TopK(g_m): g off the support of the message, zero on it."""
    E = G.copy()
    for m in range(G.shape[0]):
        idx = (words[m, : int(counts[m])] >> np.uint32(1)).astype(np.int64)
        E[m, idx] = np.float32(0.0)
    return E


def step_with_memory(G_tilde: np.ndarray, E: np.ndarray, eta, K: int, x: np.ndarray, lr) -> dict:
    """One full iteration of Algorithm 1 for all workers: compensate, remember, send, vote, update."""
    G = compensate(G_tilde, E, eta)
    out = step(G, K, x, lr)
    out["g"] = G
    out["err"] = residual(G, out["words"], out["counts"])
    return out


# ---------------------------------------------------------------------------------------------
# Momentum variant of the update (Section 4 "Effects of optimization hyper-parameters"):
#   v^t = mu * v^{t-1} + sgn[sum_m TopKSign(g_m^t)],   x^{t+1} = x^t - delta * v^t.
#
# Readings: fp32, evaluated as written with every operation rounded once: a product mu*v, a sum with
# the vote (the vote converted exactly to -1.0, 0.0 or +1.0), a product delta*v^t, a difference.
# v^{-1} = 0.  mu = 0 gives back eq. "s3gd" bit for bit.

def momentum_update(x: np.ndarray, v: np.ndarray, votes: np.ndarray, lr, mu) -> tuple[np.ndarray, np.ndarray]:
    """(x^{t+1}, v^t) from (x^t, v^{t-1}) and the vote of iteration t."""
    if x.dtype != np.float32 or v.dtype != np.float32 or x.shape != v.shape:
        raise ValueError("parameters and momentum are float32 arrays of one shape")
    decayed = (np.float32(mu) * v).astype(np.float32)
    v_new = (decayed + votes.astype(np.float32)).astype(np.float32)
    move = (np.float32(lr) * v_new).astype(np.float32)
    return (x - move).astype(np.float32), v_new


def step_with_momentum(G: np.ndarray, K: int, x: np.ndarray, v: np.ndarray, lr, mu) -> dict:
    """One iteration: encode and vote as in Algorithm 1, then the momentum form of the update."""
    words, counts = topk_sign_encode(G, K)
    tally, votes = majority_vote(words, counts, G.shape[1])
    x_new, v_new = momentum_update(x, v, votes, lr, mu)
    return dict(words=words, counts=counts, tally=tally, votes=votes, x=x_new, v=v_new)


# ---------------------------------------------------------------------------------------------
# Checks that hold at any size (used where a full sort of the row is too slow to run in a test)

def check_message_row(g: np.ndarray, K: int, words: np.ndarray, count: int) -> None:
    """Raises AssertionError unless (words, count) is exactly TopKSign(g) in the message format.

    Written from the definition, without sorting.  Let S be the selected index set and t the
    smallest selected magnitude.  S is the top-K set under (|g| descending, index ascending) iff
      (1) |S| = K;
      (2) every index with |g| > t is in S;
      (3) the members of S with |g| == t are the lowest-indexed entries of that magnitude.
    The message lists S minus its zero-valued members, ascending, with the sign bit of each.
    """
    g = _check_row(g, K)
    N = g.shape[0]
    words = np.asarray(words, dtype=np.uint32)
    assert words.shape == (K,), "row has K slots"
    assert 0 <= count <= K
    assert (words[count:] == PAD).all(), "slots past count hold the pad word"
    idx = (words[:count] >> np.uint32(1)).astype(np.int64)
    assert (idx < N).all(), "index out of range"
    assert (np.diff(idx) > 0).all(), "indices ascending and distinct"
    assert np.array_equal(words[:count] & np.uint32(1), (g[idx] < 0).astype(np.uint32)), "sign bits"
    assert not (g[idx] == 0).any(), "zero entries send nothing"
    mag = np.abs(g)
    if count < K:
        # the K selected entries include zeros: every non-zero entry must have been sent
        assert count == int(np.count_nonzero(mag)), "a non-zero entry is missing although zeros were selected"
        return
    if K == 0:
        return
    t = mag[idx].min()
    assert t > 0
    n_gt = int(np.count_nonzero(mag > t))
    sel_mag = mag[idx]
    assert int(np.count_nonzero(sel_mag > t)) == n_gt, "an entry above the threshold was left out"
    q = K - n_gt
    ties_sel = idx[sel_mag == t]
    assert ties_sel.shape[0] == q
    # lowest-indexed q entries of magnitude t: find them without touching the whole row twice
    hi = int(ties_sel[-1]) + 1
    first_q = np.nonzero(mag[:hi] == t)[0]
    assert np.array_equal(first_q, ties_sel), "ties at the threshold must go to the lowest indices"
