"""CPU oracle for RandKSign (Algorithm 2 of the paper).  TEST INFRASTRUCTURE ONLY.

RandKSign(g) = sgn(RandK(g)): K coordinates chosen at random instead of the K largest, their
signs sent, no error memory (Section 3.4 "Effect of the random-K sparsification", Algorithm 2).
The paper does not say how the K coordinates are drawn; its analysis (Assumption 4, Lemma 3)
needs every coordinate to be selected with probability K/N, independently across workers.

Reading taken here: worker m at iteration t selects the set {pi(0), ..., pi(K-1)}, where pi is a
pseudo-random permutation of [0, N) keyed by (seed, t, m).  Every selected index is distinct, the
set has exactly K members, and over the keys each coordinate is selected with probability K/N.

The permutation is a counter-based generator that both sides implement from this description:

  * domain: b = bit length of N - 1 (at least 2), h = ceil(b / 2); values below 4^h are split into
    a left half (high h bits) and a right half (low h bits);
  * 6 Feistel rounds: (left, right) <- (right, left XOR (F(right XOR key_r) AND (2^h - 1)));
  * F is the 32-bit finaliser  z ^= z >> 16; z *= 0x85EBCA6B; z ^= z >> 13; z *= 0xC2B2AE35;
    z ^= z >> 16  (arithmetic modulo 2^32);
  * round keys: k0 = F(lo32(seed) + 0x9E3779B9 * (t + 1)); k1 = F(k0 XOR hi32(seed));
    k2 = F(k1 XOR (0x85EBCA77 * (m + 1))); key_r = F(k2 + 0xC2B2AE3D * (r + 1)), r = 0..5;
  * cycle walking: apply the network again while the value is >= N (it is a bijection of
    [0, 4^h), so iterating from a value below N returns below N; 4^h < 4N keeps the walk short).

The message is then built as for TopKSign: words (index << 1) | negative in ascending index,
entries equal to +-0 send nothing, counts[m] = words sent, rows padded with 0xFFFFFFFF.
"""
from __future__ import annotations

import numpy as np

from oracle.s3gd_oracle import PAD, majority_vote, apply_update

ROUNDS = 6
_M32 = 0xFFFFFFFF


def fmix32(z: int) -> int:
    z &= _M32
    z ^= z >> 16
    z = (z * 0x85EBCA6B) & _M32
    z ^= z >> 13
    z = (z * 0xC2B2AE35) & _M32
    z ^= z >> 16
    return z


def round_keys(seed: int, t: int, m: int) -> list[int]:
    k0 = fmix32((seed & _M32) + 0x9E3779B9 * (t + 1))
    k1 = fmix32(k0 ^ ((seed >> 32) & _M32))
    k2 = fmix32(k1 ^ ((0x85EBCA77 * (m + 1)) & _M32))
    return [fmix32(k2 + 0xC2B2AE3D * (r + 1)) for r in range(ROUNDS)]


def half_bits(N: int) -> int:
    b = max(2, (N - 1).bit_length())
    return (b + 1) // 2


def feistel(v: int, h: int, keys: list[int]) -> int:
    mask = (1 << h) - 1
    left, right = v >> h, v & mask
    for k in keys:
        left, right = right, left ^ (fmix32(right ^ k) & mask)
    return (left << h) | right


def permute(i: int, N: int, keys: list[int]) -> int:
    """pi(i) for 0 <= i < N."""
    h = half_bits(N)
    v = feistel(i, h, keys)
    while v >= N:
        v = feistel(v, h, keys)
    return v


def _fmix32_np(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64) & np.uint64(_M32)
    z ^= z >> np.uint64(16)
    z = (z * np.uint64(0x85EBCA6B)) & np.uint64(_M32)
    z ^= z >> np.uint64(13)
    z = (z * np.uint64(0xC2B2AE35)) & np.uint64(_M32)
    z ^= z >> np.uint64(16)
    return z


def permute_many(i: np.ndarray, N: int, keys: list[int]) -> np.ndarray:
    """The same permutation on an array of inputs (vectorised; checked against permute())."""
    h = np.uint64(half_bits(N))
    mask = np.uint64((1 << int(h)) - 1)

    def net(v):
        left, right = v >> h, v & mask
        for k in keys:
            left, right = right, left ^ (_fmix32_np(right ^ np.uint64(k)) & mask)
        return (left << h) | right

    v = net(np.asarray(i, dtype=np.uint64))
    out = v.copy()
    todo = np.nonzero(out >= np.uint64(N))[0]
    while todo.size:
        out[todo] = net(out[todo])
        todo = todo[out[todo] >= np.uint64(N)]
    return out.astype(np.int64)


def randk_index_set(N: int, K: int, seed: int, t: int, m: int) -> np.ndarray:
    """The K selected coordinates of worker m at iteration t, ascending."""
    if not 0 <= K <= N:
        raise ValueError("0 <= K <= N")
    return np.sort(permute_many(np.arange(K), N, round_keys(seed, t, m)))


def randk_sign_encode(G: np.ndarray, K: int, seed: int, t: int) -> tuple[np.ndarray, np.ndarray]:
    """All M messages of Algorithm 2: words [M, K], counts [M]."""
    if G.ndim != 2 or G.dtype != np.float32:
        raise ValueError("gradients are a [M,N] float32 array")
    if np.isnan(G).any():
        raise ValueError("NaN in gradient: outside the input contract")
    M, N = G.shape
    words = np.full((M, K), PAD, dtype=np.uint32)
    counts = np.zeros(M, dtype=np.uint32)
    for m in range(M):
        S = randk_index_set(N, K, seed, t, m)
        g = G[m, S]
        keep = g != 0  # sgn(0) = 0: nothing to send
        w = (S[keep].astype(np.uint64) << np.uint64(1)) | (g[keep] < 0).astype(np.uint64)
        words[m, : w.shape[0]] = w.astype(np.uint32)
        counts[m] = w.shape[0]
    return words, counts


def step_randk(G: np.ndarray, K: int, x: np.ndarray, lr, seed: int, t: int) -> dict:
    """One iteration of Algorithm 2: random-K sign messages, majority vote, update."""
    words, counts = randk_sign_encode(G, K, seed, t)
    tally, votes = majority_vote(words, counts, G.shape[1])
    return dict(words=words, counts=counts, tally=tally, votes=votes, x=apply_update(x, votes, lr))
