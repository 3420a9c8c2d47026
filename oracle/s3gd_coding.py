"""CPU oracle for the compact wire format of a sparse ternary vector.  TEST INFRASTRUCTURE ONLY.

The paper counts the uplink of a worker as "K sign bits plus the support pattern", roughly
K + K*log2(N/K) bits, and the downlink as the same expression in the size of the voted support
(Section 2.2, "Gradient compression" and "Model update"; Section 1, contributions).  It names no
code that reaches this.  The format below is an Elias-Fano code of the ascending index set plus one
sign bit per entry: it spends n*(L + 1) + n + ceil(N / 2^L) + 1 bits on n entries with
L = floor(log2(N/n)), i.e. fewer than n*(4 + log2(N/n)) bits, against an information bound of
log2 C(N, n) + n.

Format of one packed vector (32-bit little-endian words; "bit p of a section" is bit p % 32 of its
word p // 32).  Shared with the library's interface as a format, not as code:

    word 0        n, the number of entries (<= N)
    word 1        L = floor(log2(N // n)) for n >= 1, else 0: the number of low index bits
    sign section  G = ceil(n / 64) groups of 64 bits; bit l of group g is 1 iff entry 64*g + l is
                  negative; unused bits are 0
    low section   G * L groups of 64 bits; group g*L + b holds bit b of (index & (2^L - 1)) of the
                  entries 64*g .. 64*g + 63, entry 64*g + l in bit l ("bit planes"); unused bits 0
    high section  H = n + ((N - 1) >> L) + 1 bits (H = 0 when n = 0); bit (index_i >> L) + i is 1 for
                  the i-th entry (i = 0 .. n-1 in ascending index), all others 0; padded with 0 to a
                  whole word

This file is written from the definition of the code; the decoder recovers an entry from the
position and rank of its 1 in the high section and never calls the encoder.
"""
from __future__ import annotations

import math

import numpy as np

HEADER_WORDS = 2


def low_bits(N: int, n: int) -> int:
    """L = floor(log2(N // n)): the largest L with n * 2^L <= N (0 when n == 0)."""
    if n == 0:
        return 0
    if not 0 < n <= N:
        raise ValueError("0 <= n <= N")
    return (N // n).bit_length() - 1


def high_bits_len(N: int, n: int) -> int:
    if n == 0:
        return 0  # an empty vector is its header alone
    return n + ((N - 1) >> low_bits(N, n)) + 1


def row_words(N: int, n: int) -> int:
    """Exact size in 32-bit words of a packed vector with n entries."""
    G = (n + 63) // 64
    return HEADER_WORDS + 2 * G * (1 + low_bits(N, n)) + (high_bits_len(N, n) + 31) // 32


def information_bits(N: int, n: int) -> int:
    """Bits that carry information (header, signs, low bits, high section), without padding."""
    return 32 * HEADER_WORDS + n + n * low_bits(N, n) + high_bits_len(N, n)


def entropy_bound_bits(N: int, n: int) -> float:
    """log2 C(N, n) + n: no code for an n-subset of [N] with n signs can use fewer bits on average."""
    lg = (math.lgamma(N + 1) - math.lgamma(n + 1) - math.lgamma(N - n + 1)) / math.log(2.0)
    return lg + n


def _check_message(words: np.ndarray, count: int, N: int) -> tuple[np.ndarray, np.ndarray]:
    w = np.asarray(words[:count], dtype=np.uint32)
    idx = (w >> np.uint32(1)).astype(np.int64)
    neg = (w & np.uint32(1)).astype(np.uint8)
    if idx.size and (idx.max() >= N or (np.diff(idx) <= 0).any()):
        raise ValueError("message indices must be ascending, distinct and below N")
    return idx, neg


def pack_row(words: np.ndarray, count: int, N: int) -> np.ndarray:
    """Packed form of one message (the first `count` words of a row in the library's word format)."""
    idx, neg = _check_message(words, count, N)
    n = int(count)
    L = low_bits(N, n)
    G = (n + 63) // 64
    out = np.zeros(row_words(N, n), dtype=np.uint32)
    out[0], out[1] = n, L
    bits64 = np.zeros((G * (1 + L), 64), dtype=np.uint8)  # one row per 64-bit group, sign groups first
    for i in range(n):  # entry i sits in lane i % 64 of its group
        g, l = divmod(i, 64)
        bits64[g, l] = neg[i]
        for b in range(L):
            bits64[G + g * L + b, l] = (int(idx[i]) >> b) & 1
    if G:
        out[HEADER_WORDS:HEADER_WORDS + 2 * G * (1 + L)] = np.packbits(bits64.reshape(-1), bitorder="little").view(np.uint32)
    H = high_bits_len(N, n)
    hb = np.zeros(((H + 31) // 32) * 32, dtype=np.uint8)
    for i in range(n):
        hb[(int(idx[i]) >> L) + i] = 1
    out[HEADER_WORDS + 2 * G * (1 + L):] = np.packbits(hb, bitorder="little").view(np.uint32)
    return out


def pack_row_fast(words: np.ndarray, count: int, N: int) -> np.ndarray:
    """The same bits as pack_row, vectorised for large rows (checked against it in the tests)."""
    idx, neg = _check_message(words, count, N)
    n = int(count)
    L = low_bits(N, n)
    G = (n + 63) // 64
    out = np.zeros(row_words(N, n), dtype=np.uint32)
    out[0], out[1] = n, L
    if n:
        planes = np.zeros((G, 1 + L, 64), dtype=np.uint8)
        flat_g, flat_l = np.arange(n) // 64, np.arange(n) % 64
        sign_part = np.zeros((G, 64), dtype=np.uint8)
        sign_part[flat_g, flat_l] = neg
        for b in range(L):
            planes[flat_g, 1 + b, flat_l] = (idx >> b) & 1
        body = np.concatenate([sign_part.reshape(-1), planes[:, 1:, :].reshape(-1)])
        out[HEADER_WORDS:HEADER_WORDS + 2 * G * (1 + L)] = np.packbits(body, bitorder="little").view(np.uint32)
    H = high_bits_len(N, n)
    hb = np.zeros(((H + 31) // 32) * 32, dtype=np.uint8)
    hb[(idx >> L) + np.arange(n)] = 1
    out[HEADER_WORDS + 2 * G * (1 + L):] = np.packbits(hb, bitorder="little").view(np.uint32)
    return out


def unpack_row(packed: np.ndarray, N: int) -> tuple[np.ndarray, int]:
    """(words, n) of a packed vector.  The i-th 1 of the high section, at position p, belongs to the
    entry of rank i; its index is ((p - i) << L) | low_i."""
    packed = np.asarray(packed, dtype=np.uint32)
    n, L = int(packed[0]), int(packed[1])
    if n > N or L != low_bits(N, n):
        raise ValueError("header does not fit N")
    G = (n + 63) // 64
    need = row_words(N, n)
    if packed.shape[0] < need:
        raise ValueError("packed vector is truncated")
    body = np.unpackbits(packed[HEADER_WORDS:HEADER_WORDS + 2 * G * (1 + L)].view(np.uint8), bitorder="little")
    sign = body[: G * 64][:n]
    planes = body[G * 64:].reshape(G, L, 64) if G else np.zeros((0, L, 64), np.uint8)
    low = np.zeros(G * 64, dtype=np.int64)
    for b in range(L):
        low |= planes[:, b, :].reshape(-1).astype(np.int64) << b
    low = low[:n]
    hb = np.unpackbits(packed[HEADER_WORDS + 2 * G * (1 + L):need].view(np.uint8), bitorder="little")
    pos = np.nonzero(hb)[0]
    if pos.shape[0] != n:
        raise ValueError("high section does not hold n ones")
    idx = ((pos - np.arange(n)) << L) | low
    if n and (idx.max() >= N or (np.diff(idx) <= 0).any()):
        raise ValueError("decoded indices are not an ascending subset of [N]")
    return ((idx.astype(np.uint64) << np.uint64(1)) | sign.astype(np.uint64)).astype(np.uint32), n


def votes_to_message(votes: np.ndarray) -> tuple[np.ndarray, int]:
    """The server's answer as a message: one word per coordinate with a non-zero vote, ascending
    (the downlink carries the voted support and its signs; Section 2.2 "Model update")."""
    votes = np.asarray(votes)
    idx = np.nonzero(votes)[0].astype(np.uint64)
    w = (idx << np.uint64(1)) | (votes[idx.astype(np.int64)] < 0).astype(np.uint64)
    return w.astype(np.uint32), int(idx.shape[0])
