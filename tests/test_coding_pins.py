"""Pins of the coding oracle (oracle/s3gd_coding.py): a hand-coded instance, exhaustive round trips
on tiny universes, injectivity, the size against the information bound and against the paper's
expression, and planted mistakes."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import s3gd_coding as C

GOLD = os.path.join(os.path.dirname(__file__), "golden", "elias_fano_example.txt")


def _gold():
    d = {}
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            d[k] = [int(t, 0) for t in v]
    return d


def _msg(idx, neg):
    return ((np.asarray(idx, dtype=np.uint64) << np.uint64(1)) | np.asarray(neg, dtype=np.uint64)).astype(np.uint32)


def test_hand_coded_instance():
    g = _gold()
    N = g["N"][0]
    words = np.array(g["words"], dtype=np.uint32)
    packed = np.array(g["packed"], dtype=np.uint32)
    assert np.array_equal(C.pack_row(words, len(words), N), packed)
    assert np.array_equal(C.pack_row_fast(words, len(words), N), packed)
    w, n = C.unpack_row(packed, N)  # the decoder alone, on bits written by hand
    assert n == len(words) and np.array_equal(w, words)
    assert C.information_bits(N, n) == g["information_bits"][0]
    assert C.row_words(N, n) == len(packed)


def test_exhaustive_round_trip_and_injectivity_on_tiny_universes():
    for N in (1, 2, 5, 6):
        seen = set()
        for n in range(N + 1):
            for idx in itertools.combinations(range(N), n):
                for neg in itertools.product((0, 1), repeat=n):
                    words = _msg(idx, neg)
                    p = C.pack_row(words, n, N)
                    assert p.shape[0] == C.row_words(N, n)
                    w, k = C.unpack_row(p, N)
                    assert k == n and np.array_equal(w, words)
                    key = p.tobytes()
                    assert key not in seen, "two different vectors share a code"
                    seen.add(key)
        assert len(seen) == 3 ** N  # every ternary vector of length N got its own code


@pytest.mark.parametrize("N,n", [(64, 0), (64, 1), (64, 64), (65, 64), (1000, 1), (1000, 999), (10_000, 100), (100_000, 1_000),
                                 (1 << 20, 1 << 10), ((1 << 20) + 7, 4097), (3_000_000, 30_000), ((1 << 31) - 2, 5)])
def test_round_trip_random_sets(N, n):
    rng = np.random.default_rng(N + n)
    if n > N // 2:
        idx = np.sort(rng.permutation(N)[:n])
    else:
        idx = np.unique(rng.integers(0, N, size=2 * n + 8))
        idx = np.sort(rng.permutation(idx)[:n])
    assert idx.shape[0] == n
    if n:
        idx[-1] = N - 1  # the last coordinate is representable
        idx = np.unique(idx)
        n = idx.shape[0]
    words = _msg(idx, rng.integers(0, 2, n))
    p = C.pack_row_fast(words, n, N)
    if n <= 5000:
        assert np.array_equal(p, C.pack_row(words, n, N))
    w, k = C.unpack_row(p, N)
    assert k == n and np.array_equal(w, words)
    # longer buffers (a row of fixed capacity) decode the same; a truncated one is refused
    w2, _ = C.unpack_row(np.concatenate([p, np.full(5, 0xDEADBEEF, np.uint32)]), N)
    assert np.array_equal(w2, words)
    if n:
        with pytest.raises(ValueError):
            C.unpack_row(p[:-1], N)


def test_structured_sets():
    N = 5000
    for idx in (np.arange(300), np.arange(N - 300, N), np.arange(0, N, 7), np.array([0]), np.array([N - 1]), np.arange(N)):
        words = _msg(idx, idx % 2)
        w, k = C.unpack_row(C.pack_row_fast(words, len(idx), N), N)
        assert k == len(idx) and np.array_equal(w, words)


@pytest.mark.parametrize("N,n", [(10_000, 100), (500_000, 500), (850_000, 42_500), (1_200_000_000, 1_200_000),
                                 (11_200_000, 112_000), (1000, 1000), (1000, 501), (1000, 3)])
def test_size_between_information_bound_and_paper_expression(N, n):
    body = C.information_bits(N, n) - 32 * C.HEADER_WORDS
    assert body >= C.entropy_bound_bits(N, n) - 1e-6          # no lossless code can beat this
    assert body <= n * (4 + math.log2(N / n)) + 1              # Elias-Fano: at most ~2 bits/entry above log2(N/n), + sign
    paper = n + n * math.log2(N / n)                           # Section 2.2: "roughly K + K log2(N/K)"
    assert paper <= body <= paper + 3 * n + 1
    assert 32 * C.row_words(N, n) - C.information_bits(N, n) < 64 * (2 + C.low_bits(N, n)) + 32  # padding: < one group per section


def test_low_bits_definition():
    for N, n in [(64, 8), (64, 9), (63, 8), (1, 1), (1000, 1), (1000, 1000), (1_200_000_000, 1_200_000)]:
        L = C.low_bits(N, n)
        assert n * 2 ** L <= N < n * 2 ** (L + 1)
    assert C.low_bits(77, 0) == 0


def test_malformed_inputs_are_rejected():
    with pytest.raises(ValueError):
        C.pack_row(_msg([5, 5], [0, 0]), 2, 10)   # repeated index
    with pytest.raises(ValueError):
        C.pack_row(_msg([7, 3], [0, 0]), 2, 10)   # descending
    with pytest.raises(ValueError):
        C.pack_row(_msg([10], [0]), 1, 10)        # index == N
    good = C.pack_row(_msg([1, 4, 9], [0, 1, 0]), 3, 10)
    bad = good.copy(); bad[1] += 1                # wrong L in the header
    with pytest.raises(ValueError):
        C.unpack_row(bad, 10)
    bad = good.copy(); bad[-1] |= 1 << 20         # an extra one in the high section
    with pytest.raises(ValueError):
        C.unpack_row(bad, 10)


def test_planted_mistakes_break_the_hand_coded_instance(monkeypatch):
    g = _gold()
    N, words, packed = g["N"][0], np.array(g["words"], np.uint32), np.array(g["packed"], np.uint32)
    # (a) one low bit too many
    real = C.low_bits
    monkeypatch.setattr(C, "low_bits", lambda N, n: real(N, n) + 1 if n else 0)
    assert not np.array_equal(C.pack_row(words, len(words), N)[: len(packed)], packed)
    monkeypatch.undo()
    # (b) a decoder that forgets to subtract the rank decodes the hand-written bits wrongly
    hb = np.unpackbits(packed[-1:].view(np.uint8), bitorder="little")
    pos = np.nonzero(hb)[0]
    low = np.array([3, 4, 7, 5, 6, 7, 5, 3])
    wrong = (pos << 3) | low
    right = ((pos - np.arange(8)) << 3) | low
    assert not np.array_equal(wrong, words >> 1) and np.array_equal(right, words >> 1)


def test_votes_to_message():
    votes = np.array([0, 1, -1, 0, 0, -1, 1, 0], dtype=np.int8)
    w, n = C.votes_to_message(votes)
    assert n == 4 and w.tolist() == [(1 << 1) | 0, (2 << 1) | 1, (5 << 1) | 1, (6 << 1) | 0]
    w0, n0 = C.votes_to_message(np.zeros(9, np.int8))
    assert n0 == 0 and w0.shape == (0,)
    # a message made from a vote gives the vote back through the server sum of one "worker"
    from oracle import s3gd_oracle as O
    tally, back = O.majority_vote(w[None, :], np.array([n], np.uint32), votes.shape[0])
    assert np.array_equal(back, votes)
