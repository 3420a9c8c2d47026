"""Communication cost per iteration in bits, as the paper's cost table states it
(Section 4, table of total communication costs, divided by T; Section 2.2 for the
uplink and downlink terms).  Reporting only: nothing on the compute path uses it."""
import math


def _pattern_bits(N: int, K: int) -> float:
    return K * math.log2(N / K) if K else 0.0


def vanilla_sgd(M: int, N: int) -> float:
    return 2.0 * 32 * M * N


def topk_sgd(M: int, N: int, K: int) -> float:
    return M * (32.0 * K + _pattern_bits(N, K)) + 32.0 * M * N


def signsgd_mv(M: int, N: int) -> float:
    return 2.0 * M * N


def s3gd_uplink(M: int, N: int, K: int) -> float:
    """M workers, each K sign bits plus the support pattern."""
    return M * (K + _pattern_bits(N, K))


def s3gd_mv(M: int, N: int, K: int) -> float:
    """Upper bound: uplink plus at most N downlink bits to each of M workers."""
    return s3gd_uplink(M, N, K) + float(M) * N


def packed_words_bits(M: int, K: int) -> float:
    """Size of the uplink as this library stores it: one 32-bit word per selected entry."""
    return 32.0 * M * K
