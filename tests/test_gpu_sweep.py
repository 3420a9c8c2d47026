"""A seeded sweep over shapes, sparsity levels and value distributions, each case run through one
of the entry-point combinations and compared with the CPU oracle bit for bit (tolerance 0).  The
cases are drawn so that every route of the encode is hit: rows below and above the smallest row the
single pass serves (2^17 entries), K on both sides of N/16 (where the pass starts to keep a bracket
instead of every candidate), K = N, K of a handful, ties, zeros, magnitudes spread over decades."""
import os

import numpy as np
import pytest
import torch

from oracle import s3gd_oracle as O
from tests.helpers import assert_same, gpu_step
from tests.test_gpu_memory import gpu_step_ec

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(9, 1 << 19, 1 << 19, device=0)
    yield c
    c.close()


def _values(rng, kind, M, N):
    if kind == 0:
        return rng.standard_normal((M, N))
    if kind == 1:  # coarse grid: heavy ties, exact zeros
        G = np.rint(rng.standard_t(3, (M, N)) * 8) / 8
        G[rng.random((M, N)) < 0.1] = 0.0
        return G
    if kind == 2:  # contiguous blocks whose scales span six decades
        nb = 37
        scale = 10.0 ** rng.uniform(-5, 1, (M, nb))
        return rng.standard_normal((M, N)) * np.repeat(scale, N // nb + 1, axis=1)[:, :N]
    if kind == 3:  # mostly zero
        return np.where(rng.random((M, N)) < 0.02, rng.standard_normal((M, N)), 0.0)
    return rng.laplace(0, 1, (M, N)) + rng.standard_normal((M, 1))  # per-worker offset


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.integers(1, 10))
    N = int(rng.choice([131_071, 131_072, 131_073, 150_001, 196_608, 262_144, 300_007, 524_288, 40_003, 4_099]))
    gamma = float(rng.choice([2e-4, 1e-3, 1e-2, 0.05, 1 / 16, 0.0626, 0.1, 0.3, 0.6, 0.95, 1.0]))
    K = max(1, min(N, int(round(gamma * N))))
    kind = int(rng.integers(0, 5))
    mode = int(rng.integers(0, 4))  # 0 fused, 1 three calls, 2 fused with memory, 3 separate calls with memory
    return rng, M, N, K, kind, mode


@pytest.mark.parametrize("seed", range(int(os.environ.get("S3GD_SWEEP_CASES", "80"))))  # more cases for a longer hunt
def test_seeded_case(ctx, seed):
    rng, M, N, K, kind, mode = _case(seed)
    what = f"seed {seed}: M={M} N={N} K={K} kind={kind} mode={mode}"
    G = _values(rng, kind, M, N).astype(np.float32)
    x = rng.standard_normal(N).astype(np.float32)
    lr = np.float32(rng.choice([1e-3, 0.25]))
    if mode < 2:
        want = O.step(G, K, x, lr)
        got = gpu_step(ctx, G, K, x, lr, fused=(mode == 0), dense_outputs=(mode == 1))
        assert_same(got, want, what=what)
    else:
        E = (_values(rng, int(rng.integers(0, 5)), M, N) * 0.5).astype(np.float32)
        eta = float(rng.choice([1.0, 0.5]))
        keys = ("words", "counts", "err", "x") if mode == 2 else ("words", "counts", "err", "tally", "votes", "x")
        for t in range(2):
            want = O.step_with_memory(G, E, eta, K, x, lr)
            got = gpu_step_ec(ctx, G, E, eta, K, x, lr, fused=(mode == 2), dense_outputs=(mode == 3))
            assert_same(got, want, keys=keys, what=f"{what} iteration {t}")
            E, x = want["err"], want["x"]
            G = _values(rng, kind, M, N).astype(np.float32)
    assert torch.cuda.is_available()
