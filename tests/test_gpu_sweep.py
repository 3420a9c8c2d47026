"""A seeded sweep over shapes, sparsity levels and value distributions, each case run through one
of the entry-point combinations (fused step, the three calls, with the memory, with momentum, random-K,
through the wire format) and compared with the CPU oracle bit for bit (tolerance 0).  The
cases are drawn so that every route of the encode is hit: rows below and above the smallest row the
single pass serves (2^17 entries), K on both sides of N/16 and N/64 (where the sample and the share
of records per candidate change), K = N, K of a handful, ties, zeros, magnitudes spread over decades."""
import os

import numpy as np
import pytest
import torch

from oracle import s3gd_coding as C
from oracle import s3gd_oracle as O
from oracle import s3gd_randk as R
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
    # 0 fused, 1 three calls, 2 fused with memory, 3 separate calls with memory, 4 momentum, 5 random-K, 6 wire format,
    # 7 memory that already holds the sum
    mode = int(rng.integers(0, 8))
    return rng, M, N, K, kind, mode


@pytest.mark.parametrize("seed", range(int(os.environ.get("S3GD_SWEEP_CASES", "80"))))  # more cases for a longer hunt
def test_seeded_case(ctx, lib, seed):
    rng, M, N, K, kind, mode = _case(seed)
    what = f"seed {seed}: M={M} N={N} K={K} kind={kind} mode={mode}"
    G = _values(rng, kind, M, N).astype(np.float32)
    x = rng.standard_normal(N).astype(np.float32)
    lr = np.float32(rng.choice([1e-3, 0.25]))
    if mode < 2:
        want = O.step(G, K, x, lr)
        got = gpu_step(ctx, G, K, x, lr, fused=(mode == 0), dense_outputs=(mode == 1))
        assert_same(got, want, what=what)
    elif mode == 7:
        E = (_values(rng, int(rng.integers(0, 5)), M, N) * 0.5).astype(np.float32)
        for t in range(2):
            want = O.step_with_memory(G, E, 1.0, K, x, lr)
            acc = torch.from_numpy(O.compensate(G, E, 1.0)).cuda()
            xd = torch.from_numpy(x.copy()).cuda()
            words = torch.empty((M, K), dtype=torch.int32, device="cuda")
            counts = torch.empty((M,), dtype=torch.int32, device="cuda")
            ctx.step_acc(acc, K, xd, float(lr), words, counts)
            torch.cuda.synchronize()
            got = dict(words=words.cpu().numpy().view(np.uint32), counts=counts.cpu().numpy().view(np.uint32),
                       err=acc.cpu().numpy(), x=xd.cpu().numpy())
            assert_same(got, want, keys=("words", "counts", "err", "x"), what=f"{what} iteration {t}")
            E, x = want["err"], want["x"]
            G = _values(rng, kind, M, N).astype(np.float32)
    elif mode == 4:
        mu = float(rng.choice([0.9, 0.5]))
        v = np.where(rng.random(N) < 0.5, 0.0, rng.standard_normal(N)).astype(np.float32)
        xd, vd = torch.from_numpy(x.copy()).cuda(), torch.from_numpy(v.copy()).cuda()
        words = torch.empty((M, K), dtype=torch.int32, device="cuda")
        counts = torch.empty((M,), dtype=torch.int32, device="cuda")
        for t in range(2):
            want = O.step_with_momentum(G, K, x, v, lr, mu)
            ctx.step_momentum(torch.from_numpy(G).cuda(), K, xd, vd, float(lr), mu, words, counts)
            torch.cuda.synchronize()
            got = dict(words=words.cpu().numpy().view(np.uint32), counts=counts.cpu().numpy().view(np.uint32),
                       x=xd.cpu().numpy(), v=vd.cpu().numpy())
            assert_same(got, want, keys=("words", "counts", "x", "v"), what=f"{what} iteration {t}")
            x, v = want["x"], want["v"]
            G = _values(rng, kind, M, N).astype(np.float32)
    elif mode == 5:
        seed, t = int(rng.integers(0, 2**63)), int(rng.integers(0, 1000))
        want = R.step_randk(G, K, x, lr, seed, t)
        xd = torch.from_numpy(x.copy()).cuda()
        words = torch.empty((M, K), dtype=torch.int32, device="cuda")
        counts = torch.empty((M,), dtype=torch.int32, device="cuda")
        ctx.step_randk(torch.from_numpy(G).cuda(), K, seed, t, xd, float(lr), words, counts)
        torch.cuda.synchronize()
        got = dict(words=words.cpu().numpy().view(np.uint32), counts=counts.cpu().numpy().view(np.uint32), x=xd.cpu().numpy())
        assert_same(got, want, keys=("words", "counts", "x"), what=what)
    elif mode == 6:
        want = O.step(G, K, x, lr)
        g = torch.from_numpy(G).cuda()
        xd = torch.from_numpy(x.copy()).cuda()
        words, counts = ctx.topk_sign_encode(g, K)
        packed = torch.full((M, lib.packed_row_words(N, K)), 0x55555555, dtype=torch.int32, device="cuda")
        ctx.pack_messages(words, counts, N, packed)
        w2, c2 = torch.empty_like(words), torch.empty_like(counts)
        ctx.unpack_messages(packed, N, K, w2, c2)
        ctx.vote_update(w2, c2, N, xd, float(lr))
        torch.cuda.synchronize()
        assert ctx.last_async_status() == 0
        pk = packed.cpu().numpy().view(np.uint32)
        for m in range(M):
            ref = C.pack_row_fast(want["words"][m], int(want["counts"][m]), N)
            assert np.array_equal(pk[m, : ref.size], ref), f"{what}: packed row {m}"
        got = dict(words=w2.cpu().numpy().view(np.uint32), counts=c2.cpu().numpy().view(np.uint32), x=xd.cpu().numpy())
        assert_same(got, want, keys=("words", "counts", "x"), what=what)
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
