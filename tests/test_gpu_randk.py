"""RandKSign (Algorithm 2) on the HIP path vs its CPU oracle: the same keyed permutation on both
sides, so index sets, words, counts, votes and parameters agree bit for bit (integer work and the
exact x -/+ lr; tolerance 0)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import s3gd_randk as R
from paper_2302_07475_amd import datagen
from tests.helpers import assert_same

pytestmark = pytest.mark.gpu
SEED = 0x1234_5678_9ABC_DEF0


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(64, 1 << 22, 1 << 22, device=0)
    yield c
    c.close()


def gpu_step_randk(ctx, G, K, x0, lr, seed, t, fused, dense_outputs=True):
    dev = torch.device("cuda:0")
    M, N = G.shape
    g = torch.from_numpy(G).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x0).copy()).to(dev)
    words = torch.full((M, K), 0x55555555, dtype=torch.int32, device=dev)
    counts = torch.full((M,), 0x55555555, dtype=torch.int32, device=dev)
    tally = votes = None
    if dense_outputs:
        tally = torch.full((N,), 0x55555555, dtype=torch.int32, device=dev)
        votes = torch.full((N,), 0x55, dtype=torch.int8, device=dev)
    if fused:
        ctx.step_randk(g, K, seed, t, x, float(lr), words, counts, tally, votes)
    else:
        ctx.randk_sign_encode(g, K, seed, t, words, counts)
        ctx.majority_vote(words, counts, N, tally, votes)
        ctx.apply_update(x, votes, float(lr))
    torch.cuda.synchronize()
    assert ctx.last_async_status() == 0
    out = dict(words=words.cpu().numpy().view(np.uint32), counts=counts.cpu().numpy().view(np.uint32), x=x.cpu().numpy())
    if dense_outputs:
        out["tally"] = tally.cpu().numpy()
        out["votes"] = votes.cpu().numpy()
    assert np.array_equal(g.cpu().numpy().view(np.uint32), G.view(np.uint32)), "gradients untouched"
    return out


SCALED = [
    datagen.C1,
    datagen.C2.scaled(M=4, N=60_001, K=600),
    datagen.C3.scaled(M=5, N=50_002, K=50, steps=3),
    datagen.C4.scaled(M=3, N=40_003, K=400),        # 5 % exact zeros: some selected entries send nothing
    datagen.C5.scaled(M=4, N=270_001, K=270),
    datagen.C2.scaled(M=16, N=300_000, K=3_000),
    datagen.C4.scaled(M=8, N=1_000_000, K=100_000),
]


@pytest.mark.parametrize("cfg", SCALED, ids=lambda c: f"{c.name}-M{c.M}-N{c.N}-K{c.K}")
@pytest.mark.parametrize("fused", [False, True], ids=["three_calls", "fused"])
def test_config_recipes_match_oracle(ctx, cfg, fused):
    x = datagen.params(cfg)
    lr = datagen.lr32(cfg)
    for t in range(cfg.steps):
        G = datagen.gradients(cfg, step=t)
        want = R.step_randk(G, cfg.K, x, lr, SEED, t)
        got = gpu_step_randk(ctx, G, cfg.K, x, lr, SEED, t, fused)
        assert_same(got, want, what=f"{cfg.name} iteration {t}")
        x = want["x"]


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 16, 17, 255, 257, 2047, 2048, 2049, 4097, 65_536, 100_003, 1 << 21, (1 << 21) + 1])
def test_every_domain_width_and_ragged_sizes(ctx, N):
    """N sets the width of the Feistel halves (odd and even bit lengths, exact powers of two) and
    the number of buckets; K runs from nothing to everything."""
    rng = np.random.default_rng(N)
    M = 3
    G = rng.standard_normal((M, N)).astype(np.float32)
    x = rng.standard_normal(N).astype(np.float32)
    for K in sorted({0, 1, min(N, 7), N // 100, N // 2, N}):
        if N > 100_000 and K == N // 2:
            continue
        want = R.step_randk(G, K, x, 1e-3, SEED + N, 4)
        got = gpu_step_randk(ctx, G, K, x, 1e-3, SEED + N, 4, fused=bool(K & 1))
        assert_same(got, want, what=f"N={N} K={K}")


def test_keys_matter_and_same_key_repeats(ctx):
    cfg = SCALED[5]
    G = datagen.gradients(cfg)
    g = torch.from_numpy(G).cuda()
    a, _ = ctx.randk_sign_encode(g, cfg.K, SEED, 0)
    b, _ = ctx.randk_sign_encode(g, cfg.K, SEED, 0)
    c, _ = ctx.randk_sign_encode(g, cfg.K, SEED, 1)
    d, _ = ctx.randk_sign_encode(g, cfg.K, SEED ^ (1 << 63), 0)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and not torch.equal(a, c) and not torch.equal(a, d)
    want, _ = R.randk_sign_encode(G, cfg.K, SEED ^ (1 << 63), 0)
    assert np.array_equal(d.cpu().numpy().view(np.uint32), want)


def test_zero_rows_and_dense_buckets(ctx):
    """K = N fills every bucket to its 2048-coordinate capacity; an all-zero row sends nothing."""
    rng = np.random.default_rng(8)
    N = 50_000
    G = rng.standard_normal((3, N)).astype(np.float32)
    G[1] = 0.0
    G[2, ::2] = -0.0
    x = rng.standard_normal(N).astype(np.float32)
    want = R.step_randk(G, N, x, 0.5, 5, 6)
    got = gpu_step_randk(ctx, G, N, x, 0.5, 5, 6, fused=True)
    assert_same(got, want, what="K=N")
    assert got["counts"].tolist() == [N, 0, N // 2]


def test_many_workers(lib):
    rng = np.random.default_rng(9)
    M, N, K = 300, 30_000, 64
    G = rng.standard_normal((M, N)).astype(np.float32)
    x = rng.standard_normal(N).astype(np.float32)
    want = R.step_randk(G, K, x, 1e-3, SEED, 2)
    with lib.Context(M, N, K, device=0) as c:
        got = gpu_step_randk(c, G, K, x, 1e-3, SEED, 2, fused=True)
    assert_same(got, want, what="M=300")


@pytest.mark.parametrize("shape", [(2, 50_000, 5_000), (3, 300_000, 150_000), (3, 300_000, 3_000)],
                         ids=["no_scratch_pool", "K_beyond_the_pool", "pool_holds_the_records"])
def test_both_forms_of_the_second_step(lib, shape):
    """A context of exactly the call's size: small rows and dense K leave no room for the per-entry
    records, so the second step evaluates the permutation again; the last shape keeps the records."""
    M, N, K = shape
    rng = np.random.default_rng(N + K)
    G = rng.standard_normal((M, N)).astype(np.float32)
    G[:, ::9] = 0.0
    x = rng.standard_normal(N).astype(np.float32)
    want = R.step_randk(G, K, x, 1e-3, SEED, 5)
    with lib.Context(M, N, K, device=0) as c:
        got = gpu_step_randk(c, G, K, x, 1e-3, SEED, 5, fused=False)
    assert_same(got, want, what=f"{shape}")


def test_nan_among_the_selected_is_reported(ctx, lib):
    G = np.ones((2, 5000), dtype=np.float32)
    S = R.randk_index_set(5000, 50, SEED, 0, 1)
    G[1, S[10]] = np.nan
    g = torch.from_numpy(G).cuda()
    ctx.randk_sign_encode(g, 50, SEED, 0)
    assert ctx.last_async_status() == lib.E_NAN


def test_argument_errors(ctx, lib):
    g = torch.zeros((2, 100), dtype=torch.float32, device="cuda")
    w = torch.zeros((2, 10), dtype=torch.int32, device="cuda")
    c = torch.zeros((2,), dtype=torch.int32, device="cuda")
    r, h = lib.raw, ctx._h
    p = lambda z: ctypes.c_void_p(z.data_ptr())
    assert r.s3gd_randk_sign_encode(h, None, 2, 100, 10, 1, 0, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_randk_sign_encode(h, p(g), 2, 100, 101, 1, 0, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_randk_sign_encode(h, p(g), 2, 100, 10, 1, 0, None, p(c), None) == lib.E_INVAL
    assert r.s3gd_step_randk(h, p(g), 2, 100, 10, 1, 0, None, 0.1, p(w), p(c), None, None, None) == lib.E_INVAL
