"""HIP path vs CPU oracle, element by element and bit for bit, at sizes the oracle finishes in
seconds.  Tolerance: 0 differing bits on words, counts, tally, votes and fp32 parameters (the
update is x -/+ lr with one rounding, so no floating-point slack is needed or allowed)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2302_07475_amd import datagen
from tests.helpers import assert_same, gpu_step, oracle_step
from tests.test_oracle_pins import check_invariants

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(64, 1 << 21, 1 << 21, device=0)
    yield c
    c.close()


SCALED = [
    datagen.C1,
    datagen.C2.scaled(M=4, N=60_001, K=600),      # odd N: rows start at every 16-byte phase
    datagen.C3.scaled(M=5, N=50_002, K=50, steps=3),
    datagen.C4.scaled(M=3, N=40_003, K=400),      # many exact ties at the threshold, exact zeros
    datagen.C5.scaled(M=4, N=70_000, K=70),
    datagen.C2.scaled(M=16, N=300_000, K=3_000),
    datagen.C4.scaled(M=8, N=1_000_000, K=10_000),
]


@pytest.mark.parametrize("cfg", SCALED, ids=lambda c: f"{c.name}-M{c.M}-N{c.N}-K{c.K}")
@pytest.mark.parametrize("fused", [False, True], ids=["three_calls", "fused"])
def test_config_recipes_match_oracle(ctx, cfg, fused):
    x = datagen.params(cfg)
    lr = datagen.lr32(cfg)
    for step in range(cfg.steps):
        G = datagen.gradients(cfg, step=step)
        want = oracle_step(G, cfg.K, x, lr)
        got = gpu_step(ctx, G, cfg.K, x, lr, fused=fused)
        assert_same(got, want, what=f"{cfg.name} step {step}")
        if step == 0:
            check_invariants(G, cfg.K, got, x, lr)
        x = want["x"]  # parameters are carried across steps (Algorithm 1 outer loop)


def test_fused_sparse_update_matches(ctx):
    """Fused call without materialised tally/votes: only x, words, counts come back."""
    for cfg in (SCALED[1], SCALED[3], SCALED[5]):
        G = datagen.gradients(cfg)
        x = datagen.params(cfg)
        want = oracle_step(G, cfg.K, x, datagen.lr32(cfg))
        got = gpu_step(ctx, G, cfg.K, x, datagen.lr32(cfg), fused=True, dense_outputs=False)
        assert_same(got, want, keys=("words", "counts", "x"), what=cfg.name)


def _edge_rows():
    rng = np.random.default_rng(77)
    N = 9000  # three tiles with a ragged tail
    rows = {
        "all_equal": np.full(N, 1.5, dtype=np.float32),
        "all_equal_neg": np.full(N, -1.5, dtype=np.float32),
        "all_zero": np.zeros(N, dtype=np.float32),
        "pm_zero_few_nonzero": np.where(rng.random(N) < 0.01, rng.standard_normal(N), rng.choice([0.0, -0.0], N)).astype(np.float32),
        "two_valued": rng.choice([1.0, -1.0, 2.0, -2.0], N).astype(np.float32),
        "inf_mix": np.where(rng.random(N) < 0.001, np.inf, rng.standard_normal(N)).astype(np.float32) * rng.choice([1, -1], N).astype(np.float32),
        "denormal": (rng.integers(-50, 50, N).astype(np.float32) * np.float32(1e-45)).astype(np.float32),
        "coarse_grid": (np.rint(rng.standard_normal(N) * 2) / 2).astype(np.float32),
        "huge_range": (rng.standard_normal(N) * 10.0 ** rng.integers(-30, 30, N)).astype(np.float32),
    }
    return rows


@pytest.mark.parametrize("name", list(_edge_rows().keys()))
def test_degenerate_rows(ctx, name):
    g = _edge_rows()[name]
    N = g.shape[0]
    G = np.stack([g, g[::-1].copy(), np.roll(g, 17)])
    x = np.linspace(-1, 1, N, dtype=np.float32)
    for K in (1, 2, 63, 64, 65, 4096, 4097, N - 1, N):
        want = oracle_step(G, K, x, 0.125)
        got = gpu_step(ctx, G, K, x, 0.125, fused=(K % 2 == 0))
        assert_same(got, want, what=f"{name} K={K}")


@pytest.mark.parametrize("N", [1, 2, 3, 5, 63, 64, 65, 1023, 1024, 1025, 4093, 4095, 4096, 4097, 8191, 8192, 8193, 12289])
def test_ragged_sizes_every_alignment(ctx, N):
    rng = np.random.default_rng(N)
    M = 5  # with odd N the five rows start at different 16-byte phases
    G = (np.rint(rng.standard_normal((M, N)) * 8) / 8).astype(np.float32)
    x = rng.standard_normal(N).astype(np.float32)
    for K in sorted({0, 1, min(N, 7), N // 2, N}):
        want = oracle_step(G, K, x, 1e-3)
        got = gpu_step(ctx, G, K, x, 1e-3)
        assert_same(got, want, what=f"N={N} K={K}")


def test_unaligned_base_pointer(ctx):
    """grads only has to be 4-byte aligned: take views that start 1, 2, 3 floats into a buffer."""
    rng = np.random.default_rng(9)
    M, N, K = 3, 10_001, 123
    for off in (1, 2, 3):
        flat = rng.standard_normal(M * N + 4).astype(np.float32)
        G = flat[off:off + M * N].reshape(M, N)
        buf = torch.from_numpy(flat).cuda()
        g_dev = buf[off:off + M * N].view(M, N)
        assert g_dev.data_ptr() % 16 == 4 * off
        x = rng.standard_normal(N).astype(np.float32)
        want = oracle_step(np.ascontiguousarray(G), K, x, 1e-3)
        got = gpu_step(ctx, G, K, x, 1e-3, g_dev=g_dev)
        assert_same(got, want, what=f"offset {off}")


def test_single_worker_and_many_workers(ctx):
    rng = np.random.default_rng(21)
    for M in (1, 2, 33, 64):
        N, K = 20_000, 200
        G = rng.standard_normal((M, N)).astype(np.float32)
        G[:, :50] = G[0, :50]  # every worker agrees on the first coordinates: hot tally slots
        x = rng.standard_normal(N).astype(np.float32)
        want = oracle_step(G, K, x, 1e-3)
        got = gpu_step(ctx, G, K, x, 1e-3, fused=bool(M & 1))
        assert_same(got, want, what=f"M={M}")


def test_same_input_twice_is_bit_identical(ctx):
    cfg = SCALED[6]
    G = datagen.gradients(cfg)
    x = datagen.params(cfg)
    a = gpu_step(ctx, G, cfg.K, x, 1e-3)
    b = gpu_step(ctx, G, cfg.K, x, 1e-3)
    assert_same(a, b, what="determinism")


def test_inputs_are_not_modified(ctx):
    cfg = SCALED[1]
    G = datagen.gradients(cfg)
    g_dev = torch.from_numpy(G).cuda()
    gpu_step(ctx, G, cfg.K, datagen.params(cfg), 1e-3, g_dev=g_dev)
    assert np.array_equal(g_dev.cpu().numpy().view(np.uint32), G.view(np.uint32))


def test_nan_is_reported_not_hidden(ctx, lib):
    G = np.ones((2, 5000), dtype=np.float32)
    G[1, 4321] = np.nan
    g = torch.from_numpy(G).cuda()
    ctx.topk_sign_encode(g, 10)
    assert ctx.last_async_status() == lib.E_NAN
    g[1, 4321] = 1.0
    ctx.topk_sign_encode(g, 10)
    assert ctx.last_async_status() == 0


def test_silent_worker_casts_no_vote(ctx):
    """A worker whose count is zero is ignored by the vote (the server only sums what arrives)."""
    cfg = SCALED[1]
    G = datagen.gradients(cfg)
    x = datagen.params(cfg)
    dev = torch.device("cuda:0")
    words, counts = ctx.topk_sign_encode(torch.from_numpy(G).to(dev), cfg.K)
    counts[2] = 0
    tally = torch.empty(cfg.N, dtype=torch.int32, device=dev)
    votes = torch.empty(cfg.N, dtype=torch.int8, device=dev)
    ctx.majority_vote(words, counts, cfg.N, tally, votes)
    want = oracle_step(np.delete(G, 2, axis=0), cfg.K, x, 1e-3)
    assert np.array_equal(tally.cpu().numpy(), want["tally"]) and np.array_equal(votes.cpu().numpy(), want["votes"])


def test_argument_errors_enqueue_nothing(ctx, lib):
    dev = torch.device("cuda:0")
    g = torch.zeros((2, 100), dtype=torch.float32, device=dev)
    w = torch.zeros((2, 10), dtype=torch.int32, device=dev)
    c = torch.zeros((2,), dtype=torch.int32, device=dev)
    x = torch.zeros((100,), dtype=torch.float32, device=dev)
    v = torch.zeros((128,), dtype=torch.int8, device=dev)
    t = torch.zeros((100,), dtype=torch.int32, device=dev)
    r, h = lib.raw, ctx._h
    p = lambda z: ctypes.c_void_p(z.data_ptr())
    assert r.s3gd_topk_sign_encode(h, None, 2, 100, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_topk_sign_encode(h, p(g), 0, 100, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_topk_sign_encode(h, p(g), 2, 100, 101, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_topk_sign_encode(h, p(g), 65, 100, 10, p(w), p(c), None) == lib.E_INVAL  # above M_max
    assert r.s3gd_topk_sign_encode(h, p(g), 2, (1 << 31) - 1, 10, p(w), p(c), None) == lib.E_RANGE
    assert r.s3gd_topk_sign_encode(h, ctypes.c_void_p(g.data_ptr() + 2), 2, 50, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_majority_vote(h, p(w), p(c), 2, 100, 10, None, None, None) == lib.E_INVAL
    assert r.s3gd_majority_vote(h, p(w), p(c), 2, 100, 10, ctypes.c_void_p(t.data_ptr() + 4), None, None) == lib.E_INVAL
    assert r.s3gd_apply_update(h, p(x), p(v), float("nan"), 100, None) == lib.E_INVAL
    assert r.s3gd_apply_update(h, p(x), p(v), -1.0, 100, None) == lib.E_INVAL
    assert r.s3gd_apply_update(h, p(x), None, 0.1, 100, None) == lib.E_INVAL
    assert r.s3gd_step(h, p(g), 2, 100, 10, None, 0.1, p(w), p(c), None, None, None) == lib.E_INVAL
    torch.cuda.synchronize()
    assert int(w.abs().sum()) == 0 and int(c.abs().sum()) == 0


# ---------------------------------------------------------------- candidate route and its fallback
def _encode_only(ctx, G, K):
    g = torch.from_numpy(G).cuda()
    words, counts = ctx.topk_sign_encode(g, K)
    torch.cuda.synchronize()
    assert ctx.last_async_status() == 0
    rows, general = ctx.last_encode_info()
    return words.cpu().numpy().view(np.uint32), counts.cpu().numpy().view(np.uint32), rows, general


@pytest.mark.parametrize("kind", ["gauss", "ties", "layers"])
@pytest.mark.parametrize("gamma", [0.07, 0.1, 0.25, 0.5, 0.9, 0.999, 1.0])
def test_dense_sparsity_levels(ctx, gamma, kind):
    """K/N from 0.07 to 1 (the paper sweeps the sparsity up to 1, signSGD with majority vote): the
    filter pass keeps records for a bracket around the K-th magnitude and only the words of what lies
    above; K = N selects nothing.  Whatever route a row ends on, words, votes and parameters are the oracle's; on
    well-spread data up to K = N/2 no row needs the general route."""
    from oracle import s3gd_oracle as O
    rng = np.random.default_rng(int(gamma * 1000))
    M, N = 3, 300_007
    if kind == "gauss":
        G = rng.standard_normal((M, N)).astype(np.float32)
    elif kind == "ties":  # coarse grid and exact zeros: thousands of entries share the K-th magnitude
        G = (np.rint(rng.standard_t(3, (M, N)) * 16) / 16).astype(np.float32)
        G[rng.random((M, N)) < 0.05] = 0.0
    else:  # magnitudes spread over four decades in contiguous blocks
        G = (rng.standard_normal((M, N)) * np.repeat(10.0 ** rng.uniform(-4, 0, (M, 60)), N // 60 + 1, axis=1)[:, :N]).astype(np.float32)
    K = min(N, int(round(gamma * N)))
    x = rng.standard_normal(N).astype(np.float32)
    want = O.step(G, K, x, np.float32(1e-3))
    got = gpu_step(ctx, G, K, x, 1e-3, fused=True, dense_outputs=False)
    assert_same(got, want, keys=("words", "counts", "x"), what=f"{kind} gamma={gamma}")
    if kind == "gauss" and gamma <= 0.5:
        assert ctx.last_encode_info() == (M, 0)
    if gamma == 1.0:
        assert ctx.last_encode_info() == (M, 0)  # nothing to select: not a fallback


def test_dense_rows_that_do_not_fit_the_bracket(ctx):
    """K/N = 0.2 on rows whose magnitudes crowd the bracket (all equal, two values, one value plus a
    sprinkle of larger ones) or leave it empty around the K-th key: each such row ends on the general
    route, the well-spread row next to them does not."""
    from oracle import s3gd_oracle as O
    rng = np.random.default_rng(77)
    N = 400_000
    K = N // 5
    G = np.empty((5, N), dtype=np.float32)
    G[0] = rng.standard_normal(N)
    G[1] = 3.0
    G[2] = rng.choice([1.0, -1.0, 1.0000001], N)
    G[3] = np.where(rng.random(N) < 0.01, rng.standard_normal(N) * 100, 0.5)
    G[4] = np.where(rng.random(N) < 0.15, 1e6, 1e-6) * rng.choice([1.0, -1.0], N)  # K-th key far below the ones above it
    x = rng.standard_normal(N).astype(np.float32)
    want = O.step(G, K, x, np.float32(1e-3))
    got = gpu_step(ctx, G, K, x, 1e-3, fused=True, dense_outputs=False)
    assert_same(got, want, keys=("words", "counts", "x"), what="crowded brackets")
    rows, general = ctx.last_encode_info()
    assert rows == 5 and 3 <= general <= 4


@pytest.mark.parametrize("N,K", [(131_072, 131), (200_003, 2_000), (1_000_000, 1_000), (2_000_001, 20_000), (2_097_152, 100_000)])
def test_candidate_route_is_taken_and_exact(ctx, N, K):
    from oracle import s3gd_oracle as O
    rng = np.random.default_rng(N + K)
    M = 3
    G = (rng.standard_normal((M, N)) * np.exp(rng.standard_normal((M, 1)))).astype(np.float32)
    words, counts, rows, general = _encode_only(ctx, G, K)
    w, c = O.topk_sign_encode(G, K)
    assert np.array_equal(words, w) and np.array_equal(counts, c)
    assert rows == M and general == 0, "ordinary data must not need the general route"


def test_rows_fall_back_independently(ctx):
    """Row 0 ordinary, row 1 all equal (every entry ties: too many candidates), row 2 mostly zero
    (lower bound 0), row 3 two-valued with the tie straddling K."""
    from oracle import s3gd_oracle as O
    rng = np.random.default_rng(5)
    N, K = 500_000, 5_000
    G = np.empty((4, N), dtype=np.float32)
    G[0] = rng.standard_normal(N)
    G[1] = -2.0
    G[2] = np.where(rng.random(N) < 0.001, rng.standard_normal(N), 0.0)
    G[3] = rng.choice([1.0, -1.0, 3.0], N, p=[0.5, 0.495, 0.005])
    words, counts, rows, general = _encode_only(ctx, G, K)
    w, c = O.topk_sign_encode(G, K)
    assert np.array_equal(counts, c)
    assert np.array_equal(words, w)
    assert general == 3


def test_threshold_ties_on_candidate_route(ctx):
    """Values on a coarse grid: hundreds of entries share the K-th magnitude; the lowest indices win."""
    from oracle import s3gd_oracle as O
    cfg = datagen.C4.scaled(M=4, N=1_500_000, K=15_000)
    G = (np.rint(datagen.gradients(cfg) * 64.0) / 64.0).astype(np.float32)  # grid 2^-6 at this small N
    words, counts, rows, general = _encode_only(ctx, G, cfg.K)
    w, c = O.topk_sign_encode(G, cfg.K)
    assert np.array_equal(words, w) and np.array_equal(counts, c)
    mag = np.abs(G[0])
    t = mag[(w[0] >> 1).astype(np.int64)].min()
    assert np.count_nonzero(mag == t) > 10, "the recipe is meant to produce ties at the threshold"
    assert general == 0


@pytest.mark.parametrize("M", [63, 64, 257, 300, 16500])
def test_many_workers_every_tally_width(lib, M):
    """The fused step packs tallies into 8-, 16- or 32-bit LDS fields depending on M, and walks the
    rows in chunks of 256; all workers agree on some coordinates so that |tally| reaches M."""
    rng = np.random.default_rng(M)
    N, K = 3000, 12
    G = rng.standard_normal((M, N)).astype(np.float32)
    G[:, 7] = 50.0      # everyone votes +1 here
    G[:, 11] = -60.0    # everyone votes -1 here
    G[::2, 13] = 70.0   # half vote +1 ...
    G[1::2, 13] = -70.0  # ... half vote -1: a tie when M is even
    x = rng.standard_normal(N).astype(np.float32)
    want = oracle_step(G, K, x, 0.5)
    assert abs(int(want["tally"][7])) == M and abs(int(want["tally"][11])) == M
    with lib.Context(M, N, K, device=0) as c:
        got = gpu_step(c, G, K, x, 0.5, fused=True, dense_outputs=False)
        assert_same(got, want, keys=("words", "counts", "x"), what=f"sparse M={M}")
        got = gpu_step(c, G, K, x, 0.5, fused=True, dense_outputs=True)
        assert_same(got, want, what=f"dense M={M}")


@pytest.mark.parametrize("M,N,K", [(10, 500_000, 500), (100, 500_000, 25_000), (5, 850_000, 8_500), (50, 850_000, 42_500)])
def test_paper_sized_models(lib, M, N, K):
    """The paper's own sizes: its CNN (N = 5e5) and ResNet-56 (N = 8.5e5) with the worker counts and
    sparsities of its cost comparison (Section 4), on the i.i.d. recipe.  Element by element."""
    cfg = datagen.C1.scaled(M=M, N=N, K=K)
    G = datagen.gradients(cfg)
    x = datagen.params(cfg)
    want = oracle_step(G, K, x, 1e-3)
    with lib.Context(M, N, K, device=0) as c:
        got = gpu_step(c, G, K, x, 1e-3, fused=True)
        assert_same(got, want, what=f"M={M} N={N} K={K}")
        got = gpu_step(c, G, K, x, 1e-3, fused=True, dense_outputs=False)
        assert_same(got, want, keys=("words", "counts", "x"), what=f"sparse M={M} N={N} K={K}")


def _banded_rows(N, K, band, rng):
    """Rows whose K largest magnitudes all sit in one narrow band (a layer with a far larger scale)."""
    G = (rng.standard_normal((3, N)) * 0.01).astype(np.float32)
    starts = [0, N // 2 - band // 2, N - band]
    for m, s in enumerate(starts):
        G[m, s:s + band] = (rng.standard_normal(band) * 5.0 + np.sign(rng.standard_normal(band)) * 3.0).astype(np.float32)
    return G


def test_skewed_rows_grow_their_segment_lists(ctx):
    """All candidates of a row come from a few waves of the single pass: those waves fill their first
    slab and reserve more (twice as large each time); the row stays on the candidate route."""
    from oracle import s3gd_oracle as O
    rng = np.random.default_rng(11)
    N, K, band = 1 << 21, 20_971, 32_768
    G = _banded_rows(N, K, band, rng)
    words, counts, rows, general = _encode_only(ctx, G, K)
    w, c = O.topk_sign_encode(G, K)
    assert np.array_equal(counts, c) and np.array_equal(words, w)
    # the magnitudes are spread widely around the threshold: the K-th lies far above the sampled
    # bound, so the radix select runs over all levels, but over the candidates, not over the row
    assert ctx.last_encode_details() == (3, 0, 3)
    idx = (w[1] >> 1).astype(np.int64)
    assert idx.min() >= N // 2 - band // 2 and idx.max() < N // 2 + band // 2, "the recipe is meant to put every selected entry in the band"


def _row_with_dense_head(N, head, rng):
    """Small noise everywhere; the first `head` entries are far larger than anything else (distinct
    magnitudes, random signs): one wave of the single pass finds a candidate in every entry it reads."""
    g = (rng.standard_normal(N, dtype=np.float32) * np.float32(0.01))
    big = (100.0 + rng.random(head) * 50.0) * np.sign(rng.standard_normal(head))
    g[:head] = big.astype(np.float32)
    return g


def _check_rows_exactly(G, K, words, counts):
    from oracle import s3gd_oracle as O
    for m in range(G.shape[0]):
        O.check_message_row(G[m], K, words[m], int(counts[m]))  # admits one answer: the sorted one


def test_one_wave_holds_a_long_chain_of_segments(lib):
    """A wave of the single pass covers dozens of consecutive 1024-entry tiles.  When every entry of 24
    of them is a candidate the wave fills its first slab at once and reserves more, each reservation
    at least twice the slab and doubling: a list of seven or eight segments, the longest a list may
    be.  The row stays on the candidate route (no row on the general one)."""
    rng = np.random.default_rng(12)
    N, K = 1 << 27, (1 << 27) // 1000
    with lib.Context(1, N, K, device=0) as c:
        plan = c.encode_plan_info(1, N, K)
        assert plan["candidates"] and not plan["chunks"], plan
        assert plan["chain"] == 8 and plan["slab"] <= 1024 and plan["tiles_per_wave"] >= 24, \
            f"shape no longer puts 24 all-candidate tiles into one wave with a small first slab: {plan}"
        G = _row_with_dense_head(N, 24 * 1024, rng)[None, :]
        words, counts, rows, general = _encode_only(c, G, K)
        assert c.last_encode_details()[:2] == (1, 0), "the chain of eight segments suffices: the row stays on the candidate route"
    _check_rows_exactly(G, K, words, counts)
    assert counts[0] == K and (words[0, :24 * 1024] >> 1 == np.arange(24 * 1024)).all()


def test_full_chain_hands_the_row_to_the_general_route(lib):
    """The same with every tile of the first wave's range a candidate tile and a range long enough to
    exhaust eight doubling segments: the wave marks the row, nothing more is kept for it, and the
    general multi-pass route serves it, with the same words."""
    rng = np.random.default_rng(13)
    M, N, K = 2, 1 << 27, (1 << 27) // 1000
    with lib.Context(M, N, K, device=0) as c:
        plan = c.encode_plan_info(M, N, K)
        assert plan["candidates"] and not plan["chunks"], plan
        tiles = plan["tiles_per_wave"]
        # a list has eight segments of slab, slab, 2 slab, ... 64 slab slots, none smaller than the tile that opens it
        longest = sum(max(plan["slab"] << max(i - 1, 0), 1024) for i in range(plan["chain"])) // 1024
        assert tiles > longest, f"a wave's range ({tiles} tiles) no longer exceeds the longest chain ({longest} tiles): {plan}"
        G = np.stack([_row_with_dense_head(N, tiles * 1024, rng),
                      (rng.standard_normal(N, dtype=np.float32))])  # an ordinary row next to it keeps its route
        words, counts, rows, general = _encode_only(c, G, K)
        assert c.last_encode_details()[:2] == (2, 1), "row 0 ends on the general route, row 1 stays on the candidate route"
    _check_rows_exactly(G, K, words, counts)


def test_candidates_the_sample_missed_exhaust_the_pool(lib):
    """A row whose sample looks ordinary while nearly every entry outside the sampled units is large:
    the sampled bound lies among the small entries, the pass finds a candidate almost everywhere, the
    row's share of the pool runs out (waves find no room for another slab) and the row is handed to
    the general route.  The sample's positions come from the library."""
    rng = np.random.default_rng(14)
    N, K = 1 << 22, (1 << 22) // 1000
    with lib.Context(2, N, K, device=0) as c:
        plan = c.encode_plan_info(2, N, K)
        assert plan["candidates"], plan
        small = (rng.standard_normal(N, dtype=np.float32) * np.float32(0.01))
        g = ((50.0 + rng.random(N) * 50.0) * np.sign(rng.standard_normal(N))).astype(np.float32)
        for u in range(plan["n_units"]):
            p = lib.encode_sample_unit_start(u, plan["unit_stride"])
            g[p:p + plan["sample_unit"]] = small[p:p + plan["sample_unit"]]
        assert N - plan["n_units"] * plan["sample_unit"] > plan["cand_stride"]
        G = np.stack([g, rng.standard_normal(N, dtype=np.float32)])
        words, counts, rows, general = _encode_only(c, G, K)
        assert c.last_encode_details()[:2] == (2, 1)
    _check_rows_exactly(G, K, words, counts)
    w, cc = __import__("oracle.s3gd_oracle", fromlist=["x"]).topk_sign_encode(G, K)
    assert np.array_equal(counts, cc) and np.array_equal(words, w)


def test_list_longer_than_one_emit_round(lib):
    """The emit pass marks the bracket's losers of 65536 candidates at a time.  One wave of the single
    pass finds 80 all-candidate tiles in a row (dense K, so its slabs are large enough to hold them):
    its list takes two rounds.  The row stays on the candidate route."""
    rng = np.random.default_rng(15)
    N = 1 << 28
    K = N // 16
    with lib.Context(1, N, K, device=0) as c:
        plan = c.encode_plan_info(1, N, K)
        assert plan["candidates"] and not plan["chunks"] and plan["tiles_per_wave"] >= 80, plan
        assert plan["slab"] * 100 > 80 * 1024 << plan["record_shift"], f"the chain of this shape no longer holds 80 tiles: {plan}"
        G = _row_with_dense_head(N, 80 * 1024, rng)[None, :]
        G[0, 80 * 1024:] *= np.float32(100.0)  # spread the rest so that the bracket holds an ordinary share of it
        words, counts, rows, general = _encode_only(c, G, K)
        assert c.last_encode_details()[:2] == (1, 0)
    _check_rows_exactly(G, K, words, counts)
    assert (words[0, :80 * 1024] >> 1 == np.arange(80 * 1024)).all()


def test_every_selected_entry_above_the_bracket(lib):
    """A row built against the sample: exactly K large entries, none of them in a sampled unit, and a
    middle level that fills the sample's upper ranks.  Both sampled bounds land on the middle level, so
    the pass takes exactly K entries for sure and the whole bracket loses: the threshold is the
    bracket's upper end and no radix select runs."""
    rng = np.random.default_rng(16)
    N, K = 1 << 22, 1 << 12
    with lib.Context(2, N, K, device=0) as c:
        plan = c.encode_plan_info(2, N, K)
        assert plan["candidates"], plan
        sampled = np.zeros(N, dtype=bool)
        for u in range(plan["n_units"]):
            p = lib.encode_sample_unit_start(u, plan["unit_stride"])
            sampled[p:p + plan["sample_unit"]] = True
        g = np.full(N, 0.001, dtype=np.float32)
        g[rng.random(N) < 1.5 * K / N] = 0.5                      # the middle level, sampled like everything else
        free = np.nonzero(~sampled)[0]
        top = rng.choice(free, size=K, replace=False)               # the K entries to select: the sample sees none
        g[top] = (100.0 + rng.random(K)).astype(np.float32) * np.sign(rng.standard_normal(K)).astype(np.float32)
        G = np.stack([g, rng.standard_normal(N, dtype=np.float32)])
        words, counts, rows, general = _encode_only(c, G, K)
        st = c.last_row_state(0)
        assert st["mode"] == 3 and st["n_cand"] - st["n_brk"] == K and st["T"] == st["U"] - 1, st
        assert c.last_encode_details()[:2] == (2, 0)
    w, cc = __import__("oracle.s3gd_oracle", fromlist=["x"]).topk_sign_encode(G, K)
    assert np.array_equal(counts, cc) and np.array_equal(words, w)
    assert np.array_equal(np.sort(top), (words[0] >> 1).astype(np.int64))


def test_fresh_context_has_clear_status(lib):
    """The status words belong to the workspace, which is not cleared as a whole: a context created
    over memory that held other data before must still report no stale flag after its first call."""
    junk = torch.full((64 << 20,), -1, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    del junk
    torch.cuda.empty_cache()
    for _ in range(4):
        with lib.Context(2, 50_000, 500, device=0) as c:
            assert c.last_async_status() == 0
            g = torch.randn((2, 50_000), device="cuda")
            c.topk_sign_encode(g, 500)
            torch.cuda.synchronize()
            assert c.last_async_status() == 0



def test_two_contexts_on_two_streams(lib):
    """One context per stream is the contract: two contexts, each with its own scratch memory, take
    steps on different inputs from two streams at once; each ends with the oracle's result."""
    cfgs = [datagen.C2.scaled(M=6, N=400_000, K=4_000), datagen.C5.scaled(M=4, N=700_001, K=700)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs = [lib.Context(c.M, c.N, c.K, device=0) for c in cfgs]
    try:
        G = [datagen.gradients(c) for c in cfgs]
        x0 = [datagen.params(c) for c in cfgs]
        g = [torch.from_numpy(a).cuda() for a in G]
        x = [torch.from_numpy(a.copy()).cuda() for a in x0]
        words = [torch.empty((c.M, c.K), dtype=torch.int32, device="cuda") for c in cfgs]
        counts = [torch.empty((c.M,), dtype=torch.int32, device="cuda") for c in cfgs]
        torch.cuda.synchronize()
        steps = 3
        for _ in range(steps):
            for i in (0, 1):
                ctxs[i].step(g[i], cfgs[i].K, x[i], float(datagen.lr32(cfgs[i])), words[i], counts[i], None, None,
                             stream=streams[i])
        torch.cuda.synchronize()
        for i in (0, 1):
            assert ctxs[i].last_async_status() == 0
            want = x0[i]
            for _ in range(steps):
                want = oracle_step(G[i], cfgs[i].K, want, datagen.lr32(cfgs[i]))["x"]
            assert np.array_equal(x[i].cpu().numpy().view(np.uint32), want.view(np.uint32))
    finally:
        for c in ctxs:
            c.close()
