"""Error-compensation memory on the HIP path vs the CPU oracle (Algorithm 1 with the two memory
lines): words, counts, the new memory, tally, votes and parameters, bit for bit.  Tolerance 0: the
compensation is one rounded product and one rounded sum on both sides, everything else is
integer work or the exact x -/+ lr."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import s3gd_oracle as O
from paper_2302_07475_amd import datagen
from tests.helpers import assert_same

pytestmark = pytest.mark.gpu

KEYS = ("words", "counts", "err", "tally", "votes", "x")


@pytest.fixture(scope="module")
def ctx(lib):
    c = lib.Context(64, 1 << 21, 1 << 21, device=0)
    yield c
    c.close()


def gpu_step_ec(ctx, Gt, E, eta, K, x0, lr, fused, dense_outputs=True, gt_dev=None, e_dev=None):
    dev = torch.device("cuda:0")
    M, N = Gt.shape
    g = torch.from_numpy(np.ascontiguousarray(Gt)).to(dev) if gt_dev is None else gt_dev
    e = torch.from_numpy(np.ascontiguousarray(E).copy()).to(dev) if e_dev is None else e_dev
    x = torch.from_numpy(np.ascontiguousarray(x0).copy()).to(dev)
    words = torch.full((M, K), 0x55555555, dtype=torch.int32, device=dev)
    counts = torch.full((M,), 0x55555555, dtype=torch.int32, device=dev)
    tally = votes = None
    if dense_outputs:
        tally = torch.full((N,), 0x55555555, dtype=torch.int32, device=dev)
        votes = torch.full((N,), 0x55, dtype=torch.int8, device=dev)
    if fused:
        ctx.step_ec(g, e, eta, K, x, float(lr), words, counts, tally, votes)
    else:
        ctx.topk_sign_encode_ec(g, e, eta, K, words, counts)
        ctx.majority_vote(words, counts, N, tally, votes)
        ctx.apply_update(x, votes, float(lr))
    torch.cuda.synchronize()
    assert ctx.last_async_status() == 0
    out = dict(words=words.cpu().numpy().view(np.uint32), counts=counts.cpu().numpy().view(np.uint32),
               err=e.cpu().numpy(), x=x.cpu().numpy(), g_dev=g)
    if dense_outputs:
        out["tally"] = tally.cpu().numpy()
        out["votes"] = votes.cpu().numpy()
    return out


SCALED = [
    datagen.C1,
    datagen.C2.scaled(M=4, N=60_001, K=600),
    datagen.C3.scaled(M=5, N=50_002, K=50, steps=3),
    datagen.C4.scaled(M=3, N=40_003, K=400),
    datagen.C5.scaled(M=4, N=270_001, K=270),       # candidate route, odd N
    datagen.C2.scaled(M=16, N=300_000, K=3_000),    # candidate route
    datagen.C4.scaled(M=8, N=1_000_000, K=10_000),  # candidate route with ties at the threshold
]


@pytest.mark.parametrize("cfg", SCALED, ids=lambda c: f"{c.name}-M{c.M}-N{c.N}-K{c.K}")
@pytest.mark.parametrize("eta", [1.0, 0.5])
def test_iterations_with_memory_match_oracle(ctx, cfg, eta):
    """Three iterations of Algorithm 1 with the memory and the parameters carried along."""
    x = datagen.params(cfg)
    lr = datagen.lr32(cfg)
    E = np.zeros((cfg.M, cfg.N), dtype=np.float32)  # e^0 = 0
    for t in range(3):
        Gt = datagen.gradients(cfg, step=t)
        want = O.step_with_memory(Gt, E, eta, cfg.K, x, lr)
        got = gpu_step_ec(ctx, Gt, E, eta, cfg.K, x, lr, fused=bool(t & 1))
        assert_same(got, want, keys=KEYS, what=f"{cfg.name} eta={eta} iteration {t}")
        assert np.array_equal(got["g_dev"].cpu().numpy().view(np.uint32), Gt.view(np.uint32)), "fresh gradients untouched"
        E, x = want["err"], want["x"]


def test_eta_zero_is_the_memoryless_encode(ctx):
    cfg = SCALED[5]
    Gt = datagen.gradients(cfg)
    E = (np.random.default_rng(1).standard_normal(Gt.shape) * 100).astype(np.float32)  # must be ignored
    x = datagen.params(cfg)
    want = O.step(Gt, cfg.K, x, 1e-3)
    got = gpu_step_ec(ctx, Gt, E, 0.0, cfg.K, x, 1e-3, fused=True)
    assert_same(got, want, keys=("words", "counts", "tally", "votes", "x"), what="eta=0")
    assert_same(got, dict(err=O.residual(O.compensate(Gt, E, 0.0), want["words"], want["counts"])), keys=("err",), what="eta=0 err")


def test_sparse_fused_step_with_memory(ctx):
    for cfg in (SCALED[1], SCALED[4], SCALED[6]):
        Gt = datagen.gradients(cfg)
        E = datagen.gradients(cfg, step=7) * np.float32(0.25)
        x = datagen.params(cfg)
        want = O.step_with_memory(Gt, E, 1.0, cfg.K, x, 1e-3)
        got = gpu_step_ec(ctx, Gt, E, 1.0, cfg.K, x, 1e-3, fused=True, dense_outputs=False)
        assert_same(got, want, keys=("words", "counts", "err", "x"), what=cfg.name)


@pytest.mark.parametrize("N", [1, 2, 3, 5, 63, 64, 65, 1023, 1024, 1025, 4095, 4096, 4097, 8193, 12289, 131_073, 140_001])
def test_ragged_sizes_every_alignment(ctx, N):
    """Odd N puts the five rows at different 16-byte phases; the last two sizes take the filter pass."""
    rng = np.random.default_rng(N)
    M = 5
    Gt = (np.rint(rng.standard_normal((M, N)) * 8) / 8).astype(np.float32)
    E = (np.rint(rng.standard_normal((M, N)) * 4) / 16).astype(np.float32)
    x = rng.standard_normal(N).astype(np.float32)
    for K in sorted({0, 1, min(N, 7), N // 200, N // 2, N}):
        want = O.step_with_memory(Gt, E, 1.0, K, x, 1e-3)
        got = gpu_step_ec(ctx, Gt, E, 1.0, K, x, 1e-3, fused=False)
        assert_same(got, want, keys=KEYS, what=f"N={N} K={K}")


@pytest.mark.parametrize("N", [196_607, 196_608, 196_613, 262_147, 589_825, 655_361])
def test_filter_chunk_boundaries(ctx, N):
    """Row lengths around multiples of a filter block (8192 entries) and of a segment list (8 blocks),
    rows at different 16-byte phases, continuous values (few ties) and a stretch of the row without
    any candidate; every row must be served by the filter pass."""
    rng = np.random.default_rng(N)
    M = 3
    Gt = rng.standard_normal((M, N)).astype(np.float32)
    E = (rng.standard_normal((M, N)) * 0.25).astype(np.float32)
    Gt[:, 20_000:90_000] *= 1e-3  # nothing here comes near the threshold: blocks with no candidate
    E[:, 20_000:90_000] *= 1e-3
    x = rng.standard_normal(N).astype(np.float32)
    for K in (N // 1000, N // 64):
        want = O.step_with_memory(Gt, E, 1.0, K, x, 1e-3)
        got = gpu_step_ec(ctx, Gt, E, 1.0, K, x, 1e-3, fused=True)
        assert_same(got, want, keys=KEYS, what=f"N={N} K={K}")
        assert ctx.last_encode_info() == (M, 0)


@pytest.mark.parametrize("gamma", [0.1, 0.3, 0.7, 1.0])
def test_dense_sparsity_levels_with_memory(ctx, gamma):
    """K/N up to 1 with the memory: the chunked filter pass keeps the words of all candidates and
    records for those between the two sampled bounds; two iterations so that the memory left by the
    first feeds the second."""
    rng = np.random.default_rng(int(gamma * 100))
    M, N = 3, 262_147
    K = min(N, int(round(gamma * N)))
    E = (rng.standard_normal((M, N)) * 0.3).astype(np.float32)
    x = rng.standard_normal(N).astype(np.float32)
    for t in range(2):
        Gt = rng.standard_normal((M, N)).astype(np.float32)
        Gt[:, ::11] = 0.0
        want = O.step_with_memory(Gt, E, 1.0, K, x, 1e-3)
        got = gpu_step_ec(ctx, Gt, E, 1.0, K, x, 1e-3, fused=(t == 0))
        assert_same(got, want, keys=KEYS, what=f"gamma={gamma} iteration {t}")
        E, x = want["err"], want["x"]
    if gamma <= 0.3 or gamma == 1.0:
        assert ctx.last_encode_info() == (M, 0)


@pytest.mark.parametrize("shape", [(3, 10_001, 100), (5, 140_001, 1_400), (3, 262_147, 26_214), (2, 300_000, 150_000),
                                   (2, 131_073, 131_073), (4, 65_537, 0), (4, 500_000, 5_000)],
                         ids=lambda t: f"M{t[0]}-N{t[1]}-K{t[2]}")
@pytest.mark.parametrize("fused", [False, True], ids=["encode", "step"])
def test_memory_already_holding_the_sum(ctx, shape, fused):
    """s3gd_topk_sign_encode_acc / s3gd_step_acc: the caller has formed g = g~ + e in the buffer.  Words,
    counts, the new memory and the parameters are those of the two-tensor call on (g~, e); every
    route of the encode is taken (small rows, single pass at sparse and dense K, K = N, K = 0, fallback rows)."""
    M, N, K = shape
    rng = np.random.default_rng(N + K)
    Gt = rng.standard_normal((M, N)).astype(np.float32)
    E = (rng.standard_normal((M, N)) * 0.4).astype(np.float32)
    if N == 500_000:  # rows the candidate checks reject
        Gt[1] = 2.0
        E[1] = 0.0
        Gt[2] = np.where(rng.random(N) < 0.001, rng.standard_normal(N), 0.0)
        E[2] = 0.0
    x = rng.standard_normal(N).astype(np.float32)
    want = O.step_with_memory(Gt, E, 1.0, K, x, 1e-3)
    acc = torch.from_numpy(O.compensate(Gt, E, 1.0)).cuda()
    words = torch.full((M, K), 0x55555555, dtype=torch.int32, device="cuda")
    counts = torch.full((M,), 0x55555555, dtype=torch.int32, device="cuda")
    xd = torch.from_numpy(x.copy()).cuda()
    if fused:
        ctx.step_acc(acc, K, xd, 1e-3, words, counts)
    else:
        ctx.topk_sign_encode_acc(acc, K, words, counts)
        ctx.vote_update(words, counts, N, xd, 1e-3)
    torch.cuda.synchronize()
    assert ctx.last_async_status() == 0
    got = dict(words=words.cpu().numpy().view(np.uint32), counts=counts.cpu().numpy().view(np.uint32), err=acc.cpu().numpy(),
               x=xd.cpu().numpy())
    assert_same(got, want, keys=("words", "counts", "err", "x"), what=f"{shape}")


def test_unaligned_base_pointers_same_phase(ctx, lib):
    rng = np.random.default_rng(19)
    M, N, K = 3, 150_001, 1_500
    for off in (1, 2, 3):
        fg = rng.standard_normal(M * N + 4).astype(np.float32)
        fe = rng.standard_normal(M * N + 4).astype(np.float32)
        bg, be = torch.from_numpy(fg).cuda(), torch.from_numpy(fe).cuda()
        gt_dev = bg[off:off + M * N].view(M, N)
        e_dev = be[off:off + M * N].view(M, N)
        Gt = fg[off:off + M * N].reshape(M, N)
        E = fe[off:off + M * N].reshape(M, N)
        x = rng.standard_normal(N).astype(np.float32)
        want = O.step_with_memory(np.ascontiguousarray(Gt), np.ascontiguousarray(E), 1.0, K, x, 1e-3)
        got = gpu_step_ec(ctx, Gt, E, 1.0, K, x, 1e-3, fused=True, gt_dev=gt_dev, e_dev=e_dev)
        assert_same(got, want, keys=KEYS, what=f"offset {off}")
        # elements around the views are not touched
        back = be.cpu().numpy()
        assert np.array_equal(back[:off].view(np.uint32), fe[:off].view(np.uint32))
        assert np.array_equal(back[off + M * N:].view(np.uint32), fe[off + M * N:].view(np.uint32))
        # another phase than the gradients is an argument error
        other = be[(off + 1) % 4:(off + 1) % 4 + M * N].view(M, N)
        w = torch.zeros((M, K), dtype=torch.int32, device="cuda")
        c = torch.zeros((M,), dtype=torch.int32, device="cuda")
        with pytest.raises(lib.S3GDError):
            ctx.topk_sign_encode_ec(gt_dev, other, 1.0, K, w, c)


def test_rows_fall_back_independently_with_memory(ctx):
    """Rows whose candidate checks fail are served by the general route reading g from the memory."""
    rng = np.random.default_rng(5)
    N, K = 500_000, 5_000
    Gt = np.empty((4, N), dtype=np.float32)
    Gt[0] = rng.standard_normal(N)
    Gt[1] = -2.0
    Gt[2] = np.where(rng.random(N) < 0.001, rng.standard_normal(N), 0.0)
    Gt[3] = rng.choice([1.0, -1.0, 3.0], N, p=[0.5, 0.495, 0.005])
    E = np.zeros_like(Gt)
    E[0] = rng.standard_normal(N) * 0.1
    E[3] = rng.choice([0.0, 1.0], N)  # g takes the values 1, -1, 3, 2, 0, 4
    x = rng.standard_normal(N).astype(np.float32)
    want = O.step_with_memory(Gt, E, 1.0, K, x, 1e-3)
    got = gpu_step_ec(ctx, Gt, E, 1.0, K, x, 1e-3, fused=True)
    assert_same(got, want, keys=KEYS, what="fallback rows")
    assert ctx.last_encode_info()[1] == 3


def _unsampled_positions(lib, plan, N):
    sampled = np.zeros(N, dtype=bool)
    for u in range(plan["n_units"]):
        p = lib.encode_sample_unit_start(u, plan["unit_stride"])
        sampled[p:p + plan["sample_unit"]] = True
    return sampled


def _memory_case_against_the_sample(lib, make_g, N, K, expect_general, expect_mode=None, formed=False):
    """Row 0 of g = g~ + e is built by `make_g(sampled, plan, rng)` against the positions the sample looks
    at; row 1 is ordinary.  The step with a memory must return the oracle's words, counts, parameters and
    memory (every coordinate: whatever the pass stored as zero and was not sent has to be back)."""
    rng = np.random.default_rng(N % 1000 + K)
    with lib.Context(2, N, K, device=0) as c:
        plan = c.encode_plan_info(2, N, K, with_memory=True)
        assert plan["candidates"] and plan["chunks"] and plan["zero_sure"], plan
        g0 = make_g(_unsampled_positions(lib, plan, N), plan, rng)
        E = np.stack([(rng.standard_normal(N) * 0.25).astype(np.float32), (rng.standard_normal(N) * 0.3).astype(np.float32)])
        E[0] = np.round(E[0] * 64) / 64        # dyadic, so that g~ = g - e and g~ + e = g are both exact in fp32
        g0 = (np.round(g0.astype(np.float64) * 4096) / 4096).astype(np.float32)
        Gt = np.stack([(g0 - E[0]).astype(np.float32), rng.standard_normal(N).astype(np.float32)])
        assert np.array_equal((Gt[0] + E[0]).astype(np.float32), g0)
        x = rng.standard_normal(N).astype(np.float32)
        want = O.step_with_memory(Gt, E, 1.0, K, x, 1e-3)
        if formed:  # the buffer already holds g~ + e (s3gd_step_acc): from K = N/32 on the pass rewrites it
            acc = torch.from_numpy(O.compensate(Gt, E, 1.0)).cuda()
            words = torch.full((2, K), 0x55555555, dtype=torch.int32, device="cuda")
            counts = torch.full((2,), 0x55555555, dtype=torch.int32, device="cuda")
            xd = torch.from_numpy(x.copy()).cuda()
            c.step_acc(acc, K, xd, 1e-3, words, counts)
            torch.cuda.synchronize()
            assert c.last_async_status() == 0
            got = dict(words=words.cpu().numpy().view(np.uint32), counts=counts.cpu().numpy().view(np.uint32),
                       err=acc.cpu().numpy(), x=xd.cpu().numpy())
        else:
            got = gpu_step_ec(c, Gt, E, 1.0, K, x, 1e-3, fused=True, dense_outputs=False)
        assert_same(got, want, keys=("words", "counts", "err", "x"), what="memory, row built against the sample")
        assert c.last_encode_details()[:2] == (2, expect_general)
        if expect_mode is not None:
            assert c.last_row_state(0)["mode"] == expect_mode, c.last_row_state(0)
    return got


def test_zeroed_entries_come_back_when_the_pool_runs_out(lib):
    """Nearly every entry outside the sampled units is large: both sampled bounds lie among the small
    entries, so the pass with a memory takes the large ones for sure and stores zeros over them, chunk after
    chunk, until the row's pool runs out.  The row is handed to the general route, which must find g
    whole: the zeroed entries are written back from the bits kept beside their words."""
    N, K = 1 << 22, (1 << 22) // 250

    def make_g(sampled, plan, rng):
        g = ((50.0 + rng.random(N) * 50.0) * np.sign(rng.standard_normal(N))).astype(np.float32)
        small = (rng.standard_normal(N) * 0.01).astype(np.float32)
        g[sampled] = small[sampled]
        assert N - int(sampled.sum()) > plan["cand_stride"]
        return g
    _memory_case_against_the_sample(lib, make_g, N, K, expect_general=1)


def _hidden_top_row(N, n_top, sampled, rng, n_mid=1500):
    """0.001 everywhere; n_mid entries of 0.5, all at sampled positions (both sampled bounds land on them); n_top
    large entries, none at a sampled position."""
    g = np.full(N, 0.001, dtype=np.float32)
    g[rng.choice(np.nonzero(sampled)[0], size=n_mid, replace=False)] = 0.5
    top = rng.choice(np.nonzero(~sampled)[0], size=n_top, replace=False)
    g[top] = ((100.0 + rng.random(n_top) * 20.0) * np.sign(rng.standard_normal(n_top))).astype(np.float32)
    return g


def test_zeroed_entries_come_back_when_too_many_were_taken_for_sure(lib):
    """K + 2000 large entries that the sample does not see: the pass takes them all for sure (more than K,
    all stored as zeros), everything fits the pool, and the verdict after the pass sends the row to the
    general route."""
    N, K = 1 << 22, 1 << 14

    def make_g(sampled, plan, rng):
        assert plan["sample_rank"] < 1500 and K + 2000 + 1500 + 2048 < plan["cand_stride"], plan
        return _hidden_top_row(N, K + 2000, sampled, rng)
    _memory_case_against_the_sample(lib, make_g, N, K, expect_general=1)


@pytest.mark.parametrize("n_extra", [0, 2000], ids=["exactly_K_for_sure", "too_many_for_sure"])
def test_rewritten_buffer_against_the_sample(lib, n_extra):
    """The same two rows through s3gd_step_acc at K = N/32, where the pass reads the one buffer and rewrites it
    with the zeros: with exactly K hidden entries nothing is left for the emit pass to zero; with 2000 more
    the row ends on the general route and every zero the pass stored is taken back."""
    N, K = 1 << 22, 1 << 17

    def make_g(sampled, plan, rng):
        n_mid = plan["sample_rank"] + 800
        assert K + n_extra + n_mid + 2048 < plan["cand_stride"], plan
        return _hidden_top_row(N, K + n_extra, sampled, rng, n_mid=n_mid)
    _memory_case_against_the_sample(lib, make_g, N, K, expect_general=1 if n_extra else 0, expect_mode=0 if n_extra else 3, formed=True)


def test_every_sent_entry_zeroed_by_the_pass_itself(lib):
    """Exactly K large entries that the sample does not see: the pass takes exactly K for sure, the whole
    bracket loses, and the emit pass has no zero left to write (threshold known after the pass: mode 3)."""
    N, K = 1 << 22, 1 << 14

    def make_g(sampled, plan, rng):
        assert plan["sample_rank"] < 1500 and K + 1500 + 2048 < plan["cand_stride"], plan
        return _hidden_top_row(N, K, sampled, rng)
    got = _memory_case_against_the_sample(lib, make_g, N, K, expect_general=0, expect_mode=3)
    assert int((got["err"][0] == 0).sum()) == K


def test_special_values(ctx):
    """Denormals stay denormal in g~ + eta * e; -0.0 and +0.0; infinities are selected and replaced
    by +0.0 in the memory; selected zeros keep their bits."""
    rng = np.random.default_rng(3)
    N = 9000
    tiny = np.float32(1e-45)
    Gt = np.stack([
        rng.integers(-50, 50, N).astype(np.float32) * tiny,
        np.where(rng.random(N) < 0.01, rng.standard_normal(N), rng.choice([0.0, -0.0], N)).astype(np.float32),
        np.where(rng.random(N) < 0.002, np.inf, rng.standard_normal(N)).astype(np.float32) * rng.choice([1, -1], N).astype(np.float32),
        (rng.standard_normal(N) * 10.0 ** rng.integers(-30, 30, N)).astype(np.float32),
    ])
    E = np.stack([
        rng.integers(-50, 50, N).astype(np.float32) * tiny,
        rng.choice([0.0, -0.0], N).astype(np.float32),
        rng.standard_normal(N).astype(np.float32),
        (rng.standard_normal(N) * 10.0 ** rng.integers(-30, 30, N)).astype(np.float32),
    ])
    x = rng.standard_normal(N).astype(np.float32)
    for eta in (1.0, 0.3):
        for K in (1, 64, 100, 4500, N):
            want = O.step_with_memory(Gt, E, eta, K, x, 0.25)
            got = gpu_step_ec(ctx, Gt, E, eta, K, x, 0.25, fused=(K % 2 == 0))
            assert_same(got, want, keys=KEYS, what=f"eta={eta} K={K}")


def test_nan_from_inf_minus_inf_is_reported(ctx, lib):
    Gt = np.ones((2, 200_000), dtype=np.float32)
    E = np.zeros_like(Gt)
    Gt[1, 123_456] = np.inf
    E[1, 123_456] = -np.inf
    g, e = torch.from_numpy(Gt).cuda(), torch.from_numpy(E).cuda()
    ctx.topk_sign_encode_ec(g, e, 1.0, 100)
    assert ctx.last_async_status() == lib.E_NAN


def test_argument_errors(ctx, lib):
    dev = torch.device("cuda:0")
    g = torch.zeros((2, 100), dtype=torch.float32, device=dev)
    e = torch.zeros((2, 100), dtype=torch.float32, device=dev)
    w = torch.zeros((2, 10), dtype=torch.int32, device=dev)
    c = torch.zeros((2,), dtype=torch.int32, device=dev)
    x = torch.zeros((100,), dtype=torch.float32, device=dev)
    r, h = lib.raw, ctx._h
    p = lambda z: ctypes.c_void_p(z.data_ptr())
    assert r.s3gd_topk_sign_encode_ec(h, p(g), None, 1.0, 2, 100, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_topk_sign_encode_ec(h, None, p(e), 1.0, 2, 100, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_topk_sign_encode_ec(h, p(g), p(e), -0.5, 2, 100, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_topk_sign_encode_ec(h, p(g), p(e), float("nan"), 2, 100, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_topk_sign_encode_ec(h, p(g), p(e), float("inf"), 2, 100, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_topk_sign_encode_ec(h, p(g), p(g), 1.0, 2, 100, 10, p(w), p(c), None) == lib.E_INVAL  # overlap
    assert r.s3gd_topk_sign_encode_ec(h, p(g), ctypes.c_void_p(e.data_ptr() + 4), 1.0, 2, 90, 10, p(w), p(c), None) == lib.E_INVAL
    assert r.s3gd_step_ec(h, p(g), p(e), 1.0, 2, 100, 10, None, 0.1, p(w), p(c), None, None, None) == lib.E_INVAL
    assert r.s3gd_step_ec(h, p(g), p(e), 1.0, 2, 100, 101, p(x), 0.1, p(w), p(c), None, None, None) == lib.E_INVAL
    torch.cuda.synchronize()
    assert int(w.abs().sum()) == 0 and int(c.abs().sum()) == 0 and float(e.abs().sum()) == 0.0
