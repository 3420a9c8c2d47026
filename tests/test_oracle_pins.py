"""Pins for the CPU oracle: things the paper and the mathematics fix, none of them
computed by the HIP path.  Each test names the mistake it is there to catch."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import s3gd_oracle as O
from paper_2302_07475_amd import datagen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kv(path):
    out = {}
    with open(os.path.join(GOLDEN, path)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                out[k] = float(v)
    return out


# ---------------------------------------------------------------- paper-printed example
def test_example1_paper_values():
    """Section 2.3, Example 1.  Catches: a flipped sign bit, a vote that sums values
    instead of signs, a selection that ignores magnitude."""
    ex = _kv("example1.txt")
    col = np.array([ex["g_1"], ex["g_2"], ex["g_3"]], dtype=np.float32)
    assert np.sign(col.mean()) == ex["sign_of_mean"]
    # coordinate 0 carries the example; coordinate 1 gives the two unsure workers a
    # larger entry elsewhere, so that K=1 makes exactly the confident worker vote on 0.
    G = np.stack([col, np.array([0.5, 5.0, 5.0], dtype=np.float32)], axis=1)
    x = np.zeros(2, dtype=np.float32)
    dense = O.step(G, 2, x, 1e-3)  # K = N: every worker sends every sign (signSGD-MV)
    assert dense["tally"][0] == -1 and dense["votes"][0] == ex["signsgd_vote"]
    sparse = O.step(G, 1, x, 1e-3)
    assert (np.abs(col) > ex["confidence"]).tolist() == [True, False, False]
    assert sparse["tally"].tolist() == [1, 2]
    assert sparse["votes"][0] == ex["sparse_vote"]
    # the update moves against the vote (eq. "s3gd")
    assert sparse["x"][0] < 0 and dense["x"][0] > 0


# ---------------------------------------------------------------- reductions to textbook routines
@pytest.mark.parametrize("M", [1, 2, 3, 4, 7])
def test_k_equals_n_is_signsgd_mv(M):
    """gamma = 1 (Section 3, special cases of Theorem 1): vote = sign(sum_m sign(g_m)).
    Catches: dropped workers, sign convention, tie handling for even M."""
    rng = np.random.default_rng(M)
    N = 257
    G = rng.standard_normal((M, N)).astype(np.float32)
    G[:, 5] = 0.0
    G[0, 7] = -0.0
    x = rng.standard_normal(N).astype(np.float32)
    r = O.step(G, N, x, 1e-3)
    want_tally = np.sign(G).astype(np.int32).sum(axis=0)
    assert np.array_equal(r["tally"], want_tally)
    assert np.array_equal(r["votes"], np.sign(want_tally).astype(np.int8))
    assert np.array_equal(r["counts"], (G != 0).sum(axis=1).astype(np.uint32))


def test_single_worker_is_sparse_signsgd():
    """M = 1 (Section 3, special case M = 1): vote = TopKSign(g_1).  Library cross-check of
    the index set on tie-free data with torch.topk and numpy.argpartition."""
    rng = np.random.default_rng(11)
    N, K = 5000, 137
    g = rng.standard_normal(N).astype(np.float32)
    mag = np.abs(g)
    srt = np.sort(mag)[::-1]
    assert srt[K - 1] > srt[K], "test needs distinct K-th and (K+1)-th magnitudes"
    x = rng.standard_normal(N).astype(np.float32)
    r = O.step(g[None, :], K, x, 0.25)
    S_torch = np.sort(torch.topk(torch.from_numpy(mag), K).indices.numpy())
    S_part = np.sort(np.argpartition(-mag, K)[:K])
    S = (r["words"][0] >> 1).astype(np.int64)
    assert np.array_equal(S, S_torch) and np.array_equal(S, S_part)
    mask = np.zeros(N, dtype=np.int8)
    mask[S_torch] = 1
    assert np.array_equal(r["votes"], np.sign(g).astype(np.int8) * mask)
    assert np.array_equal(r["x"], (x - np.float32(0.25) * r["votes"].astype(np.float32)).astype(np.float32))
    # sign bit of each word
    assert np.array_equal(r["words"][0] & 1, (g[S] < 0).astype(np.uint32))


# ---------------------------------------------------------------- brute force on tiny inputs
def _tiny_cases():
    rng = np.random.default_rng(3)
    cases = []
    cases.append(("all_equal", np.full(9, 2.5, dtype=np.float32)))
    cases.append(("all_equal_mixed_sign", np.array([1, -1, 1, -1, -1, 1, 1], dtype=np.float32)))
    cases.append(("all_zero", np.zeros(8, dtype=np.float32)))
    cases.append(("pm_zero", np.array([0.0, -0.0, 3.0, -0.0, 0.0, -3.0], dtype=np.float32)))
    cases.append(("two_valued", np.array([1, 2, 1, 2, 2, 1, 1, 2, 1, 1], dtype=np.float32)))
    cases.append(("two_valued_neg", np.array([-1, 2, 1, -2, 2, -1, 1, -2, 1, 1], dtype=np.float32)))
    cases.append(("inf", np.array([np.inf, 1, -np.inf, 3, -2, np.inf], dtype=np.float32)))
    den = np.array([1e-45, -3e-45, 0, 1e-39, -1e-39, 1.1754944e-38, 2e-45], dtype=np.float32)
    cases.append(("denormal", den))
    cases.append(("quantised", (np.rint(rng.standard_normal(40) * 4) / 4).astype(np.float32)))
    cases.append(("random", rng.standard_normal(33).astype(np.float32)))
    return cases


@pytest.mark.parametrize("name,g", _tiny_cases(), ids=[c[0] for c in _tiny_cases()])
def test_sort_equals_rank_definition(name, g):
    """Catches: wrong tie direction, ascending instead of descending sort, signed instead of
    absolute value, off-by-one at K, mishandled zeros."""
    N = g.shape[0]
    for K in range(N + 1):
        S = O.topk_index_set(g, K)
        B = O.topk_index_set_brute_force(g, K)
        assert np.array_equal(S, B), (name, K)
        assert len(S) == K
        for n in S[:3]:
            assert O.rank_of(g, int(n)) < K
        words, count = O.encode_row(g, K)
        sel_nonzero = [int(n) for n in B if g[n] != 0]
        assert count == len(sel_nonzero)
        assert (words[:count] >> 1).tolist() == sel_nonzero
        assert (words[:count] & 1).tolist() == [int(g[n] < 0) for n in sel_nonzero]
        assert (words[count:] == 0xFFFFFFFF).all()
        dense = O.topk_sign_dense(g, K)
        assert int(np.count_nonzero(dense)) == count


def test_all_equal_selects_lowest_indices():
    g = np.full(12, -4.0, dtype=np.float32)
    assert O.topk_index_set(g, 5).tolist() == [0, 1, 2, 3, 4]
    w, c = O.encode_row(g, 5)
    assert c == 5 and w.tolist() == [1, 3, 5, 7, 9]


def test_hand_worked_ties_and_votes():
    """A case small enough to do by hand.  M = 4 (even), N = 6, K = 2.
    rows:        n=0   1    2    3    4    5
      w0:         5   -5    1    0    0    2     -> {0,1}   (+,-)
      w1:        -5    1    5    1    1    1     -> {0,2}   (-,+)
      w2:         1    1   -7    7    0    0     -> {2,3}   (-,+)
      w3:         0    0    0    0    0    9     -> {0,5}: 0 selected by index order, no vote
    tally: n0 = +1-1 = 0, n1 = -1, n2 = +1-1 = 0, n3 = +1, n4 = 0, n5 = +1"""
    G = np.array([[5, -5, 1, 0, 0, 2], [-5, 1, 5, 1, 1, 1], [1, 1, -7, 7, 0, 0], [0, 0, 0, 0, 0, 9]],
                 dtype=np.float32)
    x = np.arange(6, dtype=np.float32)
    r = O.step(G, 2, x, 0.5)
    assert r["counts"].tolist() == [2, 2, 2, 1]
    assert r["words"][0].tolist() == [0, 3]
    assert r["words"][1].tolist() == [1, 4]
    assert r["words"][2].tolist() == [5, 6]
    assert r["words"][3].tolist() == [10, 0xFFFFFFFF]
    assert r["tally"].tolist() == [0, -1, 0, 1, 0, 1]
    assert r["votes"].tolist() == [0, -1, 0, 1, 0, 1]
    assert r["x"].tolist() == [0.0, 1.5, 2.0, 2.5, 4.0, 4.5]


# ---------------------------------------------------------------- two routes, one result
@pytest.mark.parametrize("M,N,K", [(1, 50, 7), (2, 64, 64), (3, 100, 0), (4, 333, 33), (5, 1000, 999)])
def test_message_route_equals_dense_definition(M, N, K):
    """eq. "s3gd" on dense ternary vectors vs the word/count message route.
    Catches: index packing, sign bit, padding read as data, count mistakes."""
    rng = np.random.default_rng(M * 1000 + N)
    G = (np.rint(rng.standard_normal((M, N)) * 3) / 3).astype(np.float32)  # many ties and zeros
    x = rng.standard_normal(N).astype(np.float32)
    a = O.step(G, K, x, 1e-3)
    b = O.step_dense(G, K, x, 1e-3)
    for k in ("tally", "votes", "x"):
        assert np.array_equal(a[k], b[k]), k
    t2, v2 = O.majority_vote_loops(a["words"], a["counts"], N)
    assert np.array_equal(t2, a["tally"]) and np.array_equal(v2, a["votes"])


# ---------------------------------------------------------------- invariants of the method
def check_invariants(G, K, r, x_before, lr):
    """Properties that hold for any input (Sections 2.1, 2.2).  Reused on GPU outputs."""
    M, N = G.shape
    mag = np.abs(G)
    voters = np.zeros(N, dtype=np.int64)
    for m in range(M):
        c = int(r["counts"][m])
        w = r["words"][m]
        idx = (w[:c] >> 1).astype(np.int64)
        assert (w[c:] == 0xFFFFFFFF).all()
        assert (np.diff(idx) > 0).all() and (idx < N).all()
        assert np.array_equal(w[:c] & 1, (G[m, idx] < 0).astype(np.uint32))
        assert c <= K
        nz = int(np.count_nonzero(G[m]))
        assert c == min(K, nz)  # counts = K minus the selected zeros
        if c:
            lo = mag[m, idx].min()
            rest = np.ones(N, dtype=bool)
            rest[idx] = False
            if c == K and rest.any():
                assert lo >= mag[m, rest].max()
                tied_out = np.nonzero(rest & (mag[m] == lo))[0]
                tied_in = idx[mag[m, idx] == lo]
                if tied_out.size:
                    assert tied_in.max() < tied_out.min()
        voters[idx] += 1
    t = r["tally"].astype(np.int64)
    assert (np.abs(t) <= voters).all() and ((t - voters) % 2 == 0).all()
    assert voters.sum() == int(r["counts"].astype(np.int64).sum())
    assert (r["votes"][voters == 0] == 0).all()
    assert np.array_equal(r["votes"], np.sign(t).astype(np.int8))
    changed = r["x"] != x_before
    assert changed.sum() <= np.count_nonzero(r["votes"]) <= min(N, M * K)
    lr = np.float32(lr)
    assert np.array_equal(r["x"][r["votes"] == 0].view(np.uint32), x_before[r["votes"] == 0].view(np.uint32))
    assert np.array_equal(r["x"][r["votes"] > 0], (x_before[r["votes"] > 0] - lr).astype(np.float32))
    assert np.array_equal(r["x"][r["votes"] < 0], (x_before[r["votes"] < 0] + lr).astype(np.float32))


@pytest.mark.parametrize("cfg", [datagen.C1,
                                 datagen.C2.scaled(M=4, N=60_000, K=600),
                                 datagen.C3.scaled(M=5, N=50_000, K=50, steps=1),
                                 datagen.C4.scaled(M=3, N=40_000, K=400),
                                 datagen.C5.scaled(M=4, N=70_000, K=70)], ids=lambda c: c.name)
def test_invariants_on_config_recipes(cfg):
    G = datagen.gradients(cfg, threads=2)
    x = datagen.params(cfg, threads=1)
    r = O.step(G, cfg.K, x, datagen.lr32(cfg))
    check_invariants(G, cfg.K, r, x, datagen.lr32(cfg))


# ---------------------------------------------------------------- closed-form statistics
def test_voter_count_is_binomial_on_iid_input():
    """Lemma 3 and Example 2: with selections uniform over coordinates, the number of
    voters per coordinate is Binomial(M, K/N); the empty fraction is (1 - K/N)^M.
    Catches: workers sharing one index set, K applied to the wrong axis."""
    cfg = datagen.C1
    G = datagen.gradients(cfg, threads=1)
    words, counts = O.topk_sign_encode(G, cfg.K)
    voters = np.zeros(cfg.N, dtype=np.int64)
    for m in range(cfg.M):
        voters[(words[m, : counts[m]] >> 1).astype(np.int64)] += 1
    gam = cfg.K / cfg.N
    empty = np.mean(voters == 0)
    assert abs(empty - (1 - gam) ** cfg.M) < 1e-3  # 0.9703; exact count fixes it to ~3e-4
    for u in range(cfg.M + 1):
        p = math.comb(cfg.M, u) * gam**u * (1 - gam) ** (cfg.M - u)
        sd = math.sqrt(p * (1 - p) / cfg.N)
        assert abs(np.mean(voters == u) - p) < 6 * sd + 2e-4, u


# ---------------------------------------------------------------- update arithmetic
def test_update_is_one_fp32_rounding():
    """eq. "s3gd" in fp32.  The exact real result x -/+ lr, rounded once to fp32, computed here
    through float64 (53 bits hold the exact sum of two fp32 numbers of these ranges)."""
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(1000) * 0.01, [0.0, -0.0, 1e-3, -1e-3, 1e30, 1e-40]]).astype(np.float32)
    votes = rng.integers(-1, 2, size=x.shape[0]).astype(np.int8)
    lr = np.float32(1e-3)
    assert lr.view(np.uint32) == 0x3A83126F
    got = O.apply_update(x, votes, lr)
    want = (x.astype(np.float64) - float(lr) * votes.astype(np.float64)).astype(np.float32)
    assert np.array_equal(got, want)
    keep = votes == 0
    assert np.array_equal(got[keep].view(np.uint32), x[keep].view(np.uint32))  # -0.0 survives


def test_nan_is_rejected_and_k_range():
    g = np.array([1, np.nan, 2], dtype=np.float32)
    with pytest.raises(ValueError):
        O.topk_index_set(g, 1)
    with pytest.raises(ValueError):
        O.topk_index_set(np.ones(3, dtype=np.float32), 4)
    assert O.topk_index_set(np.ones(3, dtype=np.float32), 0).size == 0


# ---------------------------------------------------------------- planted mistakes are caught
def test_planted_mistakes_fail_a_pin(monkeypatch):
    """Each plausible slip, planted in the oracle on the CPU, must break at least one pin."""
    g_tie = np.array([1, 2, 1, 2, 2, 1, 1, 2, 1, 1], dtype=np.float32)

    # (a) ties broken towards the highest index
    def bad_ties(g, K):
        order = np.lexsort((-np.arange(g.shape[0]), -np.abs(g)))
        return np.sort(order[:K])
    assert not np.array_equal(bad_ties(g_tie, 2), O.topk_index_set_brute_force(g_tie, 2))

    # (b) signed value instead of magnitude
    def bad_abs(g, K):
        return np.sort(np.lexsort((np.arange(g.shape[0]), -g))[:K])
    g = np.array([1, -5, 2], dtype=np.float32)
    assert not np.array_equal(bad_abs(g, 1), O.topk_index_set_brute_force(g, 1))

    # (c) sign bit inverted: Example 1 flips
    monkeypatch.setattr(O, "sgn", lambda u: -((np.asarray(u) > 0).astype(np.int8) - (np.asarray(u) < 0).astype(np.int8)))
    with pytest.raises(AssertionError):
        test_example1_paper_values()
    monkeypatch.undo()

    # (d) vote sums values instead of signs: Example 1 (K = N) would give +1
    col = np.array([3, -0.3, -0.03], dtype=np.float32)
    assert np.sign(col.sum()) == 1 and O.step(col[:, None], 1, np.zeros(1, np.float32), 1.0)["votes"][0] == -1

    # (e) update with the wrong sign
    r = O.step(np.array([[2.0]], dtype=np.float32), 1, np.array([1.0], dtype=np.float32), 0.5)
    assert r["x"][0] == 0.5


# ---------------------------------------------------------------- the any-size checker is itself pinned
def test_row_checker_accepts_the_sorted_answer_and_rejects_neighbours():
    """check_message_row is what full-size GPU tests rely on, so it is pinned against the sort
    on small inputs: it accepts the oracle's message and rejects every single-word perturbation."""
    rng = np.random.default_rng(12)
    for name, g in _tiny_cases() + [("grid", (np.rint(rng.standard_normal(300) * 4) / 4).astype(np.float32))]:
        N = g.shape[0]
        for K in sorted({0, 1, 2, N // 3, N // 2, N - 1, N}):
            words, count = O.encode_row(g, K)
            O.check_message_row(g, K, words, count)  # accepts
            sel = set((words[:count] >> 1).tolist())
            others = [n for n in range(N) if n not in sel and g[n] != 0]
            if count and others:
                # swap one selected index for an unselected one: must be rejected
                for victim in (0, count - 1):
                    bad = words.copy()
                    keep = [int(w) >> 1 for w in bad[:count]]
                    keep[victim] = others[0]
                    keep = sorted(set(keep))
                    if len(keep) != count:
                        continue
                    bad[:count] = np.array([(n << 1) | int(g[n] < 0) for n in keep], dtype=np.uint32)
                    with pytest.raises(AssertionError):
                        O.check_message_row(g, K, bad, count)
            if count:
                bad = words.copy()
                bad[0] ^= 1  # wrong sign
                with pytest.raises(AssertionError):
                    O.check_message_row(g, K, bad, count)
                bad = words.copy()
                bad[count - 1] = 0xFFFFFFFF  # dropped word
                with pytest.raises(AssertionError):
                    O.check_message_row(g, K, bad, count - 1)


# ---------------------------------------------------------------- error-compensation memory
def test_memory_hand_worked_three_iterations():
    """Algorithm 1 with eta = 1, K = 1, one worker, constant gradient (3, 2, 1): the unselected
    components pile up in the memory until they win the selection.
      t0: g=(3,2,1) -> sel 0, e=(0,2,1)
      t1: g=(3,4,2) -> sel 1, e=(3,0,2)
      t2: g=(6,2,3) -> sel 0, e=(0,2,3)
      t3: g=(3,4,4) -> tie at 4: lowest index 1 wins, e=(3,0,4)
      t4: g=(6,2,5) -> sel 0, e=(0,2,5)
      t5: g=(3,4,6) -> sel 2, e=(3,4,0)"""
    gt = np.array([[3.0, 2.0, 1.0]], dtype=np.float32)
    e = np.zeros_like(gt)
    x = np.zeros(3, dtype=np.float32)
    picks, errs = [], []
    for _ in range(6):
        r = O.step_with_memory(gt, e, 1.0, 1, x, 1.0)
        picks.append(int(r["words"][0, 0] >> 1))
        errs.append(r["err"][0].tolist())
        e, x = r["err"], r["x"]
    assert picks == [0, 1, 0, 1, 0, 2]
    assert errs == [[0, 2, 1], [3, 0, 2], [0, 2, 3], [3, 0, 4], [0, 2, 5], [3, 4, 0]]
    assert x.tolist() == [-3.0, -2.0, -1.0]  # every vote was +1: x moved by -lr each time it was selected


def test_compensate_rounds_the_product_then_the_sum():
    """tests/golden/compensate_rounding_example.txt: hand-worked (g~, e, eta) where a rounded product
    followed by a rounded sum and a fused multiply-add differ in the last bit (eq. "gradupdate",
    evaluated in fp32 as written).  The fused value is reproduced here in exact rational arithmetic
    and must differ, so that an oracle that fuses the two operations fails."""
    import os
    from fractions import Fraction
    cases = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "compensate_rounding_example.txt")) as f:
        for line in f:
            tok = line.split()
            if tok and tok[0] == "case":
                cases.append([int(v, 16) for v in tok[1:]])
    assert len(cases) == 3
    for eta_b, g_b, e_b, want, fused in cases:
        eta = np.array([eta_b], dtype=np.uint32).view(np.float32)[0]
        g = np.array([[g_b]], dtype=np.uint32).view(np.float32)
        e = np.array([[e_b]], dtype=np.uint32).view(np.float32)
        got = O.compensate(g, e, eta).view(np.uint32)[0, 0]
        assert got == want, (hex(got), hex(want))
        assert want != fused
        # one rounding of the exact value lands on the other bits: the two readings really differ here
        exact = Fraction(float(g[0, 0])) + Fraction(float(eta)) * Fraction(float(e[0, 0]))
        f_fused = Fraction(float(np.array([fused], np.uint32).view(np.float32)[0]))
        f_want = Fraction(float(np.array([want], np.uint32).view(np.float32)[0]))
        assert abs(exact - f_fused) <= abs(exact - f_want)


@pytest.mark.parametrize("eta", [0.0, 1.0, 0.5])
def test_memory_identities(eta):
    """(a) eta = 0 is the memoryless step; (b) g = e' + TopK(g) exactly (nothing is lost or counted
    twice); (c) e' vanishes exactly on the support of the message; (d) with eta = 1 the running
    sum of gradients equals memory + everything ever selected."""
    rng = np.random.default_rng(8)
    M, N, K = 3, 400, 17
    x = rng.standard_normal(N).astype(np.float32)
    E = (rng.standard_normal((M, N)) * 0.5).astype(np.float32)
    Gt = rng.standard_normal((M, N)).astype(np.float32)
    r = O.step_with_memory(Gt, E, eta, K, x, 1e-3)
    if eta == 0.0:
        plain = O.step(Gt, K, x, 1e-3)
        for k in ("words", "counts", "tally", "votes", "x"):
            assert np.array_equal(r[k], plain[k])
    G = r["g"]
    assert np.array_equal(G, (Gt + np.float32(eta) * E).astype(np.float32))
    topk_vec = np.zeros_like(G)
    for m in range(M):
        idx = (r["words"][m, : r["counts"][m]] >> 1).astype(np.int64)
        topk_vec[m, idx] = G[m, idx]
        assert (r["err"][m, idx] == 0).all()
        rest = np.ones(N, dtype=bool)
        rest[idx] = False
        assert np.array_equal(r["err"][m, rest].view(np.uint32), G[m, rest].view(np.uint32))
    assert np.array_equal(r["err"] + topk_vec, G)
    if eta == 1.0:  # integers keep fp32 exact: sum of gradients == memory + sum of selected values
        Gi = rng.integers(-8, 9, size=(1, 50)).astype(np.float32)
        e = np.zeros_like(Gi)
        sent = np.zeros_like(Gi)
        for t in range(12):
            rr = O.step_with_memory(Gi, e, 1.0, 5, np.zeros(50, np.float32), 1.0)
            idx = (rr["words"][0, : rr["counts"][0]] >> 1).astype(np.int64)
            sent[0, idx] += rr["g"][0, idx]
            e = rr["err"]
            assert np.array_equal(e + sent, Gi * (t + 1))


def test_memory_selected_zero_and_negative_zero_keep_their_bits():
    g = np.array([[0.0, -0.0, 5.0, -0.0]], dtype=np.float32)
    words, counts = O.topk_sign_encode(g, 3)  # the 5 and, by index order, the first two zeros
    assert counts[0] == 1  # only the 5 sends a sign
    e = O.residual(g, words, counts)
    assert e[0].view(np.uint32).tolist() == [0, 0x80000000, 0, 0x80000000]
    # compensation itself follows IEEE: -0.0 + eta * (+0.0) is +0.0
    assert O.compensate(g, np.zeros_like(g), 1.0)[0].view(np.uint32).tolist() == [0, 0, 0x40A00000, 0]


# ---------------------------------------------------------------- momentum form of the update
def test_momentum_hand_worked_geometric_series():
    """mu = 1/2, delta = 1/4, a coordinate voted +1 at every iteration, one voted -1 once, one never:
    v = 1, 3/2, 7/4, 15/8 (partial sums of the geometric series), x = -(1/4) * running sum of v.
    All values are dyadic, so fp32 is exact and the expected numbers are written out by hand."""
    x = np.zeros(3, dtype=np.float32)
    v = np.zeros(3, dtype=np.float32)
    seen_v, seen_x = [], []
    for t in range(4):
        votes = np.array([1, -1 if t == 0 else 0, 0], dtype=np.int8)
        x, v = O.momentum_update(x, v, votes, 0.25, 0.5)
        seen_v.append(v.tolist())
        seen_x.append(x.tolist())
    assert seen_v == [[1.0, -1.0, 0.0], [1.5, -0.5, 0.0], [1.75, -0.25, 0.0], [1.875, -0.125, 0.0]]
    assert seen_x == [[-0.25, 0.25, 0.0], [-0.625, 0.375, 0.0], [-1.0625, 0.4375, 0.0], [-1.53125, 0.46875, 0.0]]


def test_momentum_zero_is_the_plain_update_and_fp64_agrees():
    rng = np.random.default_rng(12)
    M, N, K = 4, 500, 40
    G = rng.standard_normal((M, N)).astype(np.float32)
    x = rng.standard_normal(N).astype(np.float32)
    x[3] = -0.0
    v_prev = rng.standard_normal(N).astype(np.float32)  # must be forgotten when mu = 0
    plain = O.step(G, K, x, 1e-3)
    mom = O.step_with_momentum(G, K, x, v_prev, 1e-3, 0.0)
    assert np.array_equal(mom["x"].view(np.uint32), plain["x"].view(np.uint32))
    assert np.array_equal(mom["v"], plain["votes"].astype(np.float32))
    # against the real-valued formula in fp64: roundings of 2^-24 relative to the operands (the sum may cancel)
    mu, lr = 0.9, np.float32(1e-3)
    r = O.step_with_momentum(G, K, x, v_prev, lr, mu)
    v64 = float(np.float32(mu)) * v_prev.astype(np.float64) + r["votes"]
    x64 = x.astype(np.float64) - float(lr) * v64
    assert np.allclose(r["v"], v64, rtol=0, atol=2 ** -22 * (np.abs(v_prev).max() + 1))
    assert np.allclose(r["x"], x64, rtol=0, atol=2 ** -22 * (np.abs(x64).max() + 1))
    # a planted mistake (momentum added after the step instead of before) fails the series pin
    xb, vb = np.zeros(1, np.float32), np.zeros(1, np.float32)
    for _ in range(2):
        xb = xb - np.float32(0.25) * vb  # wrong: uses v^{t-1}
        vb = np.float32(0.5) * vb + np.float32(1)
    assert xb.tolist() != [-0.625]
