"""Pins of the RandKSign oracle (oracle/s3gd_randk.py).  The paper fixes no sampling law; what it
does fix, and what is checked here: exactly K distinct coordinates per worker, every coordinate
selected with probability K/N independently across workers (Assumption 4; then the number of
voters of a coordinate is Binomial(M, K/N), Lemma 3), K = N is signSGD with majority vote, and
the message / vote / update semantics of Algorithm 1 otherwise."""
import numpy as np
import pytest
from scipy import stats

from oracle import s3gd_oracle as O
from oracle import s3gd_randk as R

SEED = 0x1234_5678_9ABC_DEF0


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 16, 17, 255, 256, 257, 1000, 4097, 65_536, 100_003])
def test_permutation_is_a_bijection(N):
    for t, m in [(0, 0), (3, 1), (7, 15)]:
        keys = R.round_keys(SEED, t, m)
        out = R.permute_many(np.arange(N), N, keys)
        assert np.array_equal(np.sort(out), np.arange(N))
        for i in list(range(min(N, 20))) + [N - 1]:
            assert R.permute(i, N, keys) == out[i]  # scalar definition == vectorised form


def test_network_is_a_bijection_of_its_whole_domain():
    keys = R.round_keys(SEED, 1, 2)
    h = R.half_bits(1000)
    D = 4 ** h
    img = {R.feistel(v, h, keys) for v in range(D)}
    assert img == set(range(D))


def test_index_sets_exact_size_distinct_sorted_and_keyed():
    N, K = 50_000, 777
    a = R.randk_index_set(N, K, SEED, 0, 0)
    assert a.shape == (K,) and (np.diff(a) > 0).all() and a[0] >= 0 and a[-1] < N
    assert np.array_equal(a, R.randk_index_set(N, K, SEED, 0, 0))             # a pure function of the key
    for other in (R.randk_index_set(N, K, SEED, 1, 0), R.randk_index_set(N, K, SEED, 0, 1),
                  R.randk_index_set(N, K, SEED + 1, 0, 0), R.randk_index_set(N, K, SEED + (1 << 40), 0, 0)):
        assert len(np.intersect1d(a, other)) < 60                             # ~K^2/N = 12 expected by chance
    assert R.randk_index_set(N, 0, SEED, 0, 0).shape == (0,)
    assert np.array_equal(R.randk_index_set(300, 300, SEED, 5, 5), np.arange(300))
    # nested in K: the first K' outputs of the permutation
    assert set(R.randk_index_set(N, 100, SEED, 0, 0)) <= set(a)


def test_every_coordinate_is_selected_with_probability_k_over_n():
    """Assumption 4: inclusion frequency over many (iteration, worker) keys, chi-square against K/N."""
    N, K, trials = 200, 20, 4000
    hits = np.zeros(N)
    for i in range(trials):
        hits[R.randk_index_set(N, K, SEED, i // 8, i % 8)] += 1
    expect = trials * K / N
    chi2 = ((hits - expect) ** 2 / (expect * (1 - K / N))).sum()
    assert stats.chi2.sf(chi2, N - 1) > 1e-4, chi2
    # pairs of coordinates: joint inclusion K(K-1)/(N(N-1)) -- catches a law that always picks neighbours
    joint = 0
    for i in range(trials):
        s = R.randk_index_set(N, K, SEED, 1000 + i, 0)
        joint += np.count_nonzero(np.diff(s) == 1)
    exp_adj = trials * (N - 1) * K * (K - 1) / (N * (N - 1))
    assert abs(joint - exp_adj) < 6 * np.sqrt(exp_adj)


def test_voter_count_is_binomial():
    """Lemma 3: with M workers the number of voters of a coordinate is Binomial(M, K/N)."""
    M, N, K = 16, 20_000, 2_000
    G = np.ones((M, N), dtype=np.float32)
    words, counts = R.randk_sign_encode(G, K, SEED, 3)
    assert (counts == K).all()
    voters = np.zeros(N, dtype=np.int64)
    for m in range(M):
        voters[(words[m] >> 1).astype(np.int64)] += 1
    obs = np.bincount(voters, minlength=M + 1)[:8]
    exp = stats.binom.pmf(np.arange(8), M, K / N) * N
    chi2 = ((obs - exp) ** 2 / exp).sum()
    assert stats.chi2.sf(chi2, 7) > 1e-4, (obs, exp)
    assert abs((voters == 0).mean() - (1 - K / N) ** M) < 0.01       # Example 2: empty fraction (1 - K/N)^M


def test_k_equals_n_is_signsgd_with_majority_vote():
    rng = np.random.default_rng(2)
    M, N = 5, 300
    G = rng.standard_normal((M, N)).astype(np.float32)
    G[0, 7] = 0.0
    x = rng.standard_normal(N).astype(np.float32)
    r = R.step_randk(G, N, x, 1e-3, SEED, 0)
    votes = np.sign(np.sign(G).sum(axis=0)).astype(np.int8)
    assert np.array_equal(r["votes"], votes)
    assert np.array_equal(r["x"], (x - np.float32(1e-3) * votes.astype(np.float32)).astype(np.float32))
    assert r["counts"].tolist() == [N - 1, N, N, N, N]               # the zero entry sends nothing


def test_single_worker_message_is_sign_on_the_selected_set():
    rng = np.random.default_rng(3)
    N, K = 5000, 50
    g = rng.standard_normal((1, N)).astype(np.float32)
    S = R.randk_index_set(N, K, SEED, 9, 0)
    g[0, S[:3]] = [0.0, -0.0, -2.5]
    r = R.step_randk(g, K, np.zeros(N, np.float32), 1.0, SEED, 9)
    dense = np.zeros(N, dtype=np.int8)
    dense[S] = O.sgn(g[0, S])
    assert np.array_equal(r["votes"], dense)
    assert r["counts"][0] == K - 2
    assert (r["words"][0, K - 2:] == 0xFFFFFFFF).all()
    w = r["words"][0, : K - 2]
    assert (np.diff(w >> 1) > 0).all() and np.array_equal(w & 1, (g[0, (w >> 1).astype(np.int64)] < 0).astype(np.uint32))


def test_planted_mistake_breaks_the_bijection(monkeypatch):
    """A round that drops the XOR with the other half is not injective: the bijection pin catches it."""
    def broken(v, h, keys):
        mask = (1 << h) - 1
        left, right = v >> h, v & mask
        for k in keys:
            left, right = right, (R.fmix32(left ^ k) & mask)  # drops the XOR with the old left half
        return (left << h) | right
    h = R.half_bits(1000)
    img = {broken(v, h, R.round_keys(SEED, 0, 0)) for v in range(4 ** h)}
    assert len(img) < 4 ** h


# ---- the exact bits of the generator: a worked instance ------------------------------------------
def _worked_example():
    """tests/golden/randk_permutation_example.txt: every round key, every value of the round function
    and the network on its whole domain for one tiny instance, worked outside the oracle."""
    import os
    ex = {"fmix": [], "round": {}}
    with open(os.path.join(os.path.dirname(__file__), "golden", "randk_permutation_example.txt")) as f:
        for line in f:
            tok = line.split()
            if not tok or tok[0].startswith("#"):
                continue
            if tok[0] == "fmix":
                ex["fmix"].append((int(tok[1], 16), int(tok[2], 16)))
            elif tok[0] == "round":
                ex["round"][int(tok[1])] = [int(v, 16) for v in tok[2:]]
            elif tok[0] in ("k", "keys"):
                ex[tok[0]] = [int(v, 16) for v in tok[1:]]
            elif tok[0] in ("net", "pi", "index_set"):
                ex[tok[0]] = [int(v) for v in tok[1:]]
            else:
                ex[tok[0]] = int(tok[1], 0)
    return ex


def test_finaliser_matches_published_vectors_and_worked_values():
    ex = _worked_example()
    for z, want in ex["fmix"]:
        assert R.fmix32(z) == want
    for r, key in enumerate(ex["keys"]):
        for right in range(4):
            assert R.fmix32(right ^ key) == ex["round"][r][right]
    z = np.array([a for a, _ in ex["fmix"]] + ex["keys"], dtype=np.uint64)
    assert R._fmix32_np(z).tolist() == [R.fmix32(int(v)) for v in z]


def test_round_keys_match_the_worked_instance():
    ex = _worked_example()
    assert R.round_keys(ex["seed"], ex["t"], ex["m"]) == ex["keys"]
    # each of seed's halves, t and m enters: changing one changes the keys
    for other in (R.round_keys(ex["seed"] ^ 1, ex["t"], ex["m"]), R.round_keys(ex["seed"] ^ (1 << 32), ex["t"], ex["m"]),
                  R.round_keys(ex["seed"], ex["t"] + 1, ex["m"]), R.round_keys(ex["seed"], ex["t"], ex["m"] + 1)):
        assert other != ex["keys"]


def test_network_and_cycle_walk_match_the_worked_instance():
    ex = _worked_example()
    N, keys = ex["N"], ex["keys"]
    assert R.half_bits(N) == ex["h"]
    assert [R.feistel(v, ex["h"], keys) for v in range(4 ** ex["h"])] == ex["net"]
    assert [R.permute(i, N, keys) for i in range(N)] == ex["pi"]
    assert R.permute_many(np.arange(N), N, keys).tolist() == ex["pi"]
    assert R.randk_index_set(N, ex["K"], ex["seed"], ex["t"], ex["m"]).tolist() == ex["index_set"]
    g = np.array([[0.5, -1.0, 2.0, 3.0, -4.0, -0.25]] * 3, dtype=np.float32)  # worker m = 2 is the third row
    words, counts = R.randk_sign_encode(g, ex["K"], ex["seed"], ex["t"])
    assert counts[2] == 3 and words[2].tolist() == [(1 << 1) | 1, (2 << 1) | 0, (5 << 1) | 1]


@pytest.mark.parametrize("mistake", ["constant", "shift", "key_order", "round_count", "halves", "no_walk"])
def test_planted_mistakes_fail_the_worked_instance(mistake, monkeypatch):
    """A wrong constant, shift, key derivation, round count, half order or a missing cycle walk keeps
    every property pin green (the result is still a keyed bijection); only the worked instance fails."""
    ex = _worked_example()
    N, keys, h = ex["N"], ex["keys"], ex["h"]
    if mistake == "constant":
        def f(z):
            z &= 0xFFFFFFFF; z ^= z >> 16; z = (z * 0x85EBCA77) & 0xFFFFFFFF; z ^= z >> 13
            z = (z * 0xC2B2AE35) & 0xFFFFFFFF; z ^= z >> 16
            return z
        monkeypatch.setattr(R, "fmix32", f)
    elif mistake == "shift":
        def f(z):
            z &= 0xFFFFFFFF; z ^= z >> 16; z = (z * 0x85EBCA6B) & 0xFFFFFFFF; z ^= z >> 15
            z = (z * 0xC2B2AE35) & 0xFFFFFFFF; z ^= z >> 16
            return z
        monkeypatch.setattr(R, "fmix32", f)
    elif mistake == "key_order":  # the halves of the seed enter the key derivation the other way round
        swapped = ((ex["seed"] & 0xFFFFFFFF) << 32) | (ex["seed"] >> 32)
        keys = R.round_keys(swapped, ex["t"], ex["m"])
        assert keys != ex["keys"]
    elif mistake == "round_count":
        keys = keys[:5]
    elif mistake == "halves":
        def net(v, hh, ks):
            mask = (1 << hh) - 1
            right, left = v >> hh, v & mask  # halves taken the other way round
            for k in ks:
                left, right = right, left ^ (R.fmix32(right ^ k) & mask)
            return (left << hh) | right
        monkeypatch.setattr(R, "feistel", net)
    if mistake == "no_walk":
        got = [R.feistel(i, h, keys) % N for i in range(N)]
    else:
        if mistake in ("constant", "shift"):
            keys = R.round_keys(ex["seed"], ex["t"], ex["m"])
        got = [R.permute(i, N, keys) for i in range(N)]
    assert got != ex["pi"]
