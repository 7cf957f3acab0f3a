"""Pins of the oracle's distribution-level functions against what the paper prints and what
the mathematics fixes (no GPU)."""
import math
import os

import numpy as np
import pytest

from oracle import ssd_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


# ----------------------------------------------------------------- the generator

def test_mix64_matches_splitmix64_vectors():
    with open(os.path.join(GOLD, "splitmix64.txt")) as f:
        want = [int(l, 16) for l in f if l.strip() and not l.startswith("#")]
    got = [O._mix64(((n + 1) * 0x9E3779B97F4A7C15) & (2 ** 64 - 1)) for n in range(3)]
    assert got == want
    vec = O._mix64_vec(np.array([((n + 1) * 0x9E3779B97F4A7C15) & (2 ** 64 - 1) for n in range(3)],
                                dtype=np.uint64))
    assert [int(v) for v in vec] == want


def test_draw_u_is_open_interval_fp32_exact_and_uniform():
    u = O.draw_u(7, O.STREAM_BONUS, 3, 1, np.arange(200000))
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)      # exact in fp32
    assert abs(u.mean() - 0.5) < 4 * math.sqrt(1 / 12 / u.size)
    hist = np.histogram(u, bins=16, range=(0, 1))[0]
    assert np.all(np.abs(hist - u.size / 16) < 5 * math.sqrt(u.size / 16))
    # streams, seeds and coordinates all decorrelate
    for other in (O.draw_u(8, O.STREAM_BONUS, 3, 1, np.arange(1000)),
                  O.draw_u(7, O.STREAM_DRAFT, 3, 1, np.arange(1000)),
                  O.draw_u(7, O.STREAM_BONUS, 4, 1, np.arange(1000)),
                  O.draw_u(7, O.STREAM_BONUS, 3, 2, np.arange(1000))):
        assert np.mean(other == u[:1000]) < 0.01
    # scalar and vector forms agree
    assert float(O.draw_u(7, O.STREAM_BONUS, 3, 1, 12345)) == u[12345]


def test_gumbel_moments():
    g = O.gumbel(11, O.STREAM_DRAFT, 0, 0, 400000)
    assert abs(g.mean() - 0.5772156649) < 0.01          # Euler-Mascheroni
    assert abs(g.var() - math.pi ** 2 / 6) < 0.02


# ----------------------------------------------------------------- Construction 1

def test_construction1_sigma_FC_and_acceptance():
    gold = _read_golden("construction1.txt")
    p_t, p_d = np.array(gold["p_t"]), np.array(gold["p_d"])
    C = gold["C"][0] / gold["C"][1]
    F = int(gold["F"][0])
    p_dp = O.sigma_FC(np.log(p_d), F, C)
    np.testing.assert_allclose(p_dp, gold["p_d_prime"], atol=1e-12)
    # the logit-shift form of the same scheme
    np.testing.assert_allclose(O.softmax_T(O.sigma_FC_logits(np.log(p_d), F, C), 1.0), gold["p_d_prime"], atol=1e-12)
    np.testing.assert_allclose(O.softmax_T(O.sigma_FC_logits(np.log(p_d) * 2.0, F, C, T=2.0), 2.0),
                               gold["p_d_prime"], atol=1e-12)
    assert O.acceptance_rate(p_t, p_d) == pytest.approx(gold["accept"][0], abs=1e-12)
    assert O.acceptance_rate(p_t, p_dp) == pytest.approx(gold["accept_prime"][0], abs=1e-12)
    # Theorem 1's second form (with the factor one half)
    assert 1 - 0.5 * np.abs(p_t - p_d).sum() == pytest.approx(gold["accept"][0], abs=1e-12)
    assert 1 - 0.5 * np.abs(p_t - p_dp).sum() == pytest.approx(gold["accept_prime"][0], abs=1e-12)


def test_construction1_residuals_cache_and_hit_rates():
    gold = _read_golden("construction1.txt")
    p_t, p_d, p_dp = (np.array(gold[k]) for k in ("p_t", "p_d", "p_d_prime"))
    r, rp = O.residual(p_t, p_d), O.residual(p_t, p_dp)
    np.testing.assert_allclose(r, gold["r"], atol=1e-12)
    np.testing.assert_allclose(rp, gold["r_prime"], atol=1e-12)
    # token 1 drawn from p_d and rejected: cache = top-2 of p_d without token 1
    cache = O.top_f_ids(np.log(p_d), 2, exclude=0) + 1
    assert list(cache) in ([int(x) for x in gold["cache"]], [int(x) for x in gold["cache_alt"]])
    assert list(cache) == [2, 3]                       # our tie rule: lower id first
    assert r[cache - 1].sum() == pytest.approx(gold["hit"][0])
    # token 3 drawn from p_d' and rejected
    cache_p = O.top_f_ids(np.log(p_dp), 2, exclude=2) + 1
    assert sorted(cache_p) == [int(x) for x in gold["cache_prime"]]
    assert rp[cache_p - 1].sum() == pytest.approx(gold["hit_prime"][0])
    # the token the verifier rejected can never be the bonus token (Sec. 4.1.1)
    assert r[0] == 0.0 and rp[2] == 0.0


def test_theorem1_identity_random():
    g = np.random.default_rng(0)
    for _ in range(50):
        n = int(g.integers(2, 50))
        a, b = g.dirichlet(np.ones(n)), g.dirichlet(np.ones(n) * 0.3)
        assert O.acceptance_rate(a, b) == pytest.approx(1 - 0.5 * np.abs(a - b).sum(), abs=1e-12)


def test_sigma_FC_monotone_hit_rate():
    # Theorem "cache hit rate increases as C -> 0": residual mass inside top-F is nonincreasing in C
    g = np.random.default_rng(1)
    for _ in range(20):
        z = g.normal(size=12)
        p_t = g.dirichlet(np.ones(12))
        S = O.top_f_ids(z, 3)
        prev = 2.0
        for C in (0.0, 0.1, 0.3, 0.6, 1.0):
            res = np.maximum(p_t - O.sigma_FC(z, 3, C), 0)
            hit = 1.0 if res.sum() == 0 else res[S].sum() / res.sum()
            assert hit <= prev + 1e-12
            prev = hit


# ----------------------------------------------------------------- top-F

def test_top_f_brute_force_with_ties_and_exclusion():
    g = np.random.default_rng(2)
    for trial in range(40):
        V = int(g.integers(5, 300))
        z = g.integers(-3, 4, size=V).astype(np.float32)      # many ties
        F = int(g.integers(1, 5))
        ex = None if trial % 3 == 0 else int(g.integers(0, V))
        want = sorted((t for t in range(V) if t != ex), key=lambda t: (-float(z[t]), t))[:F]
        assert list(O.top_f_ids(z, F, exclude=ex)) == want


def test_top_f_nan_ranks_last():
    z = np.array([1.0, np.nan, 3.0, np.nan, 2.0], dtype=np.float32)
    assert list(O.top_f_ids(z, 5)) == [2, 4, 0, 1, 3]


# ----------------------------------------------------------------- verification

def test_verify_greedy_cases():
    V, K = 9, 3
    zt = np.full((K + 1, V), -1.0)
    spec = [4, 2, 7]
    for i, s in enumerate(spec):
        zt[i, s] = 5.0
    zt[K, 1] = 5.0
    out = O.verify(zt, None, spec, 0.0, seed=0)
    assert (out.accept_len, out.bonus) == (K, 1)               # all accepted, bonus from row K
    zt2 = zt.copy()
    zt2[1, 6] = 9.0                                            # mismatch at position 1
    out = O.verify(zt2, None, spec, 0.0, seed=0)
    assert (out.accept_len, out.bonus) == (1, 6)
    zt3 = zt.copy()
    zt3[0, 3] = 5.0                                            # tie at position 0: lower id (3) wins
    out = O.verify(zt3, None, spec, 0.0, seed=0)
    assert (out.accept_len, out.bonus) == (0, 3)


def _inverse_cdf(p, u):
    return int(min(np.searchsorted(np.cumsum(p), u, side="right"), len(p) - 1))


def test_verify_sampling_is_lossless_monte_carlo():
    """K = 1.  Token 1 of the output (s_1 if accepted, else the bonus) must follow the target's
    row 0; the bonus after an acceptance must follow the target's row 1; the bonus after a
    rejection must follow the residual (Sec. 2.1)."""
    g = np.random.default_rng(3)
    V, T, N = 6, 0.8, 40000
    zt = g.normal(size=(2, V)) * 1.5
    zd = g.normal(size=(1, V)) * 1.5
    p0, p1, q0 = O.softmax_T(zt[0], T), O.softmax_T(zt[1], T), O.softmax_T(zd[0], T)
    first = np.zeros(V)
    after_acc = np.zeros(V)
    after_rej = np.zeros(V)
    us = g.random(N)
    for n in range(N):
        s = _inverse_cdf(q0, us[n])
        out = O.verify(zt, zd, [s], T, seed=1000 + n)
        if out.accept_len == 1:
            first[s] += 1
            after_acc[out.bonus] += 1
        else:
            first[out.bonus] += 1
            after_rej[out.bonus] += 1

    def close(counts, p):
        n = counts.sum()
        return np.all(np.abs(counts / n - p) < 4.5 * np.sqrt(p * (1 - p) / n) + 1e-9)

    assert close(first, p0)
    assert close(after_acc, p1)
    assert close(after_rej, O.residual(p0, q0))
    # acceptance frequency = Theorem 1
    assert abs(after_acc.sum() / N - O.acceptance_rate(p0, q0)) < 4.5 * math.sqrt(0.25 / N)


def test_verify_identical_distributions_accept_everything():
    g = np.random.default_rng(4)
    V, K = 20, 4
    z = g.normal(size=(K + 1, V))
    for seed in range(30):
        spec = [int(g.integers(0, V)) for _ in range(K)]
        out = O.verify(z, z[:K], spec, 1.0, seed)
        assert out.accept_len == K


def test_verify_zero_probability_token_is_rejected_and_never_bonus():
    V = 5
    zt = np.array([[0.0, 0.0, 0.0, 0.0, -1e9], [0.0] * V])
    zd = np.array([[0.0] * V])
    for seed in range(50):
        out = O.verify(zt, zd, [4], 1.0, seed)
        assert out.accept_len == 0 and out.bonus != 4


# ----------------------------------------------------------------- random-token backup speculator (Sec. 4.3)

def test_random_speculation_is_uniform_reproducible_and_keyed_by_sequence_and_step():
    V, K = 7, 5
    counts = np.zeros(V)
    for seed in range(6000):
        toks, logits = O.random_speculation(seed, 0, K, V)
        assert len(toks) == K and all(0 <= t < V for t in toks)
        assert logits.shape == (K, V) and not logits.any()              # the uniform distribution, as logits
        counts += np.bincount(toks, minlength=V)
    n = counts.sum()
    assert np.all(np.abs(counts / n - 1 / V) < 4.5 * math.sqrt((1 / V) * (1 - 1 / V) / n))
    # by hand from the generator's definition: token i of sequence b = hash(seed, stream 4, b, i, 0) mod V
    V = 128256
    toks, _ = O.random_speculation(99, 3, 4, V)
    assert toks == [int(O.draw_bits(99, 4, 3, i, 0)) % V for i in range(4)]
    assert toks == O.random_speculation(99, 3, 4, V)[0]
    assert toks != O.random_speculation(99, 2, 4, V)[0] and toks != O.random_speculation(98, 3, 4, V)[0]
    assert len(set(toks)) > 1


def test_verifying_random_tokens_against_the_uniform_distribution_is_lossless_monte_carlo():
    """The random backup's tokens verified with zero draft logits (the uniform q they were drawn from): token 1 of
    the output follows the target's row 0, and the acceptance frequency is Theorem 1 with q uniform."""
    g = np.random.default_rng(5)
    V, T, N = 6, 0.9, 40000
    zt = g.normal(size=(2, V)) * 1.5
    p0 = O.softmax_T(zt[0], T)
    first = np.zeros(V)
    accepted = 0
    for n in range(N):
        toks, zd = O.random_speculation(70000 + n, 0, 1, V)
        out = O.verify(zt, zd, toks, T, seed=n)
        first[toks[0] if out.accept_len == 1 else out.bonus] += 1
        accepted += out.accept_len
    assert np.all(np.abs(first / N - p0) < 4.5 * np.sqrt(p0 * (1 - p0) / N) + 1e-9)
    assert abs(accepted / N - O.acceptance_rate(p0, np.full(V, 1 / V))) < 4.5 * math.sqrt(0.25 / N)
