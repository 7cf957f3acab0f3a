"""Pins of the oracle's cache shape (Sec. 4.1.2, Theorem "Geometric Fan-Out") and of the round with a fan-out that
differs per accept length (no GPU).

The closed form is checked against what defines it: a numerical constrained maximiser of the hit-rate objective the
theorem optimises, the stationarity conditions of its proof, hand-worked small cases, and, for the integer shape,
brute force over every integer composition.  The ragged round is checked against the uniform round (already pinned
elsewhere), of which it is a sub-cache when decoding is greedy."""
import itertools
import math

import numpy as np
import pytest
from scipy.optimize import minimize

import ssd_inputs as I
from oracle import ssd_oracle as O


def test_hit_rate_objective_by_hand():
    # K = 1, a = 1/2, r = 1: P(accept 0) = 1/2 with miss 1/F_0, P(accept 1) = 1/2 with miss 1/F_1
    assert O.cache_hit_rate([2, 4], 0.5, 1.0) == pytest.approx(0.5 * (1 - 1 / 2) + 0.5 * (1 - 1 / 4))
    # one candidate never hits under the power law (miss rate 1^-r = 1)
    assert O.cache_hit_rate([1, 1, 1], 0.7, 0.4) == pytest.approx(0.0)
    # accept-length probabilities sum to one: an unbounded cache always hits
    assert O.cache_hit_rate([1e30] * 6, 0.8, 0.5) == pytest.approx(1.0)


@pytest.mark.parametrize("K,a,r,budget", [(5, 0.8, 0.5, 24.0), (3, 0.6, 1.0, 40.0), (7, 0.9, 0.3, 64.0), (1, 0.25, 1.0, 10.0)])
def test_closed_form_is_the_constrained_maximiser(K, a, r, budget):
    f = O.geometric_fan_out_real(budget, K, a, r)
    assert f.sum() == pytest.approx(budget, rel=1e-12)
    q = a ** (1 / (1 + r))
    np.testing.assert_allclose(f[1:K] / f[:K - 1], q, rtol=1e-12)
    assert f[K] / f[0] == pytest.approx(q ** K * (1 - a) ** (-1 / (1 + r)), rel=1e-12)
    # stationarity (proof of the general theorem): weight_k * d/dF (1 - F^-r) is the same for every k
    wk = np.array([a ** k * (1 - a) for k in range(K)] + [a ** K])
    np.testing.assert_allclose(wk * r * f ** (-r - 1), (wk * r * f ** (-r - 1))[0], rtol=1e-10)
    # a numerical maximiser started from the uniform shape lands on it
    res = minimize(lambda x: -O.cache_hit_rate(x, a, r), np.full(K + 1, budget / (K + 1)), method="SLSQP",
                   bounds=[(1e-3, budget)] * (K + 1), constraints=[{"type": "eq", "fun": lambda x: x.sum() - budget}],
                   options={"ftol": 1e-14, "maxiter": 500})
    assert res.success
    assert O.cache_hit_rate(f, a, r) >= -res.fun - 1e-9
    np.testing.assert_allclose(res.x, f, rtol=2e-3)
    # and moving budget between any two accept lengths lowers the hit rate
    best = O.cache_hit_rate(f, a, r)
    for i, j in itertools.permutations(range(K + 1), 2):
        g = f.copy()
        g[i] += 0.05
        g[j] -= 0.05
        assert O.cache_hit_rate(g, a, r) < best


def test_closed_form_hand_worked_cases():
    # K = 0: the whole budget sits on the only accept length
    np.testing.assert_allclose(O.geometric_fan_out_real(7.0, 0, 0.5, 1.0), [7.0])
    # K = 1, a = 1/4, r = 1: a^(1/2) = 1/2 and (1-a)^(-1/2) = 2/sqrt(3), so F_1 / F_0 = 1/sqrt(3)
    f = O.geometric_fan_out_real(1 + 1 / math.sqrt(3), 1, 0.25, 1.0)
    np.testing.assert_allclose(f, [1.0, 1 / math.sqrt(3)], rtol=1e-12)
    # K = 2, a = 1/4, r = 1: F = F_0 (1, 1/2, 1/(2 sqrt 3))
    f = O.geometric_fan_out_real(3.0, 2, 0.25, 1.0)
    np.testing.assert_allclose(f / f[0], [1.0, 0.5, 0.5 / math.sqrt(3)], rtol=1e-12)


def _compositions(total, parts, lo, hi):
    if parts == 1:
        if lo <= total <= hi:
            yield (total,)
        return
    for x in range(lo, min(hi, total - lo * (parts - 1)) + 1):
        for rest in _compositions(total - x, parts - 1, lo, hi):
            yield (x,) + rest


@pytest.mark.parametrize("K,a,r,budget,f_max", [(3, 0.8, 0.5, 16, 16), (3, 0.5, 1.0, 14, 8), (4, 0.7, 0.4, 15, 16),
                                                (2, 0.3, 0.8, 9, 16), (5, 0.8, 0.5, 24, 16)])
def test_integer_shape_against_brute_force(K, a, r, budget, f_max):
    fan = O.geometric_fan_out(budget, K, a, r, f_max)
    assert fan.sum() == budget and fan.min() >= 1 and fan.max() <= f_max
    assert all(fan[k] >= fan[k + 1] for k in range(K - 1))          # geometric part does not grow with k
    got = O.cache_hit_rate(fan, a, r)
    best = max(O.cache_hit_rate(c, a, r) for c in _compositions(budget, K + 1, 1, f_max))
    uniform = O.cache_hit_rate([budget / (K + 1)] * (K + 1), a, r)
    assert got <= best + 1e-12
    assert best - got < 0.01, (fan, got, best)                       # rounding costs under one point of hit rate
    assert got >= uniform - 1e-12 or budget % (K + 1)                # never worse than the uniform shape of that budget


def test_integer_shape_bounds_bind_and_budget_is_kept():
    # a low acceptance rate puts the real F_0 above the cap: it is held at the cap, the rest is shared
    fan = O.geometric_fan_out(48, 5, 0.5, 0.5, f_max=16)
    assert fan[0] == 16 and fan.sum() == 48 and fan.min() >= 1
    real = O.geometric_fan_out_real(48, 5, 0.5, 0.5)
    assert real[0] > 16
    # a tight budget leaves one candidate per accept length
    np.testing.assert_array_equal(O.geometric_fan_out(6, 5, 0.8, 0.5), np.ones(6, np.int64))
    # a full budget fills every accept length to the cap
    np.testing.assert_array_equal(O.geometric_fan_out(12, 2, 0.8, 0.5, f_max=4), np.full(3, 4))


# ----------------------------------------------------------------- the round with F_0..F_K

def _tiny(seed=101):
    shape = I.WORKLOADS["tiny_f32"].draft
    return shape, O.Model.from_weights(shape, I.make_weights(shape, seed))


def test_ragged_round_is_a_sub_cache_of_the_uniform_round_when_greedy():
    shape, m = _tiny()
    K, P = 3, 9
    fan = np.array([4, 2, 1, 3])
    prompt = I.make_prompt(shape, 1, P, 5)[0]
    _, trunk = O.prefill(m, prompt)
    pending = I.make_pending(shape, 1, K, 6)[0]
    full = O.prespeculate(m, trunk, pending, 4, 0.0, 1)
    rag = O.prespeculate(m, trunk, pending, fan, 0.0, 1)
    assert rag.keys.shape == (K + 1, 4) and list(rag.fan) == list(fan)
    for k in range(K + 1):
        f = fan[k]
        np.testing.assert_array_equal(rag.keys[k, :f], full.keys[k, :f])
        assert (rag.keys[k, f:] == -1).all()
        np.testing.assert_array_equal(rag.tokens[k, :f], full.tokens[k, :f])
        np.testing.assert_array_equal(rag.logits[k, :f], full.logits[k, :f])
        assert not rag.logits[k, f:].any()
        # lookup: cached outcomes hit at their rank, the uniform round's further keys miss
        for j in range(4):
            assert O.cache_lookup(rag.keys, k, int(full.keys[k, j])) == (j if j < f else -1)


def test_ragged_round_numbers_its_rows_by_running_offsets_when_sampling():
    shape, m = _tiny(seed=103)
    K, P, T, seed = 3, 7, 0.9, 44
    fan = np.array([3, 1, 2, 2])
    _, trunk = O.prefill(m, I.make_prompt(shape, 1, P, 8)[0])
    pending = I.make_pending(shape, 1, K, 9)[0]
    rag = O.prespeculate(m, trunk, pending, fan, T, seed, row_base=8)
    _, _, glue = O.glue_extend(m, trunk, pending)
    off = [0, 3, 4, 6]
    for k in range(K + 1):
        for j in range(fan[k]):
            t, l, _, _ = O.decode_branch(m, glue, P, k, rag.keys[k, j], K, T, seed, 8 + off[k] + j)
            np.testing.assert_array_equal(rag.tokens[k, j], t)
            np.testing.assert_array_equal(rag.logits[k, j], l)
    # different rows draw different noise: two branches with the same first token and accept length would still differ
    assert len({tuple(rag.tokens[k, j]) for k in range(K + 1) for j in range(fan[k])}) > 1


def test_greedy_ssd_with_a_geometric_cache_is_lossless():
    shape, mt = _tiny(seed=11)
    wd = I.make_weights(shape, 12, perturb_of=I.make_weights(shape, 11), perturb_std=0.002)
    md = O.Model.from_weights(shape, wd)
    K = I.WORKLOADS["tiny_f32"].round.K
    fan = O.geometric_fan_out((K + 1) * 3, K, 0.7, 0.5, f_max=8)
    assert len(set(fan.tolist())) > 1
    prompt = I.make_prompt(shape, 1, 12, 21)[0]
    want = O.ar_generate(mt, prompt, 24)
    got, st = O.ssd_generate(mt, md, prompt, 24, K, fan)
    assert got == want
    assert 0 < st.hits <= st.rounds
