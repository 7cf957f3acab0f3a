"""Pins of the oracle's sampling at temperature > 0 (no GPU): the Gumbel-max draw of `sample_token` and every routine
that drafts with it must follow softmax(logits / T) (Sec. 4.2.1, Def. "sampling scheme"), and the sampled SSD loop
must emit the target's own distribution (Sec. 2.1: speculative decoding is lossless).

The expected distributions are written out from the definition here (a softmax of the model's logits, products of
conditionals by enumeration of every prefix); a draw whose noise is scaled by T, or whose logits are not divided by
it, ends up at softmax(z) or softmax(z / T^2) and fails these at T = 0.6 and T = 2."""
import numpy as np
import pytest

import ssd_inputs as I
from oracle import ssd_oracle as O


def _softmax(x):
    e = np.exp(x - np.max(x))
    return e / e.sum()


def _close(counts, p, sigmas=4.5):
    n = counts.sum()
    return bool(np.all(np.abs(counts / n - p) <= sigmas * np.sqrt(p * (1 - p) / n) + 1e-9))


def _wrong_forms_fail(counts, z, T):
    """The two plausible mistakes, softmax(z) and softmax(z / T^2), are far outside the band the counts satisfy."""
    return not _close(counts, _softmax(z)) and not _close(counts, _softmax(z / T ** 2))


@pytest.mark.parametrize("T", [0.6, 2.0])
def test_sample_token_follows_softmax_of_logits_over_T(T):
    V, N = 6, 100000
    z = np.array([1.3, -0.2, 0.7, 2.1, -1.5, 0.1])
    counts = np.zeros(V)
    margins_ok = True
    for n in range(N):
        tok, margin = O.sample_token(z, T, O.gumbel(n, O.STREAM_DRAFT, 3, 1, V))
        counts[tok] += 1
        margins_ok &= margin >= 0.0
    assert margins_ok
    assert _close(counts, _softmax(z / T))
    assert _wrong_forms_fail(counts, z, T)


def test_sample_token_greedy_ignores_noise_and_breaks_ties_by_lower_id():
    z = np.array([0.5, 2.0, 2.0, -1.0])
    assert O.sample_token(z, 0.0, None) == (1, 0.0)
    tok, margin = O.sample_token(np.array([0.5, 2.0, 1.25, -1.0]), 0.0, None)
    assert tok == 1 and margin == pytest.approx(0.75)


TINY = I.ModelShape(n_layers=1, d_model=8, n_q_heads=2, n_kv_heads=1, head_dim=4, d_ffn=8, vocab=5, dtype="f32",
                    rope_theta=10000.0, tie_embeddings=False)


def _tiny_model(seed, std=0.9):
    return O.Model.from_weights(TINY, I.make_weights(TINY, seed, std=std))


def _next_logits(m, tokens):
    """Logits after `tokens` by full recomputation (the dense causal forward, pinned in test_oracle_model.py)."""
    return O.prefill(m, tokens)[0][-1]


@pytest.mark.parametrize("T", [0.6, 2.0])
def test_decode_branch_draws_follow_the_models_conditionals(T):
    """Two steps of one branch: token 1 ~ softmax(l(prefix + c) / T), token 2 given token 1 ~ softmax(l(.. + token 1) / T)."""
    m = _tiny_model(5)
    V, N = TINY.vocab, 15000
    prompt = [1, 4, 2]
    _, trunk = O.prefill(m, prompt)
    k, first, row = 1, 3, 7
    P = len(prompt) - 1 - k          # the branch sees trunk positions 0 .. P + k: the whole prompt
    p1 = _softmax(_next_logits(m, prompt + [first]) / T)
    p2 = [_softmax(_next_logits(m, prompt + [first, t]) / T) for t in range(V)]
    c1 = np.zeros(V)
    c2 = np.zeros((V, V))
    for n in range(N):
        toks, logits, _, _ = O.decode_branch(m, trunk, P, k, first, 2, T, seed=n, row=row)
        c1[toks[0]] += 1
        c2[toks[0], toks[1]] += 1
        if n == 0:
            np.testing.assert_allclose(logits[0], _next_logits(m, prompt + [first]), atol=1e-9)
    assert _close(c1, p1)
    assert _wrong_forms_fail(c1, _next_logits(m, prompt + [first]), T)
    for t in range(V):
        if c2[t].sum() > 1000:
            assert _close(c2[t], p2[t])


@pytest.mark.parametrize("T", [0.6, 2.0])
def test_speculate_draws_follow_the_models_conditionals(T):
    m = _tiny_model(6)
    V, N = TINY.vocab, 15000
    prompt = [0, 3, 3, 1]
    _, trunk = O.prefill(m, prompt[:-1])
    p1 = _softmax(_next_logits(m, prompt) / T)
    p2 = [_softmax(_next_logits(m, prompt + [t]) / T) for t in range(V)]
    c1 = np.zeros(V)
    c2 = np.zeros((V, V))
    for n in range(N):
        toks, _ = O.speculate(m, trunk, prompt[-1], 2, T, seed=n)
        c1[toks[0]] += 1
        c2[toks[0], toks[1]] += 1
    assert _close(c1, p1)
    assert _wrong_forms_fail(c1, _next_logits(m, prompt), T)
    for t in range(V):
        if c2[t].sum() > 1000:
            assert _close(c2[t], p2[t])


@pytest.mark.parametrize("backup", ["primary", "random"])
def test_sampled_ssd_loop_emits_the_targets_distribution(backup):
    """Alg. 1 at temperature 0.8 with an unrelated draft, K = 2, F = 2: the first three emitted tokens span two rounds
    (verification of a just-in-time speculation, then of a cached or a backup one).  Their joint distribution must be
    the target's: p(x1) p(x2 | x1) p(x3 | x1, x2), enumerated over all 125 prefixes."""
    T, K, F, N = 0.8, 2, 2, 4000
    target, draft = _tiny_model(11), _tiny_model(12)
    V = TINY.vocab
    prompt = [2, 0, 4]
    want = np.zeros((V, V, V))
    p1 = _softmax(_next_logits(target, prompt) / T)
    for a in range(V):
        p2 = _softmax(_next_logits(target, prompt + [a]) / T)
        for b in range(V):
            want[a, b] = p1[a] * p2[b] * _softmax(_next_logits(target, prompt + [a, b]) / T)
    got = np.zeros((V, V, V))
    hits = rounds = 0
    for n in range(N):
        out, stats = O.ssd_generate(target, draft, prompt, 3, K, F, T=T, seed=50000 + 17 * n, backup=backup)
        got[tuple(out)] += 1
        hits += stats.hits
        rounds += stats.rounds
    assert 0 < hits < rounds                                 # both the cached and the fallback speculation occur
    # marginals of each position and the joint, each cell within its binomial band
    for axis_sum in ((1, 2), (0, 2), (0, 1)):
        assert _close(got.sum(axis=axis_sum), want.sum(axis=axis_sum))
    assert _close(got.reshape(-1), want.reshape(-1), sigmas=5.0)
    # and it is not the draft's distribution
    q1 = _softmax(_next_logits(draft, prompt) / T)
    assert not _close(got.sum(axis=(1, 2)), q1)
