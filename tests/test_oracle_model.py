"""Pins of the oracle's transformer and of the pre-speculation round's structure (no GPU).

Every check is against something other than the routine itself: a closed form, a special
case with a textbook answer, a second independent code path, or brute force."""
import math

import numpy as np
import pytest

import ssd_inputs as I
from oracle import ssd_oracle as O


def _tiny(seed=101, **over):
    shape = I.WORKLOADS["tiny_f32"].draft
    if over:
        shape = I.ModelShape(**{**shape.__dict__, **over})
    return shape, O.Model.from_weights(shape, I.make_weights(shape, seed))


# ----------------------------------------------------------------- building blocks

def test_rmsnorm_unit_rms_and_gain():
    g = np.random.default_rng(0)
    x = g.normal(size=(3, 64)) * 7
    y = O.rmsnorm(x, np.ones(64), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(-1)), 1.0, atol=1e-12)
    gain = g.normal(size=64)
    np.testing.assert_allclose(O.rmsnorm(x, gain, 0.0), y * gain, atol=1e-12)
    # eps enters under the square root, next to the mean square
    one = O.rmsnorm(np.full((1, 4), 2.0), np.ones(4), 5.0)
    np.testing.assert_allclose(one, 2.0 / 3.0, atol=1e-12)


def test_rope_identity_norm_relative_and_pairing():
    g = np.random.default_rng(1)
    D = 8
    x = g.normal(size=(5, 2, D))
    np.testing.assert_allclose(O.rope(x, np.zeros(5), 10000.0), x, atol=1e-15)       # position 0
    y = O.rope(x, np.arange(5) * 13, 10000.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)
    # <rope(q,m), rope(k,n)> depends on m - n only
    q, k = g.normal(size=(1, 1, D)), g.normal(size=(1, 1, D))
    d1 = (O.rope(q, [7], 100.0) * O.rope(k, [3], 100.0)).sum()
    d2 = (O.rope(q, [104], 100.0) * O.rope(k, [100], 100.0)).sum()
    assert d1 == pytest.approx(d2, abs=1e-10)
    # pair (i, i + D/2), frequency theta^(-2i/D): a unit vector on coordinate i turns by pos * freq_i
    for i in range(D // 2):
        e = np.zeros((1, 1, D))
        e[0, 0, i] = 1.0
        r = O.rope(e, [3], 10000.0)[0, 0]
        ang = 3 * 10000.0 ** (-2 * i / D)
        want = np.zeros(D)
        want[i], want[i + D // 2] = math.cos(ang), math.sin(ang)
        np.testing.assert_allclose(r, want, atol=1e-12)


def test_attention_uniform_onehot_and_gqa_mapping():
    g = np.random.default_rng(2)
    T, S, Hq, Hkv, D = 3, 5, 4, 2, 6
    keys, vals = g.normal(size=(S, Hkv, D)), g.normal(size=(S, Hkv, D))
    mask = np.zeros((T, S), bool)
    mask[0, :2] = True
    mask[1, :] = True
    mask[2, 3] = True
    # zero queries: uniform weights over the visible keys
    out = O.attention(np.zeros((T, Hq, D)), keys, vals, mask)
    for hq in range(Hq):
        hk = hq // 2                                            # heads 0,1 -> kv 0; heads 2,3 -> kv 1
        np.testing.assert_allclose(out[0, hq], vals[:2, hk].mean(0), atol=1e-12)
        np.testing.assert_allclose(out[1, hq], vals[:, hk].mean(0), atol=1e-12)
        np.testing.assert_allclose(out[2, hq], vals[3, hk], atol=1e-12)   # a single visible key
    # scores scale as 1/sqrt(D): two keys, q.k1 - q.k0 = sqrt(D) * ln 3  =>  weights 1/4, 3/4
    q = np.zeros((1, 1, D)); q[0, 0, 0] = 1.0
    k2 = np.zeros((2, 1, D)); k2[1, 0, 0] = math.sqrt(D) * math.log(3.0)
    v2 = np.zeros((2, 1, D)); v2[0, 0, 0] = 1.0; v2[1, 0, 1] = 1.0
    o = O.attention(q, k2, v2, np.ones((1, 2), bool))[0, 0]
    np.testing.assert_allclose(o[:2], [0.25, 0.75], atol=1e-12)


def test_swiglu_closed_form():
    # scalar case: silu(1) = 1/(1+e^-1), silu(-1) = -1/(1+e), silu(0) = 0
    x = np.array([[1.0]])
    val = O.swiglu(x, np.array([[1.0], [-1.0], [0.0]]), np.array([[3.0], [2.0], [5.0]]),
                   np.array([[1.0, 0.0, 0.0]]))
    assert val[0, 0] == pytest.approx(3.0 / (1 + math.exp(-1.0)), abs=1e-14)
    val = O.swiglu(x, np.array([[1.0], [-1.0], [0.0]]), np.array([[3.0], [2.0], [5.0]]),
                   np.array([[0.0, 1.0, 1.0]]))
    assert val[0, 0] == pytest.approx(-2.0 / (1 + math.e), abs=1e-14)
    # shapes: w_gate/w_up [ffn][d], w_down [d][ffn]
    g = np.random.default_rng(3)
    out = O.swiglu(g.normal(size=(4, 5)), g.normal(size=(7, 5)), g.normal(size=(7, 5)), g.normal(size=(5, 7)))
    assert out.shape == (4, 5)


def test_forward_special_cases_reduce_to_closed_forms():
    shape = I.ModelShape(n_layers=1, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ffn=8, vocab=11,
                         dtype="f32", rope_theta=10000.0, rms_eps=1e-5)
    w = {k: v.astype(np.float64) for k, v in I.make_weights(shape, 5, std=0.5).items()}
    toks = [3, 7, 7, 1]
    # (a) attention and MLP switched off: logits = rmsnorm(rmsnorm-free residual) @ lm_head
    w0 = dict(w); w0["l0.wo"] = np.zeros_like(w["l0.wo"]); w0["l0.w_down"] = np.zeros_like(w["l0.w_down"])
    m0 = O.Model.from_weights(shape, w0)
    logits, hid, _ = O.forward(m0, toks, range(4), O.KV.empty(m0), O.causal_mask(0, 4))
    e = w["embed"][toks]
    want_hid = e / np.sqrt((e * e).mean(-1, keepdims=True) + 1e-5)
    np.testing.assert_allclose(hid, want_hid, atol=1e-12)
    np.testing.assert_allclose(logits, want_hid @ w["lm_head"].T, atol=1e-12)
    # (b) zero queries, V = first Hkv*D coordinates of the normed input, identity output projection,
    #     MLP off: h_t = e_t + (mean over s <= t of x_s[kv head of each query head])
    w1 = dict(w0)
    w1["l0.wq"] = np.zeros_like(w["l0.wq"])
    wv = np.zeros_like(w["l0.wv"]); wv[np.arange(8), np.arange(8)] = 1.0
    w1["l0.wv"] = wv
    w1["l0.wo"] = np.eye(16)
    m1 = O.Model.from_weights(shape, w1)
    _, hid1, kv1 = O.forward(m1, toks, range(4), O.KV.empty(m1), O.causal_mask(0, 4))
    x = want_hid
    h = e.copy()
    for t in range(4):
        mean_v = x[:t + 1, :8].mean(0)                          # [Hkv*D]
        for hq in range(4):
            hk = hq // 2
            h[t, hq * 4:(hq + 1) * 4] += mean_v[hk * 4:(hk + 1) * 4]
    np.testing.assert_allclose(hid1, h / np.sqrt((h * h).mean(-1, keepdims=True) + 1e-5), atol=1e-12)
    np.testing.assert_allclose(kv1.v[0].reshape(4, 8), x[:, :8], atol=1e-12)
    # (c) one token: softmax over a single key is 1, so attention returns that token's V whatever wq is
    w2 = dict(w1); w2["l0.wq"] = w["l0.wq"]
    m2 = O.Model.from_weights(shape, w2)
    _, hid2, _ = O.forward(m2, toks[:1], [9], O.KV.empty(m2), np.ones((1, 1), bool))
    np.testing.assert_allclose(hid2[0], (h[0] / np.sqrt((h[0] ** 2).mean() + 1e-5)), atol=1e-12)


def test_dense_forward_equals_token_by_token_decode():
    shape, m = _tiny()
    toks = I.make_prompt(shape, 1, 24, 9)[0]
    full, kv_full = O.prefill(m, toks)
    past = O.KV.empty(m)
    for t, tok in enumerate(toks):
        logits, _, kv = O.forward(m, [tok], [t], past, np.ones((1, t + 1), bool))
        past = past.concat(kv)
        np.testing.assert_allclose(logits[0], full[t], rtol=0, atol=1e-10)
    for l in range(m.n_layers):
        np.testing.assert_allclose(past.k[l], kv_full.k[l], atol=1e-12)
    # chunked extend (what the glue step does) is the same thing
    _, kv_a = O.prefill(m, toks[:10])
    lg, _, _ = O.glue_extend(m, kv_a, toks[10:16])
    np.testing.assert_allclose(lg, full[10:16], atol=1e-10)


def test_tied_embeddings_share_one_matrix():
    shape, m = _tiny(tie_embeddings=True)
    assert m.w["lm_head"] is m.w["embed"]
    assert "lm_head" not in I.weight_names(shape)


# ----------------------------------------------------------------- structure of the round

def test_branch_mask_matches_the_paper_figure_description():
    P, K, F, i = 7, 3, 4, 2                                    # the figure's B=1, K=3, F=4, depth i=2
    mask = O.branch_mask(P, K, F, i)
    M = (K + 1) * F
    assert mask.shape == (M, P + K + 1 + 3 * M)
    for r in range(M):
        k = r // F
        assert mask[r, :P].all()                                # left block: the verified prefix
        assert mask[r, P:P + k + 1].all() and not mask[r, P + k + 1:P + K + 1].any()   # glue 0..k
        band = mask[r, P + K + 1:].reshape(3, M)
        assert np.array_equal(band, np.tile(np.eye(M, dtype=bool)[r], (3, 1)))         # diagonal bands
        assert mask[r].sum() == P + k + 1 + i + 1


def test_fan_out_excludes_the_pending_token_and_is_brute_force_top_f():
    g = np.random.default_rng(6)
    K, F, V = 4, 3, 50
    z = g.integers(-2, 3, size=(K + 1, V)).astype(np.float64)
    pending = [5] + [int(np.argmax(z[k])) for k in range(K)]     # greedy draft: s_{k+1} is the row's top-1
    keys = O.fan_out(z, pending, F)
    assert keys.shape == (K + 1, F)
    for k in range(K + 1):
        ex = pending[k + 1] if k < K else None
        want = sorted((t for t in range(V) if t != ex), key=lambda t: (-z[k, t], t))[:F]
        assert list(keys[k]) == want
        if k < K:
            assert pending[k + 1] not in keys[k]
    assert keys[K][0] == int(np.argmax(z[K]))                   # nothing is excluded at k = K


def test_prespeculate_branches_are_exact_greedy_continuations_and_counts():
    shape, m = _tiny()
    wl = I.WORKLOADS["tiny_f32"].round
    K, F = wl.K, wl.F
    prompt = I.make_prompt(shape, 1, 40, 3)[0]
    _, trunk = O.prefill(m, prompt[:-1])
    spec, _ = O.speculate(m, trunk, prompt[-1], K, 0.0, 0)
    pending = [int(prompt[-1])] + spec
    cache = O.prespeculate(m, trunk, pending, F, 0.0, seed=0)
    # App. C: (K+1) F outcomes, K tokens each, V logits per token
    assert cache.keys.shape == (K + 1, F) and cache.tokens.shape == (K + 1, F, K)
    assert cache.tokens.size == 1 * K * (K + 1) * F
    assert cache.tokens.size + cache.logits.size == 1 * F * K * (K + 1) * (shape.vocab + 1)
    # a second routine (full recomputation, no KV reuse) gives the same continuation per outcome
    for k in range(K + 1):
        for j in range(F):
            ctx = list(prompt) + spec[:k] + [int(cache.keys[k, j])]
            assert O.ar_generate(m, ctx, K) == list(cache.tokens[k, j])
    # the trunk after the round holds prefix + glue
    assert cache.trunk.length == len(prompt) - 1 + K + 1


def test_paper_mask_formulation_equals_one_branch_at_a_time():
    shape, m = _tiny()
    K, F = 3, 4
    prompt = I.make_prompt(shape, 1, 20, 4)[0]
    _, trunk = O.prefill(m, prompt[:-1])
    P = trunk.length
    spec, _ = O.speculate(m, trunk, prompt[-1], K, 0.0, 0)
    cache = O.prespeculate(m, trunk, [int(prompt[-1])] + spec, F, 0.0, seed=0)
    step_tokens = list(cache.keys.reshape(-1))
    earlier = O.KV.empty(m)
    for i in range(K):
        logits, kv = O.branch_step_dense(m, cache.trunk, P, K, F, i, step_tokens, earlier)
        np.testing.assert_allclose(logits, cache.logits[:, :, i].reshape((K + 1) * F, -1), atol=1e-10)
        earlier = earlier.concat(kv)
        step_tokens = list(cache.tokens[:, :, i].reshape(-1))


def test_cache_lookup_brute_force_over_every_outcome():
    g = np.random.default_rng(7)
    K, F, V = 4, 2, 1024
    keys = np.stack([g.choice(V, size=F, replace=False) for _ in range(K + 1)]).astype(np.int32)
    for k in range(K + 1):
        for t in range(V):
            j = O.cache_lookup(keys, k, t)
            if t in keys[k]:
                assert keys[k, j] == t
            else:
                assert j == -1


# ----------------------------------------------------------------- losslessness of the whole loop

@pytest.mark.parametrize("seed", [11, 12, 13])
def test_greedy_ssd_equals_greedy_autoregressive_target(seed):
    shape = I.WORKLOADS["tiny_f32"].draft
    target = O.Model.from_weights(shape, I.make_weights(shape, seed))
    tw = I.make_weights(shape, seed)
    draft = O.Model.from_weights(shape, I.make_weights(shape, seed + 50, perturb_of=tw, perturb_std=0.004))
    prompt = I.make_prompt(shape, 1, 16, seed)[0]
    n_new = 48
    want = O.ar_generate(target, prompt, n_new)
    got, stats = O.ssd_generate(target, draft, prompt, n_new, K=4, F=2)
    assert got == want
    # a close-but-different draft exercises acceptance, rejection, hits and misses
    assert 0 < stats.accepted < stats.rounds * 4
    assert 0 < stats.hits


def test_unrelated_draft_is_still_lossless():
    shape = I.WORKLOADS["tiny_f32"].draft
    target = O.Model.from_weights(shape, I.make_weights(shape, 21))
    draft = O.Model.from_weights(shape, I.make_weights(shape, 22))
    prompt = I.make_prompt(shape, 1, 12, 21)[0]
    got, stats = O.ssd_generate(target, draft, prompt, 24, K=4, F=2)
    assert got == O.ar_generate(target, prompt, 24)


def test_draft_equal_to_target_accepts_all_and_always_hits():
    shape = I.WORKLOADS["tiny_f32"].draft
    target = O.Model.from_weights(shape, I.make_weights(shape, 31))
    prompt = I.make_prompt(shape, 1, 16, 31)[0]
    got, stats = O.ssd_generate(target, target, prompt, 40, K=4, F=2)
    assert got == O.ar_generate(target, prompt, 40)
    assert all(k == 4 for k in stats.accept_lens)
    assert stats.hits == stats.rounds                            # outcome (K, top-1) is always cached


def test_saguaro_sampling_inside_the_round():
    """Sec. 4.2.1: branches decoded with sigma_{F,C}.  Pinned by consequences of the definition rather than by the
    formula: C = 1 changes nothing; under teacher forcing the returned logits differ from the model's own by exactly
    T log C on the model's top-F tokens and by nothing elsewhere; with C = 0 a top-F token is never drawn; and the
    fan-out keys (ranked on the model's own logits) do not depend on C."""
    shape, m = _tiny(7)
    wl = I.WORKLOADS["tiny_f32"].round
    K, F, T = wl.K, wl.F, 1.0
    prompt = I.make_prompt(shape, 1, 30, 4)[0]
    _, trunk = O.prefill(m, prompt[:-1])
    spec, _ = O.speculate(m, trunk, prompt[-1], K, T, 5)
    pending = [int(prompt[-1])] + spec
    base = O.prespeculate(m, trunk, pending, F, T, seed=9)
    same = O.prespeculate(m, trunk, pending, F, T, seed=9, C=1.0)
    assert np.array_equal(base.tokens, same.tokens) and np.array_equal(base.logits, same.logits)
    Cw = 0.25
    forced = O.prespeculate(m, trunk, pending, F, T, seed=9, C=Cw, forced_tokens=base.tokens)
    raw = O.prespeculate(m, trunk, pending, F, T, seed=9, forced_tokens=base.tokens)
    assert np.array_equal(forced.keys, base.keys)
    diff = forced.logits - raw.logits
    for k in range(K + 1):
        for j in range(F):
            for i in range(K):
                top = set(int(t) for t in O.top_f_ids(raw.logits[k, j, i], F))
                moved = set(int(t) for t in np.nonzero(diff[k, j, i])[0])
                assert moved == top
                np.testing.assert_allclose(diff[k, j, i][sorted(top)], T * math.log(Cw), rtol=0, atol=1e-12)
    # greedy rows are untouched by the scheme (its shift is T log C)
    g0 = O.prespeculate(m, trunk, pending, F, 0.0, seed=9)
    g1 = O.prespeculate(m, trunk, pending, F, 0.0, seed=9, C=Cw)
    assert np.array_equal(g0.tokens, g1.tokens) and np.array_equal(g0.logits, g1.logits)
    # C = 0: no drafted token is one of the F tokens the model itself ranks first at that step
    zero = O.prespeculate(m, trunk, pending, F, T, seed=9, C=0.0)
    raw0 = O.prespeculate(m, trunk, pending, F, T, seed=9, forced_tokens=zero.tokens)
    for k in range(K + 1):
        for j in range(F):
            for i in range(K):
                assert int(zero.tokens[k, j, i]) not in set(int(t) for t in O.top_f_ids(raw0.logits[k, j, i], F))


def test_greedy_ssd_with_the_random_token_backup_is_lossless():
    # Sec. 4.3: after a miss the next speculation is K random tokens; the text is still the target's own
    shape = I.WORKLOADS["tiny_f32"].draft
    tw = I.make_weights(shape, 5)
    target = O.Model.from_weights(shape, tw)
    draft = O.Model.from_weights(shape, I.make_weights(shape, 55, perturb_of=tw, perturb_std=0.004))
    prompt = I.make_prompt(shape, 1, 16, 5)[0]
    n_new = 40
    got, stats = O.ssd_generate(target, draft, prompt, n_new, K=4, F=2, backup="random")
    assert got == O.ar_generate(target, prompt, n_new)
    _, jit = O.ssd_generate(target, draft, prompt, n_new, K=4, F=2, backup="primary")
    assert 0 < stats.hits < stats.rounds            # misses happened, so random speculations were verified
    assert stats.rounds >= jit.rounds               # random tokens are (almost) never accepted: more rounds, same text
