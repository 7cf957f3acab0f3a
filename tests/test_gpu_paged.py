"""Paged trunk KV, block tables, page rollback and the join / leave of sequences (App. B: the paged attention and
continuous batching the paper's system inherits from its serving stack).

A paged context computes with the same kernels in the same order as a contiguous one and only addresses the stored keys
through its block table, so the bar is bit equality with the contiguous context (which the other parity tests hold to
the oracle), whatever order the pages were handed out in; one round is also compared with the oracle directly."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import ssd_inputs as I
from oracle import ssd_oracle as O
from tests.gpu_util import TOL, TOL_BF16_OWN_PREFILL, dev_f32, dev_i32, row_rel_err

pytestmark = pytest.mark.gpu

SMALL_BF16 = I.ModelShape(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1024,
                          vocab=4112, dtype="bf16", rope_theta=500000.0, tie_embeddings=True)
NAMES = ("keys", "tokens", "logits", "hidden", "glue_logits", "trunk_len")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_03251_amd import binding
    return binding


def _cache(B, ctx):
    return {k: v.cpu().numpy() for k, v in B.read_cache(ctx).items()}


def _pages_in_use(lens):
    return sum((n + 31) // 32 for n in lens)


def _scramble_pool(B, ctx, shape, batch, seed):
    """Take and return pages in an interleaved order, so that the blocks of a sequence end up scattered over the pool."""
    rng = np.random.default_rng(seed)
    total, free = B.ssd_ctx_kv_pages(ctx)
    for b, n in enumerate(rng.permutation(batch)):
        B.ssd_ctx_prefill_sequence(ctx, int(n), dev_i32(I.make_prompt(shape, 1, 33 + 32 * b, seed + b)[0]))
    for n in rng.permutation(batch):
        B.ssd_ctx_release_sequence(ctx, int(n))
    assert B.ssd_ctx_kv_pages(ctx) == (total, free)


@pytest.mark.parametrize("name,batch,K,F,lens", [
    ("narrow passes", 2, 3, 2, [61, 30]),
    ("wide passes", 3, 4, 5, [70, 33, 95]),
])
def test_paged_trunk_equals_contiguous_trunk_over_rounds_with_rollback(B, name, batch, K, F, lens):
    """Five rounds with accept lengths that walk the trunks over page boundaries, in a contiguous context and in a
    paged one whose pool was scrambled first: the same bits in every output of every round, and after each refresh the
    pool holds exactly the pages of the verified text (the pages behind it were rolled back)."""
    shape, seed = SMALL_BF16, 41
    w = I.make_weights(shape, seed)
    model = B.ssd_model_create(shape, w)
    max_trunk = max(lens) + 6 * (K + 1) + 2 * K + 4
    n_pages = 1 + _pages_in_use([n + 7 * (K + 1) for n in lens])
    plain = B.ssd_ctx_create(model, batch, K, F, max_trunk)
    paged = B.ssd_ctx_create(model, batch, K, F, max_trunk, 0, n_pages)
    try:
        assert B.ssd_ctx_kv_pages(plain) == (0, 0)
        assert B.ssd_ctx_kv_pages(paged) == (n_pages, n_pages - 1)
        assert B.ssd_ctx_views(paged).pass_rows == (48 if name == "narrow passes" else 384)
        _scramble_pool(B, paged, shape, batch, seed)
        prompt = I.make_prompt(shape, batch, max(lens), seed)
        for ctx in (plain, paged):
            B.ssd_ctx_prefill(ctx, dev_i32(prompt), lens)
        assert B.ssd_ctx_kv_pages(paged)[1] == n_pages - 1 - _pages_in_use(lens)
        temps = dev_f32(np.zeros(batch, np.float32))
        now = list(lens)
        rng = np.random.default_rng(seed)
        for rnd in range(5):
            accepts = [K, 0, 2][:batch] if rnd == 0 else [int(a) for a in rng.integers(0, K + 1, batch)]
            pending = dev_i32(I.make_pending(shape, batch, K, seed + rnd))
            outs = []
            for ctx in (plain, paged):
                B.ssd_prespeculate(ctx, pending, temps, rnd)
                outs.append(_cache(B, ctx))
                B.ssd_ctx_commit(ctx, dev_i32(np.array(accepts, np.int32)))
                B.ssd_ctx_refresh_bounds(ctx)
            for key in NAMES:
                assert np.array_equal(outs[0][key], outs[1][key]), (rnd, key)
            now = [n + a + 1 for n, a in zip(now, accepts)]
            assert B.ssd_ctx_kv_pages(paged)[1] == n_pages - 1 - _pages_in_use(now), (rnd, now)
        # rollback by hand: every sequence back to a prefix; the pages behind it return
        back = [max(1, n - 40) for n in now]
        for ctx in (plain, paged):
            B.ssd_ctx_truncate_trunk(ctx, back)
            B.ssd_prespeculate(ctx, pending, temps, 9)
        assert B.ssd_ctx_kv_pages(paged)[1] == n_pages - 1 - _pages_in_use([n + K + 1 for n in back])
        a, b_ = _cache(B, plain), _cache(B, paged)
        for key in NAMES:
            assert np.array_equal(a[key], b_[key]), ("after truncate", key)
    finally:
        B.ssd_ctx_destroy(plain)
        B.ssd_ctx_destroy(paged)
        B.ssd_model_destroy(model)


def test_paged_round_against_the_oracle(B):
    """One round of a paged context (scrambled pool, ragged prompts prefilled on the GPU) against the float64 oracle."""
    shape, seed, batch, K, F, lens = SMALL_BF16, 43, 3, 3, 2, [45, 2, 67]
    w = I.make_weights(shape, seed)
    om = O.Model.from_weights(shape, w)
    model = B.ssd_model_create(shape, w)
    ctx = B.ssd_ctx_create(model, batch, K, F, 128, 0, 12)
    try:
        _scramble_pool(B, ctx, shape, batch, seed)
        prompt = I.make_prompt(shape, batch, max(lens), seed)
        B.ssd_ctx_prefill(ctx, dev_i32(prompt), lens)
        pending = I.make_pending(shape, batch, K, seed)
        caches = []
        for b in range(batch):
            _, trunk = O.prefill(om, prompt[b, :lens[b]])
            caches.append(O.prespeculate(om, trunk, pending[b], F, 0.0, seed=seed, row_base=b * (K + 1) * F))
        # (the context keeps the pointers, not the tensors: they stay alive in these names until the round has run)
        f_keys, f_toks = dev_i32(np.stack([c.keys for c in caches])), dev_i32(np.stack([c.tokens for c in caches]))
        B.ssd_ctx_set_forced(ctx, f_keys, f_toks)
        B.ssd_prespeculate(ctx, dev_i32(pending), dev_f32(np.zeros(batch, np.float32)), seed)
        B.ssd_ctx_set_forced(ctx, None, None)
        got = _cache(B, ctx)
        for b in range(batch):
            e_g = row_rel_err(got["glue_logits"][b], caches[b].glue_logits)
            e_l = row_rel_err(got["logits"][b], caches[b].logits)
            print(f"[paged] seq {b}: glue {e_g:.3e}, branches {e_l:.3e}", flush=True)
            assert e_g < TOL_BF16_OWN_PREFILL and e_l < TOL_BF16_OWN_PREFILL and e_l < TOL["bf16"]
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


@pytest.mark.parametrize("pages", [0, 14, -1])
def test_a_sequence_leaves_and_another_joins_its_slot(B, pages):
    """Continuous batching: after a round, sequence 1 finishes and a new request takes its slot while sequences 0 and 2
    keep their trunks.  The next round equals, bit for bit, the round of a context in which the three requests were
    placed directly; in the paged context the leaver's pages are back in the pool in between."""
    shape, seed, batch, K, F = SMALL_BF16, 47, 3, 3, 2
    lens, new_len = [40, 90, 33], 52
    w = I.make_weights(shape, seed)
    model = B.ssd_model_create(shape, w)
    prompts = [I.make_prompt(shape, 1, n, seed + i)[0] for i, n in enumerate(lens)]
    joiner = I.make_prompt(shape, 1, new_len, seed + 9)[0]
    temps = dev_f32(np.zeros(batch, np.float32))
    pending = dev_i32(I.make_pending(shape, batch, K, seed))
    flags = B.SSD_CTX_PER_OPERATOR if pages < 0 else 0     # -1: the same on the per-operator kernels (contiguous trunk)
    pages = max(pages, 0)
    direct = B.ssd_ctx_create(model, batch, K, F, 128, flags)
    served = B.ssd_ctx_create(model, batch, K, F, 128, flags, pages)
    try:
        for b, toks in enumerate([prompts[0], joiner, prompts[2]]):
            B.ssd_ctx_prefill_sequence(direct, b, dev_i32(toks))
        B.ssd_prespeculate(direct, pending, temps, 1)
        want = _cache(B, direct)

        for b, toks in enumerate(prompts):
            B.ssd_ctx_prefill_sequence(served, b, dev_i32(toks))
        B.ssd_prespeculate(served, pending, temps, 0)
        first = _cache(B, served)
        B.ssd_ctx_refresh_bounds(served)
        if pages:
            assert B.ssd_ctx_kv_pages(served)[1] == pages - 1 - _pages_in_use(lens)
        B.ssd_ctx_release_sequence(served, 1)
        if pages:
            assert B.ssd_ctx_kv_pages(served)[1] == pages - 1 - _pages_in_use([lens[0], lens[2]])
        with pytest.raises(B.SsdError):          # a round with an empty slot is refused
            B.ssd_prespeculate(served, pending, temps, 1)
        B.ssd_ctx_prefill_sequence(served, 1, dev_i32(joiner))
        B.ssd_prespeculate(served, pending, temps, 1)
        got = _cache(B, served)
        assert list(got["trunk_len"]) == [lens[0], new_len, lens[2]]
        for key in NAMES:
            assert np.array_equal(got[key], want[key]), key
        # the stayers' outcomes did not depend on their neighbour: same glue logits before and after the change
        for b in (0, 2):
            assert np.array_equal(first["glue_logits"][b], got["glue_logits"][b])
    finally:
        B.ssd_ctx_destroy(direct)
        B.ssd_ctx_destroy(served)
        B.ssd_model_destroy(model)


def test_pool_exhaustion_is_an_error_and_recoverable(B):
    shape, seed, batch, K, F = SMALL_BF16, 53, 3, 3, 2
    w = I.make_weights(shape, seed)
    model = B.ssd_model_create(shape, w)
    # 6 usable pages: two sequences of 70 positions take 3 each
    ctx = B.ssd_ctx_create(model, batch, K, F, 128, 0, 7)
    try:
        toks = dev_i32(I.make_prompt(shape, 1, 70, seed)[0])
        B.ssd_ctx_prefill_sequence(ctx, 0, toks)
        B.ssd_ctx_prefill_sequence(ctx, 1, toks)
        assert B.ssd_ctx_kv_pages(ctx) == (7, 0)
        with pytest.raises(B.SsdError) as err:
            B.ssd_ctx_prefill_sequence(ctx, 2, toks)
        assert err.value.status == -4 and "out of KV pages" in str(err.value)
        B.ssd_ctx_release_sequence(ctx, 2)       # gives back what the failed call had taken (nothing here)
        B.ssd_ctx_release_sequence(ctx, 0)
        assert B.ssd_ctx_kv_pages(ctx) == (7, 3)
        B.ssd_ctx_prefill_sequence(ctx, 2, toks[:60])
        assert B.ssd_ctx_kv_pages(ctx) == (7, 1)
        assert list(B.read_cache(ctx)["trunk_len"].cpu().numpy()) == [0, 70, 60]
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)
    with pytest.raises(B.SsdError):      # the per-operator path has no paged trunk
        c2 = None
        m2 = B.ssd_model_create(shape, w)
        try:
            c2 = B.ssd_ctx_create(m2, 1, K, F, 128, B.SSD_CTX_PER_OPERATOR, 8)
        finally:
            if c2:
                B.ssd_ctx_destroy(c2)
            B.ssd_model_destroy(m2)


@pytest.mark.parametrize("name,P,nb,F,ragged", [
    ("headline shape", 1024, 1, 4, False),
    ("long prefix, key splits and merge", 8192, 1, 8, False),
    ("batch 16, wide passes, ragged", 2048, 16, 4, True),
])
def test_full_size_paged_round_equals_contiguous_round(B, name, P, nb, F, ragged):
    """The 1B-shaped workloads of the benchmark with the trunk in pages handed out in a shuffled order: two rounds with
    a commit between them give the bits of the contiguous trunk (logits, hidden states, tokens, keys)."""
    shape, K, seed = I.LLAMA_1B, 5, 61
    g = np.random.default_rng(P + nb)
    lens = [int(x) for x in g.integers(200, P + 1, nb)] if ragged else [P] * nb
    max_trunk = P + 4 * K + 8
    n_pages = 1 + sum((n + 3 * (K + 1) + 31) // 32 for n in lens) + 2 * nb
    model = B.ssd_model_create_random(shape, seed)
    outs = []
    try:
        for pages in (0, n_pages):
            ctx = B.ssd_ctx_create(model, nb, K, F, max_trunk, 0, pages)
            try:
                if pages:
                    # shuffle the free list: take pages for every slot in turn, return them slot by slot in another order
                    for b in g.permutation(nb):
                        B.ssd_ctx_prefill_sequence(ctx, int(b), dev_i32(I.make_prompt(shape, 1, 30 + int(b), seed)[0]))
                    for b in g.permutation(nb):
                        B.ssd_ctx_release_sequence(ctx, int(b))
                B.ssd_ctx_fill_synthetic_kv(ctx, lens, seed + 1)
                temps = dev_f32(np.full(nb, 0.0, np.float32))
                got = []
                for rnd in range(2):
                    B.ssd_prespeculate(ctx, dev_i32(I.make_pending(shape, nb, K, seed + rnd)), temps, rnd)
                    got.append({k: v.clone() for k, v in B.read_cache(ctx).items()})
                    B.ssd_ctx_commit(ctx, dev_i32(np.asarray([(b + rnd) % (K + 1) for b in range(nb)], np.int32)))
                    B.ssd_ctx_refresh_bounds(ctx)
                outs.append(got)
                if pages:
                    total, free = B.ssd_ctx_kv_pages(ctx)
                    now = [n + b % (K + 1) + 1 + (b + 1) % (K + 1) + 1 for b, n in enumerate(lens)]
                    assert free == total - 1 - _pages_in_use(now)
            finally:
                B.ssd_ctx_destroy(ctx)
        for rnd in range(2):
            for key in NAMES:
                assert torch.equal(outs[0][rnd][key], outs[1][rnd][key]), (name, rnd, key)
            assert bool(torch.isfinite(outs[1][rnd]["logits"]).all())
    finally:
        B.ssd_model_destroy(model)
