"""Alg. 1 run for many rounds through the C-ABI on the tiny fp32 pair: every round verifies the pending speculation
with the target, pre-speculates with the draft, looks the realised outcome up, commits, and on a miss falls back to
just-in-time drafting with the same draft (Sec. 4.3: backup speculator = primary).  Only the loop is Python; every
step runs in the library's kernels.

What is fixed independently of any implementation (Sec. 2.1, lossless verification): with greedy decoding the
generated text equals the target's own greedy autoregressive text, whatever the draft proposes, and a draft that
equals the target has every speculation accepted in full and (F >= 1) every outcome in the cache."""
import numpy as np
import pytest
import torch

import ssd_inputs as I
from oracle import ssd_oracle as O
from tests.gpu_util import dev_f32, dev_i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2603_03251_amd import binding
    return binding


class Side:
    """One model with its context: trunk KV of the verified text, extend / commit."""

    def __init__(self, B, shape, weights, K, F, max_trunk):
        self.B, self.shape, self.K = B, shape, K
        self.model = B.ssd_model_create(shape, weights)
        if np.ndim(F) == 0:
            self.ctx = B.ssd_ctx_create(self.model, 1, K, F, max_trunk)
        else:
            self.ctx = B.ssd_ctx_create_fanout(self.model, 1, K, [int(f) for f in F], max_trunk)

    def close(self):
        self.B.ssd_ctx_destroy(self.ctx)
        self.B.ssd_model_destroy(self.model)

    def extend(self, tokens, offset=0):
        t = dev_i32(np.asarray(tokens, np.int32)[None, :])
        z = torch.empty((1, len(tokens), self.shape.vocab), dtype=torch.float32, device="cuda")
        self.B.ssd_ctx_extend(self.ctx, t, offset, z)
        return z

    def commit(self, k_dev):
        self.B.ssd_ctx_commit(self.ctx, k_dev)
        self.B.ssd_ctx_refresh_bounds(self.ctx)


def jit_speculate(B, draft, last, K, temps):
    """Ordinary drafting: K tokens after `last`, one forward each, greedy."""
    toks, tok = [], int(last)
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    for i in range(K):
        z = draft.extend([tok], offset=i)
        B.ssd_sample(z[0], temps, 0, 0, i, out)
        tok = int(out[0])
        toks.append(tok)
    return toks


def gpu_ssd_generate(B, target, draft, prompt, n_new, K, F, backup="primary", round_seed=lambda rnd: rnd):
    V = target.shape.vocab
    temps = dev_f32(np.zeros(1, np.float32))
    X = [int(t) for t in prompt]
    n0 = len(X)
    for side in (target, draft):
        B.ssd_ctx_prefill(side.ctx, dev_i32(np.asarray(X[:-1], np.int32)[None, :]), [n0 - 1])
    spec = jit_speculate(B, draft, X[-1], K, temps)
    acc = torch.zeros(1, dtype=torch.int32, device="cuda")
    bonus = torch.zeros(1, dtype=torch.int32, device="cuda")
    hit = torch.zeros(1, dtype=torch.uint8, device="cuda")
    branch = torch.zeros(1, dtype=torch.int32, device="cuda")
    nxt = torch.zeros((1, K), dtype=torch.int32, device="cuda")
    ws = torch.empty(B.ssd_verify_workspace_bytes(1, K), dtype=torch.uint8, device="cuda")
    s_draft, s_target = torch.cuda.Stream(), torch.cuda.Stream()
    rounds = hits = accepted = 0
    accept_lens = []
    while len(X) - n0 < n_new:
        rounds += 1
        pending = dev_i32(np.asarray([X[-1]] + spec, np.int32)[None, :])
        torch.cuda.synchronize()
        # the target verifies on one stream while the draft pre-speculates on the other
        zt = torch.empty((1, K + 1, V), dtype=torch.float32, device="cuda")
        B.ssd_ctx_extend(target.ctx, pending, 0, zt, stream=s_target)
        B.ssd_verify(zt, None, pending[:, 1:].contiguous(), temps, round_seed(rounds), acc, bonus, ws, stream=s_target)
        B.ssd_prespeculate(draft.ctx, pending, temps, round_seed(rounds), stream=s_draft)
        torch.cuda.synchronize()
        B.ssd_cache_lookup(draft.ctx, acc, bonus, hit, branch, nxt)
        torch.cuda.synchronize()
        k, t = int(acc[0]), int(bonus[0])
        X += spec[:k] + [t]
        accepted += k
        accept_lens.append(k)
        target.commit(acc)
        draft.commit(acc)
        if int(hit[0]):
            hits += 1
            spec = [int(x) for x in nxt[0].cpu().numpy()]
        elif backup == "primary":
            spec = jit_speculate(B, draft, t, K, temps)
        else:
            B.ssd_backup_random(round_seed(rounds), V, nxt)
            spec = [int(x) for x in nxt[0].cpu().numpy()]
    return X[n0:n0 + n_new], dict(rounds=rounds, hits=hits, accepted=accepted, accept_lens=accept_lens)


def test_greedy_ssd_text_equals_the_targets_autoregressive_text(B):
    wl = I.WORKLOADS["tiny_f32"]
    shape, K, F = wl.draft, wl.round.K, wl.round.F
    n_new, P = 40, 24
    wt = I.make_weights(shape, 11)
    wd = I.make_weights(shape, 12, perturb_of=wt, perturb_std=0.002)     # a draft close to, not equal to, its target
    prompt = I.make_prompt(shape, 1, P, 21)[0]
    ot, od = O.Model.from_weights(shape, wt), O.Model.from_weights(shape, wd)
    want = O.ar_generate(ot, prompt, n_new)
    want_ssd, st = O.ssd_generate(ot, od, prompt, n_new, K, F)
    assert want_ssd == want                                              # the oracle's own invariant
    target = Side(B, shape, wt, K, 1, P + n_new + 4 * K + 8)
    draft = Side(B, shape, wd, K, F, P + n_new + 4 * K + 8)
    try:
        got, gs = gpu_ssd_generate(B, target, draft, prompt, n_new, K, F)
        print(f"[gpu] rounds {gs['rounds']} hits {gs['hits']} accept lengths {gs['accept_lens']}", flush=True)
        print(f"[oracle] rounds {st.rounds} hits {st.hits} accept lengths {st.accept_lens}", flush=True)
        assert got == want
        # the same decisions round by round (fp32 logits against float64: no near-tie in this seeded run)
        assert gs["accept_lens"] == st.accept_lens and gs["hits"] == st.hits
        assert len(set(gs["accept_lens"])) >= 4 and 0 < gs["hits"] < gs["rounds"]      # accept lengths 0..K, hits and misses
    finally:
        target.close()
        draft.close()


def test_identical_draft_has_everything_accepted_and_every_outcome_cached(B):
    wl = I.WORKLOADS["tiny_f32"]
    shape, K, F = wl.draft, wl.round.K, wl.round.F
    n_new, P = 30, 17
    w = I.make_weights(shape, 31)
    prompt = I.make_prompt(shape, 1, P, 22)[0]
    want = O.ar_generate(O.Model.from_weights(shape, w), prompt, n_new)
    target = Side(B, shape, w, K, 1, P + n_new + 4 * K + 8)
    draft = Side(B, shape, w, K, F, P + n_new + 4 * K + 8)
    try:
        got, gs = gpu_ssd_generate(B, target, draft, prompt, n_new, K, F)
        assert got == want
        assert all(k == K for k in gs["accept_lens"])
        assert gs["hits"] == gs["rounds"]                                   # the bonus token is the draft's own top choice
        assert gs["rounds"] == -(-n_new // (K + 1))
    finally:
        target.close()
        draft.close()


def test_greedy_ssd_with_a_geometric_cache_is_lossless_and_decides_like_the_oracle(B):
    """Sec. 4.1.2: the cache shape changes which outcomes hit, never the text."""
    wl = I.WORKLOADS["tiny_f32"]
    shape, K = wl.draft, wl.round.K
    fan = B.ssd_geometric_fanout((K + 1) * wl.round.F, K, 0.6, 0.5, 8)
    assert len(set(fan)) > 1
    n_new, P = 40, 24
    wt = I.make_weights(shape, 11)
    wd = I.make_weights(shape, 12, perturb_of=wt, perturb_std=0.002)
    prompt = I.make_prompt(shape, 1, P, 21)[0]
    ot, od = O.Model.from_weights(shape, wt), O.Model.from_weights(shape, wd)
    want = O.ar_generate(ot, prompt, n_new)
    _, st = O.ssd_generate(ot, od, prompt, n_new, K, fan)
    target = Side(B, shape, wt, K, 1, P + n_new + 4 * K + 8)
    draft = Side(B, shape, wd, K, fan, P + n_new + 4 * K + 8)
    try:
        got, gs = gpu_ssd_generate(B, target, draft, prompt, n_new, K, fan)
        print(f"[gpu] fan-out {fan}: rounds {gs['rounds']} hits {gs['hits']} accept lengths {gs['accept_lens']}", flush=True)
        assert got == want
        assert gs["accept_lens"] == st.accept_lens and gs["hits"] == st.hits
    finally:
        target.close()
        draft.close()


def test_greedy_ssd_with_the_random_token_backup_decides_like_the_oracle(B):
    """Sec. 4.3: the low-latency backup speculator.  Same random tokens as the oracle's (same generator, same round
    seeds), so the same accept lengths and hits round by round, and the target's own text."""
    wl = I.WORKLOADS["tiny_f32"]
    shape, K, F = wl.draft, wl.round.K, wl.round.F
    n_new, P = 40, 24
    wt = I.make_weights(shape, 11)
    wd = I.make_weights(shape, 12, perturb_of=wt, perturb_std=0.002)
    prompt = I.make_prompt(shape, 1, P, 21)[0]
    ot, od = O.Model.from_weights(shape, wt), O.Model.from_weights(shape, wd)
    want = O.ar_generate(ot, prompt, n_new)
    _, st = O.ssd_generate(ot, od, prompt, n_new, K, F, seed=0, backup="random")
    target = Side(B, shape, wt, K, 1, P + 2 * n_new + 4 * K + 8)
    draft = Side(B, shape, wd, K, F, P + 2 * n_new + 4 * K + 8)
    try:
        got, gs = gpu_ssd_generate(B, target, draft, prompt, n_new, K, F, backup="random",
                                   round_seed=lambda rnd: 1000003 * rnd)          # the oracle's round seeds
        print(f"[gpu] rounds {gs['rounds']} hits {gs['hits']} accept lengths {gs['accept_lens']}", flush=True)
        assert got == want
        assert gs["accept_lens"] == st.accept_lens and gs["hits"] == st.hits
        assert 0 < gs["hits"] < gs["rounds"]
    finally:
        target.close()
        draft.close()


def test_greedy_ssd_for_a_batch_whose_sequences_diverge(B):
    """Alg. 1 for three sequences in one context pair: accept lengths, hits and misses differ per sequence, so the
    trunk lengths drift apart round by round (the per-sequence rollback of App. B).  Every sequence must still
    reproduce its own greedy autoregressive text."""
    wl = I.WORKLOADS["tiny_f32"]
    shape, K, F = wl.draft, wl.round.K, wl.round.F
    nb, n_new, P, V = 3, 30, 18, wl.draft.vocab
    wt = I.make_weights(shape, 41)
    wd = I.make_weights(shape, 42, perturb_of=wt, perturb_std=0.003)
    prompts = I.make_prompt(shape, nb, P, 23)
    lens = [P, P - 5, P - 9]
    ot = O.Model.from_weights(shape, wt)
    want = [O.ar_generate(ot, prompts[b][:lens[b]], n_new) for b in range(nb)]
    cap = P + n_new + 5 * K + 8
    mt, md = B.ssd_model_create(shape, wt), B.ssd_model_create(shape, wd)
    ct, cd = B.ssd_ctx_create(mt, nb, K, 1, cap), B.ssd_ctx_create(md, nb, K, F, cap)
    try:
        X = [[int(t) for t in prompts[b][:lens[b]]] for b in range(nb)]
        body = np.zeros((nb, P), np.int32)
        for b in range(nb):
            body[b, :lens[b] - 1] = X[b][:-1]
        for c in (ct, cd):
            B.ssd_ctx_prefill(c, dev_i32(body), [n - 1 for n in lens])
        temps = dev_f32(np.zeros(nb, np.float32))
        out = torch.zeros(nb, dtype=torch.int32, device="cuda")

        def jit(last):                               # K greedy tokens after `last` for every sequence, one extend each
            toks, cur = [], np.asarray(last, np.int32)
            for i in range(K):
                z = torch.empty((nb, 1, V), dtype=torch.float32, device="cuda")
                B.ssd_ctx_extend(cd, dev_i32(cur[:, None]), i, z)
                B.ssd_sample(z[:, 0].contiguous(), temps, 0, 0, i, out)
                cur = out.cpu().numpy().copy()
                toks.append(cur)
            return np.stack(toks, axis=1)            # [nb][K]

        spec = jit([x[-1] for x in X])
        acc = torch.zeros(nb, dtype=torch.int32, device="cuda")
        bonus = torch.zeros(nb, dtype=torch.int32, device="cuda")
        hit = torch.zeros(nb, dtype=torch.uint8, device="cuda")
        branch = torch.zeros(nb, dtype=torch.int32, device="cuda")
        nxt = torch.zeros((nb, K), dtype=torch.int32, device="cuda")
        ws = torch.empty(B.ssd_verify_workspace_bytes(nb, K), dtype=torch.uint8, device="cuda")
        rounds, accept_sets, hits = 0, [set() for _ in range(nb)], np.zeros(nb, int)
        while min(len(X[b]) - lens[b] for b in range(nb)) < n_new:
            rounds += 1
            pending = dev_i32(np.concatenate([np.array([[x[-1]] for x in X], np.int32), spec], axis=1))
            zt = torch.empty((nb, K + 1, V), dtype=torch.float32, device="cuda")
            B.ssd_ctx_extend(ct, pending, 0, zt)
            B.ssd_verify(zt, None, pending[:, 1:].contiguous(), temps, rounds, acc, bonus, ws)
            B.ssd_prespeculate(cd, pending, temps, rounds)
            B.ssd_cache_lookup(cd, acc, bonus, hit, branch, nxt)
            torch.cuda.synchronize()
            k, t, h = acc.cpu().numpy(), bonus.cpu().numpy(), hit.cpu().numpy()
            for b in range(nb):
                X[b] += [int(s) for s in spec[b, :k[b]]] + [int(t[b])]
                accept_sets[b].add(int(k[b]))
            hits += h
            for c in (ct, cd):
                B.ssd_ctx_commit(c, acc)
                B.ssd_ctx_refresh_bounds(c)
            cached = nxt.cpu().numpy()
            fresh = jit(t) if not h.all() else cached
            spec = np.where(h[:, None].astype(bool), cached, fresh).astype(np.int32)
        for b in range(nb):
            assert X[b][lens[b]:lens[b] + n_new] == want[b], b
        tl = B.read_cache(cd, with_logits=False)["trunk_len"].cpu().numpy()
        assert list(tl) == [len(x) - 1 for x in X] and len(set(tl)) > 1          # the sequences have drifted apart
        assert all(len(s) >= 2 for s in accept_sets) and 0 < hits.sum() < rounds * nb
    finally:
        B.ssd_ctx_destroy(ct)
        B.ssd_ctx_destroy(cd)
        B.ssd_model_destroy(mt)
        B.ssd_model_destroy(md)


SMALL_BF16 = I.ModelShape(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1024,
                          vocab=4112, dtype="bf16", rope_theta=500000.0, tie_embeddings=True)


def gpu_ar_generate(B, side, prompt, n_new):
    """The model's own greedy autoregressive text on the GPU: one single-token extend per token."""
    X = [int(t) for t in prompt]
    B.ssd_ctx_prefill(side.ctx, dev_i32(np.asarray(X[:-1], np.int32)[None, :]), [len(X) - 1])
    temps = dev_f32(np.zeros(1, np.float32))
    out = torch.zeros(1, dtype=torch.int32, device="cuda")
    zero = torch.zeros(1, dtype=torch.int32, device="cuda")
    for _ in range(n_new):
        z = side.extend([X[-1]])
        B.ssd_sample(z[0], temps, 0, 0, 0, out)
        X.append(int(out[0]))
        side.commit(zero)                              # accept length 0: the trunk grows by the one token
    return X[len(prompt):]


def test_bf16_pair_on_the_fused_pass_hundreds_of_rounds_greedy(B):
    """Alg. 1 for more than 200 rounds on a small bf16 pair whose every forward (prefill chunks, verification extends, glue
    extends, branch steps) runs through the persistent fused pass.  Losslessness (Sec. 2.1): the text equals the same
    target's own greedy autoregressive text, computed on the same GPU token by token; all accept lengths, hits and
    misses occur on the way, and the trunk walks across dozens of 32-position blocks of the value layout."""
    shape, K, F, P, n_new = SMALL_BF16, 4, 3, 19, 1100
    wt = I.make_weights(shape, 41)
    wd = I.make_weights(shape, 42, perturb_of=wt, perturb_std=0.006)
    prompt = I.make_prompt(shape, 1, P, 43)[0]
    cap = P + n_new + 4 * K + 8
    ref = Side(B, shape, wt, K, 1, cap)
    try:
        assert B.ssd_ctx_views(ref.ctx).fused_pass == 2
        want = gpu_ar_generate(B, ref, prompt, n_new)
    finally:
        ref.close()
    target, draft = Side(B, shape, wt, K, 1, cap), Side(B, shape, wd, K, F, cap)
    try:
        assert B.ssd_ctx_views(draft.ctx).fused_pass == 2 and B.ssd_ctx_views(target.ctx).fused_pass == 2
        got, gs = gpu_ssd_generate(B, target, draft, prompt, n_new, K, F)
        hist = np.bincount(gs["accept_lens"], minlength=K + 1)
        print(f"[gpu bf16] rounds {gs['rounds']} hits {gs['hits']} accepted {gs['accepted']} accept-length histogram {hist.tolist()}",
              flush=True)
        assert got == want
        # (a random-init model soon repeats itself, so accept lengths cluster at 0 and K; the ones between still occur)
        assert gs["rounds"] >= 200 and (hist > 0).sum() >= 3 and 0 < gs["hits"] < gs["rounds"]
        B.ssd_ctx_status(draft.ctx)
        B.ssd_ctx_status(target.ctx)
    finally:
        target.close()
        draft.close()


def test_bf16_pair_sampled_rounds_decide_like_the_oracle_on_the_same_logits(B):
    """Alg. 1 at temperature 0.25 on the bf16 pair: every round's verification outcome (k, t*) equals what the oracle's
    rejection sampling decides on the very logits the kernels produced (target's verification logits, and the logits the
    pending speculation was drawn from: the cache's on a hit, the just-in-time ones on a miss), near-ties excepted; hits
    and misses both occur, and the trunk lengths of both sides stay in step with the text."""
    shape, K, F, P, T, n_rounds = SMALL_BF16, 3, 8, 23, 0.25, 40
    wt = I.make_weights(shape, 51)
    wd = I.make_weights(shape, 52, perturb_of=wt, perturb_std=0.003)
    prompt = [int(t) for t in I.make_prompt(shape, 1, P, 53)[0]]
    V = shape.vocab
    cap = P + n_rounds * (K + 1) + 4 * K + 8
    target, draft = Side(B, shape, wt, K, 1, cap), Side(B, shape, wd, K, F, cap)
    temps = dev_f32(np.full(1, T, np.float32))
    acc = torch.zeros(1, dtype=torch.int32, device="cuda")
    bonus = torch.zeros(1, dtype=torch.int32, device="cuda")
    hit = torch.zeros(1, dtype=torch.uint8, device="cuda")
    branch = torch.zeros(1, dtype=torch.int32, device="cuda")
    nxt = torch.zeros((1, K), dtype=torch.int32, device="cuda")
    ptr = torch.zeros(1, dtype=torch.int64, device="cuda")
    ws = torch.empty(B.ssd_verify_workspace_bytes(1, K), dtype=torch.uint8, device="cuda")
    out = torch.zeros(1, dtype=torch.int32, device="cuda")

    def jit(last, seed):
        toks, logits, tok = [], [], int(last)
        for i in range(K):
            z = draft.extend([tok], offset=i)
            B.ssd_sample(z[0], temps, seed, 0, i, out)
            tok = int(out[0])
            toks.append(tok)
            logits.append(z[0, 0].clone())
        return toks, torch.stack(logits)[None].contiguous()

    try:
        X = list(prompt)
        for side in (target, draft):
            B.ssd_ctx_prefill(side.ctx, dev_i32(np.asarray(X[:-1], np.int32)[None, :]), [len(X) - 1])
        spec, zd = jit(X[-1], 7)
        s_draft, s_target = torch.cuda.Stream(), torch.cuda.Stream()
        hits = n_checked = 0
        ks = []
        for rnd in range(1, n_rounds + 1):
            pending = dev_i32(np.asarray([X[-1]] + spec, np.int32)[None, :])
            zt = torch.empty((1, K + 1, V), dtype=torch.float32, device="cuda")
            torch.cuda.synchronize()
            B.ssd_ctx_extend(target.ctx, pending, 0, zt, stream=s_target)
            B.ssd_verify(zt, zd, pending[:, 1:].contiguous(), temps, 1000 + rnd, acc, bonus, ws, stream=s_target)
            B.ssd_prespeculate(draft.ctx, pending, temps, 1000 + rnd, stream=s_draft)
            torch.cuda.synchronize()
            k, t = int(acc[0]), int(bonus[0])
            tr = O.verify(zt[0].cpu().numpy().astype(np.float64), zd[0].cpu().numpy().astype(np.float64), spec, T, 1000 + rnd, 0)
            if min(tr.accept_margin + [1.0]) > 1e-4 and tr.bonus_margin > 1e-4:
                assert (k, t) == (tr.accept_len, tr.bonus), (rnd, k, t, tr)
                n_checked += 1
            B.ssd_cache_lookup(draft.ctx, acc, bonus, hit, branch, nxt, ptr)
            torch.cuda.synchronize()
            X += spec[:k] + [t]
            ks.append(k)
            target.commit(acc)
            draft.commit(acc)
            tl = [int(B.read_cache(s.ctx, with_logits=False)["trunk_len"][0]) for s in (target, draft)]
            assert tl == [len(X) - 1, len(X) - 1]
            if int(hit[0]):
                hits += 1
                spec = [int(x) for x in nxt[0].cpu().numpy()]
                # the hit branch's logits leave the cache before the next round rewrites it (the payload of App. B)
                zd = B.device_copy(int(ptr[0]), (1, K, V), torch.float32)
            else:
                spec, zd = jit(t, 2000 + rnd)
        print(f"[gpu bf16 sampled] {n_rounds} rounds, {hits} hits, accept lengths {ks}, {n_checked} outcomes compared", flush=True)
        assert n_checked >= n_rounds - 2 and 0 < hits < n_rounds and len(set(ks)) >= 3
    finally:
        target.close()
        draft.close()
