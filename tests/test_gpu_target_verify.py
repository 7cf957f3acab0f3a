"""The target's side of a round at the 70B layer shape (Sec. 2.1 and Alg. 1: verification of K speculated tokens is one forward
of the target over K+1 positions, running while the draft pre-speculates).

The oracle cannot run 80 layers of this shape in seconds, so parity is taken on a model with the 70B per-layer shape
(d 8192, 64 query / 8 KV heads of 128, FFN 28672) but 2 layers and a 16384-token vocabulary: every kernel runs at its
real shape, only the layer loop and the LM head are shorter.  The full-depth model is timed by
`bench.py --workload 70b_verify_1b_draft`, not compared ("parity unpinned" at 80 layers)."""
import numpy as np
import pytest
import torch

import ssd_inputs as I
from oracle import ssd_oracle as O
from tests.gpu_util import TOL, dev_f32, dev_i32, kv_to_device, oracle_trunk_from_arrays, row_rel_err

pytestmark = pytest.mark.gpu

TARGET_2L = I.ModelShape(n_layers=2, d_model=8192, n_q_heads=64, n_kv_heads=8, head_dim=128, d_ffn=28672,
                         vocab=16384, dtype="bf16", rope_theta=500000.0, tie_embeddings=False)


@pytest.fixture(scope="module")
def B():
    from paper_2603_03251_amd import binding
    return binding


def test_target_forward_over_pending_block_and_verify(B):
    shape, P, K, seed = TARGET_2L, 300, 5, 77
    print(f"[case] target verify forward: 70B layer shape x {shape.n_layers} layers, prefix {P}, K={K}", flush=True)
    w = I.make_weights(shape, seed)
    print("[weights] generated", flush=True)
    model = B.ssd_model_create(shape, w)
    om = O.Model.from_weights(shape, w)
    del w
    k, v = I.make_prefix_kv(shape, 1, P, seed)
    ctx = B.ssd_ctx_create(model, 1, K, 1, P + 2 * K + 2)
    try:
        B.ssd_ctx_load_trunk(ctx, kv_to_device(k, "bf16"), kv_to_device(v, "bf16"), P)
        pending = I.make_pending(shape, 1, K, seed)                      # {last verified token, s_1..s_K}
        want, _, _ = O.glue_extend(om, oracle_trunk_from_arrays(om, k, v, 0), pending[0])
        print("[oracle] done", flush=True)
        logits = torch.empty((1, K + 1, shape.vocab), dtype=torch.float32, device="cuda")
        B.ssd_ctx_extend(ctx, dev_i32(pending), 0, logits)
        torch.cuda.synchronize()
        got = logits.cpu().numpy()[0]
        e = row_rel_err(got, want)
        print(f"[target logits] rel err {e:.3e}", flush=True)
        assert e < TOL["bf16"]

        # greedy verification of the pending block against these logits (Sec. 2.1): accept while the target's argmax
        # equals the speculated token; compared where the GPU's logit error cannot flip the argmax
        spec = pending[:, 1:]
        tr = O.verify(want, None, spec[0], 0.0, seed, 0)
        acc = torch.zeros(1, dtype=torch.int32, device="cuda")
        bonus = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = torch.empty(B.ssd_verify_workspace_bytes(1, K), dtype=torch.uint8, device="cuda")
        B.ssd_verify(logits, None, dev_i32(spec), dev_f32(np.zeros(1, np.float32)), seed, acc, bonus, ws)
        torch.cuda.synchronize()
        err = np.abs(got - want).max(axis=-1)
        top2 = np.sort(want, axis=-1)[:, -2:]
        decided = (top2[:, 1] - top2[:, 0]) > 2 * err
        if decided[: tr.accept_len + 1].all():
            assert int(acc[0]) == tr.accept_len and int(bonus[0]) == tr.bonus
        # and bit-exactly on the oracle's own logits (as fp32, the type the kernel consumes)
        want32 = want.astype(np.float32)
        tr32 = O.verify(want32.astype(np.float64), None, spec[0], 0.0, seed, 0)
        B.ssd_verify(dev_f32(want32[None]), None, dev_i32(spec), dev_f32(np.zeros(1, np.float32)), seed, acc, bonus, ws)
        torch.cuda.synchronize()
        assert int(acc[0]) == tr32.accept_len and int(bonus[0]) == tr32.bonus
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


DRAFT_SMALL = I.ModelShape(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1024, vocab=16384,
                           dtype="bf16", rope_theta=500000.0, tie_embeddings=True)


def test_round_with_sampled_verification_on_the_targets_logits(B):
    """The round of workload 70b_verify_1b_draft as stated: the target (70B layer shape) forwards the K+1 pending positions
    on one stream while the draft pre-speculates on another; the pending tokens were drawn from the draft at temperature 1;
    rejection sampling (Sec. 2.1) runs on the target's logits against the draft's logits of the same positions (the glue
    rows of the draft's round: the distributions s_1..s_K were drawn from); the outcome is looked up in the draft's cache.
    Checked: both models' logits against the oracle; the kernel's decision against the oracle's decision on the very
    logits the kernel saw (margin rule); and against the oracle's decision on its own logits wherever the margins exceed
    what the logit error can move."""
    tshape, dshape, P, K, F, T, seed = TARGET_2L, DRAFT_SMALL, 200, 5, 4, 1.0, 31
    wt, wd = I.make_weights(tshape, seed), I.make_weights(dshape, seed + 1)
    print("[weights] generated", flush=True)
    target, draft = B.ssd_model_create(tshape, wt), B.ssd_model_create(dshape, wd)
    omt, omd = O.Model.from_weights(tshape, wt), O.Model.from_weights(dshape, wd)
    del wt, wd
    kt, vt = I.make_prefix_kv(tshape, 1, P, seed)
    kd, vd = I.make_prefix_kv(dshape, 1, P, seed + 1)
    tctx = B.ssd_ctx_create(target, 1, K, 1, P + 2 * K + 2)
    dctx = B.ssd_ctx_create(draft, 1, K, F, P + 2 * K + 2)
    try:
        B.ssd_ctx_load_trunk(tctx, kv_to_device(kt, "bf16"), kv_to_device(vt, "bf16"), P)
        B.ssd_ctx_load_trunk(dctx, kv_to_device(kd, "bf16"), kv_to_device(vd, "bf16"), P)
        trunk_t, trunk_d = oracle_trunk_from_arrays(omt, kt, vt, 0), oracle_trunk_from_arrays(omd, kd, vd, 0)
        # the pending speculation: drawn by the oracle's draft at temperature T from the last verified token
        last = int(I.make_pending(dshape, 1, K, seed)[0, 0])
        spec, zd_want = O.speculate(omd, trunk_d, last, K, T, seed)
        pending = np.array([[last] + [int(t) for t in spec]], np.int32)
        zt_want, _, _ = O.glue_extend(omt, trunk_t, pending[0])
        print("[oracle] target and draft logits done", flush=True)
        d_pending, temps = dev_i32(pending), dev_f32(np.full(1, T, np.float32))
        zt = torch.empty((1, K + 1, tshape.vocab), dtype=torch.float32, device="cuda")
        s_target, s_draft = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        B.ssd_ctx_extend(tctx, d_pending, 0, zt, stream=s_target)          # verifier's forward ...
        B.ssd_prespeculate(dctx, d_pending, temps, seed, stream=s_draft)   # ... while the draft pre-speculates
        torch.cuda.synchronize()
        view = B.ssd_ctx_views(dctx)
        zd = B.device_copy(view.d_glue_logits, (1, K + 1, dshape.vocab), torch.float32)[:, :K].contiguous()
        got_t, got_d = zt.cpu().numpy()[0], zd.cpu().numpy()[0]
        e_t, e_d = row_rel_err(got_t, zt_want), row_rel_err(got_d, zd_want)
        print(f"[logits] target rel err {e_t:.3e}, draft rel err {e_d:.3e}", flush=True)
        assert e_t < TOL["bf16"] and e_d < TOL["bf16"]

        acc = torch.zeros(1, dtype=torch.int32, device="cuda")
        bonus = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = torch.empty(B.ssd_verify_workspace_bytes(1, K), dtype=torch.uint8, device="cuda")
        d_spec = dev_i32(pending[:, 1:])
        n_same = 0
        for vseed in range(seed, seed + 12):                      # several draws of the acceptance uniforms and the noise
            B.ssd_verify(zt, zd, d_spec, temps, vseed, acc, bonus, ws, stream=s_target)
            torch.cuda.synchronize()
            k_gpu, t_gpu = int(acc[0]), int(bonus[0])
            # the oracle on the very logits the kernel consumed: the same decision unless it is a near-tie in fp64
            tr = O.verify(got_t.astype(np.float64), got_d.astype(np.float64), pending[0, 1:], T, vseed, 0)
            if min(tr.accept_margin + [1.0]) > 1e-4 and tr.bonus_margin > 1e-4:
                assert (k_gpu, t_gpu) == (tr.accept_len, tr.bonus), (vseed, k_gpu, t_gpu, tr)
            # the oracle on its own logits: the accept length wherever no tested position is within reach of the logit
            # error (a relative change of p/q by about twice the absolute logit error), the bonus token wherever the
            # winner's lead exceeds what that error moves a log-residual by
            tr0 = O.verify(zt_want, zd_want, pending[0, 1:], T, vseed, 0)
            reach = 2 * (np.abs(got_t - zt_want).max() + np.abs(got_d - zd_want).max()) / T
            if min(tr0.accept_margin + [1.0]) > 4 * reach:
                assert k_gpu == tr0.accept_len, (vseed, k_gpu, tr0)
                n_same += 1
            # the realised outcome against the draft's cache
            hit = torch.zeros(1, dtype=torch.uint8, device="cuda")
            branch = torch.zeros(1, dtype=torch.int32, device="cuda")
            toks = torch.zeros((1, K), dtype=torch.int32, device="cuda")
            B.ssd_cache_lookup(dctx, acc, bonus, hit, branch, toks)
            torch.cuda.synchronize()
            keys = B.device_copy(view.d_keys, (K + 1, F), torch.int32).cpu().numpy()
            assert int(branch[0]) == O.cache_lookup(keys, k_gpu, t_gpu)
        print(f"[verify] accept length equal to the oracle's own in {n_same} of 12 draws that were not near-ties", flush=True)
        assert n_same >= 6
    finally:
        B.ssd_ctx_destroy(tctx)
        B.ssd_ctx_destroy(dctx)
        B.ssd_model_destroy(target)
        B.ssd_model_destroy(draft)
