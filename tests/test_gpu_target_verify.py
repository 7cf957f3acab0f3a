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
