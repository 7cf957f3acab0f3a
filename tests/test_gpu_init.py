"""Weights and prefix KV generated on the device (ssd_model_create_random, ssd_ctx_fill_synthetic_kv) against the host
twin of the same integer hash (ssd_inputs.make_hashed_*): a model created from the twin's arrays and a trunk loaded from
them must give the same bits, and the round on them must match the oracle like any other."""
import numpy as np
import pytest
import torch

import ssd_inputs as I
from oracle import ssd_oracle as O
from tests.gpu_util import TOL_FUSED_BF16, dev_f32, dev_i32, kv_to_device, oracle_trunk_from_arrays, row_rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2603_03251_amd import binding
    return binding


SHAPES = [
    I.ModelShape(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1024, vocab=4112, dtype="bf16",
                 rope_theta=500000.0, tie_embeddings=True),
    I.ModelShape(n_layers=2, d_model=512, n_q_heads=4, n_kv_heads=1, head_dim=128, d_ffn=512, vocab=2064, dtype="bf16",
                 rope_theta=500000.0, tie_embeddings=False),
    I.WORKLOADS["tiny_f32"].draft,
]


@pytest.mark.parametrize("shape", SHAPES, ids=["bf16 fused", "bf16 head_dim 128 untied", "fp32"])
def test_device_generated_model_and_prefix_equal_the_host_twin(B, shape):
    seed, nb, K, F = 911, 2, 3, 2
    lens = [37, 12]
    twin = I.make_hashed_weights(shape, seed)
    k, v = I.make_hashed_prefix_kv(shape, nb, max(lens), seed + 1)
    pending = dev_i32(I.make_pending(shape, nb, K, seed))
    temps = dev_f32(np.zeros(nb, np.float32))
    outs = []
    for on_device in (True, False):
        model = B.ssd_model_create_random(shape, seed) if on_device else B.ssd_model_create(shape, twin)
        ctx = B.ssd_ctx_create(model, nb, K, F, 96)
        try:
            if on_device:
                B.ssd_ctx_fill_synthetic_kv(ctx, lens, seed + 1)
            else:
                B.ssd_ctx_load_trunk(ctx, kv_to_device(k, shape.dtype), kv_to_device(v, shape.dtype), max(lens))
                B.ssd_ctx_truncate_trunk(ctx, lens)
            B.ssd_prespeculate(ctx, pending, temps, 1)
            outs.append({k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()})
        finally:
            B.ssd_ctx_destroy(ctx)
            B.ssd_model_destroy(model)
    for name in ("trunk_len", "keys", "tokens", "logits", "hidden", "glue_logits"):
        assert np.array_equal(outs[0][name], outs[1][name]), name
    # and the oracle agrees on the twin's arrays (sequence 1, teacher forcing not needed for the glue logits)
    om = O.Model.from_weights(shape, twin)
    trunk = oracle_trunk_from_arrays(om, k, v, 1).slice(lens[1])
    want, _, _ = O.glue_extend(om, trunk, pending.cpu().numpy()[1])
    e = row_rel_err(outs[0]["glue_logits"][1], want)
    print(f"[init] glue logits of the device-generated model against the oracle on the host twin: {e:.3e}", flush=True)
    assert e < (1e-4 if shape.dtype == "f32" else TOL_FUSED_BF16)


def test_fill_synthetic_kv_argument_checks(B):
    shape = I.WORKLOADS["tiny_f32"].draft
    model = B.ssd_model_create_random(shape, 1)
    ctx = B.ssd_ctx_create(model, 2, 4, 2, 40)
    try:
        for lens in ([0, 5], [5, 31]):
            with pytest.raises(B.SsdError) as e:
                B.ssd_ctx_fill_synthetic_kv(ctx, lens, 3)
            assert e.value.status == B.SSD_EINVAL
        B.ssd_ctx_fill_synthetic_kv(ctx, [30, 1], 3)
        torch.cuda.synchronize()
        assert list(B.read_cache(ctx, with_logits=False)["trunk_len"].cpu().numpy()) == [30, 1]
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


def test_model_gives_up_the_per_operator_weight_copies(B):
    """A model that only serves fused contexts frees the tile-order copies of its linear layers: the fused round is
    unchanged bit for bit, a context that needs the per-operator kernels is refused, and so is the release while such a
    context lives or for a shape the fused passes do not take."""
    shape = I.ModelShape(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1024, vocab=4112,
                         dtype="bf16", rope_theta=500000.0, tie_embeddings=True)
    nb, K, F = 2, 3, 2
    model = B.ssd_model_create_random(shape, 5)
    pending = torch.from_numpy(I.make_pending(shape, nb, K, 5)).cuda()
    temps = torch.zeros(nb, dtype=torch.float32, device="cuda")

    def round_of(ctx):
        B.ssd_ctx_fill_synthetic_kv(ctx, [40, 33], 6)
        B.ssd_prespeculate(ctx, pending, temps, 1)
        return {k: v.cpu() for k, v in B.read_cache(ctx).items()}

    try:
        free0 = torch.cuda.mem_get_info()[0]
        per_op = B.ssd_ctx_create(model, nb, K, F, 64, B.SSD_CTX_PER_OPERATOR)
        with pytest.raises(B.SsdError):
            B.ssd_model_release_operator_weights(model)        # a per-operator context is alive
        B.ssd_ctx_destroy(per_op)
        fused = B.ssd_ctx_create(model, nb, K, F, 64)
        before = round_of(fused)
        B.ssd_model_release_operator_weights(model)
        B.ssd_model_release_operator_weights(model)            # idempotent
        assert torch.cuda.mem_get_info()[0] > free0
        after = round_of(fused)
        for key in before:
            assert torch.equal(before[key], after[key]), key
        B.ssd_ctx_destroy(fused)
        with pytest.raises(B.SsdError):
            B.ssd_ctx_create(model, nb, K, F, 64, B.SSD_CTX_PER_OPERATOR)
    finally:
        B.ssd_model_destroy(model)
    d128 = I.ModelShape(n_layers=1, d_model=512, n_q_heads=4, n_kv_heads=1, head_dim=128, d_ffn=512, vocab=4112,
                        dtype="bf16", rope_theta=500000.0, tie_embeddings=False)
    m2 = B.ssd_model_create_random(d128, 5)
    try:
        with pytest.raises(B.SsdError):
            B.ssd_model_release_operator_weights(m2)           # its only copy
    finally:
        B.ssd_model_destroy(m2)
