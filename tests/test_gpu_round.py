"""GPU parity of the pre-speculation round against the float64 oracle, through the C ABI.

Protocol: (i) selection is compared on the oracle's logits (test_gpu_select.py) and, inside the round,
wherever the oracle's margin is not a near-tie; (ii) numerics are teacher-forced: the GPU runs every step on
the oracle's input tokens, so logits and hidden states must agree within the benchmark spec's tolerance
(rel 2e-2 in bf16, 1e-4 in fp32, relative to each row's largest magnitude); (iii) the fp32 tiny workload also
runs free and must reproduce the oracle's tokens wherever the oracle's top-2 margin exceeds 1e-4."""
import numpy as np
import pytest
import torch

import ssd_inputs as I
from oracle import ssd_oracle as O
from tests.gpu_util import (MARGIN, TOL, TOL_BF16_OWN_PREFILL, TOL_FUSED_BF16, TOL_ONE_PLANE_BF16, TOL_WIDE_BF16, dev_f32, dev_i32, elem_rel_err, kv_to_device,
                            oracle_trunk_from_arrays, rms_rel_err, row_rel_err)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2603_03251_amd import binding
    return binding


SMALL_BF16 = I.ModelShape(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1024,
                          vocab=4112, dtype="bf16", rope_theta=500000.0, tie_embeddings=True)
SMALL_BF16_D128 = I.ModelShape(n_layers=1, d_model=512, n_q_heads=8, n_kv_heads=1, head_dim=128, d_ffn=512,
                               vocab=2064, dtype="bf16", rope_theta=500000.0, tie_embeddings=False)


def _key_margin(z, keys_row, exclude):
    """Gap between the F-th selected logit and the best one left out (a near-tie makes the key set ambiguous)."""
    zz = np.array(z, dtype=np.float64)
    if exclude is not None:
        zz[exclude] = -np.inf
    sel = zz[keys_row]
    zz[keys_row] = -np.inf
    gaps = np.concatenate([-np.diff(sel), [sel[-1] - zz.max()]])
    return float(gaps.min())


def _in_row_order(a, fan):
    """Oracle cache array [K+1][max F_k]... -> the library's row order [sum F_k]... (accept length by accept length)."""
    return np.concatenate([a[k, :f] for k, f in enumerate(fan)])


def _run_round_parity(B, shape, batch, P, K, F, seed, synthetic_kv, temperature=0.0, lens=None, flags=0):
    """F: the uniform fan-out, or F_0..F_K (Sec. 4.1.2).  lens: prompt length per sequence (real prefill only;
    default P for all).  flags: ssd_round_config.flags (which kernels serve the context)."""
    tol = TOL[shape.dtype]
    w = I.make_weights(shape, seed)
    om = O.Model.from_weights(shape, w)
    model = B.ssd_model_create(shape, w)
    fan = [F] * (K + 1) if np.ndim(F) == 0 else [int(f) for f in F]
    if np.ndim(F) == 0:
        ctx = B.ssd_ctx_create(model, batch, K, F, P + 4 * K + 8, flags)
    else:
        ctx = B.ssd_ctx_create_fanout(model, batch, K, fan, P + 4 * K + 8, flags)
    assert B.ssd_ctx_fanout(ctx) == fan
    which = B.ssd_ctx_views(ctx).fused_pass
    wide = B.ssd_ctx_views(ctx).pass_rows > 48
    one_plane = (flags & B.SSD_CTX_ONE_PLANE_ALL) == B.SSD_CTX_ONE_PLANE_ALL
    if shape.dtype == "bf16":
        tol = min(tol, TOL_ONE_PLANE_BF16 if one_plane and not wide else
                  TOL_WIDE_BF16 if wide else (TOL_FUSED_BF16 if synthetic_kv else TOL_BF16_OWN_PREFILL))
    assert which == 0 if flags & B.SSD_CTX_PER_OPERATOR else True
    try:
        if synthetic_kv:
            k, v = I.make_prefix_kv(shape, batch, P, seed)
            B.ssd_ctx_load_trunk(ctx, kv_to_device(k, shape.dtype), kv_to_device(v, shape.dtype), P)
            trunks = [oracle_trunk_from_arrays(om, k, v, b) for b in range(batch)]
        else:
            prompt = I.make_prompt(shape, batch, P, seed)
            lens = [P] * batch if lens is None else list(lens)
            B.ssd_ctx_prefill(ctx, dev_i32(prompt), lens)
            trunks = [O.prefill(om, prompt[b][:lens[b]])[1] for b in range(batch)]
        pending = I.make_pending(shape, batch, K, seed)
        # make the pending tokens what a greedy draft would have proposed, so that exclusion bites
        for b in range(batch):
            spec, _ = O.speculate(om, trunks[b], pending[b, 0], K, 0.0, 0)
            pending[b, 1:] = spec
        caches = [O.prespeculate(om, trunks[b], pending[b], F, temperature, seed=seed, row_base=b * sum(fan))
                  for b in range(batch)]
        temps = dev_f32(np.full(batch, temperature, np.float32))

        # ---- free run: selection and sampling on the GPU's own logits
        B.ssd_prespeculate(ctx, dev_i32(pending), temps, seed)
        free = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()}
        assert list(free["trunk_len"]) == ([P] * batch if lens is None else lens)
        n_keys_checked = 0
        for b in range(batch):
            assert row_rel_err(free["glue_logits"][b], caches[b].glue_logits) < tol
            for k in range(K + 1):
                ex = int(pending[b, k + 1]) if k < K else None
                err = np.abs(free["glue_logits"][b, k] - caches[b].glue_logits[k]).max()
                # an ordering gap wider than twice the largest logit error cannot be flipped by it
                if _key_margin(caches[b].glue_logits[k], caches[b].keys[k, :fan[k]], ex) > 2 * err + 1e-12:
                    assert np.array_equal(free["keys"][b, k], caches[b].keys[k]), (b, k)
                    n_keys_checked += 1
                if k < K:
                    assert pending[b, k + 1] not in free["keys"][b, k]
        assert n_keys_checked > 0 or wide or one_plane       # (one bf16 plane: the error can exceed every gap of a small model's top F + 1)

        # ---- teacher-forced run: every row consumes the oracle's tokens
        f_keys = dev_i32(np.stack([_in_row_order(c.keys, fan) for c in caches]))
        f_toks = dev_i32(np.stack([_in_row_order(c.tokens, fan) for c in caches]))
        B.ssd_ctx_set_forced(ctx, f_keys, f_toks)
        B.ssd_prespeculate(ctx, dev_i32(pending), temps, seed)
        B.ssd_ctx_set_forced(ctx, None, None)
        forced = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()}
        worst = 0.0
        for b in range(batch):
            e_l = row_rel_err(forced["logits"][b], caches[b].logits)
            e_h = row_rel_err(forced["hidden"][b], caches[b].hidden)
            worst = max(worst, e_l, e_h)
            print(f"[parity] seq {b} ({('wide fused pass' if wide else 'fused pass') if which else 'per-operator kernels'}): logits {e_l:.3e}, hidden {e_h:.3e} "
                  f"(row-max metric); {elem_rel_err(forced['logits'][b], caches[b].logits):.3e}, "
                  f"{elem_rel_err(forced['hidden'][b], caches[b].hidden):.3e} (elementwise, atol 1e-2 row RMS)", flush=True)
            assert e_l < tol and e_h < tol, (b, e_l, e_h)
            assert rms_rel_err(forced["logits"][b], caches[b].logits) < tol
            # sampled tokens agree wherever the decision is not a near-tie at this precision (at T > 0 the scores are
            # logits / T + Gumbel noise keyed by the branch's row number)
            err = np.abs(forced["logits"][b] - caches[b].logits).max(axis=-1)
            decided = caches[b].margins > 2 * err / (temperature if temperature > 0 else 1.0) + 1e-12
            assert decided.any()
            assert np.array_equal(forced["tokens"][b][decided], caches[b].tokens[decided])
        return free, forced, caches, worst
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


def test_tiny_f32_workload_teacher_forced_and_free_running(B):
    wl = I.WORKLOADS["tiny_f32"]
    r = wl.round
    free, forced, caches, worst = _run_round_parity(B, wl.draft, r.batch, r.prefix - 1, r.K, r.F, wl.seed,
                                                     synthetic_kv=False)
    assert worst < 1e-4
    # free-running fp32: tokens equal the oracle's unless an earlier decision of that branch was a near-tie
    c = caches[0]
    n_equal = 0
    for k in range(r.K + 1):
        for j in range(r.F):
            if free["keys"][0, k, j] != c.keys[k, j]:
                continue
            for i in range(r.K):
                if c.margins[k, j, i] < MARGIN:
                    break
                assert free["tokens"][0, k, j, i] == c.tokens[k, j, i]
                n_equal += 1
    assert n_equal >= r.K * (r.K + 1) * r.F - 4


def test_small_bf16_ragged_rows_synthetic_prefix(B):
    # M = 2 * 4 * 3 = 24 rows, prefix 203 (not a multiple of anything), GQA group 4
    _run_round_parity(B, SMALL_BF16, batch=2, P=203, K=3, F=3, seed=7, synthetic_kv=True)


def test_small_bf16_many_rows_and_real_prefill(B):
    # M = 3 * 5 * 5 = 75 rows: more than one 64-row GEMM pass, last 16-row tile ragged
    _run_round_parity(B, SMALL_BF16, batch=3, P=37, K=4, F=5, seed=8, synthetic_kv=False)


def test_small_bf16_fused_pass_with_real_prefill(B):
    # M = 2 * 4 * 2 = 16 rows: the context is served by the fused pass, so the prefill chunks, the glue extend (causal
    # rows whose keys exist only in the pass) and the branch steps all run through its attention and K/V append
    _run_round_parity(B, SMALL_BF16, batch=2, P=37, K=3, F=2, seed=11, synthetic_kv=False)


def test_small_bf16_fused_pass_group_of_two_and_long_lookahead(B):
    # GQA group 2 (8 rows per query tile) and K + 1 = 9 > 8: sixteen fresh-key slots per row, two fresh blocks
    shape = I.ModelShape(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=4, head_dim=64, d_ffn=1024,
                         vocab=4112, dtype="bf16", rope_theta=500000.0, tie_embeddings=True)
    _run_round_parity(B, shape, batch=1, P=70, K=3, F=3, seed=12, synthetic_kv=True)
    _run_round_parity(B, SMALL_BF16, batch=1, P=45, K=8, F=2, seed=13, synthetic_kv=False)


def test_small_bf16_round_with_key_splits_merged_by_the_last_unit(B):
    # 700 and 1500 stored keys: 3 and 6 key splits per (sequence, KV head, query tile) in the narrow pass
    _run_round_parity(B, SMALL_BF16, batch=2, P=700, K=3, F=3, seed=31, synthetic_kv=True)
    _run_round_parity(B, SMALL_BF16, batch=1, P=1500, K=4, F=2, seed=32, synthetic_kv=True)


def test_small_bf16_narrow_pass_plane_configurations(B):
    """The precision of what the narrow pass hands from phase to phase: default (xn, att, act one fp16 plane; q, p two
    bf16 planes) and SSD_CTX_TWO_PLANES (head + remainder everywhere): same round, each within its bound, ordered as
    their significant bits say.  A combination that is not compiled in is refused at creation."""
    _, _, _, dflt = _run_round_parity(B, SMALL_BF16, batch=2, P=203, K=3, F=3, seed=7, synthetic_kv=True)
    _, _, _, two = _run_round_parity(B, SMALL_BF16, batch=2, P=203, K=3, F=3, seed=7, synthetic_kv=True,
                                     flags=B.SSD_CTX_TWO_PLANES)
    print(f"[planes] worst error: default {dflt:.3e}, two planes {two:.3e}", flush=True)
    assert dflt > two                        # the flag did change the arithmetic
    model = B.ssd_model_create(SMALL_BF16, I.make_weights(SMALL_BF16, 7))
    try:
        for flags in (B.SSD_CTX_TWO_PLANES | 0x100,     # only xn as one plane
                      B.SSD_CTX_ONE_PLANE_ALL):         # q and p as one bf16 plane too: a build option
            with pytest.raises(B.SsdError):
                B.ssd_ctx_create(model, 2, 3, 3, 256, flags)
    finally:
        B.ssd_model_destroy(model)


@pytest.mark.parametrize("rows_per_seq", ["narrow", "wide"])
def test_activations_beyond_the_fp16_range_saturate(B, rows_per_seq):
    """The fused passes hand activations to their linear layers as fp16: with RMSNorm gains of 1e6 the normalised
    residual stream and the SwiGLU output lie far beyond +-65504.  They saturate there instead of turning into
    infinities, so every logit and hidden state of the round stays finite (no comparison with the oracle, which has no
    such limit: this pins the documented behaviour at the edge of the number format, narrow and wide passes)."""
    shape, seed, nb, P, K = SMALL_BF16, 41, 2, 40, 3
    F = 3 if rows_per_seq == "narrow" else 16                  # 2 x 4 x 16 = 128 branch rows: wide passes
    w = I.make_weights(shape, seed)
    for name in w:
        if name.endswith("attn_norm") or name.endswith("mlp_norm"):
            w[name] = I.round_to_bf16(np.full_like(w[name], 1.0e6))
    model = B.ssd_model_create(shape, w)
    ctx = B.ssd_ctx_create(model, nb, K, F, P + 4 * K + 8)
    try:
        assert (B.ssd_ctx_views(ctx).pass_rows > 48) == (rows_per_seq == "wide")
        k, v = I.make_prefix_kv(shape, nb, P, seed)
        B.ssd_ctx_load_trunk(ctx, kv_to_device(k, "bf16"), kv_to_device(v, "bf16"), P)
        pending = dev_i32(I.make_pending(shape, nb, K, seed))
        B.ssd_prespeculate(ctx, pending, dev_f32(np.zeros(nb, np.float32)), seed)
        out = B.read_cache(ctx)
        B.ssd_ctx_refresh_bounds(ctx)
        for name in ("logits", "hidden", "glue_logits"):
            x = out[name].cpu().numpy()
            assert np.isfinite(x).all(), name
            assert np.abs(x).max() > 0, name
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


@pytest.mark.parametrize("P", [50, 700])
def test_fused_pass_phase_by_phase_equals_persistent(B, P):
    # the same pass as one launch per phase (no grid barrier) and as one persistent launch: identical bits, since
    # every sum is taken in a fixed order.  700 stored keys are scored as 3 key splits per query tile, which the unit that
    # arrives last merges, in split order whichever unit that is; run twice, the bits are the same again.
    shape, seed, nb, K, F = SMALL_BF16, 21, 2, 3, 3
    w = I.make_weights(shape, seed)
    k, v = I.make_prefix_kv(shape, nb, P, seed)
    pending = dev_i32(I.make_pending(shape, nb, K, seed))
    temps = dev_f32(np.zeros(nb, np.float32))
    outs = []
    for mode in ("phases", "persistent"):
        model = B.ssd_model_create(shape, w)
        ctx = B.ssd_ctx_create(model, nb, K, F, P + 4 * K + 8, B.SSD_CTX_FUSED_PHASES if mode == "phases" else 0)
        assert B.ssd_ctx_views(ctx).fused_pass == (1 if mode == "phases" else 2)
        try:
            B.ssd_ctx_load_trunk(ctx, kv_to_device(k, "bf16"), kv_to_device(v, "bf16"), P)
            B.ssd_prespeculate(ctx, pending, temps, seed)
            if mode == "persistent":
                B.ssd_ctx_enable_phase_clocks(ctx, True)
                B.ssd_prespeculate(ctx, pending, temps, seed)
                clocks = B.ssd_ctx_read_phase_clocks(ctx)
                assert clocks.shape[0] == 2 + 6 * shape.n_layers and clocks.shape[1] == 8
                assert (clocks[0, 2] >= clocks[0, 0]).all() and (clocks[-1, 2] > clocks[0, 0]).all()
            outs.append({k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()})
            B.ssd_ctx_refresh_bounds(ctx)            # would report a grid-barrier time-out
            if mode == "persistent":
                B.ssd_ctx_truncate_trunk(ctx, [P] * nb)
                B.ssd_prespeculate(ctx, pending, temps, seed)
                again = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()}
                for name in ("keys", "tokens", "logits", "hidden", "glue_logits"):
                    assert np.array_equal(outs[-1][name], again[name]), name
        finally:
            B.ssd_ctx_destroy(ctx)
            B.ssd_model_destroy(model)
    for name in ("keys", "tokens", "logits", "hidden", "glue_logits"):
        assert np.array_equal(outs[0][name], outs[1][name]), name


def test_wide_passes_agree_with_narrow_passes_and_repeat_bit_for_bit(B):
    """75 branch rows (3 sequences of 25): more than a narrow pass holds, so the context is served by wide passes (up to
    384 rows, one stream of the weights per step, one launch per phase).  The same round as narrow passes of whole
    sequences agrees to rounding (other summation order), and a second wide round gives the same bits
    (every sum is taken in a fixed order)."""
    shape, seed, nb, P, K, F = SMALL_BF16, 23, 3, 50, 4, 5
    w = I.make_weights(shape, seed)
    k, v = I.make_prefix_kv(shape, nb, P, seed)
    pending = dev_i32(I.make_pending(shape, nb, K, seed))
    temps = dev_f32(np.zeros(nb, np.float32))
    model = B.ssd_model_create(shape, w)
    outs = {}
    try:
        for mode, flags in (("wide", 0), ("wide again", 0), ("narrow", B.SSD_CTX_NARROW_PASSES)):
            ctx = B.ssd_ctx_create(model, nb, K, F, P + 4 * K + 8, flags)
            try:
                view = B.ssd_ctx_views(ctx)
                assert (view.pass_rows, view.fused_pass) == ((48, 2) if mode == "narrow" else (384, 1))
                B.ssd_ctx_load_trunk(ctx, kv_to_device(k, "bf16"), kv_to_device(v, "bf16"), P)
                print(f"[wide] {mode}", flush=True)
                B.ssd_prespeculate(ctx, pending, temps, seed)
                outs[mode] = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()}
                B.ssd_ctx_refresh_bounds(ctx)
            finally:
                B.ssd_ctx_destroy(ctx)
    finally:
        B.ssd_model_destroy(model)
    for name in ("keys", "tokens", "logits", "hidden", "glue_logits"):
        assert np.array_equal(outs["wide"][name], outs["wide again"][name]), name
    e = row_rel_err(outs["wide"]["glue_logits"], outs["narrow"]["glue_logits"])
    print(f"[wide] glue logits, wide against narrow passes: {e:.3e}", flush=True)
    assert e < TOL["bf16"]


def test_small_bf16_ragged_prompt_lengths_in_one_batch(B):
    # five sequences whose prompts differ in length (one a single token): three fused passes of 2 + 2 + 1 sequences,
    # every row with its own visible trunk length
    _run_round_parity(B, SMALL_BF16, batch=5, P=70, K=3, F=2, seed=19, synthetic_kv=False, lens=[70, 33, 1, 64, 17])


def test_small_bf16_ragged_prompt_lengths_per_operator_path(B):
    _run_round_parity(B, SMALL_BF16, batch=3, P=45, K=3, F=2, seed=29, synthetic_kv=False, lens=[45, 2, 31], temperature=0.7,
                      flags=B.SSD_CTX_PER_OPERATOR)


def test_fused_pass_barrier_epoch_wraps_around(B):
    """The grid barrier of the fused pass numbers its barriers on from launch to launch in 32 bits.  A context whose
    count starts shortly before 2^32 passes the wrap inside its second round and must give bit-identical results."""
    shape, batch, P, K, F, seed = SMALL_BF16, 2, 40, 3, 2, 5
    w = I.make_weights(shape, seed)
    model = B.ssd_model_create(shape, w)
    k, v = I.make_prefix_kv(shape, batch, P, seed)
    pending = dev_i32(I.make_pending(shape, batch, K, seed))
    temps = dev_f32(np.zeros(batch, np.float32))
    outs = []
    try:
        for epoch0 in (0, 2 ** 32 - 40):
            ctx = B.ssd_ctx_create(model, batch, K, F, P + 4 * K + 8)
            B.ssd_ctx_debug_set(ctx, B.SSD_DEBUG_BARRIER_EPOCH, epoch0)
            try:
                B.ssd_ctx_load_trunk(ctx, kv_to_device(k, shape.dtype), kv_to_device(v, shape.dtype), P)
                for rnd in range(3):                       # 4 launches of 11 barriers each per round
                    B.ssd_prespeculate(ctx, pending, temps, seed)
                torch.cuda.synchronize()
                B.ssd_ctx_refresh_bounds(ctx)              # raises if a barrier wait expired
                outs.append({k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()})
            finally:
                B.ssd_ctx_destroy(ctx)
        for name in ("keys", "tokens", "logits", "hidden"):
            assert np.array_equal(outs[0][name], outs[1][name]), name
    finally:
        B.ssd_model_destroy(model)


def _small(**over):
    return I.ModelShape(**{**SMALL_BF16.__dict__, **over})


@pytest.mark.parametrize("name,shape,kw", [
    ("shortest round", SMALL_BF16, dict(batch=1, P=5, K=1, F=1, seed=1, synthetic_kv=False)),
    ("longest lookahead", _small(n_layers=1), dict(batch=1, P=40, K=15, F=3, seed=2, synthetic_kv=True)),
    ("widest fan-out", _small(n_layers=1), dict(batch=1, P=33, K=2, F=16, seed=3, synthetic_kv=True)),
    ("one KV head for 8 query heads", _small(n_kv_heads=1), dict(batch=2, P=70, K=3, F=2, seed=4, synthetic_kv=True)),
    ("multi-head attention", _small(n_kv_heads=8), dict(batch=1, P=65, K=3, F=4, seed=5, synthetic_kv=True)),
    ("one-token prompts", SMALL_BF16, dict(batch=3, P=1, K=2, F=2, seed=6, synthetic_kv=False)),
    ("two key splits", _small(n_layers=1), dict(batch=1, P=2100, K=2, F=4, seed=7, synthetic_kv=True)),
    ("wider model", _small(d_model=1024, n_q_heads=16, n_kv_heads=4, d_ffn=1536), dict(batch=1, P=90, K=4, F=4, seed=8, synthetic_kv=True)),
    ("48 rows, the most of a fused pass", SMALL_BF16, dict(batch=1, P=100, K=5, F=8, seed=10, synthetic_kv=True)),
    ("56 rows per sequence: per-operator kernels", _small(n_layers=1), dict(batch=1, P=50, K=6, F=8, seed=11, synthetic_kv=True)),
    ("seven sequences of different lengths", _small(n_layers=1),
     dict(batch=7, P=12, K=2, F=2, seed=14, synthetic_kv=False, lens=[12, 1, 5, 9, 2, 12, 7])),
])
def test_small_bf16_corner_shapes(B, name, shape, kw):
    print(f"[case] {name}", flush=True)
    _run_round_parity(B, shape, **kw)


def test_small_bf16_head_dim_128_untied(B):
    _run_round_parity(B, SMALL_BF16_D128, batch=1, P=70, K=2, F=2, seed=9, synthetic_kv=True)


def test_small_bf16_geometric_cache_shape(B):
    """Sec. 4.1.2: a round whose fan-out follows the theorem's geometric shape; the library's integer shape equals the
    oracle's, the rows run accept length by accept length, and the fused pass serves the 13 rows per sequence."""
    K = 3
    fan = B.ssd_geometric_fanout(13, K, 0.7, 0.5, 8)
    assert fan == O.geometric_fan_out(13, K, 0.7, 0.5, 8).tolist() and len(set(fan)) > 2
    free, forced, caches, _ = _run_round_parity(B, SMALL_BF16, batch=2, P=203, K=K, F=fan, seed=7, synthetic_kv=True)
    for k in range(K + 1):
        assert (free["keys"][:, k, fan[k]:] == -1).all() and (free["keys"][:, k, :fan[k]] >= 0).all()


def test_small_bf16_geometric_cache_shape_sampled_per_operator_path(B):
    # temperature > 0: the Gumbel noise of a branch is keyed by its row number in the ragged order; kernels launched
    # one by one instead of the fused pass
    _run_round_parity(B, SMALL_BF16, batch=3, P=77, K=4, F=[6, 1, 3, 2, 9], seed=23, synthetic_kv=False, temperature=0.8,
                      flags=B.SSD_CTX_PER_OPERATOR)


def test_tiny_f32_geometric_cache_shape_lookup(B):
    """Every cached outcome of a ragged cache is found at its rank and returns its own speculation and logits
    pointer; the keys a wider cache would have held at that accept length miss."""
    shape = I.WORKLOADS["tiny_f32"].draft
    w = I.make_weights(shape, 3)
    model = B.ssd_model_create(shape, w)
    K, fan, nb, P = 4, [3, 1, 4, 2, 1], 2, 20
    R, off = sum(fan), np.concatenate([[0], np.cumsum(fan)])
    ctx = B.ssd_ctx_create_fanout(model, nb, K, fan, 128)
    wide = B.ssd_ctx_create(model, nb, K, max(fan), 128)
    try:
        prompt = I.make_prompt(shape, nb, P, 5)
        pending = I.make_pending(shape, nb, K, 5)
        for c in (ctx, wide):
            B.ssd_ctx_prefill(c, dev_i32(prompt), [P, P - 3])
            B.ssd_prespeculate(c, dev_i32(pending), dev_f32(np.zeros(nb)), 0)
        got = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx, with_logits=False).items()}
        ref = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(wide, with_logits=False).items()}
        v = B.ssd_ctx_views(ctx)
        hit = torch.zeros(nb, dtype=torch.uint8, device="cuda")
        branch = torch.zeros(nb, dtype=torch.int32, device="cuda")
        spec = torch.zeros((nb, K), dtype=torch.int32, device="cuda")
        ptrs = torch.zeros(nb, dtype=torch.int64, device="cuda")
        for k in range(K + 1):
            # greedy branches do not depend on their row number: the ragged cache is a sub-cache of the wide one
            assert np.array_equal(got["keys"][:, k, :fan[k]], ref["keys"][:, k, :fan[k]])
            assert np.array_equal(got["tokens"][:, k, :fan[k]], ref["tokens"][:, k, :fan[k]])
            for j in range(max(fan)):
                probe = [int(ref["keys"][b, k, j]) for b in range(nb)]
                B.ssd_cache_lookup(ctx, dev_i32([k] * nb), dev_i32(probe), hit, branch, spec, ptrs)
                torch.cuda.synchronize()
                want = [O.cache_lookup(got["keys"][b], k, probe[b]) for b in range(nb)]
                assert want == [j if j < fan[k] else -1] * nb
                assert list(branch.cpu().numpy()) == want
                for b in range(nb):
                    if want[b] >= 0:
                        assert np.array_equal(spec.cpu().numpy()[b], got["tokens"][b, k, j])
                        assert int(ptrs[b]) == v.d_logits + (b * R + off[k] + j) * K * shape.vocab * 4
                    else:
                        assert int(hit[b]) == 0 and int(ptrs[b]) == 0
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_ctx_destroy(wide)
        B.ssd_model_destroy(model)


def test_lookup_and_commit(B):
    shape = I.WORKLOADS["tiny_f32"].draft
    w = I.make_weights(shape, 3)
    model = B.ssd_model_create(shape, w)
    K, F, nb, P = 4, 2, 3, 20
    ctx = B.ssd_ctx_create(model, nb, K, F, 128)
    try:
        acc = dev_i32([0, 1, 2])
        bonus = dev_i32([1, 2, 3])
        hit = torch.zeros(nb, dtype=torch.uint8, device="cuda")
        branch = torch.zeros(nb, dtype=torch.int32, device="cuda")
        spec = torch.zeros((nb, K), dtype=torch.int32, device="cuda")
        with pytest.raises(B.SsdError) as e:
            B.ssd_cache_lookup(ctx, acc, bonus, hit, branch, spec)
        assert e.value.status == B.SSD_ESTATE                     # lookup before any pre-speculation
        with pytest.raises(B.SsdError) as e:
            B.ssd_prespeculate(ctx, dev_i32(np.zeros((nb, K + 1))), dev_f32(np.zeros(nb)), 0)
        assert e.value.status == B.SSD_ESTATE                     # empty trunk
        prompt = I.make_prompt(shape, nb, P, 5)
        B.ssd_ctx_prefill(ctx, dev_i32(prompt), [P, P - 3, P - 7])    # ragged lengths
        pending = I.make_pending(shape, nb, K, 5)
        B.ssd_prespeculate(ctx, dev_i32(pending), dev_f32(np.zeros(nb)), 0)
        cache = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx, with_logits=False).items()}
        assert list(cache["trunk_len"]) == [P, P - 3, P - 7]
        keys, toks = cache["keys"], cache["tokens"]
        # every (k, token) outcome of sequence 1: hit iff the oracle's linear search finds it
        ptrs = torch.zeros(nb, dtype=torch.int64, device="cuda")
        v = B.ssd_ctx_views(ctx)
        for k in range(K + 1):
            probe = [int(keys[0, k, F - 1]), int((keys[1, k].max() + 1) % shape.vocab), int(keys[2, k, 0])]
            B.ssd_cache_lookup(ctx, dev_i32([k] * nb), dev_i32(probe), hit, branch, spec, ptrs)
            torch.cuda.synchronize()
            want = [O.cache_lookup(keys[b], k, probe[b]) for b in range(nb)]
            assert list(branch.cpu().numpy()) == want
            assert list(hit.cpu().numpy()) == [1 if j >= 0 else 0 for j in want]
            sp = spec.cpu().numpy()
            for b in range(nb):
                if want[b] >= 0:
                    assert np.array_equal(sp[b], toks[b, k, want[b]])
                    row = (b * (K + 1) + k) * F + want[b]
                    assert int(ptrs[b]) == v.d_logits + row * K * shape.vocab * 4
                else:
                    assert (sp[b] == -1).all() and int(ptrs[b]) == 0
        # an accept length outside 0..K is a miss
        B.ssd_cache_lookup(ctx, dev_i32([K + 1, -1, 0]), dev_i32([int(keys[0, 0, 0])] * nb), hit, branch, spec)
        torch.cuda.synchronize()
        assert list(hit.cpu().numpy())[:2] == [0, 0]
        # commit: trunk grows by k + 1 (clamped)
        B.ssd_ctx_commit(ctx, dev_i32([0, K, K + 5]))
        torch.cuda.synchronize()
        tl = B.read_cache(ctx, with_logits=False)["trunk_len"].cpu().numpy()
        assert list(tl) == [P + 1, P - 3 + K + 1, P - 7 + K + 1]
        B.ssd_ctx_refresh_bounds(ctx)
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


def test_argument_validation(B):
    shape = I.WORKLOADS["tiny_f32"].draft
    model = B.ssd_model_create(shape, I.make_weights(shape, 3))
    try:
        for bad in [(0, 4, 2, 128), (1, 0, 2, 128), (1, 16, 2, 128), (1, 4, 17, 128), (1, 4, 2, 5)]:
            with pytest.raises(B.SsdError) as e:
                B.ssd_ctx_create(model, *bad)
            assert e.value.status == B.SSD_EINVAL
        ctx = B.ssd_ctx_create(model, 1, 4, 2, 40)
        with pytest.raises(B.SsdError) as e:      # prompt does not leave room for a round
            B.ssd_ctx_prefill(ctx, dev_i32(np.zeros((1, 35))), [35])
        assert e.value.status == B.SSD_EINVAL
        B.ssd_ctx_destroy(ctx)
        # a fan-out per accept length: K+1 entries, each within 1..SSD_MAX_F
        for fan in ([2, 2, 2, 2, 0], [2, 2, 2, 2, 17]):
            with pytest.raises(B.SsdError) as e:
                B.ssd_ctx_create_fanout(model, 1, 4, fan, 128)
            assert e.value.status == B.SSD_EINVAL
        # trunk truncation: lengths within 1 .. what the trunk holds
        ctx = B.ssd_ctx_create(model, 2, 4, 2, 64)
        B.ssd_ctx_prefill(ctx, dev_i32(I.make_prompt(shape, 2, 20, 1)), [20, 12])
        for lens in ([0, 5], [21, 5]):
            with pytest.raises(B.SsdError) as e:
                B.ssd_ctx_truncate_trunk(ctx, lens)
            assert e.value.status == B.SSD_EINVAL
        B.ssd_ctx_truncate_trunk(ctx, [20, 20])       # within the bound: positions 12..19 of sequence 1 hold padding KV
        B.ssd_ctx_truncate_trunk(ctx, [7, 3])
        torch.cuda.synchronize()
        assert list(B.read_cache(ctx, with_logits=False)["trunk_len"].cpu().numpy()) == [7, 3]
        B.ssd_ctx_destroy(ctx)
    finally:
        B.ssd_model_destroy(model)


@pytest.mark.parametrize("fan", [None, [2, 4, 1, 3]])
def test_small_bf16_saguaro_sampling_scheme(B, fan):
    """Sec. 4.2.1: branches drawn from sigma_{F,C}; with a fan-out per accept length, depth i lowers its top F_i.  Teacher-forced on the oracle's tokens, the cached logits must be the
    oracle's lowered logits wherever the step's top-F set is not a near-tie at this precision (there, lowering a
    different token is equally right: the row is then compared with the shift taken out on both sides)."""
    shape, batch, P, K, F, seed, T, Cw = SMALL_BF16, 2, 61, 3, 3, 17, 1.0, 0.3
    tol = TOL[shape.dtype]
    w = I.make_weights(shape, seed)
    om = O.Model.from_weights(shape, w)
    model = B.ssd_model_create(shape, w)
    fans = [F] * (K + 1) if fan is None else fan
    F = F if fan is None else fan                    # what the oracle's prespeculate takes
    RB = sum(fans)
    ctx = B.ssd_ctx_create(model, batch, K, F, P + 4 * K + 8) if fan is None else \
        B.ssd_ctx_create_fanout(model, batch, K, fans, P + 4 * K + 8)
    try:
        k, v = I.make_prefix_kv(shape, batch, P, seed)
        B.ssd_ctx_load_trunk(ctx, kv_to_device(k, shape.dtype), kv_to_device(v, shape.dtype), P)
        trunks = [oracle_trunk_from_arrays(om, k, v, b) for b in range(batch)]
        pending = I.make_pending(shape, batch, K, seed)
        rb = lambda b: b * RB
        caches = [O.prespeculate(om, trunks[b], pending[b], F, T, seed=seed, row_base=rb(b), C=Cw) for b in range(batch)]
        raws = [O.prespeculate(om, trunks[b], pending[b], F, T, seed=seed, row_base=rb(b), forced_tokens=caches[b].tokens)
                for b in range(batch)]
        temps = dev_f32(np.full(batch, T, np.float32))
        f_keys = dev_i32(np.stack([_in_row_order(c.keys, fans) for c in caches]))     # kept alive while the context points at them
        f_toks = dev_i32(np.stack([_in_row_order(c.tokens, fans) for c in caches]))
        B.ssd_ctx_set_saguaro(ctx, Cw)
        B.ssd_ctx_set_forced(ctx, f_keys, f_toks)
        B.ssd_prespeculate(ctx, dev_i32(pending), temps, seed)
        B.ssd_ctx_set_forced(ctx, None, None)
        got = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()}
        shift = T * np.log(Cw)
        n_exact = n_tie = n_tok = 0
        for b in range(batch):
            for kk in range(K + 1):
                for j in range(fans[kk]):
                    for i in range(K):
                        z_got, z_want, z_raw = got["logits"][b, kk, j, i], caches[b].logits[kk, j, i], raws[b].logits[kk, j, i]
                        scale = np.abs(z_raw).max()
                        F = fans[i]                  # depth i is verified at accept length i of the next round
                        top = O.top_f_ids(z_raw, F + 1)
                        # what the GPU lowered: the entries that sit about `shift` below the oracle's raw logits
                        lowered = np.nonzero(z_got - z_raw < shift / 2)[0]
                        assert len(lowered) == F
                        unshifted = z_got.astype(np.float64).copy()
                        unshifted[lowered] -= shift
                        err = np.abs(unshifted - z_raw).max()
                        assert err / scale < tol
                        if z_raw[top[F - 1]] - z_raw[top[F]] > 2 * err:
                            assert set(lowered) == set(int(t) for t in top[:F])
                            assert np.abs(z_got - z_want).max() / scale < tol
                            n_exact += 1
                            if caches[b].margins[kk, j, i] > 2 * err / T:
                                assert got["tokens"][b, kk, j, i] == caches[b].tokens[kk, j, i]
                                n_tok += 1
                        else:
                            n_tie += 1
        assert n_exact > 10 * max(n_tie, 1) and n_tok > 0
        # the scheme off again: the next round's logits are the model's own
        B.ssd_ctx_set_saguaro(ctx, 1.0)
        B.ssd_ctx_set_forced(ctx, f_keys, f_toks)
        B.ssd_prespeculate(ctx, dev_i32(pending), temps, seed)
        B.ssd_ctx_set_forced(ctx, None, None)
        again = B.read_cache(ctx)["logits"].cpu().numpy()
        for b in range(batch):
            assert row_rel_err(again[b], raws[b].logits) < tol
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


@pytest.mark.parametrize("fused", [True, False])
def test_small_bf16_rounds_in_sequence_with_rollback(B, fused):
    """Several rounds on one context (App. B "Glue & Recurrence"): after each round the trunk keeps the glue positions
    0..k of the realised accept length and the next glue extend overwrites the rest.  Accept lengths 0, K, 2, 1, K walk
    the trunk across a 32-position block boundary of the value layout; every round's cache must match the oracle's
    round on the oracle's own trunk."""
    shape, batch, P, K, F, seed = SMALL_BF16, 2, 27, 3, 2, 33
    tol = TOL[shape.dtype]
    w = I.make_weights(shape, seed)
    om = O.Model.from_weights(shape, w)
    model = B.ssd_model_create(shape, w)
    ctx = B.ssd_ctx_create(model, batch, K, F, P + 6 * (K + 1) + 2 * K + 4, 0 if fused else B.SSD_CTX_PER_OPERATOR)
    assert (B.ssd_ctx_views(ctx).fused_pass == 2) == fused
    try:
        k, v = I.make_prefix_kv(shape, batch, P, seed)
        B.ssd_ctx_load_trunk(ctx, kv_to_device(k, shape.dtype), kv_to_device(v, shape.dtype), P)
        trunks = [oracle_trunk_from_arrays(om, k, v, b) for b in range(batch)]
        temps = dev_f32(np.zeros(batch, np.float32))
        for rnd, accepts in enumerate([(0, K), (K, 2), (2, 0), (1, 1), (K, K)]):
            pending = I.make_pending(shape, batch, K, seed + rnd)
            caches = [O.prespeculate(om, trunks[b], pending[b], F, 0.0, seed=rnd, row_base=b * (K + 1) * F) for b in range(batch)]
            f_keys = dev_i32(np.stack([c.keys for c in caches]))
            f_toks = dev_i32(np.stack([c.tokens for c in caches]))
            d_pending = dev_i32(pending)
            B.ssd_ctx_set_forced(ctx, f_keys, f_toks)
            B.ssd_prespeculate(ctx, d_pending, temps, rnd)
            B.ssd_ctx_set_forced(ctx, None, None)
            got = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()}
            assert list(got["trunk_len"]) == [t.length for t in trunks]
            for b in range(batch):
                e_g = row_rel_err(got["glue_logits"][b], caches[b].glue_logits)
                e_l = row_rel_err(got["logits"][b], caches[b].logits)
                assert e_g < tol and e_l < tol, (rnd, b, e_g, e_l)
            B.ssd_ctx_commit(ctx, dev_i32(np.array(accepts, np.int32)))
            B.ssd_ctx_refresh_bounds(ctx)
            trunks = [caches[b].trunk.slice(trunks[b].length + accepts[b] + 1) for b in range(batch)]
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


def test_fused_pass_expired_wait_is_reported_and_recovered(B):
    """Error path of the persistent kernel, forced from the host without hanging anything: with a spin limit of one
    poll the bounded waits of the next launch expire, every workgroup sets the fault word and leaves the kernel
    normally.  From then on the hot calls fail with EHIP (instead of handing out a half-written cache), ssd_ctx_status
    reports the fault without blocking, and after ssd_ctx_recover the context computes the same bits as before."""
    shape, nb, P, K, F, seed = SMALL_BF16, 2, 50, 3, 2, 41
    w = I.make_weights(shape, seed)
    model = B.ssd_model_create(shape, w)
    ctx = B.ssd_ctx_create(model, nb, K, F, P + 4 * K + 8)
    try:
        assert B.ssd_ctx_views(ctx).fused_pass == 2
        k, v = I.make_prefix_kv(shape, nb, P, seed)
        kd, vd = kv_to_device(k, "bf16"), kv_to_device(v, "bf16")
        B.ssd_ctx_load_trunk(ctx, kd, vd, P)
        pending = dev_i32(I.make_pending(shape, nb, K, seed))
        temps = dev_f32(np.zeros(nb, np.float32))
        B.ssd_prespeculate(ctx, pending, temps, seed)
        good = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()}
        B.ssd_ctx_status(ctx)                                  # healthy: no exception
        B.ssd_ctx_debug_set(ctx, B.SSD_DEBUG_SPIN_LIMIT, 1)
        print("[fault] launching one round whose bounded waits expire after one poll", flush=True)
        B.ssd_prespeculate(ctx, pending, temps, seed)          # enqueues fine; the kernels give up and end
        torch.cuda.synchronize()
        with pytest.raises(B.SsdError) as e:
            B.ssd_ctx_status(ctx)
        assert e.value.status == B.SSD_EHIP
        hit = torch.zeros(nb, dtype=torch.uint8, device="cuda")
        branch = torch.zeros(nb, dtype=torch.int32, device="cuda")
        spec = torch.zeros((nb, K), dtype=torch.int32, device="cuda")
        zero = dev_i32(np.zeros(nb))
        for call in (lambda: B.ssd_prespeculate(ctx, pending, temps, seed),
                     lambda: B.ssd_cache_lookup(ctx, zero, zero, hit, branch, spec),
                     lambda: B.ssd_ctx_commit(ctx, zero),
                     lambda: B.ssd_ctx_refresh_bounds(ctx)):
            with pytest.raises(B.SsdError) as e:
                call()
            assert e.value.status == B.SSD_EHIP and "ssd_ctx_recover" in str(e.value)
        B.ssd_ctx_debug_set(ctx, B.SSD_DEBUG_SPIN_LIMIT, 0)    # back to the default
        B.ssd_ctx_recover(ctx)
        B.ssd_ctx_status(ctx)
        with pytest.raises(B.SsdError) as e:                   # the cache was invalidated
            B.ssd_cache_lookup(ctx, zero, zero, hit, branch, spec)
        assert e.value.status == B.SSD_ESTATE
        B.ssd_ctx_load_trunk(ctx, kd, vd, P)                   # the aborted glue extend may have left slots half written
        B.ssd_prespeculate(ctx, pending, temps, seed)
        again = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctx).items()}
        B.ssd_ctx_refresh_bounds(ctx)
        for name in ("keys", "tokens", "logits", "hidden", "glue_logits"):
            assert np.array_equal(good[name], again[name]), name
    finally:
        B.ssd_ctx_destroy(ctx)
        B.ssd_model_destroy(model)


def test_two_fused_contexts_on_two_streams_take_turns(B):
    """Two contexts served by the persistent kernel, driven from two streams at once (a draft beside a small target):
    the library makes each persistent launch wait for the previous one of the process, so neither starves the other's
    grid barrier, and both give the bits they give alone."""
    shape, nb, P, K, F = SMALL_BF16, 2, 60, 3, 2
    models, ctxs, pend, alone = [], [], [], []
    temps = dev_f32(np.zeros(nb, np.float32))
    try:
        for seed in (51, 52):
            w = I.make_weights(shape, seed)
            models.append(B.ssd_model_create(shape, w))
            ctxs.append(B.ssd_ctx_create(models[-1], nb, K, F, P + 4 * K + 8))
            k, v = I.make_prefix_kv(shape, nb, P, seed)
            B.ssd_ctx_load_trunk(ctxs[-1], kv_to_device(k, "bf16"), kv_to_device(v, "bf16"), P)
            pend.append(dev_i32(I.make_pending(shape, nb, K, seed)))
            B.ssd_prespeculate(ctxs[-1], pend[-1], temps, seed)
            alone.append({k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctxs[-1]).items()})
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        for rep in range(4):
            for i in (0, 1):
                B.ssd_prespeculate(ctxs[i], pend[i], temps, 51 + i, stream=streams[i])
        torch.cuda.synchronize()
        for i in (0, 1):
            B.ssd_ctx_status(ctxs[i])
            got = {k_: v_.cpu().numpy() for k_, v_ in B.read_cache(ctxs[i]).items()}
            for name in ("keys", "tokens", "logits", "hidden"):
                assert np.array_equal(alone[i][name], got[name]), (i, name)
    finally:
        for c in ctxs:
            B.ssd_ctx_destroy(c)
        for m in models:
            B.ssd_model_destroy(m)
