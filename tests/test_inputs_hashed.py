"""The hashed input family (ssd_inputs.hashed_normal and friends): statistics, determinism, and the integer definition
worked by hand for one element, so that the device generator can be held to it bit for bit (tests/test_gpu_init.py)."""
import numpy as np

import ssd_inputs as I


def _mix64_py(x):
    x &= (1 << 64) - 1
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & ((1 << 64) - 1)
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & ((1 << 64) - 1)
    x ^= x >> 31
    return x


def test_hashed_normal_matches_the_definition_in_plain_integers():
    seed, tid, std = 77, 16 + 16 * 3 + 4, 0.02
    prefix = _mix64_py(seed + 0x9E3779B97F4A7C15 * (tid + 1))
    idx = np.array([0, 1, 2, 12345678901, (5 << 40) + 17], dtype=np.uint64)
    got = I.hashed_normal(seed, tid, idx, std, bf16=False)
    for i, g in zip(idx.tolist(), got.tolist()):
        bits = _mix64_py(prefix + i)
        S = (bits & 0xFFFF) + ((bits >> 16) & 0xFFFF) + ((bits >> 32) & 0xFFFF) + (bits >> 48)
        want = np.float32(S - 131070) * np.float32(std / np.sqrt(4.0 * (65536.0 ** 2 - 1.0) / 12.0))
        assert np.float32(g) == want


def test_hashed_normal_statistics_and_bf16():
    x = I.hashed_normal(3, 0, np.arange(400000, dtype=np.uint64), 0.02, bf16=False)
    assert abs(x.mean()) < 4 * 0.02 / np.sqrt(x.size)
    assert abs(x.std() / 0.02 - 1.0) < 0.01
    assert abs(np.mean(np.abs(x) < 0.02) - 0.6827) < 0.02            # bell-shaped: a sum of 4 uniforms is close to normal
    y = I.hashed_normal(3, 0, np.arange(4096, dtype=np.uint64), 0.02, bf16=True)
    assert np.array_equal(I.round_to_bf16(y), y) and np.abs(y - x[:4096]).max() <= np.abs(x[:4096]).max() * 2.0 ** -8
    # tensors and seeds decorrelate
    z = I.hashed_normal(3, 1, np.arange(4096, dtype=np.uint64), 0.02, bf16=False)
    assert abs(np.corrcoef(x[:4096], z)[0, 1]) < 0.08


def test_hashed_weights_and_kv_have_the_models_shapes():
    shape = I.ModelShape(n_layers=2, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=32, d_ffn=96, vocab=50, dtype="bf16",
                         rope_theta=10000.0, tie_embeddings=False)
    w = I.make_hashed_weights(shape, 5)
    assert set(w) == set(I.weight_names(shape))
    assert w["l1.w_down"].shape == (64, 96) and (w["l0.attn_norm"] == 1).all()
    assert not np.array_equal(w["l0.wq"], w["l1.wq"]) and not np.array_equal(w["embed"], w["lm_head"])
    k, v = I.make_hashed_prefix_kv(shape, 3, 7, 5)
    assert k.shape == v.shape == (2, 3, 7, 1, 32)
    assert abs(k.std() - 1.0) < 0.05 and not np.array_equal(k, v)
    k2, _ = I.make_hashed_prefix_kv(shape, 3, 9, 5)               # a longer prefix extends a shorter one
    assert np.array_equal(k2[:, :, :7], k)
