"""ssd_verify_static (verification without any allocation: its workspace is a static device array) against ssd_verify
(workspace brought by the caller), through the C ABI: the same accept lengths and bonus tokens, bit for bit, on two
calls in a row, the second one smaller (it runs over what the first left in the shared array)."""
import numpy as np
import pytest
import torch

import ssd_inputs as I
from tests.gpu_util import dev_f32, dev_i32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2603_03251_amd import binding
    return binding


def _case(B, nb, K, V, seed, temps):
    zt_h = I.make_logits(nb * (K + 1), V, seed).reshape(nb, K + 1, V)
    zd_h = I.make_logits(nb * K, V, seed + 1).reshape(nb, K, V)
    # drafted tokens: the draft's own most likely ones, so that acceptance is neither always 0 nor always K
    spec_h = zd_h.argmax(axis=-1).astype(np.int32)
    zt_h[:, :K][np.arange(nb)[:, None], np.arange(K)[None, :], spec_h] += 4.0       # the target likes most of them too
    zt, zd, spec, T = dev_f32(zt_h), dev_f32(zd_h), dev_i32(spec_h), dev_f32(np.asarray(temps, np.float32))
    out = []
    for static in (False, True):
        k = torch.full((nb,), -7, dtype=torch.int32, device="cuda")
        t = torch.full((nb,), -7, dtype=torch.int32, device="cuda")
        if static:
            B.ssd_verify_static(zt, zd, spec, T, seed, k, t)
        else:
            ws = torch.empty(B.ssd_verify_workspace_bytes(nb, K), dtype=torch.uint8, device="cuda")
            B.ssd_verify(zt, zd, spec, T, seed, k, t, ws)
        torch.cuda.synchronize()
        out.append((k.cpu().numpy().copy(), t.cpu().numpy().copy()))
    (k0, t0), (k1, t1) = out
    print(f"[case] B={nb} K={K} V={V}: accept lengths {k0.tolist()}", flush=True)
    assert np.array_equal(k0, k1) and np.array_equal(t0, t1)
    assert (k0 >= 0).all() and (k0 <= K).all() and (t0 >= 0).all() and (t0 < V).all()
    return k0


def test_verify_static_equals_verify_on_two_calls_the_second_smaller(B):
    assert B.ssd_verify_static_capacity() >= B.ssd_verify_workspace_bytes(16, 5)
    # first call: batch 16 at the full vocabulary, greedy and sampled sequences mixed
    ks = _case(B, 16, 5, 128256, 11, [0.0, 1.0, 0.7, 0.0] * 4)
    assert len(set(ks.tolist())) > 1
    # second call, smaller in every size, over the first call's leftovers in the shared array
    _case(B, 3, 2, 4099, 12, [1.0, 0.0, 1.3])
    # and the first shape once more
    _case(B, 16, 5, 128256, 13, [1.0] * 16)


def test_verify_static_rejects_sizes_beyond_its_buffer(B):
    nb, K, V = 400, 15, 8
    assert B.ssd_verify_workspace_bytes(nb, K) > B.ssd_verify_static_capacity()
    z = torch.zeros((nb, K + 1, V), dtype=torch.float32, device="cuda")
    k = torch.zeros(nb, dtype=torch.int32, device="cuda")
    with pytest.raises(B.SsdError) as e:
        B.ssd_verify_static(z, None, torch.zeros((nb, K), dtype=torch.int32, device="cuda"),
                            torch.zeros(nb, dtype=torch.float32, device="cuda"), 0, k, k.clone())
    assert e.value.status == B.SSD_EINVAL
