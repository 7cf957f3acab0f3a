"""The C-ABI library loads here (no GPU needed) and exports every function include/ssd.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ssd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ssd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2603_03251_amd import binding
    names = _declared()
    assert len(names) >= 15
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in ssd.h but not exported"
    # the binding covers the same set, under the same names
    assert sorted(binding.EXPORTS) == names
    for n in names:
        if n != "ssd_last_error":
            assert callable(getattr(binding, n)), n


def test_argument_errors_are_reported_without_a_gpu():
    from paper_2603_03251_amd import binding as b
    assert b.lib.ssd_verify(None, None, None, None, 1, 1, 8, 0, None, None, None, None) == b.SSD_EINVAL
    assert b"null" in b.lib.ssd_last_error()
    assert b.lib.ssd_top_f(None, 8, None, 1, 8, 1, None, None, None) == b.SSD_EINVAL
    assert b.lib.ssd_top_f_workspace_bytes(0) == 0 and b.lib.ssd_top_f_workspace_bytes(6) > 0
    assert b.lib.ssd_ctx_create(None, None, None) == b.SSD_EINVAL
    assert b.lib.ssd_verify_workspace_bytes(0, 3) == 0
    assert b.lib.ssd_verify_workspace_bytes(2, 5) > 0


def test_geometric_cache_shape_equals_the_oracles_integer_shape():
    """Sec. 4.1.2 theorem: the library's host-side calculator against the oracle over a grid, and its argument checks."""
    from oracle import ssd_oracle as O
    from paper_2603_03251_amd import binding as b
    n = 0
    for K in (1, 3, 5, 7):
        for a in (0.3, 0.5, 0.7, 0.8, 0.9):
            for r in (0.3, 0.5, 1.0):
                for budget in (K + 1, 2 * (K + 1) + 1, 4 * (K + 1), 6 * (K + 1) - 1, 8 * (K + 1)):
                    for f_max in (8, 16):
                        if budget > (K + 1) * f_max:
                            continue
                        got = b.ssd_geometric_fanout(budget, K, a, r, f_max)
                        assert got == O.geometric_fan_out(budget, K, a, r, f_max).tolist(), (K, a, r, budget, f_max)
                        n += 1
    assert n > 400
    import pytest
    for bad in [(3, 5, 0.8, 0.5, 16), (200, 5, 0.8, 0.5, 16), (24, 5, 1.0, 0.5, 16), (24, 5, 0.8, 0.0, 16)]:
        with pytest.raises(b.SsdError) as e:
            b.ssd_geometric_fanout(*bad)
        assert e.value.status == b.SSD_EINVAL


def test_bench_byte_count_of_the_headline_step_by_hand():
    """The roofline's numerator for workload 1b_p1024_f4, worked out by hand: every weight once, the trunk KV once per
    sequence, the fp32 logits kept, the branches' private suffix KV."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    import ssd_inputs as I
    wl = I.WORKLOADS["1b_p1024_f4"]
    d, f, V, L, kvd = 2048, 8192, 128256, 16, 512
    weights = (L * ((2048 + 2 * kvd) * d + d * 2048 + 3 * d * f) + V * d) * 2          # bf16, LM head tied to the embedding
    trunk = L * (1024 + 6) * 2 * kvd * 2                                             # prefix + glue positions, K and V
    logits = 24 * V * 4
    suffix = 24 * L * 5 * 2 * kvd * 2
    assert weights == 2_471_493_632
    assert bench.algorithmic_bytes_per_decode_step(wl.draft, wl.round) == weights + trunk + logits + suffix == 2_521_489_408
    # a prefix length per sequence replaces batch x prefix by the sum of the lengths
    assert bench.algorithmic_bytes_per_decode_step(wl.draft, wl.round, [500]) == weights + L * (500 + 6) * 2 * kvd * 2 + logits + suffix
