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
    assert b.lib.ssd_top_f(None, 8, None, 1, 8, 1, None, None) == b.SSD_EINVAL
    assert b.lib.ssd_ctx_create(None, None, None) == b.SSD_EINVAL
    assert b.lib.ssd_verify_workspace_bytes(0, 3) == 0
    assert b.lib.ssd_verify_workspace_bytes(2, 5) > 0
