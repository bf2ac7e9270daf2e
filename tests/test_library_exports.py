"""The C-ABI library loads and exports every symbol include/sled.h declares (no GPU needed)."""
import os
import re

from paper_2506_09397_amd import sled

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sled.h")).read()
    return sorted(set(re.findall(r"SLED_API\s+[\w\s\*]+?\b(sled_\w+)\s*\(", text)))


def test_header_declares_the_three_entry_points():
    names = _declared()
    for must in ("sled_verify_batch", "sled_accept", "sled_kv_append"):
        assert must in names
    assert len(names) >= 15


def test_library_exports_every_declared_symbol():
    L = sled.lib()
    for name in _declared():
        assert hasattr(L, name), f"libsled.so does not export {name}"
    assert sorted(sled.EXPORTS) == _declared()


def test_error_strings_without_gpu():
    L = sled.lib()
    assert L.sled_strerror(0) == b"ok"
    assert b"invalid" in L.sled_strerror(-1)
    assert isinstance(L.sled_last_error(), bytes)
    # argument validation happens on the host before any device call
    assert L.sled_accept(7, 1, None, 10, 1.0, None, None, None, None, None, None, None, None, 0, None) == sled.EINVAL
    assert L.sled_accept_workspace_bytes(0, 0, 0) == 0
