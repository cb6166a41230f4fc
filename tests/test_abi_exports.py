"""The C-ABI library loads and exports every symbol include/nm_conv.h declares
(no GPU needed, no compute call made)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nm_conv.h")
LIB = os.path.join(ROOT, "paper_2507_17301_amd", "libnmconv.so")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nm_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_entry_points():
    names = _declared()
    for must in ("nm_prune", "nm_conv2d", "nm_autotune"):
        assert must in names


@pytest.mark.skipif(not os.path.exists(LIB), reason="libnmconv.so not built (python -m paper_2507_17301_amd.build)")
def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(LIB)
    for name in _declared():
        assert hasattr(L, name), f"{name} declared in nm_conv.h but not exported"


@pytest.mark.skipif(not os.path.exists(LIB), reason="libnmconv.so not built")
def test_host_side_argument_checks_need_no_gpu():
    from paper_2507_17301_amd import binding as nm
    L = nm.lib()
    assert L.nm_variant_count() > 0
    assert nm.nm_variant_name(0).startswith("NB")
    assert nm.nm_variant_name(-1) is None and nm.nm_variant_name(10 ** 6) is None
    import numpy as np
    w = np.ones((4, 1, 1, 6), dtype=np.float32)
    with pytest.raises(nm.NMError) as e:
        nm.nm_prune(w, 2, 4, 2)              # K % M != 0 is rejected before any GPU work
    assert e.value.code == -1
    with pytest.raises(nm.NMError):
        nm.nm_prune(w, 3, 2, 2)              # n > m
    w[0, 0, 0, 0] = float("inf")
    with pytest.raises(nm.NMError):
        nm.nm_prune(w, 1, 2, 2)
    with pytest.raises(nm.NMError):
        nm.nm_force_variant(10 ** 6)
    nm.nm_cache_clear()
    assert nm.nm_cache_size() == 0
