"""The C-ABI library loads and exports every symbol include/harli.h declares (CPU only)."""
import ctypes
import os
import re

import pytest

from paper_2511_11729_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(harli_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 20
    l = ctypes.CDLL(binding.LIB_PATH)
    missing = [n for n in names if not hasattr(l, n)]
    assert not missing, missing


def test_binding_covers_every_declared_symbol():
    assert set(declared_functions()) <= set(binding._SIGS)


def test_status_strings_and_errors():
    l = binding.lib()
    assert l.harli_status_str(0) == b"ok"
    assert b"memory" in l.harli_status_str(2)
    assert b"gfx950" in l.harli_version()
    with pytest.raises(binding.HarliError) as e:
        binding.Pool(0x1000, 100, n_layers=1, kv_row_bytes=64, block_bytes=4096)   # slab holds no chunk
    assert e.value.status == binding.HARLI_ERR_INVALID and "chunk" in str(e.value)
    with pytest.raises(binding.HarliError):
        binding.Pool(0x1000, 1 << 20, n_layers=1, kv_row_bytes=64, block_bytes=3000)  # not granule * 2^k
