"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol,
rejects bad arguments before launching anything, and reports sane workspace sizes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", name) for name in sorted(os.listdir(os.path.join(ROOT, "include")))
           if name.endswith(".h")]


@pytest.fixture(scope="module")
def L():
    from paper_2602_01801_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_01801_amd.build import build
        build()
    return binding.lib()


def declared_functions():
    text = "\n".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)))


def test_header_declares_the_expected_entry_points():
    from paper_2602_01801_amd import EXPORTS
    assert declared_functions() == sorted(EXPORTS)
    for name in ("tempcache_compress", "ann_select_self", "ann_select_cross", "sparse_attn_fwd"):
        assert name in EXPORTS


def test_library_exports_every_declared_symbol(L):
    for name in declared_functions():
        assert hasattr(L, name), name
    assert L.fastar_version().decode().startswith("fastar")
    assert L.fastar_strerror(-3).decode() == "workspace too small"


def test_workspace_sizes(L):
    from paper_2602_01801_amd import OP_COMPRESS, OP_SELECT_CROSS, OP_SELECT_SELF, workspace_bytes
    # AnnSA at the Wan-shaped layer: summaries + one int32 per (query block, key block)
    w = workspace_bytes(OP_SELECT_SELF, 12, 4680, 32760, 32, 128, 64, 4)
    assert w >= 12 * 37 * 512 * 4 + 12 * 37 * 4 * 32 and w % 256 == 0
    w = workspace_bytes(OP_SELECT_CROSS, 12, 4680, 512, 32, 128)
    assert w >= 12 * 37 * 512 * 4
    w = workspace_bytes(OP_COMPRESS, 12, 1560, 37440, 32)
    assert w >= 12 * 37440 * 12 + 12 * 1560 * (32 + 8 + 16)
    assert workspace_bytes(99, 1, 1, 1) == 0


def test_null_and_inconsistent_arguments_return_error_codes_without_a_gpu(L):
    null = ctypes.c_void_p(0)
    assert L.ann_select_self(null, 128, null, null, 1, 256, 32, 128, 4, 64, 2, null, null, null, 0, null) == -1
    assert L.ann_select_cross(null, 128, null, 64, 1, 32, 128, 4, null, null, null, 0, null) == -1
    assert L.sparse_attn_fwd(null, 1, null, null, null, null, 1, 1, 128, 1, null, null, 128, 64, 1,
                             ctypes.c_float(1.0), null, null, null) == -1
    assert L.fastar_encode(null, 1, 16, 128, None, 32, null, null) == -1
    assert L.tempcache_compress(None, None, null, null, null, 1, null, 0, 0, 0, 0, 0, null, null, null, null, 0,
                                0, null) == -1


def test_cache_beyond_the_32_bit_row_offsets_is_rejected_before_any_launch(L):
    # bf16 tiles are addressed by 32-bit byte offsets inside a head: C * d * 2 >= 2^32 must come back as unsupported
    # (the pointers are never dereferenced: the check precedes every launch)
    fake = ctypes.c_void_p(0x10000)
    assert L.sparse_attn_fwd(fake, 128, fake, fake, None, fake, 1, 1 << 24, 128, 1, fake, fake, 128, 64, 1,
                             ctypes.c_float(1.0), fake, None, None) == -2
    assert L.sparse_attn_fwd(fake, 128, fake, fake, None, fake, 1, 1 << 25, 64, 1, fake, fake, 128, 64, 1,
                             ctypes.c_float(1.0), fake, None, None) == -2


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2602_01801_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libfastar.so")
    with pytest.raises(binding.FastarError, match="no fallback"):
        binding.lib()
