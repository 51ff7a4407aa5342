"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the header
declares, sizes its workspaces from host fields, and rejects bad arguments before any HIP call.
(Every call below is built to fail validation, so nothing is ever launched.)"""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2605_07719_amd import fluxion as F

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "fluxion.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fx_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert {"fx_summarize", "fx_select", "fx_sparse_decode", "fx_status_string"} <= set(names)
    lib = F.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert set(F.EXPORTS) == set(names)


def test_status_strings():
    assert F.status_string(F.FX_OK) == "ok"
    texts = {F.status_string(s) for s in range(6)}
    assert len(texts) == 6 and all(texts)
    assert F.status_string(99)


class HostLayout:
    """An fx_layout whose 'device' arrays are host dummies: only for calls that fail validation."""

    def __init__(self, batch=2, hq=8, hkv=2, d=128, max_seq_len=4096, gran=(32, 32), token_stride=None,
                 kv_head_stride=None):
        self.seq_len = np.full(batch, max_seq_len, np.int32)
        self.seq_base = np.zeros(batch, np.int64)
        self.sum_base = np.zeros(batch * hkv, np.int64)
        self.gran = np.asarray(gran, np.int32)
        self.c = F._CLayout(batch, hq, hkv, d, max_seq_len, self.seq_len.ctypes.data, self.seq_base.ctypes.data,
                            kv_head_stride if kv_head_stride is not None else max_seq_len * d,
                            token_stride if token_stride is not None else d, self.sum_base.ctypes.data,
                            self.gran.ctypes.data)


def ws_bytes(L, k_max=64, sink=64, window=256):
    lib = F.lib()
    return (lib.fx_select_workspace_bytes(ctypes.byref(L.c)),
            lib.fx_decode_workspace_bytes(ctypes.byref(L.c), k_max, sink, window))


def test_workspace_sizes_follow_host_fields():
    a = ws_bytes(HostLayout())
    assert a[0] > 0 and a[1] > 0
    assert ws_bytes(HostLayout(max_seq_len=8192))[0] == 2 * a[0]            # per (b, h, block) scratch
    assert ws_bytes(HostLayout(batch=4))[0] == 2 * a[0]
    assert ws_bytes(HostLayout(), k_max=128)[1] >= a[1]
    # select: fp32 score (tiles of 16) + u64 key per (batch, q head, block), fp32 magnitude per 16 blocks
    assert a[0] == 2 * 8 * (4096 // 32) * 12 + 2 * 8 * 8 * 4
    assert ws_bytes(HostLayout(gran=(32, 24)))[0] == 0                       # invalid layout -> 0


@pytest.mark.parametrize("kwargs, status", [
    (dict(d=96), F.FX_ERR_UNSUPPORTED),
    (dict(hq=7), F.FX_ERR_INVALID_ARG),
    (dict(hq=32, hkv=2, gran=(32, 32)), F.FX_ERR_UNSUPPORTED),              # group of 16
    (dict(gran=(32, 20)), F.FX_ERR_UNSUPPORTED),
    (dict(gran=(32, 256)), F.FX_ERR_UNSUPPORTED),
    (dict(max_seq_len=(1 << 19) + 1), F.FX_ERR_UNSUPPORTED),
    (dict(token_stride=64), F.FX_ERR_INVALID_ARG),                           # < head_dim
    (dict(token_stride=132), F.FX_ERR_INVALID_ARG),                          # not a multiple of 8
    (dict(batch=0), F.FX_ERR_INVALID_ARG),
])
def test_bad_layouts_are_rejected(kwargs, status):
    L = HostLayout(**kwargs)
    buf = np.zeros(64, np.uint8)
    p = ctypes.c_void_p(buf.ctypes.data)
    lib = F.lib()
    assert lib.fx_summarize(ctypes.byref(L.c), p, p, None) == status
    assert lib.fx_select(ctypes.byref(L.c), p, p, p, None, 64, 256, 8, p, p, p, 1 << 40, None) == status
    assert lib.fx_sparse_decode(ctypes.byref(L.c), p, p, p, p, p, 8, 64, 256, p, p, 1 << 40, None) == status


def test_bad_arguments_are_rejected_before_any_launch():
    L = HostLayout()
    lib = F.lib()
    buf = np.zeros(256, np.uint8)
    base = buf.ctypes.data + (-buf.ctypes.data % 16)
    p = ctypes.c_void_p(base)
    odd = ctypes.c_void_p(base + 2)
    need_sel, need_dec = ws_bytes(L, k_max=8)
    INV, SMALL = F.FX_ERR_INVALID_ARG, F.FX_ERR_WORKSPACE_TOO_SMALL
    assert lib.fx_summarize(None, p, p, None) == INV
    assert lib.fx_summarize(ctypes.byref(L.c), None, p, None) == INV
    assert lib.fx_summarize(ctypes.byref(L.c), odd, p, None) == INV
    # select: both / neither budget, k_max, sink/window, null outputs, alignment, workspace size
    sel = lambda *a: lib.fx_select(ctypes.byref(L.c), *a)
    assert sel(p, p, p, p, 64, 256, 8, p, p, p, need_sel, None) == INV
    assert sel(p, p, None, None, 64, 256, 8, p, p, p, need_sel, None) == INV
    assert sel(p, p, p, None, 64, 256, 0, p, p, p, need_sel, None) == INV
    assert sel(p, p, p, None, -1, 256, 8, p, p, p, need_sel, None) == INV
    assert sel(p, p, p, None, 64, 256, 8, None, p, p, need_sel, None) == INV
    assert sel(odd, p, p, None, 64, 256, 8, p, p, p, need_sel, None) == INV
    assert sel(p, p, p, None, 64, 256, 8, p, p, p, need_sel - 1, None) == SMALL
    dec = lambda *a: lib.fx_sparse_decode(ctypes.byref(L.c), *a)
    assert dec(p, p, p, p, p, 8, 64, 256, None, p, need_dec, None) == INV
    assert dec(p, odd, p, p, p, 8, 64, 256, p, p, need_dec, None) == INV
    assert dec(p, p, p, p, p, 8, 64, -5, p, p, need_dec, None) == INV
    assert dec(p, p, p, p, p, 8, 64, 256, p, p, need_dec - 1, None) == SMALL
    # the variant with built-in scratch: same checks, and a problem no launch size could fit is refused on the host
    stat = lambda L_, *a: lib.fx_sparse_decode_static(ctypes.byref(L_.c), *a)
    assert stat(L, p, p, p, p, p, 8, 64, 256, None, None) == INV
    assert stat(L, p, odd, p, p, p, 8, 64, 256, p, None) == INV
    assert stat(L, p, p, p, p, p, 0, 64, 256, p, None) == INV
    huge = HostLayout(batch=512, hq=8, hkv=8, d=64, max_seq_len=1 << 19, gran=(16,) * 8)  # 4096 union lists of 32768 entries
    assert stat(huge, p, p, p, p, p, 1 << 15, 64, 256, p, None) == F.FX_ERR_SCRATCH_LIMIT
    # measurement aids
    assert lib.fx_profile_read(None, 5) == INV
    assert lib.fx_probe_read(None, 1024, p, 4, None) == INV
    assert lib.fx_probe_read_streaming(None, 1024, p, 4, None) == INV
    assert lib.fx_probe_copy(p, p, 8, 4, None) == INV


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(F, "_lib", None)
    monkeypatch.setattr(F, "LIB_PATH", "/nonexistent/libfluxion.so")
    with pytest.raises(ImportError):
        F.lib()


def test_product_and_oracle_do_not_reach_into_each_other():
    """The oracle is test infrastructure: nothing under the package may import, load or run it, and the oracle
    may not use the package's code (only the seeded input generators are shared, by the tests)."""
    import pathlib
    import re

    root = pathlib.Path(__file__).resolve().parents[1]
    pkg = root / "paper_2605_07719_amd"
    for path in list(pkg.rglob("*.py")) + list(pkg.rglob("*.hip")) + list(pkg.rglob("*.hpp")) + list(pkg.rglob("*.cpp")):
        text = path.read_text()
        assert not re.search(r"^\s*(from|import)\s+oracle\b", text, re.M), path
        assert "fx_oracle" not in text and "libfx_oracle" not in text, path
    for path in (root / "oracle").rglob("*"):
        if path.suffix in (".py", ".cpp", ".h", ".hpp"):
            text = path.read_text()
            assert "paper_2605_07719_amd" not in text and "libfluxion" not in text and "fluxion.h" not in text, path
