"""Host-side checks of the C interface that need no GPU: the library loads, exports every
symbol the header declares, and its host helpers behave (no compute calls here)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2105_08764_amd as s2v

    if not os.path.exists(s2v.LIB_PATH):
        from paper_2105_08764_amd import build

        build.build()
    return s2v.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "s2v.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(s2v_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    import paper_2105_08764_amd as s2v

    names = declared_functions()
    assert set(names) == set(s2v.EXPORTS)
    for name in names:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    import paper_2105_08764_amd as s2v

    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -6):
        text = s2v.s2v_status_str(code)
        assert text and text not in seen
        seen.add(text)
    assert s2v.s2v_status_str(-99) == "unknown status"


def test_adaptive_d_table(lib):
    # Sec. 4.5.1: d = 8 / 4 / 2 / 1 by |C| against N/2, N/4, N/8 (table kept in tests/golden)
    import paper_2105_08764_amd as s2v

    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "adaptive_d_table.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 10
    for c, n, d in rows:
        assert s2v.s2v_adaptive_d(int(c), int(n)) == int(d), (c, n, d)


def test_create_without_gpu_reports_no_device(lib):
    import torch

    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    handle = ctypes.c_void_p()
    rc = lib.s2v_create(None, ctypes.byref(handle))
    assert rc == -5 and not handle.value
    assert lib.s2v_create(None, None) == -1


def test_workspace_bytes_is_host_only_and_monotone(lib):
    import paper_2105_08764_amd as s2v

    def need(n, nnz, G, p, T, S, k, training):
        g = s2v.CGraph(n, nnz, None, None, None, G, None)
        out = ctypes.c_size_t(0)
        rc = lib.s2v_workspace_bytes(None, ctypes.byref(g), p, T, S, k, int(training), ctypes.byref(out))
        return rc, out.value

    rc, a = need(1000, 10000, 1, 32, 3, 1, 1, False)
    assert rc == 0 and a >= 1000 * 32 * 4
    rc, b = need(1000, 10000, 1, 32, 3, 1, 1, True)
    assert rc == 0 and b > a
    rc, c = need(2_000_000, 60_000_000, 1, 64, 4, 1, 19000, False)
    assert rc == 0 and 2_000_000 * 64 * 4 <= c < 2 * 2_000_000 * 64 * 4      # about one extra embedding
    assert need(1000, 10000, 1, 48, 3, 1, 1, False)[0] == -2                    # unsupported p
    assert need(1000, 10000, 0, 32, 3, 1, 1, False)[0] == -1                    # G < 1
    assert need(1000, 10000, 1, 32, 0, 1, 1, False)[0] == -1                    # T < 1
    assert need(2**27, 10, 1, 64, 2, 16, 1, False)[0] == -2                     # N*S >= 2^31


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    import paper_2105_08764_amd as s2v

    monkeypatch.setattr(s2v, "_lib", None)
    monkeypatch.setattr(s2v, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(FileNotFoundError):
        s2v.load_library()
