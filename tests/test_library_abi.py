"""The C-ABI library loads and exports every symbol that include/poly.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2507_14959_amd", "libpoly.so")


def _declared():
    names = set()
    for header in ("poly.h", "poly_profile.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(poly_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_entry_points():
    names = _declared()
    for n in ("poly_select", "poly_forward", "poly_lora_linear", "poly_forward_workspace_bytes", "poly_status_string"):
        assert n in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail("libpoly.so is not built: run `python -m paper_2507_14959_amd.build`")
    lib = ctypes.CDLL(LIB)
    for n in _declared():
        assert hasattr(lib, n), n
    from paper_2507_14959_amd import binding
    assert sorted(binding.EXPORTS) == _declared()
    # host-only calls: sizes and strings
    assert binding.status_string(0) == "ok" and "range" in binding.status_string(-2)
    assert binding.poly_select_state_bytes(80) == 16 + 16
    assert binding.poly_lora_linear_workspace_bytes(4, 197, 16, 8, 1) > 8 * 197 * 16 * 2


def test_workspace_size_grows_with_rows_and_rejects_bad_models():
    from paper_2507_14959_amd import binding, synth
    import ctypes as C
    cfg = synth.CFG2
    d = binding.ModelDesc(cfg.H, cfg.W, cfg.patch, cfg.D, cfg.heads, cfg.L, cfg.Dm, 0, cfg.targets, cfg.r, cfg.n_adapters,
                          cfg.C, cfg.dtype, 1.0, 1e-6, 0)
    f = binding.lib().poly_forward_workspace_bytes
    a, b = f(C.byref(d), 32, 58), f(C.byref(d), 32, 96)
    assert 0 < a < b
    d.D = 200      # not 64 * heads
    assert f(C.byref(d), 32, 58) == 0
