"""The C-ABI library builds, loads and exports every symbol include/rad.h
declares; no compute call is made (no GPU here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    hdr = open(os.path.join(ROOT, "include", "rad.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return sorted(set(re.findall(r"\b(rad_[A-Za-z_0-9]+)\s*\(", hdr)))


@pytest.fixture(scope="module")
def lib():
    from paper_2007_10412_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2007_10412_amd import binding
    names = _declared()
    assert len(names) >= 25
    for n in names:
        assert hasattr(lib, n), n
        assert n in binding.SIGNATURES, n + " missing from the Python binding"
        assert hasattr(binding, n), n


def test_fixed_k_host_function(lib):
    from oracle import rad_oracle as R
    for p, d in [(0.1, 784), (0.1, 300), (0.1, 16384), (0.5, 4096), (0.02, 4096), (1.0, 10), (0.1, 1)]:
        assert lib.rad_fixed_k(p, d) == R.fixed_k(p, d)


def test_null_and_missing_device_are_status_codes(lib):
    from paper_2007_10412_amd import binding as B
    assert lib.rad_ctx_destroy(None) == B.RAD_ERR_NULL
    assert lib.rad_ctx_create(None, None) == B.RAD_ERR_NULL
    assert lib.rad_last_error(None) == b"no context"
    import torch
    if not torch.cuda.is_available():
        ctx = ctypes.c_void_p()
        assert lib.rad_ctx_create(ctypes.byref(ctx), None) == B.RAD_ERR_DEVICE   # no CPU fallback
        assert not ctx.value


def test_product_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2007_10412_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"(import|from)\s+oracle|oracle[./]", text), f
    assert "paper_2007_10412_amd" not in open(os.path.join(ROOT, "oracle", "rad_oracle.py")).read()
