"""The C-ABI library loads, exports every symbol include/flare.h declares, and rejects bad
arguments on the host before anything is launched (no GPU needed, no compute calls)."""
import ctypes
import os
import re

import pytest

from paper_2508_12594_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2508_12594_amd import build
        build.build_library(verbose=False)
    return binding.load()


def _declared(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(flare_[a-z_]+)\s*\(", text))


def test_header_symbols_are_exported(lib):
    """Every function an include/*.h declares is exported by the library it belongs to, and the bindings
    list exactly those: flare.h (the operator) and flare_profile.h (timing hooks) -> libflare.so,
    flare_rates.h (machine-rate micro-benchmarks) -> libflare_rates.so."""
    headers = sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h"))
    assert headers == ["flare.h", "flare_profile.h", "flare_rates.h"]
    declared = sorted(_declared("flare.h") | _declared("flare_profile.h"))
    assert declared == sorted(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    from paper_2508_12594_amd import rates
    rl = rates.load()
    assert sorted(_declared("flare_rates.h")) == sorted(rates.EXPORTS)
    for name in rates.EXPORTS:
        assert hasattr(rl, name), name
    assert rl.flare_rates_count() == len(rates.names()) > 10


def test_version_and_strerror(lib):
    assert binding.version() >= 200
    assert binding.strerror(0) == "success"
    for code in (-1, -2, -3, -4, -5, -6, -99):
        assert len(binding.strerror(code)) > 0


def test_workspace_bytes_and_shape_checks(lib):
    f, b = binding.workspace_bytes(1, 8, 1000000, 256, 16, binding.FLARE_BF16)
    assert 0 < f < 64 << 20 and b > 0
    f1, _ = binding.workspace_bytes(1, 4, 1024, 64, 32, binding.FLARE_F32)
    assert f1 > 0 and f1 % 256 == 0
    bad = [(0, 1, 1, 1, 16, 0, -1), (1, 1, 1, 1, 5, 0, -2), (1, 1, 1, 1, 16, 7, -2), (70000, 1, 1, 1, 16, 0, -2)]
    for B, H, N, M, d, dt, want in bad:
        shp = binding.FlareShape(B, H, N, M, d, dt)
        assert lib.flare_workspace_bytes(ctypes.byref(shp), None, None) == want
    assert lib.flare_workspace_bytes(None, None, None) == -1
    shp = binding.FlareShape(1, 1, 8, 32, 16, binding.FLARE_F32, 0, 2)      # shared_latents must be 0 or 1
    assert lib.flare_workspace_bytes(ctypes.byref(shp), None, None) == -1
    shp = binding.FlareShape(1, 1, 8, 32, 16, binding.FLARE_F32, 0, 0, 0, 4)   # unknown variant bit
    assert lib.flare_workspace_bytes(ctypes.byref(shp), None, None) == -1
    shp = binding.FlareShape(1, 1, 8, 32, 16, binding.FLARE_F32, 0, 0, 0, 3)   # both known bits
    assert lib.flare_workspace_bytes(ctypes.byref(shp), None, None) == 0


def test_null_and_misaligned_pointers_are_rejected(lib):
    shp = binding.FlareShape(1, 1, 8, 32, 16, binding.FLARE_F32)
    p = ctypes.c_void_p(4096)        # never dereferenced: the checks fail first
    odd = ctypes.c_void_p(4100)
    one = ctypes.c_float(1)
    assert lib.flare_forward(ctypes.byref(shp), None, p, p, p, p, p, None, one, p, 1 << 20, None) == -1
    assert lib.flare_forward(ctypes.byref(shp), p, p, p, None, p, p, None, one, p, 1 << 20, None) == -1
    assert lib.flare_forward(ctypes.byref(shp), p, odd, p, p, p, p, None, one, p, 1 << 20, None) == -3
    assert lib.flare_forward(ctypes.byref(shp), p, p, p, p, p, p, odd, one, p, 1 << 20, None) == -3
    assert lib.flare_forward(ctypes.byref(shp), p, p, p, p, p, p, None, one, p, 16, None) == -4
    assert lib.flare_forward(ctypes.byref(shp), p, p, p, p, p, p, None, one, None, 0, None) == -4
    assert lib.flare_decode(ctypes.byref(shp), p, p, None, p, None, one, None, 0, None) == -1
    # the entry point with the static scratch: shape and size checks come before anything touches a device
    big = binding.FlareShape(1, 8, 1 << 20, 2048, 8, binding.FLARE_BF16)
    assert lib.flare_forward_static(ctypes.byref(big), p, p, p, p, p, p, None, one, None) == -6
    assert lib.flare_forward_static(None, p, p, p, p, p, p, None, one, None) == -1
    assert lib.flare_backward(ctypes.byref(shp), p, p, p, None, None, None, p, p, p, p, p, one, p,
                              1 << 20, None) == -1
    assert lib.flare_backward(ctypes.byref(shp), p, p, p, None, None, p, p, p, p, p, p, one, p,
                              16, None) == -4
