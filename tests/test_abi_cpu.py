"""CPU-only checks of the C ABI: the library loads, exports what include/floe.h declares, and rejects
bad arguments before touching the device (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2505_05950_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2505_05950_amd import build
        build.build()
    return binding.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "floe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(floe_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"floe_quantize_expert", "floe_expert_ffn_sparse", "floe_moe_layer_decode", "floe_stage_channels"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings_and_version(lib):
    assert lib.floe_abi_version() >= 1
    seen = {lib.floe_status_string(s) for s in range(0, -7, -1)}
    assert len(seen) == 7 and all(seen)


def test_argument_validation_happens_before_any_device_work(lib):
    from paper_2505_05950_amd.binding import _Expert, _Shape
    fake = C.c_void_p(4096)            # never dereferenced: every call below must fail validation first

    def q(d, f, bits, group):
        s = _Shape(d, f, bits, group)
        return lib.floe_quantize_expert(C.byref(s), fake, fake, fake, fake, None)

    assert q(4096, 16, 5, 64) == -3            # bits
    assert q(4096, 16, 2, 48) == -3            # group not a power of two in range
    assert q(4096 + 64, 16, 2, 128) == -2      # d % group
    assert q(4096 + 64, 16, 2, 64) == -2       # d % 512
    assert q(16384, 16, 2, 64) == -3           # d too large
    assert q(4096, 0, 2, 64) == -1
    s = _Shape(4096, 16, 2, 64)
    assert lib.floe_quantize_expert(C.byref(s), None, fake, fake, fake, None) == -1
    assert lib.floe_up_gemv(C.byref(s), fake, fake, fake, fake, -1, fake, None) == -1
    assert lib.floe_up_gemv(C.byref(s), fake, fake, fake, C.c_void_p(4098), 1, fake, None) == -1   # misaligned x
    assert lib.floe_select_channels(fake, 0, 1, fake, fake, fake, None) == -1
    e = _Expert(s, 4096, 4096, 4096, 4096, 0, 16)
    ws = C.c_void_p(1 << 20)
    need = lib.floe_expert_workspace_bytes(C.byref(s), 1)
    assert need > 0
    assert lib.floe_expert_ffn_sparse(C.byref(e), fake, 1, fake, None, fake, fake, fake, ws, need - 1, None) == -4
    e_bad = _Expert(s, 4096, 4096, 4096, 4096, 0, 15)                                   # gd_rows != f
    assert lib.floe_expert_ffn_sparse(C.byref(e_bad), fake, 1, fake, None, fake, fake, fake, ws, need, None) == -1
    assert lib.floe_stage_channels(None, 4096, 16, fake, fake, 4, fake, None, None, None) == -1
    assert lib.floe_expert_workspace_bytes(C.byref(_Shape(4096, 16, 7, 64)), 1) == 0
