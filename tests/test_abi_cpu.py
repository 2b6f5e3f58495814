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


def test_tuning_switch_validates_its_arguments(lib):
    bad = [(1, 4), (1, -1), (2, 4097), (2, -1), (3, 3), (3, -1), (4, 257), (4, -1), (0, 0), (9, 0)]
    for key, value in bad:
        assert lib.floe_tuning(key, value) == -1, (key, value)
    try:
        for key, values in ((1, (1, 2, 3)), (2, (1, 32, 4096)), (3, (1, 2)), (4, (1, 16, 256))):
            for v in values:
                assert lib.floe_tuning(key, v) == 0, (key, v)
    finally:
        for key in (1, 2, 3, 4):
            assert lib.floe_tuning(key, 0) == 0


def test_layer_workspace_query_for_every_path_the_dispatch_can_take(lib):
    """The workspace plan (host logic only) for the two layer shapes of the benchmark at batch sizes on both sides of
    every dispatch boundary, under every tuning: a size is returned, it holds at least the partial results of one block
    per (token, slot), and it is the same when asked twice (the decode call sizes its pointers with the same routine)."""
    from paper_2505_05950_amd.binding import _Layer, _Shape
    lib.floe_layer_workspace_bytes.restype = C.c_size_t
    fake = C.c_void_p(4096)
    shapes = [(4096, 14336, 2, 64, 8, 2, 0), (2048, 1408, 3, 32, 64, 6, 2), (1024, 300, 4, 128, 3, 1, 1),
              (1536, 700, 8, 64, 100, 4, 0)]
    try:
        for fused_tasks in (0, 16, 256):
            for grouped in (0, 1, 2):
                for union in (0, 1, 2, 3):
                    lib.floe_tuning(4, fused_tasks), lib.floe_tuning(3, grouped), lib.floe_tuning(1, union)
                    for d, f, bits, group, n, top_k, n_shared in shapes:
                        L = _Layer(n, top_k, n_shared, 1, _Shape(d, f, bits, group), 4096, None, 4096, 0, 4096, 0)
                        slots = top_k + n_shared
                        for T in (1, 2, 3, 4, 8, 9, 16, 17, 32, 33, 64, 128, 500, 4096):
                            need = lib.floe_layer_workspace_bytes(C.byref(L), T)
                            assert need >= T * slots * d * 4, (d, f, bits, n, T, fused_tasks, grouped, union)
                            assert need == lib.floe_layer_workspace_bytes(C.byref(L), T)
                            assert need < (64 << 30)
                        assert lib.floe_layer_workspace_bytes(C.byref(L), -1) == 0
                        assert lib.floe_moe_layer_decode(C.byref(L), fake, 1, fake, None, fake, 16, None) == -4
    finally:
        for key in (1, 3, 4):
            lib.floe_tuning(key, 0)
