"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2411_01288_amd import build as bld
    if not os.path.exists(bld.LIB):
        bld.build_library()
    from paper_2411_01288_amd import binding
    return binding


def header_functions():
    text = open(os.path.join(ROOT, "include", "hexa_moe.h")).read()
    return sorted(set(re.findall(r"HEXA_API[^;(]*?\b(hexa_moe_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol(B):
    names = header_functions()
    assert len(names) >= 8
    assert sorted(B.EXPORTS) == names
    for n in names:
        assert getattr(B.lib, n) is not None


def test_size_queries_and_shape_validation(B):
    ok = B.make_shape(4096, 384, 1536, 8, 2, "bf16")
    assert B.workspace_bytes(ok) > 4096 * 2 * 1536 * 2 * 2
    assert B.index_scratch_bytes(ok) >= 8 * 4
    f32 = B.make_shape(7, 5, 3, 2, 1, "f32")            # fp32 takes any positive sizes
    assert B.workspace_bytes(f32) > 0
    for bad in (B.make_shape(0, 64, 64, 4, 1, "bf16"), B.make_shape(8, 64, 64, 0, 1, "bf16"),
                B.make_shape(8, 64, 64, 4, 0, "bf16"), B.make_shape(8, -64, 64, 4, 1, "bf16"),
                B.make_shape(8, 64, 64, 2000, 1, "bf16"),          # E > 1024
                B.make_shape(2 ** 30, 64, 64, 4, 4, "bf16"),       # T*k overflows int32
                B.make_shape(8, 60, 64, 4, 1, "bf16"),             # bf16 needs multiples of 64
                B.Shape(8, 64, 64, 4, 1, 7, 0),                    # unknown dtype
                B.make_shape(8, 64, 64, 4, 1, "bf16", 3)):         # unknown activation
        assert B.workspace_bytes(bad) == 0 and B.index_scratch_bytes(bad) == 0


def test_error_codes_without_touching_a_gpu(B):
    lib = B.lib
    ok = B.make_shape(8, 64, 64, 4, 1, "bf16")
    none = B.Idx()
    P = ctypes.c_void_p
    assert lib.hexa_moe_index(None, None, none, None, 0, None) == 1                      # NULL shape
    assert lib.hexa_moe_index(ctypes.byref(ok), None, none, None, 0, None) == 1          # NULL pointers
    bad = B.make_shape(8, 60, 64, 4, 1, "bf16")
    assert lib.hexa_moe_index(ctypes.byref(bad), None, none, None, 0, None) == 3         # unsupported
    neg = B.make_shape(-1, 64, 64, 4, 1, "bf16")
    assert lib.hexa_moe_index(ctypes.byref(neg), None, none, None, 0, None) == 2         # shape
    fake = P(4096)   # never dereferenced: the size check fails first
    idx = B.Idx(fake, fake, fake, fake)
    assert lib.hexa_moe_index(ctypes.byref(ok), fake, idx, fake, 0, None) == 4           # scratch too small
    assert lib.hexa_moe_fwd(ctypes.byref(ok), fake, fake, fake, fake, fake, fake, fake, idx, fake,
                            fake, 16, None) == 4                                         # workspace too small
    assert lib.hexa_moe_bwd(ctypes.byref(ok), fake, fake, fake, fake, fake, fake, idx, fake, 16, fake,
                            fake, fake, fake, fake, None, None) == 4
    assert lib.hexa_moe_fwd(ctypes.byref(ok), None, fake, fake, fake, fake, fake, fake, idx, fake,
                            fake, 1 << 40, None) == 1
    # router front-end: k > E and k > 64 are unsupported, E > 1024 is a shape error
    assert lib.hexa_moe_route(None, fake, 0, fake, fake, None) == 1
    assert lib.hexa_moe_route(ctypes.byref(ok), None, 0, fake, fake, None) == 1
    assert lib.hexa_moe_route(ctypes.byref(B.make_shape(8, 64, 64, 4, 5, "bf16")), fake, 0, fake, fake, None) == 3
    assert lib.hexa_moe_route(ctypes.byref(B.make_shape(8, 64, 64, 128, 65, "bf16")), fake, 0, fake, fake, None) == 3
    assert lib.hexa_moe_route(ctypes.byref(ok), fake, 2, fake, fake, None) == 3
    assert lib.hexa_moe_route(ctypes.byref(B.make_shape(8, 64, 64, 2000, 2, "bf16")), fake, 0, fake, fake, None) == 2
    flop = ctypes.c_double()
    assert lib.hexa_moe_mfma_probe(0, 10, fake, None, ctypes.byref(flop)) == 2
    assert lib.hexa_moe_mfma_probe(4, 10, None, None, ctypes.byref(flop)) == 1
    for code in range(6):
        assert lib.hexa_moe_status_string(code)
    assert b"unknown" in lib.hexa_moe_status_string(99)


def test_binding_checks_tensor_shapes_on_the_host(B):
    import torch
    shape = B.make_shape(8, 64, 64, 4, 1, "bf16")
    with pytest.raises(ValueError):
        B._ptr(torch.zeros(8, 64), (8, 64), torch.bfloat16, "x")     # not a device tensor
    with pytest.raises(B.HexaError) as ei:
        B._check(3)
    assert ei.value.code == 3


def test_heterogeneous_allocation(B):
    """Eq. 1 / Eq. 2: shares proportional to 1/latency, integral, exact sum."""
    from fractions import Fraction
    assert B.allocate([1.0, 1.0, 1.0, 1.0], 128) == [32, 32, 32, 32]
    assert B.allocate([1.0, 2.0], 90) == [60, 30]                       # twice as fast, twice the batch
    assert B.allocate([2.0, 1.0, 1.0], 8192, 64) == [1664, 3264, 3264]  # 25.6 / 51.2 / 51.2 granules -> 26 / 51 / 51
    got = B.allocate([1.0, 1.0, 1.0], 10)
    assert got == [4, 3, 3]                                             # ties go to the lower device index
    lat = [0.8, 1.3, 2.9, 1.0, 5.5]
    for total, g in ((1000, 1), (4096, 64), (40, 8), (0, 1)):
        s = B.allocate(lat, total, g)
        assert sum(s) == total and all(v % g == 0 and v >= 0 for v in s)
        w = [Fraction(1) / Fraction(t) for t in lat]
        for v, wi in zip(s, w):                                        # within one granule of the ideal share
            assert abs(Fraction(v) - wi / sum(w) * total) < g
    for bad in (([1.0, 0.0], 10, 1), ([1.0, -2.0], 10, 1), ([1.0], 10, 3), ([], 10, 1), ([1.0], -1, 1)):
        with pytest.raises(B.HexaError):
            B.allocate(*bad)


def test_bench_refuses_more_than_one_gpu():
    """The measured path is one GPU's share; bench.py says so instead of running N > 1."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "single-GPU" in (r.stdout + r.stderr)
