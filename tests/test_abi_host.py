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
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, n)).read() for n in sorted(os.listdir(inc)) if n.endswith(".h"))
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
    assert B.workspace_bytes(B.make_shape((1 << 19) - 2, 4096, 64, 4, 1, "bf16")) > 0   # (T+1)*d*2 = 2^32 - 8192: the largest x
    assert B.workspace_bytes(f32) > 0
    for bad in (B.make_shape(0, 64, 64, 4, 1, "bf16"), B.make_shape(8, 64, 64, 0, 1, "bf16"),
                B.make_shape(8, 64, 64, 4, 0, "bf16"), B.make_shape(8, -64, 64, 4, 1, "bf16"),
                B.make_shape(8, 64, 64, 2000, 1, "bf16"),          # E > 1024
                B.make_shape(2 ** 30, 64, 64, 4, 4, "bf16"),       # T*k overflows int32
                B.make_shape(8, 60, 64, 4, 1, "bf16"),             # bf16 needs multiples of 64
                B.make_shape(8, 64, 1 << 23, 4, 1, "bf16"),        # 256 rows of d_ff exceed 32-bit byte offsets
                B.make_shape(1 << 21, 64, 1 << 21, 4, 1, "bf16"),  # one 256-row fp32 output window reaches 2^31 bytes
                B.make_shape((1 << 19) - 1, 4096, 64, 4, 1, "bf16"),  # x and one more row reach 2^32 bytes
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
    # the allocation-free index: same checks, and a shape beyond its built-in scratch is refused
    assert lib.hexa_moe_index_static(None, fake, idx, None) == 1
    assert lib.hexa_moe_index_static(ctypes.byref(ok), None, idx, None) == 1
    assert lib.hexa_moe_index_static(ctypes.byref(bad), fake, idx, None) == 3
    wide = B.make_shape(100000, 64, 64, 1024, 3, "bf16")
    assert B.index_scratch_bytes(wide) > B.INDEX_STATIC_SCRATCH_BYTES
    assert lib.hexa_moe_index_static(ctypes.byref(wide), fake, idx, None) == 4
    # router front-end: k > E and k > 64 are unsupported, E > 1024 is a shape error
    assert lib.hexa_moe_route(None, fake, 0, fake, fake, None) == 1
    assert lib.hexa_moe_route(ctypes.byref(ok), None, 0, fake, fake, None) == 1
    assert lib.hexa_moe_route(ctypes.byref(B.make_shape(8, 64, 64, 4, 5, "bf16")), fake, 0, fake, fake, None) == 3
    assert lib.hexa_moe_route(ctypes.byref(B.make_shape(8, 64, 64, 128, 65, "bf16")), fake, 0, fake, fake, None) == 3
    assert lib.hexa_moe_route(ctypes.byref(ok), fake, 2, fake, fake, None) == 3
    assert lib.hexa_moe_route(ctypes.byref(B.make_shape(8, 64, 64, 2000, 2, "bf16")), fake, 0, fake, fake, None) == 2
    flop = ctypes.c_double()
    assert lib.hexa_moe_mfma_probe(0, 0, 10, fake, None, ctypes.byref(flop)) == 2
    assert lib.hexa_moe_mfma_probe(0, 4, 10, None, None, ctypes.byref(flop)) == 1
    assert lib.hexa_moe_mfma_probe(3, 4, 10, fake, None, ctypes.byref(flop)) == 3
    # alignment: a workspace base off the 256-byte grid, a tensor pointer off the 16-byte grid
    big = 1 << 40
    odd_ws, odd_x = P(4096 + 64), P(4096 + 8)
    assert lib.hexa_moe_fwd(ctypes.byref(ok), fake, fake, fake, fake, fake, fake, fake, idx, fake,
                            odd_ws, big, None) == 4
    assert lib.hexa_moe_fwd(ctypes.byref(ok), odd_x, fake, fake, fake, fake, fake, fake, idx, fake,
                            fake, big, None) == 3
    assert lib.hexa_moe_bwd(ctypes.byref(ok), fake, fake, fake, fake, fake, fake, idx, odd_ws, big, fake,
                            fake, fake, fake, fake, None, None) == 4
    assert lib.hexa_moe_bwd(ctypes.byref(ok), fake, fake, fake, fake, fake, fake, idx, fake, big, fake,
                            odd_x, fake, fake, fake, None, None) == 3
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


def test_heterogeneous_allocation_against_the_oracle(B):
    """hexa_moe_allocate (Sec. 3.4 Eq. 1 / Eq. 2, largest-remainder rounding) against the exact
    rational oracle: hand cases, seeded random cases, and its error returns."""
    import numpy as np
    from oracle.allocate_oracle import allocate as ref
    hand = [([1.0, 1.0, 1.0, 1.0], 128, 1), ([1.0, 2.0], 90, 1), ([2.0, 1.0, 1.0], 8192, 64),
            ([1.0, 1.0, 1.0], 10, 1), ([1.0, 1.0, 1.0], 11, 1), ([0.5, 0.25, 1.0], 6, 1),
            ([4.58, 3.06], 100, 1), ([3.20, 3.18], 100, 1), ([3.28, 9.42], 100, 1),   # Sec. 4 Table 2
            ([5.0], 77, 7), ([1.0, 4.0], 0, 1)]
    for lat, total, g in hand:
        assert B.allocate(lat, total, g) == ref(lat, total, g), (lat, total, g)
    rng = np.random.default_rng(2024)
    for _ in range(500):
        n = int(rng.integers(1, 9))
        lat = [float(x) for x in rng.uniform(0.1, 20.0, n)]
        g = int(rng.choice([1, 8, 64]))
        total = g * int(rng.integers(0, 2000))
        assert B.allocate(lat, total, g) == ref(lat, total, g), (lat, total, g)
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
