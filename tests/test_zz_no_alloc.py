"""hexa_moe_index_static, the entry point that allocates nothing (its scratch is a fixed array in
the library's device memory), against hexa_moe_index: bit-exact, on two calls in a row that
share the array, the second on a smaller input, and once more after other work."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(B, T, k, E, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    topk_idx = torch.randint(0, E, (T, k), generator=g, device=DEV, dtype=torch.int32)
    topk_idx[topk_idx == 2] = 0                                    # an empty expert, a heavy one
    shape = B.make_shape(T, 64, 64, E, k, "bf16")
    want = B.hexa_moe_index(shape, topk_idx)
    got = B.alloc_idx(shape, DEV)
    for t in got.values():
        t.fill_(-7)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    print(f"index_static T={T} k={k} E={E}", flush=True)
    B.hexa_moe_index_static(shape, topk_idx, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name in ("counts", "offsets", "perm", "inv"):
        assert torch.equal(got[name], want[name]), (name, T, k, E)
    return got


def test_index_static_matches_index_on_consecutive_calls():
    from paper_2411_01288_amd import binding as B
    big = _both(B, 131072, 2, 64, 1)        # the largest workload's index: 1024 chunks x 64 experts
    small = _both(B, 1000, 3, 37, 2)        # then a smaller one: the array still holds the first call's histogram
    assert int(big["offsets"][-1]) == 262144 and int(small["offsets"][-1]) == 3000
    _both(B, 65, 1, 256, 3)                 # a single partial chunk row, the widest E the array always covers
    _both(B, 131072, 2, 64, 1)              # and the large one again


def test_index_static_rejects_shapes_beyond_its_scratch():
    from paper_2411_01288_amd import binding as B
    shape = B.make_shape(100000, 64, 64, 1024, 3, "bf16")       # 1024 chunks x 1024 experts x 4 B = 4 MiB
    assert B.index_scratch_bytes(shape) > B.INDEX_STATIC_SCRATCH_BYTES
    idx = B.alloc_idx(shape, DEV)
    topk_idx = torch.zeros((100000, 3), dtype=torch.int32, device=DEV)
    with pytest.raises(B.HexaError) as ei:
        B.hexa_moe_index_static(shape, topk_idx, idx)
    assert ei.value.code == 4
