"""The paper's -1-padded re-index form on the GPU against the oracle, bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("T,k,E,blk", [(10, 1, 4, 4), (1000, 2, 7, 16), (333, 3, 5, 1), (4096, 1, 64, 64),
                                       (5, 2, 9, 8), (70000, 2, 1024, 32), (131072, 2, 64, 256)])
def test_padded_index_matches_oracle(oracle, T, k, E, blk):
    from paper_2411_01288_amd import binding as B
    g = torch.Generator().manual_seed(T + E + blk)
    topk = torch.randint(0, E, (T, k), generator=g, dtype=torch.int32)
    if E > 2:
        topk[topk == 1] = 0                       # an expert without tokens
    shape = B.make_shape(T, 64, 64, E, k, "bf16")
    idx = B.hexa_moe_index(shape, topk.to(DEV))
    v, starts = B.hexa_moe_padded_index(shape, idx, blk)
    torch.cuda.synchronize()
    rv, rs = oracle.padded_index(topk.numpy(), E, blk)
    assert v.numel() == T * k + E * (blk - 1) == rv.size
    assert np.array_equal(starts.cpu().numpy(), rs)
    assert np.array_equal(v.cpu().numpy(), rv)


def test_padded_index_rejects_bad_arguments():
    from paper_2411_01288_amd import binding as B
    shape = B.make_shape(64, 64, 64, 4, 1, "bf16")
    idx = B.hexa_moe_index(shape, torch.zeros((64, 1), dtype=torch.int32, device=DEV))
    with pytest.raises(B.HexaError):
        B.hexa_moe_padded_index(shape, idx, 0)
