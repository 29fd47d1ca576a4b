"""Model-centric use of the same entry points (Sec. 3.3, tensor parallelism over the FFN hidden size):
each device would hold W1[:, :, f_i], b1[:, f_i], W2[:, f_i, :] and run the unchanged layer with
d_ff = |f_i|; GELU is elementwise in f, so the partial outputs add up (b2 counted once).  Here the
slices run one after the other on the one GPU, with unequal sizes from the heterogeneous split
(Eq. 2), and their sum / concatenation is checked against the oracle on the full layer."""
import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import MoEWorkload, generate
from gpu_util import TOL, host32, host_inputs, nrm_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_hidden_size_slices_add_up(oracle, dtype):
    from paper_2411_01288_amd import binding as B
    w = MoEWorkload("tp", 700, 128, 512, 5, 2, dtype, "zipf", 21)
    data = generate(w, DEV)
    shares = B.allocate([1.0, 2.5, 1.6], w.d_ff, 64)        # three unequal "devices"
    assert sum(shares) == w.d_ff and len(set(shares)) > 1
    shape_full = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype)
    idx = B.hexa_moe_index(shape_full, data["topk_idx"])
    y = torch.zeros((w.T, w.d_model), dtype=torch.float32, device=DEV)
    dx = torch.zeros_like(y)
    dgate = torch.zeros((w.T, w.k), dtype=torch.float32, device=DEV)
    db2 = None
    dW1, db1, dW2 = [], [], []
    lo = 0
    for r, fi in enumerate(shares):
        sl = slice(lo, lo + fi); lo += fi
        shape = B.make_shape(w.T, w.d_model, fi, w.E, w.k, w.dtype)
        W1 = data["W1"][:, :, sl].contiguous(); b1 = data["b1"][:, sl].contiguous()
        W2 = data["W2"][:, sl, :].contiguous()
        b2 = data["b2"] if r == 0 else torch.zeros_like(data["b2"])   # the bias is added on one rank
        ws = B.alloc_workspace(shape, DEV)
        yi = B.hexa_moe_fwd(shape, data["x"], data["topk_idx"], data["gate"], W1, b1, W2, b2, idx, ws)
        g = B.hexa_moe_bwd(shape, data["dY"], data["x"], data["topk_idx"], data["gate"], W1, W2, idx, ws)
        y += yi.float(); dx += g["dx"].float(); dgate += g["dgate"]
        dW1.append(g["dW1"]); db1.append(g["db1"]); dW2.append(g["dW2"])
        db2 = g["db2"] if r == 0 else db2           # every rank computes the same db2
        if r > 0:
            assert torch.equal(g["db2"], db2)
    torch.cuda.synchronize()
    c = host_inputs(data)
    args = (c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"])
    ry = oracle.fwd(*args, c["b2"])
    rdx, rdgate = oracle.bwd_tokens(*args, c["b2"], c["dY"])
    rdW1, rdb1, rdW2, rdb2 = oracle.bwd_experts(*args, c["dY"])
    tol = TOL[dtype] * 3        # three partial results, each rounded to the element type, are added
    assert nrm_err(host32(y), ry) <= tol
    assert nrm_err(host32(dx), rdx) <= tol
    assert nrm_err(host32(dgate), rdgate) <= tol
    assert nrm_err(host32(torch.cat(dW1, dim=2)), rdW1) <= TOL[dtype]
    assert nrm_err(host32(torch.cat(db1, dim=1)), rdb1) <= TOL[dtype]
    assert nrm_err(host32(torch.cat(dW2, dim=1)), rdW2) <= TOL[dtype]
    assert nrm_err(host32(db2), rdb2) <= TOL[dtype]
