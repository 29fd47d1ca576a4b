"""ReLU and SiLU through the whole layer on the GPU against the oracle (GELU-tanh, the default, is what
every other GPU test runs), fp32 and bf16."""
import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import MoEWorkload, generate
from gpu_util import TOL, host32, host_inputs, nrm_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture
def oracle_act(oracle):
    def choose(kind):
        oracle.set_activation(kind)
        return oracle
    yield choose
    oracle.set_activation(0)


@pytest.mark.parametrize("dtype,T,d,f,E,k", [("f32", 200, 24, 40, 3, 2), ("bf16", 900, 128, 320, 6, 2),
                                             ("bf16", 3000, 256, 512, 7, 2)])
@pytest.mark.parametrize("kind", [1, 2])
def test_activation_parity(oracle_act, kind, dtype, T, d, f, E, k):
    from paper_2411_01288_amd import binding as B
    O = oracle_act(kind)
    w = MoEWorkload("act", T, d, f, E, k, dtype, "zipf", 70 + kind)
    data = generate(w, DEV)
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype, activation=kind)
    idx = B.hexa_moe_index(shape, data["topk_idx"])
    ws = B.alloc_workspace(shape, DEV)
    y = B.hexa_moe_fwd(shape, data["x"], data["topk_idx"], data["gate"], data["W1"], data["b1"],
                       data["W2"], data["b2"], idx, ws)
    g = B.hexa_moe_bwd(shape, data["dY"], data["x"], data["topk_idx"], data["gate"], data["W1"],
                       data["W2"], idx, ws)
    torch.cuda.synchronize()
    c = host_inputs(data)
    args = (c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"])
    y_ref = O.fwd(*args, c["b2"])
    dx_ref, dg_ref = O.bwd_tokens(*args, c["b2"], c["dY"])
    dW1, db1, dW2, db2 = O.bwd_experts(*args, c["dY"])
    tol = TOL[dtype]
    for name, got, ref in (("y", y, y_ref), ("dx", g["dx"], dx_ref), ("dgate", g["dgate"], dg_ref),
                           ("dW1", g["dW1"], dW1), ("db1", g["db1"], db1), ("dW2", g["dW2"], dW2),
                           ("db2", g["db2"], db2)):
        assert nrm_err(host32(got), ref) <= tol, name
    # the three activations really differ: the GELU result is not within tolerance of this one
    shape0 = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype)
    y0 = B.hexa_moe_fwd(shape0, data["x"], data["topk_idx"], data["gate"], data["W1"], data["b1"],
                        data["W2"], data["b2"], idx, ws)
    torch.cuda.synchronize()
    assert nrm_err(host32(y0), y_ref) > 2.5 * tol
