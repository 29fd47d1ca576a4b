"""Router front-end on the GPU against the oracle: indices bit-exact (selection is comparisons
only), gates within fp32 rounding of the fp64 softmax; then the routed layer end to end."""
import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import MoEWorkload, generate
from gpu_util import TOL, host32, nrm_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GATE_TOL = 2e-6   # |gate - ref| with gates <= 1: exp and the division in fp32, sums of <= 1024 terms


def _logits(T, E, seed, ties=False):
    g = torch.Generator(device="cpu").manual_seed(seed)
    if ties:   # few distinct values: most comparisons are between equal logits
        return torch.randint(-2, 3, (T, E), generator=g).float()
    return torch.randn(T, E, generator=g) * 2.0


@pytest.mark.parametrize("T,E,k", [(1000, 4, 1), (4096, 8, 2), (5000, 64, 2), (777, 60, 8), (300, 100, 8),
                                   (130, 1024, 4), (50, 5, 5), (3, 64, 64), (1, 1, 1), (257, 200, 64)])
@pytest.mark.parametrize("mode", [0, 1])
def test_route_matches_oracle(oracle, T, E, k, mode):
    from paper_2411_01288_amd import binding as B
    logits = _logits(T, E, 1000 + T + E + k)
    shape = B.make_shape(T, 64, 64, E, k, "bf16")
    idx, gate = B.hexa_moe_route(shape, logits.to(DEV), mode)
    torch.cuda.synchronize()
    ridx, rgate = oracle.route(logits.numpy(), k, mode)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.abs(gate.cpu().numpy().astype(np.float64) - rgate).max() <= GATE_TOL


@pytest.mark.parametrize("T,E,k", [(2000, 12, 3), (500, 70, 5), (64, 8, 8)])
def test_route_ties_bit_exact(oracle, T, E, k):
    from paper_2411_01288_amd import binding as B
    logits = _logits(T, E, 5 + E, ties=True)
    shape = B.make_shape(T, 64, 64, E, k, "bf16")
    idx, gate = B.hexa_moe_route(shape, logits.to(DEV), 0)
    torch.cuda.synchronize()
    ridx, rgate = oracle.route(logits.numpy(), k, 0)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.abs(gate.cpu().numpy().astype(np.float64) - rgate).max() <= GATE_TOL


def test_route_full_size_c5_shape(oracle):
    """T = 131072, E = 64, top-2 (the C5 routing problem), every row checked."""
    from paper_2411_01288_amd import binding as B
    T, E, k = 131072, 64, 2
    logits = _logits(T, E, 77)
    shape = B.make_shape(T, 2048, 8192, E, k, "bf16")
    idx, gate = B.hexa_moe_route(shape, logits.to(DEV), 0)
    torch.cuda.synchronize()
    ridx, rgate = oracle.route(logits.numpy(), k, 0)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.abs(gate.cpu().numpy().astype(np.float64) - rgate).max() <= GATE_TOL
    assert np.abs(gate.cpu().numpy().sum(1) - 1).max() < 1e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_routed_layer_end_to_end(oracle, dtype):
    """logits -> route -> index -> fwd -> bwd on the GPU against logits -> oracle route -> oracle layer."""
    from paper_2411_01288_amd import binding as B
    w = MoEWorkload("routed", 900, 128, 256, 6, 2, dtype, "topk", 11)
    data = generate(w, DEV)
    logits = _logits(w.T, w.E, 12)
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype)
    tk, gate = B.hexa_moe_route(shape, logits.to(DEV), 0)
    idx = B.hexa_moe_index(shape, tk)
    ws = B.alloc_workspace(shape, DEV)
    y = B.hexa_moe_fwd(shape, data["x"], tk, gate, data["W1"], data["b1"], data["W2"], data["b2"], idx, ws)
    g = B.hexa_moe_bwd(shape, data["dY"], data["x"], tk, gate, data["W1"], data["W2"], idx, ws)
    torch.cuda.synchronize()
    ridx, rgate = oracle.route(logits.numpy(), w.k, 0)
    assert np.array_equal(tk.cpu().numpy(), ridx)
    c = {n: host32(data[n]) for n in ("x", "W1", "b1", "W2", "b2", "dY")}
    rg32 = rgate.astype(np.float32)   # the layer takes fp32 gates
    ry = oracle.fwd(c["x"], ridx, rg32, c["W1"], c["b1"], c["W2"], c["b2"])
    rdx, rdgate = oracle.bwd_tokens(c["x"], ridx, rg32, c["W1"], c["b1"], c["W2"], c["b2"], c["dY"])
    rdW1, rdb1, rdW2, rdb2 = oracle.bwd_experts(c["x"], ridx, rg32, c["W1"], c["b1"], c["W2"], c["dY"])
    tol = TOL[dtype] * (2 if dtype == "f32" else 1)   # gates differ from the oracle's by fp32 rounding
    assert nrm_err(host32(y), ry) <= tol
    assert nrm_err(host32(g["dx"]), rdx) <= tol
    assert nrm_err(host32(g["dgate"]), rdgate) <= tol
    for n, r in (("dW1", rdW1), ("db1", rdb1), ("dW2", rdW2), ("db2", rdb2)):
        assert nrm_err(host32(g[n]), r) <= tol, n
