"""GPU behaviour beyond element-wise parity: run-to-run reproducibility, repeated backward on
one saved workspace, gate == 1 (the paper's unweighted top-k sum), dropped expert ids."""
import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import MoEWorkload, generate, workload
from gpu_util import TOL, host32, host_inputs, nrm_err, run_hip_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_bitwise_reproducible_and_bwd_can_repeat():
    from paper_2411_01288_amd import binding as B
    w = MoEWorkload("rep", 3000, 256, 512, 7, 2, "bf16", "zipf", 5)
    data = generate(w, DEV)
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype)
    outs = []
    for _ in range(2):
        idx, y, g = run_hip_layer(w, data)
        outs.append((y.clone(), {k: v.clone() for k, v in g.items()}))
    assert torch.equal(outs[0][0], outs[1][0])
    for k in outs[0][1]:
        assert torch.equal(outs[0][1][k], outs[1][1][k]), k
    # backward twice on the workspace one forward left behind
    idx = B.hexa_moe_index(shape, data["topk_idx"])
    ws = B.alloc_workspace(shape, DEV)
    B.hexa_moe_fwd(shape, data["x"], data["topk_idx"], data["gate"], data["W1"], data["b1"],
                   data["W2"], data["b2"], idx, ws)
    g1 = {k: v.clone() for k, v in B.hexa_moe_bwd(shape, data["dY"], data["x"], data["topk_idx"],
                                                  data["gate"], data["W1"], data["W2"], idx, ws).items()}
    g2 = B.hexa_moe_bwd(shape, data["dY"], data["x"], data["topk_idx"], data["gate"], data["W1"],
                        data["W2"], idx, ws)
    torch.cuda.synchronize()
    for k in g1:
        assert torch.equal(g1[k], g2[k]), k


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_unit_gates_give_the_unweighted_topk_sum(oracle, dtype):
    """gate == 1 is the paper's own top-k formulation (App. B Table 5 row 3)."""
    w = MoEWorkload("g1", 500, 64, 128, 4, 3, dtype, "topk", 21)
    data = generate(w, DEV)
    data["gate"] = torch.ones_like(data["gate"])
    _, y, g = run_hip_layer(w, data)
    c = host_inputs(data)
    y_ref = oracle.fwd(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["b2"])
    dx_ref, _ = oracle.bwd_tokens(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["b2"], c["dY"])
    assert nrm_err(host32(y), y_ref) <= TOL[dtype]
    assert nrm_err(host32(g["dx"]), dx_ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_out_of_range_expert_ids_are_dropped_not_faulted(oracle, dtype):
    from paper_2411_01288_amd import binding as B
    w = MoEWorkload("drop", 700, 64, 128, 5, 2, dtype, "topk", 33)
    data = generate(w, DEV)
    bad_rows = torch.tensor([3, 77, 400, 699], device=DEV)
    data["topk_idx"][bad_rows, 0] = torch.tensor([5, -1, 1000, -7], device=DEV, dtype=torch.int32)
    idx, y, g = run_hip_layer(w, data)
    offs = idx["offsets"].cpu().numpy()
    assert offs[-1] == w.A - 4                               # detectable: offsets[E] < A
    inv = idx["inv"].cpu().numpy().reshape(w.T, w.k)
    assert all(inv[r, 0] == -1 for r in bad_rows.cpu().tolist())
    assert np.all(idx["perm"].cpu().numpy()[offs[-1]:] == -1)
    # equivalent valid problem: those four assignments contribute nothing
    c = host_inputs(data)
    ti = c["topk_idx"].copy()
    gate = c["gate"].copy()
    for r in bad_rows.cpu().tolist():
        ti[r, 0] = 0
        gate[r, 0] = 0.0
    y_ref = oracle.fwd(c["x"], ti, gate, c["W1"], c["b1"], c["W2"], c["b2"])
    dx_ref, _ = oracle.bwd_tokens(c["x"], ti, gate, c["W1"], c["b1"], c["W2"], c["b2"], c["dY"])
    assert nrm_err(host32(y), y_ref) <= TOL[dtype]
    assert nrm_err(host32(g["dx"]), dx_ref) <= TOL[dtype]
    dg = g["dgate"].cpu().numpy()
    assert all(dg[r, 0] == 0.0 for r in bad_rows.cpu().tolist())
    for n in ("dW1", "dW2", "db1", "db2"):
        assert bool(torch.isfinite(g[n]).all())
