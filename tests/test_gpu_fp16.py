"""The fp16 variant of the MFMA path (same kernels with the other 16-bit format) against the oracle."""
import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import MoEWorkload, generate, workload
from gpu_util import TOL, host32, host_inputs, nrm_err, run_hip_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("T,d,f,E,k,routing", [
    (700, 128, 192, 3, 2, "topk"), (1500, 64, 64, 5, 2, "zipf"), (2048, 320, 448, 32, 1, "forced"),
    (5, 64, 128, 4, 2, "topk"), (4096, 384, 1536, 8, 2, "topk"), (20000, 64, 64, 2, 2, "topk"),
])
def test_fp16_parity(oracle, T, d, f, E, k, routing):
    w = MoEWorkload("h", T, d, f, E, k, "f16", routing, 300 + T)
    data = generate(w, DEV)
    assert data["x"].dtype == torch.float16
    idx, y, g = run_hip_layer(w, data)
    assert y.dtype == torch.float16 and g["dx"].dtype == torch.float16
    c = host_inputs(data)
    counts, offsets, perm, inv = oracle.index(c["topk_idx"], w.E)
    assert np.array_equal(idx["perm"].cpu().numpy(), perm)
    args = (c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"])
    y_ref = oracle.fwd(*args, c["b2"])
    dx_ref, dg_ref = oracle.bwd_tokens(*args, c["b2"], c["dY"])
    dW1, db1, dW2, db2 = oracle.bwd_experts(*args, c["dY"])
    errs = {}
    for name, got, ref in (("y", y, y_ref), ("dx", g["dx"], dx_ref), ("dgate", g["dgate"], dg_ref),
                           ("dW1", g["dW1"], dW1), ("db1", g["db1"], db1), ("dW2", g["dW2"], dW2),
                           ("db2", g["db2"], db2)):
        errs[name] = nrm_err(host32(got), ref)
    print({k_: f"{v:.2e}" for k_, v in errs.items()}, flush=True)
    for name, v in errs.items():
        assert v <= TOL["f16"], name
    for e in np.nonzero(counts == 0)[0]:
        for n in ("dW1", "db1", "dW2", "db2"):
            assert float(g[n][e].abs().max()) == 0.0, (n, e)
