"""GPU parity at the full sizes of the named workloads C3, C4, C5, in the launch configuration
bench.py times.  The oracle cannot redo these sizes whole, so: the index is compared in full
(bit-exact); y, dx, dgate on sampled tokens (random ones, every token of the smallest expert,
a slice of the largest); dW1, db1, dW2, db2 on sampled experts (largest, smallest non-empty,
one more) x sampled hidden units, all rows.  Empty experts must give exact zeros.
"""
import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import generate, workload
from gpu_util import TOL, host32, nrm_err, run_hip_layer

pytestmark = pytest.mark.gpu


def sampled_parity(oracle, w, n_tokens=192, n_cols=12, seed=0):
    dev = torch.device("cuda:0")
    data = generate(w, dev)
    idx, y, g = run_hip_layer(w, data)
    ti = data["topk_idx"].cpu().numpy()
    counts, offsets, perm, inv = oracle.index(ti, w.E)
    assert np.array_equal(idx["counts"].cpu().numpy(), counts)
    assert np.array_equal(idx["offsets"].cpu().numpy(), offsets)
    assert np.array_equal(idx["perm"].cpu().numpy(), perm)
    assert np.array_equal(idx["inv"].cpu().numpy(), inv)
    assert counts.sum() == w.A

    c = {k: host32(v) for k, v in data.items() if k != "topk_idx"}
    rng = np.random.default_rng(seed)
    nonempty = np.nonzero(counts)[0]
    e_small = nonempty[np.argmin(counts[nonempty])]
    e_big = int(np.argmax(counts))
    seg = lambda e: perm[offsets[e]:offsets[e + 1]] // w.k
    tok = np.unique(np.concatenate([rng.integers(0, w.T, n_tokens), seg(e_small)[:64],
                                    seg(e_big)[:32], seg(e_big)[-32:]])).astype(np.int32)
    tol = TOL[w.dtype]
    y_ref = oracle.fwd(c["x"], ti, c["gate"], c["W1"], c["b1"], c["W2"], c["b2"], tokens=tok)
    dx_ref, dg_ref = oracle.bwd_tokens(c["x"], ti, c["gate"], c["W1"], c["b1"], c["W2"], c["b2"],
                                       c["dY"], tokens=tok)
    tok_t = torch.from_numpy(tok.astype(np.int64)).to(dev)
    errs = {"y": nrm_err(host32(y[tok_t]), y_ref), "dx": nrm_err(host32(g["dx"][tok_t]), dx_ref),
            "dgate": nrm_err(host32(g["dgate"][tok_t]), dg_ref)}

    experts = np.unique([e_big, e_small, int(rng.choice(nonempty))]).astype(np.int32)
    cols = np.sort(rng.choice(w.d_ff, n_cols, replace=False)).astype(np.int32)
    dW1, db1, dW2, db2 = oracle.bwd_experts(c["x"], ti, c["gate"], c["W1"], c["b1"], c["W2"], c["dY"],
                                            experts=experts, cols=cols)
    ex_t = torch.from_numpy(experts.astype(np.int64)).to(dev)
    co_t = torch.from_numpy(cols.astype(np.int64)).to(dev)
    errs["dW1"] = nrm_err(host32(g["dW1"][ex_t][:, :, co_t]), dW1)
    errs["db1"] = nrm_err(host32(g["db1"][ex_t][:, co_t]), db1)
    errs["dW2"] = nrm_err(host32(g["dW2"][ex_t][:, co_t, :]), dW2)
    errs["db2"] = nrm_err(host32(g["db2"][ex_t]), db2)
    print(w.name, w.routing, "tokens/expert min", int(counts.min()), "max", int(counts.max()),
          {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= tol, (k, v, tol)
    for e in np.nonzero(counts == 0)[0]:
        for n in ("dW1", "db1", "dW2", "db2"):
            assert float(g[n][int(e)].abs().max()) == 0.0, (n, e)
    for n in ("dx", "dW1", "db1", "dW2", "db2", "dgate"):
        assert bool(torch.isfinite(g[n]).all()), n
    assert bool(torch.isfinite(y.float()).all())
    return counts


def test_c3_zipf_sampled(oracle):
    sampled_parity(oracle, workload("C3"))


def test_c4_forced_imbalance_sampled(oracle):
    counts = sampled_parity(oracle, workload("C4"))
    assert counts[0] == 32768 and all(counts[e] == 0 for e in (1, 15, 16, 31))


def test_c5_large_sampled(oracle):
    sampled_parity(oracle, workload("C5"))


def test_c5_shape_under_zipf_skew_sampled(oracle):
    """The largest shape with C3's Zipf(1.2) routing: one expert holds a large share of the rows,
    which exercises the split token contraction and its fixed-order reduction at full size."""
    sampled_parity(oracle, workload("C5", routing="zipf"), n_tokens=96, n_cols=8)


def test_c5_fp16_sampled(oracle):
    """The largest shape through the fp16 instantiation of the contraction kernels (same launch
    configuration; tolerance an eighth of bf16's)."""
    sampled_parity(oracle, workload("C5", dtype="f16"), n_tokens=96, n_cols=8)
