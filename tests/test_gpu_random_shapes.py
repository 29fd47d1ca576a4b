"""Seeded random shapes through the whole layer against the oracle: odd token counts, feature sizes
that are multiples of 64 but not of the 256-wide tile, 1..40 experts, top-1..4, uniform and skewed
routing (segment lengths that are not multiples of the 64-row K block, segments longer than one
weight-gradient chunk, empty experts).  T >= 7: the tolerance is normalised by the largest reference
entry of a tensor, which means little for a dgate of one or two dot products that happen to cancel."""
import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import MoEWorkload, generate
from gpu_util import TOL, host32, host_inputs, nrm_err, run_hip_layer

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        T = int(rng.choice([7, 63, 64, 65, 255, 257, 511, 1000, 1999, 3001, 4500]))
        d = 64 * int(rng.integers(1, 9))
        f = 64 * int(rng.integers(1, 13))
        E = int(rng.choice([1, 2, 3, 5, 8, 17, 40]))
        k = int(rng.integers(1, 5))
        routing = str(rng.choice(["topk", "zipf"])) if E >= k else "topk"
        out.append((T, d, f, E, min(k, E), routing, 1000 + i))
    return out


EXTREMES = [
    (300, 64, 64, 1024, 2, "topk", 501),      # the largest expert count: almost every expert empty or one row
    (2000, 64, 128, 1024, 3, "zipf", 502),
    (20000, 64, 64, 2, 2, "topk", 503),       # long segments, several weight-gradient chunks, tiny features
    (257, 1024, 64, 3, 1, "topk", 504),       # d >> f
    (257, 64, 1536, 3, 1, "topk", 505),       # f >> d
    (500, 128, 192, 8, 8, "topk", 506),       # top-8 of 8 (the paper's largest k): every token visits every expert
    (1200, 64, 128, 32, 8, "zipf", 507),      # top-8 of 32 under skew
]


@pytest.mark.parametrize("T,d,f,E,k,routing,seed", _cases(20, 20241127) + EXTREMES)
def test_random_bf16_shape(oracle, T, d, f, E, k, routing, seed):
    w = MoEWorkload("rnd", T, d, f, E, k, "bf16", routing, seed)
    data = generate(w, DEV)
    print(f"case T={T} d={d} f={f} E={E} k={k} {routing} seed={seed}", flush=True)
    idx, y, g = run_hip_layer(w, data)
    c = host_inputs(data)
    counts, offsets, perm, inv = oracle.index(c["topk_idx"], w.E)
    assert np.array_equal(idx["perm"].cpu().numpy(), perm) and np.array_equal(idx["inv"].cpu().numpy(), inv)
    args = (c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"])
    y_ref = oracle.fwd(*args, c["b2"])
    dx_ref, dg_ref = oracle.bwd_tokens(*args, c["b2"], c["dY"])
    dW1, db1, dW2, db2 = oracle.bwd_experts(*args, c["dY"])
    tol = TOL["bf16"]
    for name, got, ref in (("y", y, y_ref), ("dx", g["dx"], dx_ref), ("dgate", g["dgate"], dg_ref),
                           ("dW1", g["dW1"], dW1), ("db1", g["db1"], db1), ("dW2", g["dW2"], dW2),
                           ("db2", g["db2"], db2)):
        assert nrm_err(host32(got), ref) <= tol, name
    for e in np.nonzero(counts == 0)[0]:
        for n in ("dW1", "db1", "dW2", "db2"):
            assert float(g[n][e].abs().max()) == 0.0, (n, e)
