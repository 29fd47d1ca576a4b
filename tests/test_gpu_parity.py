"""GPU parity: the HIP library (through the C ABI) against the CPU oracle, element by element.

Tolerances (max-abs normalised per output tensor): 1e-5 for fp32, 2e-2 for bf16 inputs with
fp32 accumulation; index outputs are compared bit for bit.
"""
import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import MoEWorkload, generate, workload
from gpu_util import TOL, host32, host_inputs, nrm_err, run_hip_layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def check_index(oracle, w, data, idx):
    ti = data["topk_idx"].cpu().numpy()
    counts, offsets, perm, inv = oracle.index(ti, w.E)
    assert np.array_equal(idx["counts"].cpu().numpy(), counts)
    assert np.array_equal(idx["offsets"].cpu().numpy(), offsets)
    assert np.array_equal(idx["perm"].cpu().numpy(), perm)
    assert np.array_equal(idx["inv"].cpu().numpy(), inv)
    return counts


def full_parity(oracle, w, data, label=""):
    idx, y, g = run_hip_layer(w, data)
    counts = check_index(oracle, w, data, idx)
    c = host_inputs(data)
    tol = TOL[w.dtype]
    y_ref = oracle.fwd(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["b2"])
    dx_ref, dg_ref = oracle.bwd_tokens(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"],
                                       c["b2"], c["dY"])
    dW1, db1, dW2, db2 = oracle.bwd_experts(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"],
                                            c["W2"], c["dY"])
    errs = {
        "y": nrm_err(host32(y), y_ref), "dx": nrm_err(host32(g["dx"]), dx_ref),
        "dgate": nrm_err(host32(g["dgate"]), dg_ref), "dW1": nrm_err(host32(g["dW1"]), dW1),
        "db1": nrm_err(host32(g["db1"]), db1), "dW2": nrm_err(host32(g["dW2"]), dW2),
        "db2": nrm_err(host32(g["db2"]), db2),
    }
    print(label or w.name, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= tol, (k, v, tol)
    for e in np.nonzero(counts == 0)[0]:       # experts without tokens: exact zeros
        for n in ("dW1", "db1", "dW2", "db2"):
            assert float(g[n][e].abs().max()) == 0.0, (n, e)
    return errs


def test_c1_fp32_full(oracle, dev):
    w = workload("C1")
    full_parity(oracle, w, generate(w, dev))


@pytest.mark.parametrize("T,d,f,E,k", [(37, 20, 52, 3, 2), (300, 64, 96, 5, 3), (1, 8, 8, 1, 1)])
def test_fp32_odd_shapes(oracle, dev, T, d, f, E, k):
    w = MoEWorkload("odd", T, d, f, E, k, "f32", "topk", 99 + T)
    full_parity(oracle, w, generate(w, dev), label=f"f32 T{T} d{d} f{f} E{E} k{k}")


@pytest.mark.parametrize("T,d,f,E,k,routing", [
    (700, 128, 192, 3, 2, "topk"),        # segments of ~470 rows: one full 256 tile + ragged tail
    (1500, 64, 64, 5, 2, "zipf"),         # smallest legal feature sizes, skewed segments
    (2048, 320, 448, 32, 1, "forced"),    # empty experts, one long segment, N tails (320, 448 % 256 != 0)
    (5, 64, 128, 4, 2, "topk"),           # fewer rows than one MFMA block
])
def test_bf16_small_shapes(oracle, dev, T, d, f, E, k, routing):
    w = MoEWorkload("small", T, d, f, E, k, "bf16", routing, 7 + T)
    full_parity(oracle, w, generate(w, dev), label=f"bf16 T{T} d{d} f{f} E{E} k{k} {routing}")


@pytest.mark.parametrize("T,d,f,E,k,routing", [
    (70000, 64, 512, 8, 2, "zipf"),       # 140 000 rows = ~550 row tiles = ~138 groups of four
    (70000, 64, 256, 64, 2, "bias"),      # the same with 64 experts (C5's count): many segment tails
])
def test_bf16_many_row_tiles_full(oracle, dev, T, d, f, E, k, routing):
    """Row GEMMs deal their 256-row tiles to the eight XCDs in groups of four, and once there are
    128 groups or more (only C5-sized problems otherwise) the last, partial round of groups is
    dealt whole instead of being cut in eight.  Small feature sizes let the oracle check every
    element of such a problem."""
    w = MoEWorkload("many-tiles", T, d, f, E, k, "bf16", routing, 4242 + E)
    data = generate(w, dev)
    counts = np.bincount(data["topk_idx"].cpu().numpy().ravel(), minlength=E)
    assert sum(-(-int(n) // 256) for n in counts) >= 4 * 128
    full_parity(oracle, w, data, label=f"bf16 T{T} d{d} f{f} E{E} k{k} {routing}")


def test_c2_bf16_full(oracle, dev):
    w = workload("C2")
    full_parity(oracle, w, generate(w, dev))


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_index_bit_exact_all_configs(oracle, dev, name):
    from paper_2411_01288_amd import binding as B
    w = workload(name)
    gen = torch.Generator(device=dev); gen.manual_seed(w.seed)
    from paper_2411_01288_amd.workloads import _route
    topk_idx, _ = _route(w, gen, dev)
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype)
    idx = B.hexa_moe_index(shape, topk_idx)
    torch.cuda.synchronize()
    counts = check_index(oracle, w, {"topk_idx": topk_idx}, idx)
    assert counts.sum() == w.A
    if name == "C4":
        assert counts[0] == w.T // 2 and all(counts[e] == 0 for e in (1, 15, 16, 31))


@pytest.mark.parametrize("T,k,E", [(1, 1, 1), (63, 1, 7), (64, 2, 64), (65, 3, 1000), (100000, 3, 1024),
                                   (70000, 1, 2)])
def test_index_edge_shapes(oracle, dev, T, k, E):
    from paper_2411_01288_amd import binding as B
    g = torch.Generator(device=dev); g.manual_seed(T * 31 + E)
    topk_idx = torch.randint(0, E, (T, k), generator=g, device=dev, dtype=torch.int32)
    if E > 4:
        topk_idx[topk_idx == 3] = 0
    shape = B.make_shape(T, 64, 64, E, k, "bf16")
    idx = B.hexa_moe_index(shape, topk_idx)
    torch.cuda.synchronize()
    check_index(oracle, MoEWorkload("i", T, 64, 64, E, k, "bf16", "topk", 0), {"topk_idx": topk_idx}, idx)
