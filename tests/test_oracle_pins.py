"""Pins for the CPU oracle: it is checked against things other than itself.

  * index      -> hand-worked fixture, numpy stable argsort, structural invariants
  * forward    -> dense "every expert for every token, then mask by routing"
                  brute force written in numpy (Sec. 3.1: both formulations give
                  each token the same output), and the E=1 case against a library MLP
  * backward   -> central finite differences of L = <y, dY> w.r.t. every input,
                  torch autograd over a per-expert python loop, closed-form invariants
  * activation -> values, symmetry, finite difference, library gelu(tanh)
None of these import or call anything of the HIP path.
"""
import os

import numpy as np
import pytest
import torch

from paper_2411_01288_amd.workloads import generate, workload
from conftest import to_np32

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def small_case(seed, T=24, d=8, f=16, E=5, k=2, dup=False):
    rng = np.random.default_rng(seed)
    c = dict(
        x=rng.standard_normal((T, d)).astype(np.float32),
        W1=(rng.standard_normal((E, d, f)) * 0.3).astype(np.float32),
        b1=(rng.standard_normal((E, f)) * 0.1).astype(np.float32),
        W2=(rng.standard_normal((E, f, d)) * 0.3).astype(np.float32),
        b2=(rng.standard_normal((E, d)) * 0.1).astype(np.float32),
        dY=rng.standard_normal((T, d)).astype(np.float32),
        gate=rng.uniform(0.1, 1.0, (T, k)).astype(np.float32),
        topk_idx=rng.integers(0, E, (T, k)).astype(np.int32),
    )
    if dup and k > 1:
        c["topk_idx"][0, 1] = c["topk_idx"][0, 0]      # one token picks an expert twice
    return c


def np_case(name, **ov):
    data = generate(workload(name, **ov))
    c = {k: to_np32(v) for k, v in data.items() if k != "topk_idx"}
    c["topk_idx"] = data["topk_idx"].numpy()
    return c


# ---------------------------------------------------------------- brute force
def gelu_np(u):
    return 0.5 * u * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (u + 0.044715 * u ** 3)))


def dense_masked_forward(c):
    """All E experts for every token (no index structures), masked by routing."""
    x = c["x"].astype(np.float64)
    T = x.shape[0]
    E = c["W1"].shape[0]
    pre = np.einsum("ti,eif->tef", x, c["W1"].astype(np.float64)) + c["b1"].astype(np.float64)[None]
    h = gelu_np(pre)
    o = np.einsum("tef,efm->tem", h, c["W2"].astype(np.float64)) + c["b2"].astype(np.float64)[None]
    m = np.zeros((T, E))
    for j in range(c["topk_idx"].shape[1]):
        np.add.at(m, (np.arange(T), c["topk_idx"][:, j]), c["gate"][:, j].astype(np.float64))
    return np.einsum("te,tem->tm", m, o), m, pre, h, o


def torch_loop_grads(c, act=None):
    """Library cross-check: autograd through a per-expert python loop, fp64."""
    act = act or (lambda z: torch.nn.functional.gelu(z, approximate="tanh"))
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=(k != "dY"))
         for k, v in c.items() if k != "topk_idx"}
    idx = torch.tensor(c["topk_idx"], dtype=torch.long)
    T, k = idx.shape
    y = torch.zeros_like(t["x"])
    for e in range(c["W1"].shape[0]):
        for j in range(k):
            rows = (idx[:, j] == e).nonzero().flatten()
            if rows.numel() == 0:
                continue
            h = act(t["x"][rows] @ t["W1"][e] + t["b1"][e])
            y = y.index_add(0, rows, t["gate"][rows, j, None] * (h @ t["W2"][e] + t["b2"][e]))
    (y * t["dY"]).sum().backward()
    g = lambda n: (t[n].grad if t[n].grad is not None else torch.zeros_like(t[n])).numpy()
    return y.detach().numpy(), {n: g(n) for n in ("x", "gate", "W1", "b1", "W2", "b2")}


def oracle_all(oracle, c):
    y = oracle.fwd(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["b2"])
    dx, dgate = oracle.bwd_tokens(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"],
                                  c["b2"], c["dY"])
    dW1, db1, dW2, db2 = oracle.bwd_experts(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"],
                                            c["W2"], c["dY"])
    return y, dict(x=dx, gate=dgate, W1=dW1, b1=db1, W2=dW2, b2=db2)


def rel(a, b):
    return np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300)


# ---------------------------------------------------------------------- index
def test_index_hand_worked_fixture(oracle):
    rows = {}
    for line in open(os.path.join(GOLD, "index_10tok_4exp.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        rows[key] = np.array(vals, dtype=np.int32)
    counts, offsets, perm, inv = oracle.index(rows["R"].reshape(-1, 1), 4)
    assert counts.tolist() == rows["counts"].tolist()
    assert offsets.tolist() == rows["offsets"].tolist()
    assert perm.tolist() == rows["perm"].tolist()
    assert inv.tolist() == rows["inv"].tolist()


@pytest.mark.parametrize("T,k,E,seed", [(1, 1, 1, 0), (7, 3, 2, 1), (1000, 2, 8, 2),
                                       (4096, 1, 64, 3), (513, 4, 5, 4)])
def test_index_is_stable_argsort_and_invariants(oracle, T, k, E, seed):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, E, (T, k)).astype(np.int32)
    if E > 3:
        idx[idx == 2] = 0                       # force an empty expert in the middle
    counts, offsets, perm, inv = oracle.index(idx, E)
    flat = idx.reshape(-1)
    A = T * k
    assert np.array_equal(perm, np.argsort(flat, kind="stable").astype(np.int32))
    assert np.array_equal(counts, np.bincount(flat, minlength=E))
    assert counts.sum() == A and offsets[0] == 0 and offsets[E] == A     # App. B, Table 4
    assert np.array_equal(np.sort(perm), np.arange(A))
    assert np.array_equal(inv[perm], np.arange(A))
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e)
        assert np.all(np.diff(seg) > 0)


def test_index_rejects_out_of_range(oracle):
    with pytest.raises(ValueError):
        oracle.index(np.array([[0], [4]], np.int32), 4)
    with pytest.raises(ValueError):
        oracle.index(np.array([[-1]], np.int32), 4)


# -------------------------------------------------------------------- forward
@pytest.mark.parametrize("seed,k,dup", [(0, 1, False), (1, 2, False), (2, 3, True)])
def test_forward_equals_dense_masked_bruteforce(oracle, seed, k, dup):
    c = small_case(seed, k=k, dup=dup)
    y = oracle.fwd(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["b2"])
    ref = dense_masked_forward(c)[0]
    assert rel(y, ref) < 1e-13


def test_forward_dense_bruteforce_on_C1(oracle):
    c = np_case("C1")
    y = oracle.fwd(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["b2"])
    assert rel(y, dense_masked_forward(c)[0]) < 1e-12


def test_forward_token_subset_is_a_slice(oracle):
    c = small_case(5, T=40)
    full = oracle.fwd(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["b2"])
    tok = np.array([39, 0, 17, 17, 3], np.int32)
    sub = oracle.fwd(c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["b2"], tokens=tok)
    assert np.array_equal(sub, full[tok])


def test_single_expert_is_a_plain_mlp(oracle):
    """E=1, k=1, gate=1: the layer is linear -> gelu(tanh) -> linear (library routine)."""
    c = small_case(7, T=33, d=12, f=20, E=1, k=1)
    c["gate"][:] = 1.0
    y, g = oracle_all(oracle, c)
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True)
         for k, v in c.items() if k in ("x", "W1", "b1", "W2", "b2")}
    h = torch.nn.functional.gelu(torch.nn.functional.linear(t["x"], t["W1"][0].T, t["b1"][0]),
                                 approximate="tanh")
    yt = torch.nn.functional.linear(h, t["W2"][0].T, t["b2"][0])
    (yt * torch.tensor(c["dY"], dtype=torch.float64)).sum().backward()
    assert rel(y, yt.detach().numpy()) < 1e-13
    for n in ("x", "W1", "b1", "W2", "b2"):
        assert rel(g[n], t[n].grad.numpy()) < 1e-12, n


# ------------------------------------------------------------------- backward
def test_backward_central_finite_differences(oracle):
    """L = <y, dY>; perturb every element of every input (float64-exact inputs)."""
    c = small_case(11, T=6, d=4, f=8, E=3, k=2, dup=True)
    c["topk_idx"][c["topk_idx"] == 1] = 2          # expert 1 is empty
    _, g = oracle_all(oracle, c)
    dY = c["dY"].astype(np.float64)

    def loss(cc):
        return float((oracle.fwd(cc["x"], cc["topk_idx"], cc["gate"], cc["W1"], cc["b1"],
                                 cc["W2"], cc["b2"]) * dY).sum())

    eps = 2.0 ** -7      # exactly representable steps on float32 inputs; the oracle is fp64 inside
    for name in ("x", "gate", "W1", "b1", "W2", "b2"):
        base = c[name]
        fd = np.zeros(base.shape, np.float64)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            # quantise the centre so +-eps stay exact in float32
            v0 = np.float32(np.round(base[i] * 64) / 64)
            cp, cm = dict(c), dict(c)
            cp[name] = base.copy(); cm[name] = base.copy()
            cp[name][i] = v0 + eps; cm[name][i] = v0 - eps
            c0 = dict(c); c0[name] = base.copy(); c0[name][i] = v0
            # Richardson: combine steps eps and eps/2 to cancel the O(eps^2) term
            ch, cmh = dict(c), dict(c)
            ch[name] = base.copy(); cmh[name] = base.copy()
            ch[name][i] = v0 + eps / 2; cmh[name][i] = v0 - eps / 2
            d1 = (loss(cp) - loss(cm)) / (2 * eps)
            d2 = (loss(ch) - loss(cmh)) / eps
            fd[i] = (4 * d2 - d1) / 3
            # analytic gradient must be taken at the quantised centre
            _, g0 = oracle_all(oracle, c0)
            ana = g0[name][i]
            assert abs(fd[i] - ana) <= 1e-6 * max(1.0, abs(ana)), (name, i, fd[i], ana)
    assert np.all(g["W1"][1] == 0) and np.all(g["W2"][1] == 0)
    assert np.all(g["b1"][1] == 0) and np.all(g["b2"][1] == 0)


@pytest.mark.parametrize("seed,k,dup", [(3, 1, False), (4, 2, True), (5, 4, True)])
def test_backward_matches_autograd_loop(oracle, seed, k, dup):
    c = small_case(seed, T=50, d=8, f=24, E=6, k=k, dup=dup)
    c["topk_idx"][c["topk_idx"] == 4] = 0          # empty expert
    y, g = oracle_all(oracle, c)
    yt, gt = torch_loop_grads(c)
    assert rel(y, yt) < 1e-13
    for n in g:
        assert rel(g[n], gt[n]) < 1e-12, n
    for n in ("W1", "b1", "W2", "b2"):
        assert np.all(g[n][4] == 0.0), n           # exact zeros, not small numbers


def test_backward_dense_masked_formulas_on_C1(oracle):
    c = np_case("C1")
    _, g = oracle_all(oracle, c)
    _, m, pre, h, o = dense_masked_forward(c)
    dY = c["dY"].astype(np.float64)
    # dW2[e] = sum_t m[t,e] h[t,e,:]^T dY[t,:]   ;  db2[e] = sum_t m[t,e] dY[t]
    assert rel(g["W2"], np.einsum("te,tef,tm->efm", m, h, dY)) < 1e-12
    assert rel(g["b2"], np.einsum("te,tm->em", m, dY)) < 1e-12
    # dgate[t,j] = <dY_t, o[t, idx[t,j]]>
    T = dY.shape[0]
    dg = np.stack([np.einsum("tm,tm->t", dY, o[np.arange(T), c["topk_idx"][:, j]])
                   for j in range(c["topk_idx"].shape[1])], 1)
    assert rel(g["gate"], dg) < 1e-12


def test_backward_invariants(oracle):
    c = small_case(21, T=64, d=8, f=16, E=6, k=2, dup=True)
    y, g = oracle_all(oracle, c)
    dY = c["dY"].astype(np.float64)
    # sum_e db2[e] = sum_t (sum_j g_tj) dY_t
    gs = c["gate"].astype(np.float64).sum(1)
    assert rel(g["b2"].sum(0), (gs[:, None] * dY).sum(0)) < 1e-13
    # permuting tokens permutes y, dx, dgate rows and leaves dW, db unchanged (up to sum order)
    p = np.random.default_rng(0).permutation(64)
    cp = dict(c)
    for n in ("x", "dY", "gate", "topk_idx"):
        cp[n] = c[n][p]
    yp, gp = oracle_all(oracle, cp)
    assert np.array_equal(yp, y[p]) and np.array_equal(gp["x"], g["x"][p])
    assert np.array_equal(gp["gate"], g["gate"][p])
    for n in ("W1", "b1", "W2", "b2"):
        assert rel(gp[n], g[n]) < 1e-13, n
    # y, dW2, db2 are linear in the gate
    c2 = dict(c); c2["gate"] = (c["gate"] * np.float32(2.0))
    y2, g2 = oracle_all(oracle, c2)
    assert rel(y2, 2 * y) < 1e-14 and rel(g2["W2"], 2 * g["W2"]) < 1e-14
    assert rel(g2["b2"], 2 * g["b2"]) < 1e-14
    # a token that picks one expert twice == one pick with the summed gate
    c3 = small_case(22, T=9, k=2)
    c3["topk_idx"][:, 1] = c3["topk_idx"][:, 0]
    c3["gate"] = np.float32(0.25) * np.ones_like(c3["gate"])
    c4 = dict(c3); c4["topk_idx"] = c3["topk_idx"][:, :1].copy()
    c4["gate"] = np.float32(0.5) * np.ones((9, 1), np.float32)
    y3, g3 = oracle_all(oracle, c3)
    y4, g4 = oracle_all(oracle, c4)
    assert rel(y3, y4) < 1e-14
    for n in ("x", "W1", "b1", "W2", "b2"):
        assert rel(g3[n], g4[n]) < 1e-13, n


def test_expert_and_column_restriction_is_a_slice(oracle):
    c = small_case(31, T=40, d=8, f=16, E=5, k=2)
    args = (c["x"], c["topk_idx"], c["gate"], c["W1"], c["b1"], c["W2"], c["dY"])
    dW1, db1, dW2, db2 = oracle.bwd_experts(*args)
    ex = np.array([3, 0], np.int32)
    cols = np.array([15, 2, 7], np.int32)
    sW1, sb1, sW2, sb2 = oracle.bwd_experts(*args, experts=ex, cols=cols)
    assert np.array_equal(sW1, dW1[ex][:, :, cols]) and np.array_equal(sb1, db1[ex][:, cols])
    assert np.array_equal(sW2, dW2[ex][:, cols, :]) and np.array_equal(sb2, db2[ex])
    full = oracle.bwd_tokens(*args[:6], c["b2"], c["dY"])
    tok = np.array([5, 39, 0], np.int32)
    sub = oracle.bwd_tokens(*args[:6], c["b2"], c["dY"], tokens=tok)
    assert np.array_equal(sub[0], full[0][tok]) and np.array_equal(sub[1], full[1][tok])


# ----------------------------------------------------------------- activation
def test_gelu_values_and_derivative(oracle):
    assert oracle.gelu(0.0) == 0.0
    assert oracle.gelu_grad(0.0) == 0.5
    for u in (0.1, 0.7, 1.3, 2.9, 6.0):
        assert abs(oracle.gelu(u) - oracle.gelu(-u) - u) < 1e-15 * max(1, u)
        lib = torch.nn.functional.gelu(torch.tensor([u, -u], dtype=torch.float64), approximate="tanh")
        assert abs(oracle.gelu(u) - lib[0].item()) < 1e-15
        assert abs(oracle.gelu(-u) - lib[1].item()) < 1e-15
        e = 1e-5
        fd = (oracle.gelu(u + e) - oracle.gelu(u - e)) / (2 * e)
        assert abs(fd - oracle.gelu_grad(u)) < 1e-9
        fd = (oracle.gelu(-u + e) - oracle.gelu(-u - e)) / (2 * e)
        assert abs(fd - oracle.gelu_grad(-u)) < 1e-9
    assert abs(oracle.gelu(30.0) - 30.0) < 1e-12 and abs(oracle.gelu(-30.0)) < 1e-12


# --------------------------------------------------------------------- router
# The paper takes the routing choice as given; the reading pinned here: k largest logits, equal
# logits to the lower expert id, slots by descending logit, softmax gates.
def _route_ref(logits, k, mode):
    """numpy / scipy only: a stable sort of the negated logits gives exactly that order."""
    from scipy.special import softmax
    order = np.argsort(-logits.astype(np.float64), axis=1, kind="stable")[:, :k]
    sel = np.take_along_axis(logits.astype(np.float64), order, axis=1)
    if mode == 0:
        gate = softmax(sel, axis=1)
    else:
        gate = np.take_along_axis(softmax(logits.astype(np.float64), axis=1), order, axis=1)
    return order.astype(np.int32), gate


@pytest.mark.parametrize("T,E,k", [(64, 4, 1), (200, 8, 2), (50, 64, 2), (33, 100, 8), (7, 5, 5)])
@pytest.mark.parametrize("mode", [0, 1])
def test_route_matches_stable_sort_and_library_softmax(oracle, T, E, k, mode):
    rng = np.random.default_rng(100 + T + E)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, gate = oracle.route(logits, k, mode)
    ridx, rgate = _route_ref(logits, k, mode)
    assert np.array_equal(idx, ridx)
    assert np.abs(gate - rgate).max() < 1e-14


def test_route_ties_go_to_the_lower_expert_id(oracle):
    rng = np.random.default_rng(7)
    logits = rng.integers(-2, 3, size=(300, 12)).astype(np.float32)   # many equal logits
    for k in (1, 3, 12):
        idx, gate = oracle.route(logits, k, 0)
        ridx, rgate = _route_ref(logits, k, 0)
        assert np.array_equal(idx, ridx)
        assert np.abs(gate - rgate).max() < 1e-14
    row = np.array([[1, 5, 5, 0, 5]], np.float32)
    idx, gate = oracle.route(row, 3, 0)
    assert idx.tolist() == [[1, 2, 4]] and np.allclose(gate, 1 / 3, atol=1e-15)


def test_route_invariants(oracle):
    rng = np.random.default_rng(8)
    logits = (3 * rng.standard_normal((128, 16))).astype(np.float32)
    idx, g0 = oracle.route(logits, 4, 0)
    _, g1 = oracle.route(logits, 4, 1)
    assert np.abs(g0.sum(1) - 1).max() < 1e-14                      # renormalised over the selection
    assert (np.diff(g0, axis=1) <= 0).all() and (g1.sum(1) < 1).all()
    assert np.abs(g1 / g1.sum(1, keepdims=True) - g0).max() < 1e-14  # same ratios in both modes
    assert all(len(set(r)) == 4 for r in idx.tolist())               # k distinct experts
    ia, ga = oracle.route(logits, 16, 0)                             # k = E: the full softmax, sorted
    _, gb = oracle.route(logits, 16, 1)
    assert np.abs(ga - gb).max() < 1e-14
    shifted, gs = oracle.route(logits + np.float32(8.0), 4, 0)       # exactly representable shift
    assert np.array_equal(shifted, idx) and np.abs(gs - g0).max() < 1e-6
    with pytest.raises(ValueError):
        oracle.route(logits, 17, 0)
    bad = logits.copy(); bad[3, 2] = np.nan
    with pytest.raises(ValueError):
        oracle.route(bad, 2, 0)


# ------------------------------------------------- the paper's padded re-index form
def test_padded_index_golden_fixture(oracle):
    """Fig. 3's dimensions (10 tokens, 4 experts, tile 4), routing and expected vectors worked by hand
    in tests/golden/index_10tok_4exp.txt."""
    import os
    vals = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "index_10tok_4exp.txt")):
        tok = line.split("#")[0].split()
        if tok:
            vals[tok[0]] = [int(t) for t in tok[1:]]
    routing = np.array(vals["R"], np.int32).reshape(-1, 1)
    v, starts = oracle.padded_index(routing, 4, 4)
    assert starts.tolist() == vals["padded_starts"]
    assert v[: starts[-1]].tolist() == vals["padded_v"]
    assert (v[starts[-1]:] == -1).all()


@pytest.mark.parametrize("T,k,E,blk", [(10, 1, 4, 4), (200, 2, 7, 16), (33, 3, 5, 1), (64, 1, 3, 64), (5, 2, 9, 8)])
def test_padded_index_against_brute_force(oracle, T, k, E, blk):
    rng = np.random.default_rng(T + E + blk)
    idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
    if E > 2:
        idx[idx == 1] = 0                                   # an empty expert
    v, starts = oracle.padded_index(idx, E, blk)
    flat = idx.reshape(-1)
    exp_v, exp_s = [], [0]
    for e in range(E):                                      # python lists, no shared code
        ids = [a for a in range(T * k) if flat[a] == e]
        pad = (-len(ids)) % blk
        exp_v += ids + [-1] * pad
        exp_s.append(len(exp_v))
    assert starts.tolist() == exp_s
    assert v[: exp_s[-1]].tolist() == exp_v and (v[exp_s[-1]:] == -1).all()
    assert all(s % blk == 0 for s in exp_s)                 # every sub-vector is tile-aligned
    # the unpadded index is the padded one with the -1 entries removed
    counts, offsets, perm, inv = oracle.index(idx, E)
    assert v[v >= 0].tolist() == perm.tolist()
    with pytest.raises(ValueError):
        oracle.padded_index(idx, E, blk, cap=exp_s[-1] - 1)


# ---------------------------------------------------- the other activations (ReLU, SiLU)
@pytest.fixture
def with_activation(oracle):
    """Sets the oracle's process-wide activation for one test and restores GELU-tanh."""
    def choose(kind):
        oracle.set_activation(kind)
    yield choose
    oracle.set_activation(0)


@pytest.mark.parametrize("kind,lib_act", [(1, torch.nn.functional.relu), (2, torch.nn.functional.silu)])
def test_other_activations_match_autograd_loop(oracle, with_activation, kind, lib_act):
    with_activation(kind)
    c = small_case(40 + kind, T=60, d=8, f=24, E=5, k=2, dup=True)
    c["topk_idx"][c["topk_idx"] == 3] = 0
    y, g = oracle_all(oracle, c)
    yt, gt = torch_loop_grads(c, act=lib_act)
    assert rel(y, yt) < 1e-13
    for n in g:
        assert rel(g[n], gt[n]) < 1e-12, n


def test_activation_scalar_values(oracle, with_activation):
    with_activation(1)
    assert [oracle.act(u) for u in (-2.0, 0.0, 3.5)] == [0.0, 0.0, 3.5]
    assert [oracle.act_grad(u) for u in (-2.0, 0.0, 3.5)] == [0.0, 0.0, 1.0]
    with_activation(2)
    for u in (-4.0, -0.3, 0.0, 0.7, 5.0):
        assert abs(oracle.act(u) - u / (1 + np.exp(-u))) < 1e-15
        e = 1e-6
        assert abs((oracle.act(u + e) - oracle.act(u - e)) / (2 * e) - oracle.act_grad(u)) < 1e-9
    assert oracle.act_grad(0.0) == 0.5
    with_activation(0)
    assert oracle.act(0.9) == oracle.gelu(0.9) and oracle.act_grad(0.9) == oracle.gelu_grad(0.9)
    with pytest.raises(ValueError):
        oracle.set_activation(7)


# ---- heterogeneous-aware allocation (Sec. 3.4 Eq. 1-2) ------------------------------------------

def _alloc_fixture():
    rows = []
    for line in open(os.path.join(GOLD, "alloc_table2.txt")):
        if line.startswith("#") or not line.strip():
            continue
        c, t0, t1, r0, r1 = line.split()
        rows.append((int(c), float(t0), float(t1), r0, r1))
    return rows


def test_allocation_reproduces_the_paper_capacity_table():
    """Sec. 4 Table 2 prints, for three power settings of its two GPUs, the measured latencies and
    the capacity proportion R = Eq. 1 / Eq. 2 with total 1, to two decimals."""
    from oracle.allocate_oracle import ideal_shares
    rows = _alloc_fixture()
    assert len(rows) == 3
    for _, t0, t1, r0, r1 in rows:
        q = ideal_shares([t0, t1], 1)
        assert sum(q) == 1
        assert f"{float(q[0]):.2f}" == r0 and f"{float(q[1]):.2f}" == r1
        # and the split of a batch of 100 in whole samples is that proportion
        from oracle.allocate_oracle import allocate
        s = allocate([t0, t1], 100)
        assert s == [round(float(q[0]) * 100), 100 - round(float(q[0]) * 100)]


def test_allocation_closed_forms_and_invariants():
    from fractions import Fraction
    from oracle.allocate_oracle import allocate, ideal_shares
    assert allocate([3.0] * 4, 128) == [32] * 4                 # equal devices, equal shares
    assert allocate([1.0, 2.0], 90) == [60, 30]                 # half the latency, twice the work
    assert allocate([1.0, 1.0, 1.0], 10) == [4, 3, 3]           # equal fractions: lower index first
    assert allocate([1.0, 1.0, 1.0], 11) == [4, 4, 3]
    assert allocate([2.0, 1.0, 1.0], 8192, 64) == [1664, 3264, 3264]   # 25.6 / 51.2 / 51.2 granules
    assert allocate([5.0], 77, 7) == [77]
    assert allocate([1.0, 4.0], 0) == [0, 0]
    rng = np.random.default_rng(12)
    for _ in range(200):
        n = int(rng.integers(1, 7))
        lat = [float(x) for x in rng.uniform(0.2, 9.0, n)]
        g = int(rng.choice([1, 8, 64]))
        total = g * int(rng.integers(0, 300))
        s = allocate(lat, total, g)
        q = ideal_shares(lat, total)
        assert sum(s) == total and sum(q) == total
        assert all(v % g == 0 and v >= 0 for v in s)
        assert all(abs(Fraction(v) - qi) < g for v, qi in zip(s, q))       # within one granule
        # scaling every latency by the same factor changes nothing (only ratios enter Eq. 1-2)
        assert allocate([2.0 * t for t in lat], total, g) == s
        # a faster device never gets less
        order = np.argsort(lat)
        assert all(s[order[i]] >= s[order[i + 1]] for i in range(n - 1))
    for bad in (([1.0, 0.0], 10, 1), ([1.0, -2.0], 10, 1), ([1.0], 10, 3), ([], 10, 1), ([1.0], -1, 1)):
        with pytest.raises(ValueError):
            allocate(*bad)


def test_allocation_against_brute_force_over_all_splits():
    """Largest-remainder rounding is the integer split closest to the ideal shares in the L1 sense;
    among equally close ones the rule hands the extra units to the lower device index, i.e. picks
    the lexicographically largest.  Enumerate every split of a few units over 2-3 devices."""
    from fractions import Fraction
    from itertools import product
    from oracle.allocate_oracle import allocate, ideal_shares
    rng = np.random.default_rng(5)
    cases = [([1.0, 1.0], 5), ([1.0, 1.0, 1.0], 7), ([1.0, 2.0, 4.0], 9), ([0.5, 0.25, 1.0], 6)]
    for _ in range(40):
        n = int(rng.integers(2, 4))
        cases.append(([float(x) for x in rng.integers(1, 9, n)], int(rng.integers(0, 13))))
    for lat, units in cases:
        q = ideal_shares(lat, units)
        best, best_cost = None, None
        for s in product(range(units + 1), repeat=len(lat)):
            if sum(s) != units:
                continue
            cost = sum(abs(Fraction(v) - qi) for v, qi in zip(s, q))
            if best is None or cost < best_cost or (cost == best_cost and s > best):
                best, best_cost = s, cost
        assert tuple(allocate(lat, units)) == best, (lat, units)
