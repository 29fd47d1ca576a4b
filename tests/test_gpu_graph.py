"""The whole step (index, forward, backward) recorded into a HIP graph and replayed: the library
allocates nothing, synchronises nothing and issues no memset nodes, so a capture of its launches
must reproduce the eager results bit for bit on every replay (launch-latency regime, workload C2)."""
import pytest
import torch

from paper_2411_01288_amd.workloads import generate, workload

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_graph_replays_equal_eager(name):
    from paper_2411_01288_amd import binding as B
    w = workload(name)
    data = generate(w, DEV)
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype)
    idx = B.alloc_idx(shape, DEV)
    scratch = torch.empty(max(B.index_scratch_bytes(shape), 256), dtype=torch.uint8, device=DEV)
    ws = B.alloc_workspace(shape, DEV)
    y = torch.empty((w.T, w.d_model), dtype=data["x"].dtype, device=DEV)
    grads = None

    def step():
        nonlocal grads
        B.hexa_moe_index(shape, data["topk_idx"], idx, scratch)
        B.hexa_moe_fwd(shape, data["x"], data["topk_idx"], data["gate"], data["W1"], data["b1"],
                       data["W2"], data["b2"], idx, ws, y)
        grads = B.hexa_moe_bwd(shape, data["dY"], data["x"], data["topk_idx"], data["gate"],
                               data["W1"], data["W2"], idx, ws, out=grads)

    step()                                   # eager: also sets the kernels' launch attributes
    torch.cuda.synchronize()
    ref = {"y": y.clone(), "perm": idx["perm"].clone(), **{k: v.clone() for k, v in grads.items()}}

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                               # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(4):
        # the program's own eager work between replays: wipe every output
        y.zero_(); idx["perm"].zero_()
        for v in grads.values():
            v.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, ref["y"]), replay
        assert torch.equal(idx["perm"], ref["perm"]), replay
        for k, v in grads.items():
            assert torch.equal(v, ref[k]), (replay, k)
