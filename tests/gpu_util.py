"""Helpers shared by the GPU parity tests: run the HIP library through its binding and
bring results to the host.  Nothing here computes any part of the layer."""
import os

import numpy as np
import torch


def poisoned(shape, dtype, device):
    """A tensor of NaNs: an output element the library never writes stays NaN and is caught by
    the comparison with the oracle (or by the finiteness sweep of the sampled tests)."""
    return torch.full(shape, float("nan"), dtype=dtype, device=device)


def run_hip_layer(w, data, want_dgate=True):
    """data: dict of device tensors from workloads.generate.  Returns (idx, y, grads) on device.

    Every output tensor and the whole workspace start out as NaN bit patterns (0xFF bytes are a
    NaN in fp32, bf16 and fp16 alike), the index outputs as -7: whatever the library does not
    write, or reads without having written, shows up in the results."""
    from paper_2411_01288_amd import binding as B
    shape = B.make_shape(w.T, w.d_model, w.d_ff, w.E, w.k, w.dtype)
    dev = data["x"].device
    dt = data["x"].dtype
    T, d, f, E, k = w.T, w.d_model, w.d_ff, w.E, w.k
    idx = B.alloc_idx(shape, dev)
    for t in idx.values():
        t.fill_(-7)
    idx = B.hexa_moe_index(shape, data["topk_idx"], idx)
    ws = B.alloc_workspace(shape, dev)
    ws.fill_(0xFF)
    y = B.hexa_moe_fwd(shape, data["x"], data["topk_idx"], data["gate"], data["W1"], data["b1"],
                       data["W2"], data["b2"], idx, ws, poisoned((T, d), dt, dev))
    f32 = torch.float32
    out = {"dx": poisoned((T, d), dt, dev), "dW1": poisoned((E, d, f), f32, dev),
           "db1": poisoned((E, f), f32, dev), "dW2": poisoned((E, f, d), f32, dev),
           "db2": poisoned((E, d), f32, dev),
           "dgate": poisoned((T, k), f32, dev) if want_dgate else None}
    g = B.hexa_moe_bwd(shape, data["dY"], data["x"], data["topk_idx"], data["gate"], data["W1"],
                       data["W2"], idx, ws, want_dgate=want_dgate, out=out)
    torch.cuda.synchronize()
    return idx, y, g


def host32(t):
    return t.detach().to("cpu").float().numpy()


def host_inputs(data):
    c = {k: host32(v) for k, v in data.items() if k != "topk_idx"}
    c["topk_idx"] = data["topk_idx"].cpu().numpy()
    return c


def nrm_err(got, ref):
    """max |got - ref| / max |ref|  (the max-abs normalised error of the tolerance statement)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    err = float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))
    log = os.environ.get("HEXA_ERR_LOG")      # optional: one line per comparison (a survey of the errors actually met)
    if log:
        with open(log, "a") as f:
            f.write(f"{err:.3e}\t{os.environ.get('PYTEST_CURRENT_TEST', '')}\n")
    return err


# fp32 and bf16: the tolerances of the benchmark statement.  fp16 (11-bit significands against bf16's
# 8) is not in that statement: its rounding errors are 8 times smaller than bf16's, so its tolerance is
# an eighth of bf16's (measured: below 8e-4, as bf16 stays below 6e-3).
TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 2.5e-3}
