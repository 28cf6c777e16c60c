"""Helpers for the GPU parity tests."""
import numpy as np

TOL = 1e-4  # max |gpu - oracle| / max |oracle| per tensor, the bar the target states for fp32


def rel_err(got, ref):
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64).reshape(ref.shape)
    scale = np.abs(ref).max()
    if scale == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / scale)


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()


def count_decision_flips(net, outs_a, outs_b):
    """Number of discrete decisions of backward propagation (Section 2.2: the chain rule through ReLU and max-pooling
    layers) that two sets of forward values take differently: ReLU inputs on opposite sides of zero, pooling windows
    whose maximum sits at different positions.  outs_*: {layer id or index: array} as the net runners return them."""
    from oracle import layers as L
    flips = 0
    for i, layer in enumerate(net["layers"]):
        src = layer["inputs"][0]
        if src < 0 or layer["type"] not in ("relu", "maxpool"):
            continue
        b = np.asarray(outs_b[src], np.float64)
        a = np.asarray(outs_a[src], np.float64).reshape(b.shape)
        if layer["type"] == "relu":
            flips += int(((a > 0) != (b > 0)).sum())
        else:
            ones = np.ones(L.maxpool_fwd(b, layer["k"], layer["stride"], layer["pad"]).shape)
            ra = L.maxpool_bwd(a, ones, layer["k"], layer["stride"], layer["pad"])
            rb = L.maxpool_bwd(b, ones, layer["k"], layer["stride"], layer["pad"])
            flips += int((ra != rb).sum() + 1) // 2
    return flips
