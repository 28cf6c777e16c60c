"""Layer-wise training step of a whole network on the CPU oracle (test infrastructure only).

Forward propagation visits layers 0..L-1 in order, backward propagation L-1..0 (Section 2.2,
"DNN training"): each layer turns dY into dX with the chain rule (Eq. chain_rule), and the
weight gradients come from the same rule.  For non-linear topologies (Fig. nonlinear_dfg) a
producer with several consumers receives the SUM of its consumers' dX.

Everything is fp64.  The runner is value-semantic: an in-place ReLU simply returns a new
array, which has the same values as overwriting would.
"""
import numpy as np

from . import layers as L


def _shape_of(net, outs, i):
    return outs[i].shape if i >= 0 else (net["batch"], net["in_c"], net["in_h"], net["in_w"])


def forward(net, x, labels, weights):
    """Returns (outs, loss): outs[i] is layer i's output Y (fp64); the last layer's is the scalar loss."""
    x = np.asarray(x, np.float64)
    outs = []

    def val(i):
        return x if i < 0 else outs[i]

    loss = None
    for i, layer in enumerate(net["layers"]):
        t = layer["type"]
        a = val(layer["inputs"][0])
        k, st, pd = layer["k"], layer["stride"], layer["pad"]
        if t == "conv":
            y = L.conv_fwd(a, weights[i], st, pd)
        elif t == "relu":
            y = L.relu_fwd(a)
        elif t == "maxpool":
            y = L.maxpool_fwd(a, k, st, pd)
        elif t == "avgpool":
            y = L.avgpool_fwd(a, k, st, pd)
        elif t == "fc":
            y = L.fc_fwd(a, weights[i]).reshape(a.shape[0], -1, 1, 1)
        elif t == "concat":
            y = np.concatenate([val(j) for j in layer["inputs"]], axis=1)
        elif t == "softmax_ce":
            loss, _ = L.softmax_ce(a.reshape(a.shape[0], -1), labels)
            y = np.array(loss)
        else:
            raise ValueError(t)
        outs.append(y)
    return outs, loss


def step(net, x, labels, weights, want_dx_input=False, outs_override=None, dy_hook=None):
    """One forward + backward pass.  Returns dict(outs, loss, dw {layer: array}, dx {tensor id: array}).

    outs_override: {layer id: array} - layer outputs to run the BACKWARD pass from instead of this
    function's own forward values (which are still returned in `outs`).  Backward propagation takes
    discrete decisions from forward values (which window element is the maximum, whether an activation
    is positive); an fp32 forward pass that differs from the fp64 one in the last bit can decide one of
    them differently, which moves a whole gradient term.  A comparison that hands the other side's
    forward values in here makes both sides decide on the same numbers.

    dy_hook: called as dy_hook(layer id, dY) with the gradient with respect to each layer's output, just before
    that layer's backward computation (observation only)."""
    x = np.asarray(x, np.float64)
    outs, loss = forward(net, x, labels, weights)
    own_outs = outs
    if outs_override:
        outs = list(outs)
        for i, a in outs_override.items():
            if net["layers"][i]["type"] != "softmax_ce":
                outs[i] = np.asarray(a, np.float64).reshape(own_outs[i].shape)
    nl = len(net["layers"])

    def val(i):
        return x if i < 0 else outs[i]

    grads = {}  # tensor id -> accumulated dLoss/dTensor

    def give(i, g):
        if i < 0 and not want_dx_input:
            return
        grads[i] = g if i not in grads else grads[i] + g

    dw = {}
    for i in range(nl - 1, -1, -1):
        layer = net["layers"][i]
        t = layer["type"]
        src = layer["inputs"][0]
        a = val(src)
        k, st, pd = layer["k"], layer["stride"], layer["pad"]
        if t == "softmax_ce":
            _, dz = L.softmax_ce(a.reshape(a.shape[0], -1), labels)
            give(src, dz.reshape(a.shape))
            continue
        dy = grads.pop(i)
        if dy_hook is not None:
            dy_hook(i, dy)
        if t == "conv":
            dw[i] = L.conv_bwd_filter(a, dy, weights[i].shape, st, pd)
            if src >= 0 or want_dx_input:
                give(src, L.conv_bwd_data(dy, weights[i], a.shape, st, pd))
        elif t == "relu":
            give(src, L.relu_bwd(outs[i], dy))
        elif t == "maxpool":
            give(src, L.maxpool_bwd(a, dy, k, st, pd))
        elif t == "avgpool":
            give(src, L.avgpool_bwd(dy, a.shape, k, st, pd))
        elif t == "fc":
            dy2 = dy.reshape(dy.shape[0], -1)
            dw[i] = L.fc_bwd_filter(a, dy2)
            give(src, L.fc_bwd_data(dy2, weights[i], a.shape))
        elif t == "concat":
            c0 = 0
            for j in layer["inputs"]:
                cj = val(j).shape[1]
                give(j, np.ascontiguousarray(dy[:, c0:c0 + cj]))
                c0 += cj
        else:
            raise ValueError(t)
    return dict(outs=own_outs, loss=loss, dw=dw, dx=grads)


def sgd_update(weights, dw, lr):
    """Section 2.2: after backward propagation reaches the first layer, the weights are adjusted with the
    weight gradients.  Plain SGD: W <- W - lr * dW."""
    return {i: np.asarray(w, np.float64) - lr * dw[i] for i, w in weights.items()}
