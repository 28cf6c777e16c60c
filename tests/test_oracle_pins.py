"""Pins for the CPU oracle: each check ties an oracle function to something other than itself
(a library routine on a special case, a closed form, an invariant, a hand-worked value, or
finite differences of the oracle's own forward pass)."""
import os

import numpy as np
import pytest
from scipy import signal, special

from oracle import layers as L
from oracle import net as onet
from synth import gen, nets

RNG = np.random.default_rng(1234)
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":")
        out[k.strip()] = np.array([float(t) for t in v.split()])
    return out


def test_conv_hand_example():
    g = _gold("conv_hand_example.txt")
    x = np.arange(1, 10, dtype=np.float64).reshape(1, 1, 3, 3)
    w = np.array([[1.0, 0.0], [0.0, -1.0]]).reshape(1, 1, 2, 2)
    assert np.array_equal(L.conv_fwd(x, w, 1, 0).ravel(), g["pad0"])
    assert np.array_equal(L.conv_fwd(x, w, 1, 1).ravel(), g["pad1"])
    dy = np.ones((1, 1, 2, 2))
    assert np.array_equal(L.conv_bwd_filter(x, dy, w.shape, 1, 0).ravel(), g["dw"])
    assert np.array_equal(L.conv_bwd_data(dy, w, x.shape, 1, 0).ravel(), g["dx"])


def _scipy_conv(x, w, stride, pad):
    n, c, h, wd = x.shape
    k = w.shape[0]
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    full = np.zeros((n, k, xp.shape[2] - w.shape[2] + 1, xp.shape[3] - w.shape[3] + 1))
    for i in range(n):
        for j in range(k):
            for ci in range(c):
                full[i, j] += signal.correlate2d(xp[i, ci], w[j, ci], mode="valid")
    return full[:, :, ::stride, ::stride]


@pytest.mark.parametrize("shape", [
    # n, c, h, w, k, r, stride, pad
    (2, 3, 7, 6, 4, 3, 1, 1),
    (1, 2, 9, 9, 3, 3, 2, 0),
    (2, 1, 11, 13, 2, 5, 1, 2),
    (1, 3, 15, 15, 2, 7, 2, 3),
    (1, 2, 23, 23, 3, 11, 4, 0),
    (2, 4, 5, 5, 3, 1, 1, 0),
])
def test_conv_fwd_vs_scipy_correlate(shape):
    n, c, h, w, k, r, st, pd = shape
    x = RNG.standard_normal((n, c, h, w))
    wt = RNG.standard_normal((k, c, r, r))
    ref = _scipy_conv(x, wt, st, pd)
    y = L.conv_fwd(x, wt, st, pd)
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_conv_special_cases():
    # one-pixel image, 3x3 pad 1: only the centre tap sees data
    x = RNG.standard_normal((3, 4, 1, 1))
    w = RNG.standard_normal((5, 4, 3, 3))
    np.testing.assert_allclose(L.conv_fwd(x, w, 1, 1)[:, :, 0, 0], x[:, :, 0, 0] @ w[:, :, 1, 1].T, rtol=1e-13)
    # 1x1 conv is a matrix product over channels
    x = RNG.standard_normal((2, 6, 4, 5))
    w = RNG.standard_normal((3, 6, 1, 1))
    np.testing.assert_allclose(L.conv_fwd(x, w), np.einsum("nchw,kc->nkhw", x, w[:, :, 0, 0]), rtol=1e-12, atol=1e-13)
    # kernel as large as the image, no padding: an FC dot product
    x = RNG.standard_normal((3, 2, 4, 4))
    w = RNG.standard_normal((5, 2, 4, 4))
    fc = L.fc_fwd(x, w.reshape(5, -1))
    np.testing.assert_allclose(L.conv_fwd(x, w)[:, :, 0, 0], fc, rtol=1e-13)
    np.testing.assert_allclose(fc, x.reshape(3, -1) @ w.reshape(5, -1).T, rtol=1e-12, atol=1e-13)
    # delta kernel at tap (r, s): a shifted copy of X (zero where the shift leaves the image)
    x = RNG.standard_normal((1, 1, 5, 6))
    for r in range(3):
        for s in range(3):
            w = np.zeros((1, 1, 3, 3))
            w[0, 0, r, s] = 1.0
            y = L.conv_fwd(x, w, 1, 1)
            xp = np.pad(x, ((0, 0), (0, 0), (1, 1), (1, 1)))
            assert np.array_equal(y, xp[:, :, r:r + 5, s:s + 6])


@pytest.mark.parametrize("shape", [(2, 3, 7, 6, 4, 3, 1, 1), (2, 2, 8, 8, 3, 5, 1, 2), (1, 2, 6, 7, 2, 2, 1, 0)])
def test_conv_bwd_vs_scipy(shape):
    """Stride-1 gradients have closed forms as library correlations / full convolutions."""
    n, c, h, w, k, r, st, pd = shape
    x = RNG.standard_normal((n, c, h, w))
    wt = RNG.standard_normal((k, c, r, r))
    y = L.conv_fwd(x, wt, st, pd)
    dy = RNG.standard_normal(y.shape)
    xp = np.pad(x, ((0, 0), (0, 0), (pd, pd), (pd, pd)))
    dw_ref = np.zeros_like(wt)
    dx_ref = np.zeros_like(xp)
    for i in range(n):
        for j in range(k):
            for ci in range(c):
                dw_ref[j, ci] += signal.correlate2d(xp[i, ci], dy[i, j], mode="valid")
                dx_ref[i, ci] += signal.convolve2d(dy[i, j], wt[j, ci], mode="full")
    dx_ref = dx_ref[:, :, pd:pd + h, pd:pd + w]
    np.testing.assert_allclose(L.conv_bwd_filter(x, dy, wt.shape, st, pd), dw_ref, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(L.conv_bwd_data(dy, wt, x.shape, st, pd), dx_ref, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("shape", [(2, 3, 9, 8, 4, 3, 2, 1), (1, 2, 23, 23, 3, 11, 4, 0), (2, 2, 7, 7, 3, 3, 1, 1),
                                   (1, 3, 15, 14, 2, 7, 2, 3), (2, 3, 6, 6, 2, 5, 1, 0)])
def test_conv_adjoint_identities(shape):
    """<conv(X,W), dY> = <X, bwd_data(dY,W)> = <W, bwd_filter(X,dY)> for the bilinear map."""
    n, c, h, w, k, r, st, pd = shape
    x = RNG.standard_normal((n, c, h, w))
    wt = RNG.standard_normal((k, c, r, r))
    y = L.conv_fwd(x, wt, st, pd)
    dy = RNG.standard_normal(y.shape)
    a = np.vdot(y, dy)
    b = np.vdot(x, L.conv_bwd_data(dy, wt, x.shape, st, pd))
    cc = np.vdot(wt, L.conv_bwd_filter(x, dy, wt.shape, st, pd))
    assert abs(a - b) <= 1e-11 * abs(a) + 1e-12
    assert abs(a - cc) <= 1e-11 * abs(a) + 1e-12


def test_softmax_ce_closed_forms():
    for classes in (10, 1000):
        z = np.zeros((4, classes))
        lab = np.array([0, 3, classes - 1, 5])
        loss, dz = L.softmax_ce(z, lab)
        assert abs(loss - np.log(classes)) < 1e-14
        np.testing.assert_allclose(dz.sum(axis=1), 0, atol=1e-14)
    z = RNG.standard_normal((6, 17)) * 5
    lab = RNG.integers(0, 17, 6)
    loss, dz = L.softmax_ce(z, lab)
    ref = np.mean(special.logsumexp(z, axis=1) - z[np.arange(6), lab])
    assert abs(loss - ref) < 1e-13
    sm = special.softmax(z, axis=1)
    sm[np.arange(6), lab] -= 1
    np.testing.assert_allclose(dz, sm / 6, rtol=1e-12, atol=1e-15)
    # shift invariance and large logits (max subtraction must not change the value)
    loss2, _ = L.softmax_ce(z + 700.0, lab)
    assert abs(loss2 - loss) < 1e-9


def test_maxpool_properties():
    x = RNG.standard_normal((2, 3, 7, 7))
    for k, st, pd in [(2, 2, 0), (3, 2, 0), (3, 2, 1), (3, 1, 1)]:
        y = L.maxpool_fwd(x, k, st, pd)
        xp = np.pad(x, ((0, 0), (0, 0), (pd, pd), (pd, pd)), constant_values=-np.inf)
        ref = np.empty_like(y)
        for p in range(y.shape[2]):
            for q in range(y.shape[3]):
                ref[:, :, p, q] = xp[:, :, p * st:p * st + k, q * st:q * st + k].max(axis=(2, 3))
        assert np.array_equal(y, ref)
        dy = RNG.standard_normal(y.shape)
        dx = L.maxpool_bwd(x, dy, k, st, pd)
        # every dY element is routed exactly once, overlapping windows or not
        assert abs(dx.sum() - dy.sum()) < 1e-12
        # gradient only lands on cells that are the maximum of some window
        assert np.all((dx == 0) | np.isin(x, y))
    # padding never wins: all-negative input keeps negative maxima
    xn = -np.abs(RNG.standard_normal((1, 1, 4, 4))) - 1
    assert np.all(L.maxpool_fwd(xn, 3, 2, 1) < 0)
    # ties: the first maximum in row-major window order takes the gradient
    xt = np.zeros((1, 1, 2, 2))
    dx = L.maxpool_bwd(xt, np.array([[[[5.0]]]]), 2, 2, 0)
    assert np.array_equal(dx.ravel(), [5.0, 0, 0, 0])
    xt = np.array([[[[1.0, 3.0], [3.0, 2.0]]]])
    dx = L.maxpool_bwd(xt, np.array([[[[5.0]]]]), 2, 2, 0)
    assert np.array_equal(dx.ravel(), [0, 5.0, 0, 0])


def test_avgpool_properties():
    x = np.full((2, 3, 8, 8), 2.5)
    assert np.array_equal(L.avgpool_fwd(x, 4, 4, 0), np.full((2, 3, 2, 2), 2.5))
    x = RNG.standard_normal((2, 3, 7, 7))
    y = L.avgpool_fwd(x, 7, 1, 0)
    np.testing.assert_allclose(y[:, :, 0, 0], x.mean(axis=(2, 3)), rtol=1e-13)
    dy = RNG.standard_normal(y.shape)
    dx = L.avgpool_bwd(dy, x.shape, 7, 1, 0)
    np.testing.assert_allclose(dx, np.broadcast_to(dy / 49.0, x.shape), rtol=1e-14)
    # adjoint identity for the linear map, with overlap and padding
    for k, st, pd in [(3, 2, 1), (2, 2, 0), (3, 1, 1)]:
        y = L.avgpool_fwd(x, k, st, pd)
        dy = RNG.standard_normal(y.shape)
        assert abs(np.vdot(y, dy) - np.vdot(x, L.avgpool_bwd(dy, x.shape, k, st, pd))) < 1e-12


def test_fc_vs_matmul():
    x = RNG.standard_normal((5, 3, 2, 2))
    w = RNG.standard_normal((7, 12))
    dy = RNG.standard_normal((5, 7))
    np.testing.assert_allclose(L.fc_fwd(x, w), x.reshape(5, -1) @ w.T, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(L.fc_bwd_data(dy, w, x.shape).reshape(5, -1), dy @ w, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(L.fc_bwd_filter(x, dy), dy.T @ x.reshape(5, -1), rtol=1e-12, atol=1e-14)


def test_relu():
    x = np.array([-1.0, 0.0, 2.0, -0.0, 1e-300])
    y = L.relu_fwd(x)
    assert np.array_equal(y, [0, 0, 2.0, 0, 1e-300])
    assert np.array_equal(L.relu_bwd(y, np.ones(5)), [0, 0, 1, 0, 1])


def _fd_check(net, seed, n_probe=24, h=1e-5):
    """Central finite differences of the oracle's own forward loss against its backward pass."""
    x, labels, weights = gen.make(net, seed=seed)
    x = x.astype(np.float64)
    weights = {k: v.astype(np.float64) for k, v in weights.items()}
    res = onet.step(net, x, labels, weights, want_dx_input=True)
    r = np.random.default_rng(seed)
    worst = 0.0

    def loss_of(xx, ww):
        return onet.forward(net, xx, labels, ww)[1]

    targets = [("x", None)] + [("w", k) for k in weights]
    for kind, key in targets:
        arr = x if kind == "x" else weights[key]
        grad = res["dx"][-1] if kind == "x" else res["dw"][key]
        assert grad.shape == arr.shape
        flat = arr.reshape(-1)
        for idx in r.choice(flat.size, size=min(n_probe, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + h
            lp = loss_of(x, weights)
            flat[idx] = old - h
            lm = loss_of(x, weights)
            flat[idx] = old
            fd = (lp - lm) / (2 * h)
            an = grad.reshape(-1)[idx]
            # relative to the element, floored at 1% of the tensor's largest gradient
            err = abs(fd - an) / max(abs(an), 1e-2 * np.abs(grad).max())
            worst = max(worst, err)
    return worst


def test_finite_differences_tiny_net():
    # The paper's Tiny-shaped net (conv-relu-pool x2, FC, softmax-CE), smaller batch for speed.
    assert _fd_check(nets.tiny(batch=2), seed=7) < 2e-6


def test_finite_differences_strided_padded_overlapping():
    # strided conv, overlapping max-pool with padding, avg-pool, two FCs with a ReLU between
    b = nets._Builder("fd2", 2, 2, 13, 13)
    b.conv(3, 5, stride=2, pad=1)
    b.maxpool(3, 2, pad=1)
    b.conv(4, 3, pad=1)
    b.avgpool(2, 1)
    b.fc(6)
    b.fc(5, relu=False)
    assert _fd_check(b.done(), seed=11) < 2e-6


def test_finite_differences_fork_join():
    # one inception-style module: fork (sum of consumer gradients) and channel concat
    assert _fd_check(nets.fork_join(batch=2), seed=13, n_probe=10) < 2e-6


def test_planted_mistakes_are_caught():
    """The pins must fail for plausible mistakes: check three mutants of the definition."""
    x = RNG.standard_normal((1, 2, 6, 6))
    w = RNG.standard_normal((2, 2, 3, 3))
    good = _scipy_conv(x, w, 1, 1)
    flipped = L.conv_fwd(x, w[:, :, ::-1, ::-1].copy(), 1, 1)      # convolution instead of correlation
    transposed = L.conv_fwd(x, w.transpose(0, 1, 3, 2).copy(), 1, 1)  # r/s swapped
    assert np.abs(flipped - good).max() > 1e-3
    assert np.abs(transposed - good).max() > 1e-3
    z = RNG.standard_normal((4, 10))
    lab = np.array([1, 2, 3, 4])
    loss, _ = L.softmax_ce(z, lab)
    assert abs(loss * 4 - np.mean(special.logsumexp(z, axis=1) - z[np.arange(4), lab])) > 1e-3  # sum vs mean


def test_backward_from_given_forward_values():
    """step(outs_override=...) with the oracle's own outputs is the plain step; with perturbed outputs the
    decisions (here: which element of a pooling window wins) follow the given values."""
    net = nets.tiny(batch=2)
    x, labels, weights = gen.make(net, seed=3)
    a = onet.step(net, x, labels, weights)
    b = onet.step(net, x, labels, weights, outs_override={i: o for i, o in enumerate(a["outs"])})
    for i in a["dw"]:
        assert np.array_equal(a["dw"][i], b["dw"][i])
    flipped = {1: -np.asarray(a["outs"][1])}          # ReLU output negated: every mask and arg-max changes
    c = onet.step(net, x, labels, weights, outs_override=flipped)
    assert np.abs(c["dw"][0] - a["dw"][0]).max() > 1e-6
    assert all(np.array_equal(p, q) for p, q in zip(a["outs"], c["outs"]))  # reported outputs stay the oracle's own


def test_decision_flips_amplify_forward_perturbations():
    """Backward propagation is discontinuous in the forward values (arg-max of a pooling window, sign test of a
    ReLU: Eq. chain_rule through those layers).  Every pre-activation is perturbed by noise of a given size relative to
    its tensor's largest element, the oracle's backward pass is run from the perturbed values, and the decisions that
    came out differently are counted.
      - 1e-10: no decision changes, and the first layer's weight gradient does not move at all (it depends on the other
        layers' forward values only through their decisions);
      - 1e-6, the size of the rounding error of an fp32 forward pass: a network of a million activations has a few values
        that close to a tie (4 here); they flip, and the weight gradient moves by 3e-3 of its largest element, three
        orders of magnitude more than the perturbation.
    This is why GPU gradients are compared with an oracle backward pass run from the GPU's own forward values, and why a
    comparison with the oracle deciding for itself shows outliers on exactly the images where decisions differ."""
    from tests.gpu_util import count_decision_flips
    net = nets.vgg(batch=8, in_hw=64, widths=(16, 32, 64, 64, 64), fc=(64, 10))
    x, labels, weights = gen.make(net, seed=11)
    a = onet.step(net, x, labels, weights)
    first = min(a["dw"])
    result = {}
    for eps in (1e-10, 1e-6):
        rng = np.random.default_rng(5)
        moved = {}
        for i, l in enumerate(net["layers"]):
            if l["type"] == "relu" and net["layers"][i - 1]["type"] == "conv":
                z = np.asarray(a["outs"][i - 1])   # the convolution's output before the ReLU
                moved[i - 1] = z + eps * np.abs(z).max() * rng.standard_normal(z.shape)
                moved[i] = np.maximum(moved[i - 1], 0.0)
        b = onet.step(net, x, labels, weights, outs_override=moved)
        outs = list(a["outs"])
        for i, v in moved.items():
            outs[i] = v
        flips = count_decision_flips(net, outs, a["outs"])
        dev = np.abs(b["dw"][first] - a["dw"][first]).max() / np.abs(a["dw"][first]).max()
        result[eps] = (flips, dev)
    assert result[1e-10] == (0, 0.0), result
    assert 1 <= result[1e-6][0] <= 20 and result[1e-6][1] > 100e-6, result
