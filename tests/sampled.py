"""Sampled-output oracle: evaluates the CPU oracle on small sub-problems cut out of large tensors, one
output element (or one filter slice) at a time.  tests/test_sampled_helpers.py checks these helpers
against the oracle run on whole (small) tensors."""
import numpy as np

from oracle import layers as L


def _patch(x, n, h0, w0, k):
    """x[n, :, h0:h0+k, w0:w0+k] with zeros outside the image, as float64 (1, C, k, k)."""
    _, c, hh, ww = x.shape
    out = np.zeros((1, c, k, k), np.float64)
    hs, he = max(h0, 0), min(h0 + k, hh)
    ws, we = max(w0, 0), min(w0 + k, ww)
    if hs < he and ws < we:
        out[0, :, hs - h0:he - h0, ws - w0:we - w0] = x[n, :, hs:he, ws:we]
    return out


def sampled_conv_fwd_check(x, w, y, stride, pad, relu, rng, samples=96):
    """Oracle value of sampled outputs: a 1x1-output convolution of the receptive field."""
    n_, k_, p_, q_ = y.shape
    r = w.shape[2]
    scale = np.abs(y).max()
    worst = 0.0
    for _ in range(samples):
        n, k, p, q = rng.integers(n_), rng.integers(k_), rng.integers(p_), rng.integers(q_)
        if _ % 4 == 0:  # make sure image borders are among the samples
            p, q = rng.choice([0, p_ - 1]), rng.choice([0, q_ - 1])
        ref = L.conv_fwd(_patch(x, n, p * stride - pad, q * stride - pad, r), w[k:k + 1], 1, 0)[0, 0, 0, 0]
        if relu:
            ref = max(ref, 0.0)
        worst = max(worst, abs(float(y[n, k, p, q]) - ref) / scale)
    return worst


def sampled_conv_bwd_data_check(dy, w, dx, pad, rng, samples=96):
    """stride 1, odd R: dX[n,c,h,w] = sum_{k,r,s} dY[n,k,h+pad-r,w+pad-s] W[k,c,r,s].  Cut the R x R window of dY
    that these terms touch (zeros outside the image); the oracle's backward-data of that window with
    padding (R-1)/2 has exactly this sum at its centre element."""
    n_, c_, h_, w_ = dx.shape
    r = w.shape[2]
    assert r % 2 == 1
    half = (r - 1) // 2
    scale = np.abs(dx).max()
    worst = 0.0
    for _ in range(samples):
        n, c, h, ww = rng.integers(n_), rng.integers(c_), rng.integers(h_), rng.integers(w_)
        if _ % 4 == 0:
            h, ww = rng.choice([0, h_ - 1]), rng.choice([0, w_ - 1])
        win = _patch(dy, n, h + pad - (r - 1), ww + pad - (r - 1), r)
        ref = L.conv_bwd_data(win, w[:, c:c + 1], (1, 1, r, r), 1, half)[0, 0, half, half]
        worst = max(worst, abs(float(dx[n, c, h, ww]) - ref) / scale)
    return worst


def sampled_conv_bwd_filter_check(x, dy, dw, stride, pad, rng, pairs=6):
    """Each sample is a (k, c) pair: the oracle's backward-filter on those two channel slices gives all taps."""
    k_, c_ = dw.shape[:2]
    scale = np.abs(dw).max()
    worst = 0.0
    for _ in range(pairs):
        k, c = rng.integers(k_), rng.integers(c_)
        ref = L.conv_bwd_filter(np.ascontiguousarray(x[:, c:c + 1]), np.ascontiguousarray(dy[:, k:k + 1]), (1, 1) + dw.shape[2:], stride, pad)
        worst = max(worst, np.abs(dw[k, c].astype(np.float64) - ref[0, 0]).max() / scale)
    return worst


