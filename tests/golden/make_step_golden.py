#!/usr/bin/env python3
"""Writes tests/golden/<workload>_b<batch>_step.json: ONE training step of a benchmark configuration at its stated
size (the seeded synthetic inputs of synth/gen.py), computed by the fp64 CPU oracle and by nothing else.  Stored:

  loss                       the mean softmax cross-entropy of the batch
  layers[i]                  per layer with weights: shape, max |dW|, ||dW||, and sampled entries of dW
  fwd[i]                     per layer: max |Y| over the whole batch and sampled entries of the layer's output Y
                             (a CONV / FC layer's output before the ReLU that follows it, the ReLU's after)
  dy[i]                      per layer: max |dY| and sampled entries of the gradient with respect to the layer's output,
                             as it arrives at the layer's backward computation (Eq. chain_rule)
  margins[i]                 per ReLU / max-pool layer: how many of the oracle's decisions are close calls: ReLU inputs
                             with |x| below a threshold, pooling windows whose two largest elements are closer than a
                             threshold (largest > 0).  A forward pass in another precision decides those differently.

Sample positions are flat indices into the full-batch NCHW tensor.

The oracle is far too slow and too large in fp64 to run such a batch in one piece, and it does not have to: every layer
treats the images of a batch independently, the loss is the mean of the per-image losses and a weight gradient is the
sum of per-image contributions.  So the batch is cut into chunks of --chunk images; oracle.net.step runs on each chunk
(where it averages over the chunk's images), and the chunk results are combined as

    loss = mean over chunks of loss_chunk,      dW = (chunk / batch) * sum over chunks of dW_chunk,
    Y    = the chunk's own,                     dY = (chunk / batch) * dY_chunk.

VGG-16 at batch 256 takes about an hour on 8 cores, the batch-128 workloads minutes.
Usage: python tests/golden/make_step_golden.py --workload vgg16|alexnet|overfeat|googlenet [--chunk 16]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import net as onet  # noqa: E402
from synth import gen, nets  # noqa: E402

THRESHOLDS = [1e-8, 1e-7, 1e-6, 1e-5, 1e-4]


def _r(v):
    return float("%.12g" % v)


class Sampler:
    """Sampled entries of per-layer tensors that only ever exist one chunk of images at a time."""

    def __init__(self, shapes, count, seed):
        rng = np.random.default_rng(seed)
        self.per_image, self.index, self.value, self.max_abs = {}, {}, {}, {}
        for i, s in shapes.items():
            size = int(np.prod(s))
            self.per_image[i] = size // s[0]
            self.index[i] = np.sort(rng.choice(size, size=min(count, size), replace=False))
            self.value[i] = np.zeros(len(self.index[i]))
            self.max_abs[i] = 0.0

    def take(self, i, first_image, arr, scale=1.0):
        flat = np.asarray(arr).reshape(-1)
        lo = first_image * self.per_image[i]
        a, b = np.searchsorted(self.index[i], [lo, lo + flat.size])
        self.value[i][a:b] = flat[self.index[i][a:b] - lo] * scale
        self.max_abs[i] = max(self.max_abs[i], float(np.abs(flat).max()) * scale)

    def dump(self):
        return {str(i): dict(max_abs=_r(self.max_abs[i]), index=[int(v) for v in self.index[i]], value=[_r(v) for v in self.value[i]])
                for i in self.index}


def _window_top2_gap(a, k, st, pd):
    """Largest element and its distance to the second largest, per pooling window (padding never wins)."""
    p = np.pad(a, ((0, 0), (0, 0), (pd, pd), (pd, pd)), constant_values=-np.inf)
    v = np.lib.stride_tricks.sliding_window_view(p, (k, k), axis=(2, 3))[:, :, ::st, ::st]
    v = v.reshape(v.shape[:4] + (k * k,))
    top = np.partition(v, k * k - 2, axis=-1)[..., -2:]
    return top[..., 1], top[..., 1] - top[..., 0]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="vgg16", choices=sorted(nets.CONFIGS))
    ap.add_argument("--batch", type=int, default=0, help="default: the workload's own")
    ap.add_argument("--chunk", type=int, default=16)
    ap.add_argument("--samples", type=int, default=400, help="sampled dW entries per layer")
    ap.add_argument("--fwd-samples", type=int, default=256)
    ap.add_argument("--dy-samples", type=int, default=2048)
    ap.add_argument("--out", default="")
    args = ap.parse_args()
    make = nets.CONFIGS[args.workload]
    net = make(args.batch) if args.batch else make()
    batch = net["batch"]
    assert batch % args.chunk == 0
    out_path = args.out or os.path.join(ROOT, "tests", "golden", "%s_b%d_step.json" % (args.workload, batch))
    x, labels, weights = gen.make(net)
    part = make(args.chunk)
    out_shapes, _ = nets.shapes(net)
    sampled = {i: s for i, s in enumerate(out_shapes) if net["layers"][i]["type"] != "softmax_ce"}
    fwd = Sampler(sampled, args.fwd_samples, 160208125)
    dys = Sampler(sampled, args.dy_samples, 160208126)
    margins = {i: dict(kind=l["type"], total=0, below=[0] * len(THRESHOLDS)) for i, l in enumerate(net["layers"]) if l["type"] in ("relu", "maxpool")}
    dw = {i: np.zeros(w.shape, np.float64) for i, w in weights.items()}
    losses = []
    scale = args.chunk / batch
    t0 = time.time()
    for c in range(batch // args.chunk):
        first = c * args.chunk
        sl = slice(first, first + args.chunk)
        r = onet.step(part, x[sl], labels[sl], weights, dy_hook=lambda i, g: dys.take(i, first, g, scale))
        losses.append(float(r["loss"]))
        for i in dw:
            dw[i] += r["dw"][i]
        for i in sampled:
            fwd.take(i, first, r["outs"][i])
        for i, m in margins.items():
            layer = net["layers"][i]
            src = layer["inputs"][0]
            a = r["outs"][src] if src >= 0 else x[sl].astype(np.float64)
            if m["kind"] == "relu":
                close, m_total = np.abs(a), a.size
            else:
                top, gap = _window_top2_gap(a, layer["k"], layer["stride"], layer["pad"])
                close, m_total = gap[top > 0], int((top > 0).sum())
            m["total"] += int(m_total)
            for j, t in enumerate(THRESHOLDS):
                m["below"][j] += int((close < t).sum())
        print("chunk %d/%d done, %.0f s" % (c + 1, batch // args.chunk, time.time() - t0), flush=True)
    rng = np.random.default_rng(160208124)
    out = dict(config="%s batch %d, synth.gen.make(nets.CONFIGS[%r](%d)) with its default seed" % (args.workload, batch, args.workload, batch),
               chunk=args.chunk, loss=float(np.mean(losses)), layers={}, fwd=fwd.dump(), dy=dys.dump(),
               thresholds=THRESHOLDS, margins={str(i): m for i, m in margins.items()})
    for i, g in dw.items():
        g = g * scale
        flat = g.reshape(-1)
        idx = np.sort(rng.choice(flat.size, size=min(args.samples, flat.size), replace=False))
        out["layers"][str(i)] = dict(shape=list(g.shape), max_abs=float(np.abs(flat).max()), l2=float(np.sqrt((flat * flat).sum())),
                                     index=[int(v) for v in idx], value=[float(flat[v]) for v in idx])
    with open(out_path, "w") as f:
        json.dump(out, f)
    print("wrote", out_path)


if __name__ == "__main__":
    main()
