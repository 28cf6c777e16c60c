#!/usr/bin/env python3
"""Writes tests/golden/vgg16_b256_step.json: the loss and sampled weight-gradient entries of ONE training step of
the benchmark configuration itself (VGG-16, batch 256, the seeded synthetic inputs of synth/gen.py), computed by the
fp64 CPU oracle and by nothing else.

The oracle is far too slow and too large in fp64 to run the batch in one piece, and it does not have to: every layer
treats the images of a batch independently, the loss is the mean of the per-image losses and a weight gradient is the
sum of per-image contributions.  So the batch is cut into chunks of --chunk images; oracle.net.step runs on each chunk
(where it averages over the chunk's images), and the chunk results are combined as

    loss = mean over chunks of loss_chunk,      dW = (chunk / batch) * sum over chunks of dW_chunk.

Takes about an hour and a half on 8 cores.  Usage: python tests/golden/make_vgg16_b256_golden.py [--chunk 16] [--samples 400]
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--chunk", type=int, default=16)
    ap.add_argument("--samples", type=int, default=400)
    ap.add_argument("--out", default=os.path.join(ROOT, "tests", "golden", "vgg16_b256_step.json"))
    args = ap.parse_args()
    assert args.batch % args.chunk == 0
    net = nets.vgg16(args.batch)
    x, labels, weights = gen.make(net)
    part = nets.vgg16(args.chunk)
    dw = {i: np.zeros(w.shape, np.float64) for i, w in weights.items()}
    losses = []
    t0 = time.time()
    for c in range(args.batch // args.chunk):
        sl = slice(c * args.chunk, (c + 1) * args.chunk)
        r = onet.step(part, x[sl], labels[sl], weights)
        losses.append(float(r["loss"]))
        for i in dw:
            dw[i] += r["dw"][i]
        print("chunk %d/%d done, %.0f s" % (c + 1, args.batch // args.chunk, time.time() - t0), flush=True)
    scale = args.chunk / args.batch
    rng = np.random.default_rng(160208124)
    out = dict(config="VGG-16 batch %d, synth.gen.make(nets.vgg16(%d)) with its default seed" % (args.batch, args.batch),
               chunk=args.chunk, loss=float(np.mean(losses)), layers={})
    for i, g in dw.items():
        g = g * scale
        flat = g.reshape(-1)
        idx = np.sort(rng.choice(flat.size, size=min(args.samples, flat.size), replace=False))
        out["layers"][str(i)] = dict(shape=list(g.shape), max_abs=float(np.abs(flat).max()), l2=float(np.sqrt((flat * flat).sum())),
                                     index=[int(v) for v in idx], value=[float(flat[v]) for v in idx])
    with open(args.out, "w") as f:
        json.dump(out, f)
    print("wrote", args.out)


if __name__ == "__main__":
    main()
