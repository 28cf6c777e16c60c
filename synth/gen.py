"""Seeded generators for inputs, labels and initial weights.

Counter-based generator: numpy's Philox4x64 keyed by the seed; normal deviates come from
numpy's Generator.standard_normal on that bit stream, cast to fp32.  The numbers are produced
once on the host and handed to the oracle and to the HIP library as arrays, so the generator
itself is not part of any parity claim.
"""
import numpy as np

from . import nets

BASE_SEED = 160208124000
CONFIG_INDEX = {"tiny": 0, "alexnet": 1, "overfeat": 2, "googlenet": 3, "vgg16": 4}


def seed_for(name):
    return BASE_SEED + CONFIG_INDEX.get(name, 99)


def rng(seed):
    return np.random.Generator(np.random.Philox(key=int(seed)))


def make(net, seed=None, classes=None):
    """Returns (x fp32 NCHW ~N(0,1), labels int32 uniform, weights {layer id: fp32 He-normal})."""
    g = rng(seed_for(net["name"]) if seed is None else seed)
    out, wshape = nets.shapes(net)
    x = g.standard_normal((net["batch"], net["in_c"], net["in_h"], net["in_w"]), dtype=np.float32)
    n_classes = out[-2][1] if classes is None else classes
    labels = g.integers(0, n_classes, size=net["batch"], dtype=np.int32)
    weights = {}
    for i, ws in enumerate(wshape):
        if ws is None:
            continue
        fan_in = int(np.prod(ws[1:]))
        w = g.standard_normal(ws, dtype=np.float32)
        w *= np.float32(np.sqrt(2.0 / fan_in))
        weights[i] = w
    return x, labels, weights
