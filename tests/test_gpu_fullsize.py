"""GPU parity at the benchmark's full sizes (VGG-16 batch 256 and the other workloads), in the launch
configuration bench.py times.  The oracle cannot run these sizes whole, so it is applied to
sampled outputs one by one (each sample is a small sub-problem cut out of the GPU's own input
tensors), and properties that hold at any size are checked on the whole tensors: the adjoint
identities of the bilinear map and bit-identical results with and without offloading."""
import zlib

import numpy as np
import pytest

from oracle import layers as L
from oracle import memsched as ms
from synth import gen, nets
from tests.gpu_util import TOL, dev, host
from tests.sampled import sampled_conv_bwd_data_check, sampled_conv_bwd_filter_check, sampled_conv_fwd_check
from tests.sched_util import check_schedule, lib_ws

pytestmark = pytest.mark.gpu
G = 1 << 30


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_1602_08124_amd import binding
    return binding


# (name, N, C, H, W, K, R, stride, pad): VGG-16 batch 256 layers spanning every tile configuration, plus the
# first layers of AlexNet / GoogLeNet and an inception 1x1 at batch 128
FULL_LAYERS = [
    ("vgg c1_1", 256, 3, 224, 224, 64, 3, 1, 1),
    ("vgg c1_2", 256, 64, 224, 224, 64, 3, 1, 1),
    ("vgg c2_1", 256, 64, 112, 112, 128, 3, 1, 1),
    ("vgg c2_2", 256, 128, 112, 112, 128, 3, 1, 1),    # F(4x4) Winograd on 128 channels, 52 KB planes staged in LDS, 15 chunks
    ("vgg c3_2", 256, 256, 56, 56, 256, 3, 1, 1),
    ("vgg c4_2", 256, 512, 28, 28, 512, 3, 1, 1),      # backward-filter in three splits of 576 grouped tiles
    ("vgg c5_1", 256, 512, 14, 14, 512, 3, 1, 1),
    ("alexnet c1", 128, 3, 227, 227, 96, 11, 4, 0),
    ("alexnet c2", 128, 96, 27, 27, 256, 5, 1, 2),
    ("googlenet stem", 128, 3, 224, 224, 64, 7, 2, 3),
    ("googlenet 4a 1x1", 128, 480, 14, 14, 192, 1, 1, 0),
    ("googlenet 4b 5x5 reduce->5x5", 128, 24, 14, 14, 64, 5, 1, 2),
    # the largest tensors the library takes: X, Y, dX and dY of 2^31 - 2^25 elements (8.5 GB) each; above 4 GiB the
    # packed-weight kernels step aside (32-bit byte offsets) and the generic ones index elements with 32 bits
    ("largest tensors", 63, 32, 1024, 1024, 32, 3, 1, 1),
]


@pytest.mark.parametrize("cfg", FULL_LAYERS, ids=[c[0] for c in FULL_LAYERS])
def test_conv_layer_full_size(B, cfg):
    import torch
    name, n, c, h, w, k, r, st, pd = cfg
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    g = torch.Generator(device="cuda").manual_seed(1234)
    x = torch.randn((n, c, h, w), device="cuda", generator=g)
    wt = torch.randn((k, c, r, r), device="cuda", generator=g) * float(np.sqrt(2.0 / (c * r * r)))
    p, q = L.out_dim(h, r, st, pd), L.out_dim(w, r, st, pd)
    y = torch.empty((n, k, p, q), device="cuda")
    dy = torch.randn((n, k, p, q), device="cuda", generator=g)
    dx = torch.empty_like(x)
    dw = torch.empty_like(wt)
    wsp = torch.empty(max(B.op_conv_fwd_workspace(x.shape, wt.shape, st, pd), B.op_conv_bwd_data_workspace(x.shape, wt.shape, st, pd), 4) // 4, device="cuda")
    wsf = torch.empty(max(B.op_conv_bwd_filter_workspace(x.shape, wt.shape, st, pd), 4) // 4, device="cuda")
    B.op_conv_fwd(x, wt, y, st, pd, True, ws=wsp)
    B.op_conv_bwd_filter(x, dy, dw, wsf, st, pd)
    xh, wh, yh, dyh, dwh = host(x), host(wt).astype(np.float64), host(y), host(dy), host(dw)
    assert np.isfinite(yh).all() and np.isfinite(dwh).all()
    assert sampled_conv_fwd_check(xh, wh, yh, st, pd, True, rng) < TOL
    assert sampled_conv_bwd_filter_check(xh, dyh, dwh, st, pd, rng) < TOL
    # adjoint identities on the whole tensors (no ReLU): <conv(X,W),dY> = <W,dW> (= <X,dX>)
    B.op_conv_fwd(x, wt, y, st, pd, False, ws=wsp)
    a = float((y.double() * dy.double()).sum())
    cc = float((wt.double() * dw.double()).sum())
    # dY is independent of Y, so <Y,dY> is one draw from a distribution around 0 whose spread is |Y| |dY| / sqrt(count):
    # rounding errors scale with that spread, not with where the draw happened to land
    spread = float(y.double().norm() * dy.double().norm()) / np.sqrt(y.numel())
    bound = 2e-5 * max(abs(a), spread) + 1e-3
    assert abs(a - cc) < bound
    if st == 1:
        B.op_conv_bwd_data(dy, wt, dx, st, pd, ws=wsp)
        dxh = host(dx)
        assert np.isfinite(dxh).all()
        assert sampled_conv_bwd_data_check(dyh, wh, dxh, pd, rng) < TOL
        b = float((x.double() * dx.double()).sum())
        assert abs(a - b) < bound


def _run(B, net, x_dev, lab_dev, weights, policy, budget, hooks=(), winograd=True, algo=None, kernels=None):
    """The library's default settings unless winograd=False (no plan uses the Winograd kernel), algo names another
    algorithm mode for a static policy, or kernels = {conv layer: (fwd, bwd-data, bwd-filter)} names the kernels."""
    n = B.Net(net, budget)
    n.set_winograd(winograd)
    if algo:
        n.set_conv_algo(algo)
    for i, names in (kernels or {}).items():
        n.set_layer_kernels(i, names)
    n.set_policy(policy)
    if policy == "fit" and budget:
        st = n.stats()
        check_schedule(net, n.trace(), st["pool_extent_bytes"], n.offload_set(), st["persistent_bytes"])
    n.attach_torch()
    for i, w in weights.items():
        n.set_weights(i, w)
    caps = {}
    for i in hooks:
        caps[i] = np.empty(n.output_count(i), np.float32)
        n.capture_output(i, caps[i])
    loss = n.forward(x_dev, lab_dev)
    n.backward()
    dw = {i: n.get_weight_grad(i, w.shape) for i, w in weights.items()}
    st = n.stats()
    st["ws"] = lib_ws(n, net)
    convs = [i for i, l in enumerate(net["layers"]) if l["type"] == "conv"]
    st["kernels"] = {i: n.layer_kernels(i) for i in convs}
    n.close()
    return loss, dw, st, caps


def test_vgg16_b256_step_under_12_gib(B):
    """The benchmark configuration itself, with the library's default settings: VGG-16, batch 256, vDNN_all / conv / dyn
    (and fit) under 12 GiB against the no-offload run: bit-identical loss and weight gradients, statistics equal to the
    memory-schedule oracle, and sampled layer outputs against the CPU oracle evaluated on the captured layer inputs."""
    import torch
    net = nets.vgg16(256)
    x, labels, weights = gen.make(net)
    xd, ld = torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda()
    out_shapes, _ = nets.shapes(net)
    hooks = (0, 1, 2, 23, 24)  # c1_1, its ReLU, c1_2 (pre-ReLU), pool4, c5_1 (pre-ReLU)
    assert [net["layers"][i]["type"] for i in hooks] == ["conv", "relu", "conv", "maxpool", "conv"]
    base_loss, base_dw, base_st, caps = _run(B, net, xd, ld, weights, "none", 0, hooks)
    assert np.isfinite(base_loss) and 5.0 < base_loss < 40.0
    rng = np.random.default_rng(7)
    c11 = caps[0].reshape(out_shapes[0])
    r11 = caps[1].reshape(out_shapes[1])
    c12 = caps[2].reshape(out_shapes[2])
    p4 = caps[23].reshape(out_shapes[23])
    c51 = caps[24].reshape(out_shapes[24])
    assert sampled_conv_fwd_check(x, weights[0].astype(np.float64), c11, 1, 1, False, rng) < TOL
    assert np.array_equal(r11, np.maximum(c11, 0))
    assert sampled_conv_fwd_check(r11, weights[2].astype(np.float64), c12, 1, 1, False, rng) < TOL
    assert sampled_conv_fwd_check(p4, weights[24].astype(np.float64), c51, 1, 1, False, rng) < TOL
    del caps, c11, r11, c12, p4, c51
    # sampled weight gradients of the last FC layer from captured tensors would need dY; instead use the
    # invariants: every dW finite, and identical bits under every offloading policy
    for i, d in base_dw.items():
        assert np.isfinite(d).all(), i
    assert base_st["n_winograd_convs"] == 10   # c2_2 ... c5_3
    for pol in ("all", "conv", "dyn", "fit"):
        loss, dw, st, _ = _run(B, net, xd, ld, weights, pol, 12 * G)
        assert st["conv_algo"] == "p" and st["kernels"] == base_st["kernels"]   # every plan of a net runs the same kernels
        if pol == "fit":
            assert st["n_offload"] > 2                         # feature maps move in pieces
            assert 0 < st["offloaded_bytes"] == st["prefetched_bytes"] < 9299820544   # fewer bytes than vDNN_conv moves
        else:
            ref = ms.simulate(net, st["effective_policy"], 12 * G, ws=st["ws"])
            assert st["peak_bytes"] == ref["peak_bytes"] <= 12 * G
            assert st["offloaded_bytes"] == ref["offloaded_bytes"] == st["prefetched_bytes"]
        assert st["peak_bytes"] <= st["pool_extent_bytes"] <= 12 * G
        if pol == "all":
            assert st["offloaded_bytes"] == 15568207872
        if pol == "dyn":
            assert st["effective_policy"] == "conv"
        # the no-hook run folds ReLU into the convolutions, the hooked base run did not for layers 0 and 2:
        # compare against a no-hook no-offload run instead
        if pol == "all":
            nh_loss, nh_dw, _, _ = _run(B, net, xd, ld, weights, "none", 0)
            assert nh_loss == base_loss
            for i in weights:
                assert np.array_equal(nh_dw[i], base_dw[i]), i
        assert loss == base_loss, pol
        for i in weights:
            assert np.array_equal(dw[i], base_dw[i]), (pol, i)


def test_vgg16_b256_direct_kernels_only(B):
    """vdnn_set_winograd(net, 0): no plan runs the Winograd kernel, the step agrees with the default one to rounding (the
    loss to 1e-5; the gradients are held to the oracle separately, in test_step_against_the_oracle_at_full_size), and
    offloading is bit-identical to no offloading here too."""
    import torch
    net = nets.vgg16(256)
    x, labels, weights = gen.make(net)
    xd, ld = torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda()
    wino_loss, _, wino_st, _ = _run(B, net, xd, ld, weights, "none", 0)
    base_loss, base_dw, base_st, _ = _run(B, net, xd, ld, weights, "none", 0, winograd=False)
    assert wino_st["n_winograd_convs"] == 10 and base_st["n_winograd_convs"] == 0
    assert base_st["peak_bytes"] < wino_st["peak_bytes"]
    assert abs(wino_loss - base_loss) < 1e-5 * abs(base_loss)
    for pol in ("conv", "fit"):
        loss, dw, st, _ = _run(B, net, xd, ld, weights, pol, 12 * G, winograd=False)
        assert st["n_winograd_convs"] == 0 and loss == base_loss
        for i in weights:
            assert np.array_equal(dw[i], base_dw[i]), (pol, i)


# The static policies run the performance-optimal kernels and fail where a workspace does not fit (the paper's vDNN_conv (p));
# where the stated budget is too small for that, the configuration runs the greedy mode (Section 3.3).
OTHER = [("alexnet", "conv", "greedy", 1 * G), ("overfeat", "all", None, 2 * G), ("overfeat", "conv", None, 2 * G),
         ("googlenet", "dyn", None, 3 * G), ("googlenet", "all", None, 3 * G), ("alexnet", "fit", None, 900 << 20),
         ("googlenet", "fit", None, 2 * G), ("vgg116_b32", "fit", None, 4 * G)]


@pytest.mark.parametrize("name,policy,algo,budget", OTHER)
def test_other_workloads_full_size(B, name, policy, algo, budget):
    """AlexNet / OverFeat / GoogLeNet shaped workloads at batch 128 under their budgets: statistics equal to the
    memory-schedule oracle, and bit-identical to a no-offload run without a budget that runs the same kernels (those of the
    performance-optimal mode by itself; those the plan reports, named layer by layer, after a greedy downgrade)."""
    import torch
    net = nets.vgg(batch=32, extra_per_group=20) if name == "vgg116_b32" else nets.CONFIGS[name]()
    x, labels, weights = gen.make(net)
    xd, ld = torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda()
    loss, dw, st, _ = _run(B, net, xd, ld, weights, policy, budget, algo=algo)
    assert np.isfinite(loss) and 1.0 < loss < 60.0
    if algo == "greedy":
        assert st["conv_algo"] == "greedy" and st["n_downgraded_convs"] > 0
    base_loss, base_dw, base_st, _ = _run(B, net, xd, ld, weights, "none", 0, kernels=None if st["conv_algo"] == "p" else st["kernels"])
    assert base_st["kernels"] == st["kernels"]
    if policy == "fit":
        # the schedule itself is checked in _run (tests/sched_util.py); here: it offloads, within the budget
        assert ms.simulate(net, "none", budget, st["conv_algo"], ws=st["ws"])["status"] == "oom" and st["offloaded_bytes"] == st["prefetched_bytes"] > 0
        assert st["peak_bytes"] <= st["pool_extent_bytes"] <= budget and st["window_fill_pm"] > 0
    else:
        ref = ms.simulate(net, st["effective_policy"], budget, st["conv_algo"], ws=st["ws"])
        assert ref["status"] == "ok"
        assert st["peak_bytes"] == ref["peak_bytes"] <= budget and st["pool_extent_bytes"] <= budget
        assert st["offloaded_bytes"] == ref["offloaded_bytes"] and st["n_ondemand_fetch"] == ref["n_ondemand_fetch"]
        assert st["n_downgraded_convs"] == ref["n_downgraded_convs"]
    assert loss == base_loss
    for i in weights:
        assert np.isfinite(dw[i]).all()
        assert np.array_equal(dw[i], base_dw[i]), i


@pytest.mark.parametrize("extra,check_identity", [(20, True), (80, False)])
def test_very_deep_vgg_batch_32(B, extra, check_identity):
    """Section 5.5: VGG-116 ... VGG-416 at batch 32.  The baseline allocation grows to tens of GB while vDNN keeps
    the GPU-side footprint to a few GB, with most feature maps on the host."""
    import torch
    net = nets.vgg(batch=32, extra_per_group=extra)
    x, labels, weights = gen.make(net, seed=gen.BASE_SEED + 50 + extra)
    xd, ld = torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda()
    loss, dw, st, _ = _run(B, net, xd, ld, weights, "all", 12 * G)
    ref = ms.simulate(net, "all", 12 * G, ws=st["ws"])
    info = ms.analyse(net)
    assert np.isfinite(loss)
    assert st["peak_bytes"] == ref["peak_bytes"] and st["offloaded_bytes"] == ref["offloaded_bytes"]
    host_fraction = st["offloaded_bytes"] / sum(info["nbytes"].values())
    assert host_fraction > 0.8
    # Section 5.5 quotes 67.1 GB for the baseline of VGG-416 (ours: 70.1 GB without cuDNN's workspace
    # accounting) and a GPU-side footprint of a few GB under vDNN
    assert st["baseline_bytes"] > (18e9 if extra == 20 else 60e9)
    assert st["peak_bytes"] < 0.2 * st["baseline_bytes"] and st["peak_bytes"] < 12 * G
    if check_identity:
        base_loss, base_dw, _, _ = _run(B, net, xd, ld, weights, "none", 0)
        assert loss == base_loss
        for i in weights:
            assert np.array_equal(dw[i], base_dw[i]), i


GOLDEN = [("vgg16", "dyn", 12 * G, 3), ("alexnet", "conv:greedy", 1 * G, 6), ("overfeat", "all", 2 * G, 6), ("googlenet", "dyn", 3 * G, 6)]


def full_size_oracle_report(B, name, policy, budget, k_images, winograd=True):
    """One step of a benchmark configuration at its stated size, policy and budget, every layer's output and every
    gradient map captured, against
      (a) tests/golden/<name>_b<batch>_step.json, which tests/golden/make_step_golden.py wrote from the fp64 CPU oracle alone:
          loss, sampled forward values, sampled gradient-map entries, sampled weight-gradient entries;
      (b) the oracle run here on k_images images of the same batch -- the first image whose golden samples all agree, and the
          images whose golden samples disagree most -- twice: deciding ReLU signs and pooling arg-max from the GPU's forward
          values ("shared"), and deciding for itself ("pure"); every element of every output and gradient map is compared;
      (c) the defining sum of sampled weight-gradient entries, evaluated in fp64 from the GPU's own X and dY of the whole batch.
    Returns the measurements; the test below asserts on them.  Error measure as everywhere: largest deviation relative to
    the largest element of the oracle's tensor."""
    import json
    import os
    import torch
    from oracle import net as onet
    from tests.gpu_util import count_decision_flips, rel_err
    make = nets.CONFIGS[name]
    net = make()
    batch = net["batch"]
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "%s_b%d_step.json" % (name, batch))
    gold = json.load(open(path))
    x, labels, weights = gen.make(net)
    n = B.Net(net, budget)
    n.set_winograd(winograd)
    if ":" in policy:
        policy, algo = policy.split(":")
        n.set_conv_algo(algo)
    n.set_policy(policy)
    n.attach_torch()
    for i, w in weights.items():
        n.set_weights(i, w)
    nl = len(net["layers"])
    outs = {i: np.empty(n.output_count(i), np.float32) for i in range(nl - 1)}
    grads = {i: np.empty(n.output_count(i), np.float32) for i in range(nl - 1)}
    for i in range(nl - 1):
        n.capture_output(i, outs[i])
        n.capture_grad(i, grads[i])
    loss = n.forward(torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda())
    n.backward()
    dw = {i: n.get_weight_grad(i, w.shape) for i, w in weights.items()}
    st = n.stats()
    n.close()
    rep = dict(name=name, stats=st, loss_err=abs(loss - gold["loss"]) / abs(gold["loss"]), fwd={}, dy={}, dw={}, images={})
    per = {i: outs[i].size // batch for i in outs}
    # (a) the golden step
    outliers = np.zeros(batch, np.int64)   # per image: sampled gradient-map entries beyond 1e-4
    for key, mine in (("fwd", outs), ("dy", grads)):
        for i, g in gold[key].items():
            idx = np.array(g["index"])
            d = np.abs(mine[int(i)][idx].astype(np.float64) - np.array(g["value"])) / g["max_abs"]
            rep[key][int(i)] = dict(max=float(d.max()), beyond=float((d > TOL).mean()), samples=len(d))
            if key == "dy":
                np.add.at(outliers, idx[d > TOL] // per[int(i)], 1)
    rep["flagged_images"] = int((outliers > 0).sum())
    for i, g in gold["layers"].items():
        flat = dw[int(i)].reshape(-1).astype(np.float64)
        assert list(dw[int(i)].shape) == g["shape"]
        d = np.abs(flat[np.array(g["index"])] - np.array(g["value"])) / g["max_abs"]
        rep["dw"][int(i)] = dict(max=float(d.max()), rms=float(np.sqrt((d * d).mean())), l2_err=abs(float(np.sqrt((flat * flat).sum())) - g["l2"]) / g["l2"])
    # (b) k images under the oracle, decisions shared and not
    clean = [int(j) for j in np.nonzero(outliers == 0)[0][:1]]
    worst = [int(j) for j in np.argsort(-outliers, kind="stable") if outliers[j] > 0][:k_images - len(clean)]
    chosen = clean + worst
    part = make(len(chosen))
    xs, ls = x[chosen], labels[chosen]
    scale = len(chosen) / batch
    ov = {i: np.ascontiguousarray(outs[i].reshape(batch, -1)[chosen]) for i in outs}
    gv = {i: grads[i].reshape(batch, -1)[chosen] for i in grads}
    shared_dy, pure_dy = {}, {}
    ref = onet.step(part, xs, ls, weights, outs_override=ov, dy_hook=lambda i, g: shared_dy.__setitem__(i, g.reshape(len(chosen), -1) * scale))
    pure = onet.step(part, xs, ls, weights, dy_hook=lambda i, g: pure_dy.__setitem__(i, g.reshape(len(chosen), -1) * scale))
    rep["shared_fwd_max"] = max(rel_err(ov[i], ref["outs"][i]) for i in ov)
    for j, img in enumerate(chosen):
        one = make(1)
        flips = count_decision_flips(one, {i: ov[i][j:j + 1] for i in ov}, [o[j:j + 1] if o.ndim else o for o in ref["outs"]])
        rep["images"][img] = dict(golden_outliers=int(outliers[img]), flips=flips,
                                  shared_dy=max(rel_err(gv[i][j], shared_dy[i][j]) * np.abs(shared_dy[i][j]).max() / np.abs(shared_dy[i]).max() for i in shared_dy if i in gv),
                                  pure_dy=max(rel_err(gv[i][j], pure_dy[i][j]) * np.abs(pure_dy[i][j]).max() / np.abs(pure_dy[i]).max() for i in pure_dy if i in gv))
    rep["shared_dy"] = {i: rel_err(gv[i], shared_dy[i]) for i in shared_dy if i in gv}
    for i in weights:
        e = (pure["dw"][i] - ref["dw"][i]).reshape(-1)
        rep["dw"][i]["decisions_on_chosen"] = float(np.abs(e).max()) * scale / gold["layers"][str(i)]["max_abs"]
    # (c) the weight gradients from the GPU's own X and dY, whole batch
    rng = np.random.default_rng(11)
    shapes, _ = nets.shapes(net)
    for i, w in weights.items():
        layer = net["layers"][i]
        src = layer["inputs"][0]
        xin = x if src < 0 else outs[src].reshape(shapes[src])
        dy = grads[i].reshape(shapes[i])
        if layer["type"] == "conv":
            rep["dw"][i]["from_own_x_dy"] = sampled_conv_bwd_filter_check(xin, dy, dw[i], layer["stride"], layer["pad"], rng, pairs=4)
        else:
            x2, dy2 = xin.reshape(batch, -1).astype(np.float64), dy.reshape(batch, -1).astype(np.float64)
            rows = rng.integers(0, dw[i].shape[0], 8)
            want = dy2[:, rows].T @ x2
            rep["dw"][i]["from_own_x_dy"] = float(np.abs(dw[i][rows].astype(np.float64) - want).max() / np.abs(dw[i]).max())
    return rep


def print_report(rep):
    print("%s: loss error %.2e; forward on the chosen images, all elements: %.2e; %d of the batch's images have gradient-map samples beyond 1e-4 of the golden file" %
          (rep["name"], rep["loss_err"], rep["shared_fwd_max"], rep["flagged_images"]))
    for img, r in rep["images"].items():
        print("  image %3d: %3d golden samples beyond 1e-4, %3d decisions differ; gradient maps vs the oracle with shared decisions %.1e, vs the oracle alone %.1e" %
              (img, r["golden_outliers"], r["flips"], r["shared_dy"], r["pure_dy"]))
    for i in sorted(rep["fwd"]):
        f, d = rep["fwd"][i], rep["dy"][i]
        line = "  layer %3d  Y max %.1e | dY vs golden: max %.1e, %.1f %% of %d samples beyond 1e-4 | dY with shared decisions %.1e" % (
            i, f["max"], d["max"], 100 * d["beyond"], d["samples"], rep["shared_dy"].get(i, float("nan")))
        if i in rep["dw"]:
            w = rep["dw"][i]
            line += " | dW vs golden: max %.1e rms %.1e; from own X, dY %.1e; decisions on the chosen images move it by %.1e" % (
                w["max"], w["rms"], w["from_own_x_dy"], w["decisions_on_chosen"])
        print(line)


@pytest.mark.parametrize("name,policy,budget,k_images", GOLDEN, ids=[g[0] for g in GOLDEN])
def test_step_against_the_oracle_at_full_size(B, name, policy, budget, k_images):
    """End-to-end parity of the four full-size configurations, each under its own policy and budget, against the fp64 oracle.

    What holds to 1e-4 without qualification: the loss and every sampled forward value of every layer.  Backward propagation
    takes discrete decisions from forward values (Eq. chain_rule through ReLU and max-pooling: which activations are positive,
    which element of a window is the largest), and an fp32 forward pass that is right to 1e-6 still puts a few of the millions of
    near-ties of an image on the other side than the fp64 pass; each such decision moves whole gradient terms of that image, in
    the layer where it happens and in every layer below.  The test shows from values that this, and nothing else, separates the
    GPU's gradients from the oracle's:
      - images whose golden gradient-map samples all agree to 1e-4 have no differing decision (checked on the first of them),
        and there the GPU's gradient maps equal the oracle's own, every element, to 1e-4;
      - images whose golden samples disagree do have differing decisions (checked on the worst of them), and with the oracle
        deciding from the GPU's forward values their gradient maps agree as well, every element, to 1e-4;
      - the weight gradients are the defining sums over the GPU's own X and dY (sampled entries, fp64, whole batch) to 1e-4.
    The distance of the weight gradients to the golden file is printed beside what the differing decisions of the chosen images
    alone do to them; it is bounded here only as a sanity check (1e-2), since its size is a property of the near-ties of the
    data, not of the kernels."""
    rep = full_size_oracle_report(B, name, policy, budget, k_images)
    print_report(rep)
    assert rep["stats"]["peak_bytes"] <= budget
    assert rep["loss_err"] < TOL
    assert max(f["max"] for f in rep["fwd"].values()) < TOL
    assert rep["shared_fwd_max"] < TOL
    assert max(rep["shared_dy"].values()) < TOL, rep["shared_dy"]
    for img, r in rep["images"].items():
        assert r["shared_dy"] < TOL, (img, r)
        if r["golden_outliers"]:
            assert r["flips"] > 0, (img, r)          # a disagreement with the golden file has its cause in a decision
        if r["flips"] == 0:
            assert r["pure_dy"] < TOL, (img, r)      # no decision differs: the oracle needs no help
    for i, w in rep["dw"].items():
        assert w["from_own_x_dy"] < TOL, (i, w)
        assert w["l2_err"] < 1e-3 and w["max"] < 1e-2, (i, w)
