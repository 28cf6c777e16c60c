"""Pins for the memory-schedule oracle (oracle/memsched.py): a hand-enumerated trace, closed
forms from the network shapes, the paper's quoted figure, and the ordering invariants the
paper states."""
import numpy as np

from oracle import memsched as ms
from synth import nets

G = 2 ** 30


def _vgg16_feature_map_elems(batch):
    """Per-layer X sizes of VGG-16 written out by hand (224x224 input, five groups)."""
    conv_in = [(3, 224), (64, 224), (64, 112), (128, 112), (128, 56), (256, 56), (256, 56),
               (256, 28), (512, 28), (512, 28), (512, 14), (512, 14), (512, 14)]
    pool_in = [(64, 224), (128, 112), (256, 56), (512, 28), (512, 14)]
    conv = sum(c * h * h for c, h in conv_in) * batch
    pool = sum(c * h * h for c, h in pool_in) * batch
    return conv, pool


def test_vgg16_offload_bytes_closed_form_and_paper_figure():
    net = nets.vgg16(256)
    conv, pool = _vgg16_feature_map_elems(256)
    r_all = ms.simulate(net, "all", 400 * G)
    r_conv = ms.simulate(net, "conv", 400 * G)
    assert r_all["offloaded_bytes"] == 4 * (conv + pool)
    assert r_conv["offloaded_bytes"] == 4 * conv
    # Section 5.1: vDNN_all offloads "up to 16 GB" for VGG-16 (256)
    assert 15.0e9 < r_all["offloaded_bytes"] < 16.5e9
    assert r_all["n_offload"] == 18 and r_conv["n_offload"] == 13
    for r in (r_all, r_conv):
        assert r["prefetched_bytes"] == r["offloaded_bytes"]
        assert r["n_prefetch"] + r["n_ondemand_fetch"] == r["n_offload"]
        assert r["cur_bytes"] == r["persistent_bytes"]


def test_vgg16_trainability_under_12_gib():
    """Section 5: VGG-16 (256) does not fit 12 GB without offloading, and does with vDNN; batch 64 and 128
    with the memory-optimal algorithm fit without it."""
    net = nets.vgg16(256)
    assert ms.simulate(net, "none", 12 * G)["status"] == "oom"
    assert ms.simulate(net, "all", 12 * G)["status"] == "ok"
    assert ms.simulate(net, "conv", 12 * G)["status"] == "ok"
    assert ms.baseline_bytes(net) > 12 * G
    assert ms.baseline_bytes(nets.vgg16(64)) < 12 * G
    assert ms.dynamic(net, 12 * G)[:2] == ("conv", "p")
    assert ms.dynamic(nets.vgg16(64), 12 * G)[:2] == ("none", "p")
    assert ms.dynamic(net, 2 * G)[0] is None


def test_hand_enumerated_trace_linear_net():
    """conv3x3(4) - relu - maxpool2 - fc(5) - loss on a 1x2x4x4 input, policy all, written out by hand.
    Sizes: input 128 B -> 256; conv out 1x4x4x4 = 256 B; pool out 1x4x2x2 = 64 B -> 256; fc out 20 B -> 256."""
    b = nets._Builder("hand", 1, 2, 4, 4)
    b.conv(4, 3, pad=1)
    b.maxpool(2, 2)
    b.fc(5, relu=False)
    net = b.done()
    r = ms.simulate(net, "all", 1 << 20)
    w0 = 4 * 4 * 2 * 9  # 288 -> 512
    w3 = 4 * 5 * 16     # 320 -> 512
    expect = [
        ("create", "alloc", "W0", 512), ("create", "alloc", "dW0", 512),
        ("create", "alloc", "W3", 512), ("create", "alloc", "dW3", 512),
        ("create", "alloc", "labels", 256), ("create", "alloc", "loss", 256),
        ("F-1", "alloc", "B-1", 256),
        ("F0", "alloc", "B0", 256), ("F0", "offload", "B-1", 128), ("F0", "compute", "conv"), ("F0", "free", "B-1", 256),
        ("F1", "compute", "relu"),
        ("F2", "alloc", "B2", 256), ("F2", "offload", "B0", 256), ("F2", "compute", "maxpool"), ("F2", "free", "B0", 256),
        ("F3", "alloc", "B3", 256), ("F3", "compute", "fc"),
        ("F4", "compute", "softmax_ce"),
        # backward of the loss: the search passes fc (3) and finds the pool (2), whose X (B0) is on the host
        ("B4", "alloc", "B0", 256), ("B4", "prefetch", "B0", 256), ("B4", "alloc", "dB3", 256),
        ("B4", "compute", "softmax_ce"), ("B4", "free", "B3", 256),
        # fc: search passes pool (nothing pending), relu, finds conv 0 with B-1 on the host
        ("B3", "alloc", "B-1", 256), ("B3", "prefetch", "B-1", 128), ("B3", "alloc", "dB2", 256),
        ("B3", "compute", "fc"), ("B3", "free", "dB3", 256), ("B3", "free", "B2", 256),
        ("B2", "alloc", "dB0", 256), ("B2", "compute", "maxpool"), ("B2", "free", "dB2", 256),
        ("B1", "compute", "relu"), ("B1", "free", "B0", 256),
        # first layer: no dX, no workspace (reduction of 16 is not split)
        ("B0", "compute", "conv"), ("B0", "free", "dB0", 256), ("B0", "free", "B-1", 256),
    ]
    assert w0 == 288 and w3 == 320
    assert r["trace"] == expect
    assert r["status"] == "ok" and r["cur_bytes"] == 4 * 512 + 2 * 256
    # peak: persistent 2560 + during B3: B0, B-1, dB3, dB2, B2 = 5 * 256
    assert r["peak_bytes"] == 2560 + 5 * 256


def test_prefetch_order_is_reverse_offload_order_and_bounded_by_conv():
    for net in (nets.vgg16(8), nets.alexnet(4), nets.overfeat(4)):
        for pol in ("all", "conv"):
            r = ms.simulate(net, pol, 400 * G)
            off = [t[2] for t in r["trace"] if t[1] == "offload"]
            pre = [t[2] for t in r["trace"] if t[1] in ("prefetch", "ondemand")]
            assert pre == off[::-1]
            # a prefetch issued before the backward computation of layer m is for a layer n < m,
            # and no CONV layer lies strictly between n's offload layer and m
            info = ms.analyse(net)
            for t in r["trace"]:
                if t[1] == "prefetch":
                    m = int(t[0][1:])
                    b = int(t[2][1:])
                    n = info["readers"][b][-1]
                    assert n < m
                    assert all(net["layers"][j]["type"] != "conv" for j in range(n + 1, m))


def test_policy_ordering_invariants():
    """Section 3.3 / 5.1: all uses the least memory, then conv, then no offloading; the network-wide
    baseline is above all of them."""
    for mk in (nets.tiny, nets.alexnet, nets.overfeat, nets.googlenet, nets.vgg16, nets.fork_join):
        net = mk()
        peaks = {p: ms.simulate(net, p, 400 * G) for p in ("all", "conv", "none")}
        assert peaks["all"]["peak_bytes"] <= peaks["conv"]["peak_bytes"] <= peaks["none"]["peak_bytes"]
        assert peaks["all"]["avg_bytes_layerstep"] <= peaks["conv"]["avg_bytes_layerstep"] <= peaks["none"]["avg_bytes_layerstep"]
        assert peaks["none"]["peak_bytes"] <= ms.baseline_bytes(net)
        assert peaks["none"]["offloaded_bytes"] == 0
        assert peaks["conv"]["offloaded_bytes"] <= peaks["all"]["offloaded_bytes"]
        for r in peaks.values():
            assert r["status"] == "ok" and r["cur_bytes"] == r["persistent_bytes"]
            assert r["prefetched_bytes"] == r["offloaded_bytes"]


def test_offload_only_at_last_consumer():
    """Fig. nonlinear_dfg: a feature map with several consumers is offloaded once, by its last consumer."""
    net = nets.fork_join()
    info = ms.analyse(net)
    for pol in ("all", "conv"):
        r = ms.simulate(net, pol, 400 * G)
        seen = set()
        for t in r["trace"]:
            if t[1] == "offload":
                b = int(t[2][1:])
                assert b not in seen
                seen.add(b)
                assert int(t[0][1:]) == info["readers"][b][-1]
        # the forked feature map (4 consumers) is among them under both policies
        forked = [b for b, rd in info["readers"].items() if len(rd) == 4]
        assert len(forked) == 1 and forked[0] in seen


def test_oom_is_reported_where_it_happens():
    net = nets.tiny(8)
    r = ms.simulate(net, "none", 300 * 1024)
    assert r["status"] == "oom" and r["oom_at"] == "F0"
    r = ms.simulate(net, "all", 1100 * 1024)
    assert r["status"] == "oom" and r["oom_at"].startswith("B")
    assert ms.simulate(net, "all", 4 * 2 ** 20)["status"] == "ok"


def test_very_deep_vgg_host_fraction():
    """Section 5.4: for VGG-116..416 at batch 32 most of the allocations live on the host (81-92 %)."""
    fracs = []
    for extra in (20, 40):
        net = nets.vgg(batch=32, extra_per_group=extra)
        r = ms.simulate(net, "all", 400 * G)
        info = ms.analyse(net)
        total = sum(info["nbytes"].values())
        fracs.append(r["offloaded_bytes"] / total)
    assert all(f > 0.8 for f in fracs)


def test_dynamic_policy_phases():
    """Section 3.3: budgets chosen so that each phase of vDNN_dyn decides."""
    net = nets.alexnet(8)
    none_p = ms.simulate(net, "none", 1 << 50, "p")["peak_bytes"]
    conv_p = ms.simulate(net, "conv", 1 << 50, "p")["peak_bytes"]
    all_p = ms.simulate(net, "all", 1 << 50, "p")["peak_bytes"]
    all_m = ms.simulate(net, "all", 1 << 50, "m")["peak_bytes"]
    assert all_m < all_p <= conv_p <= none_p
    assert ms.dynamic(net, none_p)[:2] == ("none", "p")                 # phase 2, first try
    assert ms.dynamic(net, none_p - 256)[:2] == ("conv", "p")           # phase 2, second try
    pol, algo, r = ms.dynamic(net, all_p - 256)                           # phase 3: greedy downgrade
    assert algo == "greedy" and r["status"] == "ok" and r["n_memopt_convs"] >= 1 and r["peak_bytes"] <= all_p - 256
    assert ms.dynamic(net, all_m - 256)[0] is None                        # phase 1 fails: not trainable
    # the memory-optimal algorithm allocates no convolution workspace at all
    tr = ms.simulate(net, "all", 1 << 50, "m")["trace"]
    conv_layers = {i for i, l in enumerate(net["layers"]) if l["type"] == "conv"}
    assert not [t for t in tr if t[1] == "alloc" and t[2] == "WS" and int(t[0][1:]) in conv_layers]


def test_winograd_workspace_closed_forms():
    """The Winograd workspace rules evaluated by hand for VGG-16 (256) layers: transformed filter 16*C*K floats, then
    16*(C + K) floats per 2x2 output tile for as many images as fit 512 MiB; backward-filter: the 16 products once
    plus once per reduction split, then the same chunk."""
    MiB = 1 << 20
    # c4_2: 512 -> 512 at 28 x 28: 196 tiles per image, 16 * 1024 * 196 * 4 = 12 845 056 bytes per image, 41 images per chunk
    assert ms.winograd_workspace(256, 512, 28, 28, 512, 3, 1, 1) == 16 * 512 * 512 * 4 + 41 * 12845056
    assert 41 * 12845056 <= 512 * MiB < 42 * 12845056
    # c5: 14 x 14, 49 tiles: 3 211 264 bytes per image, 167 images per chunk
    assert ms.winograd_workspace(256, 512, 14, 14, 512, 3, 1, 1) == 16 * 512 * 512 * 4 + 167 * 3211264
    # a batch smaller than the chunk: all of it
    assert ms.winograd_workspace(8, 512, 14, 14, 512, 3, 1, 1) == 16 * 512 * 512 * 4 + 8 * 3211264
    # 13 x 13 (odd sides): 7 x 7 tiles as well
    assert ms.winograd_workspace(8, 384, 13, 13, 256, 3, 1, 1) == 16 * 384 * 256 * 4 + 8 * 16 * 640 * 49 * 4
    # not wide enough, not 3x3, strided, unpadded: no Winograd
    for args in ((256, 128, 28, 28, 512, 3, 1, 1), (256, 512, 28, 28, 64, 3, 1, 1), (256, 512, 28, 28, 512, 5, 1, 2),
                 (256, 512, 28, 28, 512, 3, 2, 1), (256, 512, 28, 28, 512, 3, 1, 0), (256, 520, 28, 28, 512, 3, 1, 1)):
        assert ms.winograd_workspace(*args) == 0, args
    # backward-filter of c4_2: 4 x 4 tiles of 128 x 128 per product, 16 products: 256 workgroups -> 4 splits of the
    # 41 * 196 = 8036 tile positions
    assert ms.winograd_filter_workspace(256, 512, 28, 28, 512, 3, 1, 1) == 16 * 512 * 512 * 4 * (1 + 4) + 41 * 12845056
    # c3_2: 256 -> 256 at 56 x 56: 784 tiles, 25 690 112 bytes per image, 20 per chunk; 2 x 2 tiles x 16 = 64 workgroups -> 16 splits
    assert ms.winograd_filter_workspace(256, 256, 56, 56, 256, 3, 1, 1) == 16 * 256 * 256 * 4 * (1 + 16) + 20 * 25690112
    assert ms.winograd_filter_workspace(256, 192, 56, 56, 256, 3, 1, 1) == 0      # input channels not a multiple of 128
    assert ms.winograd_filter_workspace(256, 256, 56, 56, 128, 3, 1, 1) == 0      # fewer than 256 output channels
