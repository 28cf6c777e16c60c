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
    assert net["layers"] == _hand_net()["layers"]
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
    """Section 5.5: for VGG-116..416 at batch 32 most of the allocations live on the host (81-92 %)."""
    fracs = []
    for extra in (20, 40):
        net = nets.vgg(batch=32, extra_per_group=extra)
        r = ms.simulate(net, "all", 400 * G)
        info = ms.analyse(net)
        total = sum(info["nbytes"].values())
        fracs.append(r["offloaded_bytes"] / total)
    assert all(f > 0.8 for f in fracs)


def _hand_net():
    b = nets._Builder("hand", 1, 2, 4, 4)
    b.conv(4, 3, pad=1)
    b.maxpool(2, 2)
    b.fc(5, relu=False)
    return b.done()


def test_workspace_and_algorithm_modes_by_hand():
    """Section 2.2 / 3.3 on the hand net above, with workspace sizes given by hand: the conv layer can run three ways
    in each direction (fastest first, the last without workspace), the FC layer needs 256 bytes in forward.
    Live bytes when the conv asks for its workspace: forward 2560 + B-1 + B0 = 3072, backward 2560 + dB0 + B-1 = 3072."""
    net = _hand_net()
    ws = {(0, "fwd"): [1024, 512, 0], (0, "bwd"): [2048, 256, 0], (3, "fwd"): [256]}
    r = ms.simulate(net, "all", 1 << 20, "p", ws=ws)
    tr = r["trace"]
    f0 = [t for t in tr if t[0] == "F0"]
    assert f0 == [("F0", "alloc", "B0", 256), ("F0", "alloc", "WS", 1024), ("F0", "offload", "B-1", 128), ("F0", "compute", "conv"),
                  ("F0", "free", "WS", 1024), ("F0", "free", "B-1", 256)]
    assert [t for t in tr if t[0] == "F3"] == [("F3", "alloc", "B3", 256), ("F3", "alloc", "WS", 256), ("F3", "compute", "fc"), ("F3", "free", "WS", 256)]
    assert [t for t in tr if t[0] == "B0"] == [("B0", "alloc", "WS", 2048), ("B0", "compute", "conv"), ("B0", "free", "WS", 2048),
                                               ("B0", "free", "dB0", 256), ("B0", "free", "B-1", 256)]
    # peak: backward of the conv, 3072 + 2048
    assert r["peak_bytes"] == 5120 and r["n_memopt_convs"] == 0 and r["n_downgraded_convs"] == 0
    # without any workspace the step peaks at 3840 (backward of the FC layer, five 256-byte blocks live)
    assert ms.simulate(net, "all", 1 << 20)["peak_bytes"] == 3840
    # performance-optimal under 3840: the 1024 bytes in F0 do not fit (3072 + 1024)
    r = ms.simulate(net, "all", 3840, "p", ws=ws)
    assert r["status"] == "oom" and r["oom_at"] == "F0"
    # greedy under 3840: forward takes the second entry (3072 + 512 fits), backward the second (2048 does not, 256 does)
    r = ms.simulate(net, "all", 3840, "greedy", ws=ws)
    assert r["status"] == "ok" and r["peak_bytes"] == 3840
    assert [t[3] for t in r["trace"] if t[1] == "alloc" and t[2] == "WS"] == [512, 256, 256]
    assert r["n_downgraded_convs"] == 1 and r["n_memopt_convs"] == 0
    # no entry with workspace fits in backward: the memory-optimal algorithm is what is left
    r = ms.simulate(net, "all", 3840, "greedy", ws={(0, "fwd"): [1024, 512, 0], (0, "bwd"): [2048, 1024, 0], (3, "fwd"): [256]})
    assert [t[3] for t in r["trace"] if t[1] == "alloc" and t[2] == "WS"] == [512, 256]
    assert r["n_downgraded_convs"] == 1 and r["n_memopt_convs"] == 1
    # memory-optimal: no workspace for the conv in either direction; the FC layer keeps its own
    r = ms.simulate(net, "all", 3840, "m", ws=ws)
    assert [(t[0], t[3]) for t in r["trace"] if t[1] == "alloc" and t[2] == "WS"] == [("F3", 256)]
    assert r["n_memopt_convs"] == 1 and r["peak_bytes"] == 3840
    # the baseline allocates one workspace of the largest performance-optimal size (Fig. mem_allocation_policy_global):
    # feature maps 4 x 256, W and dW 4 x 512, two gradient maps of 256, workspace 2048
    assert ms.baseline_bytes(net, ws) == 4 * 256 + 4 * 512 + 2 * 256 + 2048
    assert ms.baseline_bytes(net) == 4 * 256 + 4 * 512 + 2 * 256
    # trace_stats recounts a trace: the hand-computed figures again
    st = ms.trace_stats(ms.simulate(net, "all", 1 << 20, "p", ws=ws)["trace"])
    assert st["peak_bytes"] == 5120 and st["cur_bytes"] == 2560 and st["offloaded_bytes"] == 128 + 256 == st["prefetched_bytes"]
    assert (st["n_offload"], st["n_prefetch"], st["n_ondemand_fetch"]) == (2, 2, 0)


def _alexnet_ws(net):
    """Hand-made workspace lists for the dyn test: every conv layer can run with 6 MiB, 1 MiB or nothing."""
    ws = {}
    for i, l in enumerate(net["layers"]):
        if l["type"] == "conv":
            ws[i, "fwd"] = [4 << 20, 1 << 20, 0]
            ws[i, "bwd"] = [6 << 20, 1 << 20, 0]
    return ws


def test_dynamic_policy_phases():
    """Section 3.3: budgets chosen so that each phase of vDNN_dyn decides."""
    net = nets.alexnet(8)
    ws = _alexnet_ws(net)
    none_p = ms.simulate(net, "none", 1 << 50, "p", ws=ws)["peak_bytes"]
    conv_p = ms.simulate(net, "conv", 1 << 50, "p", ws=ws)["peak_bytes"]
    all_p = ms.simulate(net, "all", 1 << 50, "p", ws=ws)["peak_bytes"]
    all_m = ms.simulate(net, "all", 1 << 50, "m", ws=ws)["peak_bytes"]
    assert all_m < all_p <= conv_p <= none_p
    assert ms.dynamic(net, none_p, ws)[:2] == ("none", "p")                 # phase 2, first try
    assert ms.dynamic(net, none_p - 256, ws)[:2] == ("conv", "p")           # phase 2, second try
    pol, algo, r = ms.dynamic(net, all_p - 256, ws)                           # phase 3: greedy downgrade
    assert algo == "greedy" and r["status"] == "ok" and r["n_downgraded_convs"] >= 1 and r["peak_bytes"] <= all_p - 256
    assert ms.dynamic(net, all_m - 256, ws)[0] is None                        # phase 1 fails: not trainable
    # the memory-optimal algorithm allocates no convolution workspace at all
    tr = ms.simulate(net, "all", 1 << 50, "m", ws=ws)["trace"]
    conv_layers = {i for i, l in enumerate(net["layers"]) if l["type"] == "conv"}
    assert not [t for t in tr if t[1] == "alloc" and t[2] == "WS" and int(t[0][1:]) in conv_layers]
