"""CPU tests of the library's host logic: the C ABI loads and exports every declared symbol, the
planner's op sequence and byte statistics equal the memory-schedule oracle's for the paper's policies (the
library's workspace sizes go into the oracle as a parameter), schedules beyond the paper keep the contract any vDNN
schedule has to keep (tests/sched_util.py), placements never overlap live blocks, and error paths return statuses."""
import ctypes as C
import os
import re

import pytest

from oracle import memsched as ms
from synth import nets
from tests.sched_util import check_placement, check_schedule, lib_ws

binding = pytest.importorskip("paper_1602_08124_amd.binding")
G = 2 ** 30
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "vdnn.h")).read()
    declared = set(re.findall(r"\b(vdnn_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 30
    for name in declared:
        assert hasattr(binding.lib, name), name
    assert declared == set(binding.EXPORTS), declared ^ set(binding.EXPORTS)


CASES = [(nets.tiny, 8), (nets.alexnet, 128), (nets.overfeat, 128), (nets.googlenet, 128), (nets.vgg16, 256),
         (nets.fork_join, 4), (lambda b: nets.vgg(b, extra_per_group=20), 32)]


@pytest.mark.parametrize("mk,batch", CASES)
@pytest.mark.parametrize("policy", ["none", "conv", "all"])
def test_plan_equals_memory_schedule_oracle(mk, batch, policy):
    net = mk(batch)
    n = binding.Net(net, 0)
    n.set_policy(policy)
    ws = lib_ws(n, net)
    ref = ms.simulate(net, policy, 1 << 50, ws=ws)
    tr = n.trace()
    assert [t[:4] for t in tr] == [tuple(t) for t in ref["trace"]]
    st = n.stats()
    for k in ("peak_bytes", "offloaded_bytes", "prefetched_bytes", "n_offload", "n_prefetch", "n_ondemand_fetch"):
        assert st[k] == ref[k], k
    assert st["cur_bytes"] == ref["cur_bytes"] == st["persistent_bytes"]
    assert abs(st["avg_bytes_layerstep"] - ref["avg_bytes_layerstep"]) < 1e-6 * ref["avg_bytes_layerstep"]
    assert st["baseline_bytes"] == ms.baseline_bytes(net, ws)
    assert st["pool_extent_bytes"] >= st["peak_bytes"]
    chosen = {int(t[2][1:]) for t in tr if t[1] == "offload"}
    mine = check_schedule(net, tr, st["pool_extent_bytes"], chosen, st["persistent_bytes"])
    assert mine["peak_bytes"] == st["peak_bytes"]
    n.close()


@pytest.mark.parametrize("mk,batch,budget", [(nets.tiny, 8, 4 << 20), (nets.alexnet, 128, G), (nets.overfeat, 128, 2 * G),
                                             (nets.googlenet, 128, 3 * G), (nets.vgg16, 256, 12 * G), (nets.vgg16, 256, 2 * G),
                                             (nets.vgg16, 128, 12 * G)])
def test_trainability_and_dyn_match_oracle(mk, batch, budget):
    net = mk(batch)
    n = binding.Net(net, budget)
    ws = lib_ws(n, net)
    for policy in ("none", "conv", "all"):
        ref = ms.simulate(net, policy, budget, ws=ws)
        s = n.try_policy(policy)
        assert (s == binding.OK) == (ref["status"] == "ok"), (policy, n.last_error())
        if s != binding.OK:
            assert s == binding.ERR_OOM_DEVICE
            assert n.last_error().startswith(ref["oom_at"] + ":")
        else:
            assert n.stats()["pool_extent_bytes"] <= budget
    pol, algo, ref = ms.dynamic(net, budget, ws)
    s = n.try_policy("dyn")
    if pol is None:
        assert s == binding.ERR_OOM_DEVICE
    else:
        st = n.stats()
        assert s == binding.OK and st["effective_policy"] == pol and st["conv_algo"] == algo
        assert st["peak_bytes"] == ref["peak_bytes"]
        assert [t[:4] for t in n.trace()] == [tuple(t) for t in ref["trace"]]
    n.close()


def test_dyn_phases_and_algorithm_modes_match_oracle():
    """Budgets placed so that each phase of vDNN_dyn decides; static policies under each algorithm mode."""
    net = nets.alexnet(8)
    n_conv = sum(l["type"] == "conv" for l in net["layers"])
    peaks = {}
    for pol in ("none", "conv", "all"):
        for algo in ("p", "m"):
            n = binding.Net(net, 0)
            n.set_conv_algo(algo)
            n.set_policy(pol)
            ws = lib_ws(n, net)
            ref = ms.simulate(net, pol, 1 << 50, algo, ws=ws)
            st = n.stats()
            assert [t[:4] for t in n.trace()] == [tuple(t) for t in ref["trace"]]
            assert st["peak_bytes"] == ref["peak_bytes"] and st["conv_algo"] == algo
            assert st["n_memopt_convs"] == ref["n_memopt_convs"] == (n_conv if algo == "m" else 0)
            peaks[pol, algo] = st["peak_bytes"]
            n.close()
    assert peaks["all", "m"] < peaks["all", "p"] < peaks["conv", "p"] < peaks["none", "p"]
    seen = set()
    for budget in (peaks["none", "p"], peaks["none", "p"] - 256, peaks["conv", "p"] - 256, peaks["all", "p"] - 256,
                   peaks["all", "m"], peaks["all", "m"] - 256):
        pol, algo, ref = ms.dynamic(net, budget, ws)
        seen.add((pol, algo))
        n = binding.Net(net, budget)
        s = n.try_policy("dyn")
        if pol is None:
            assert s == binding.ERR_OOM_DEVICE
        else:
            st = n.stats()
            assert (st["effective_policy"], st["conv_algo"]) == (pol, algo), budget
            assert st["peak_bytes"] == ref["peak_bytes"] and st["n_memopt_convs"] == ref["n_memopt_convs"]
            assert st["n_downgraded_convs"] == ref["n_downgraded_convs"]
            assert [t[:4] for t in n.trace()] == [tuple(t) for t in ref["trace"]]
            assert st["pool_extent_bytes"] <= budget
        n.close()
    assert seen == {("none", "p"), ("conv", "p"), ("all", "p"), ("conv", "greedy"), (None, None)}


def test_vgg16_b256_fits_12_gib_with_all_and_conv():
    net = nets.vgg16(256)
    n = binding.Net(net, 12 * G)
    assert n.try_policy("none") == binding.ERR_OOM_DEVICE
    for p in ("all", "conv"):
        n.set_policy(p)
        st = n.stats()
        assert st["pool_extent_bytes"] <= 12 * G
    n.set_policy("dyn")
    assert n.stats()["effective_policy"] == "conv" and n.stats()["conv_algo"] == "p"
    n.close()


def test_invalid_descriptions_are_rejected():
    def status(net):
        desc, keep = binding.make_desc(net)
        h = C.c_void_p()
        s = binding.lib.vdnn_create(C.byref(desc), 0, C.byref(h))
        if s == binding.OK:
            binding.lib.vdnn_destroy(h)
        return s
    good = nets.tiny(2)
    assert status(good) == binding.OK
    bad = nets.tiny(2)
    bad["layers"][-1]["type"] = "relu"          # no loss at the end
    assert status(bad) == binding.ERR_INVALID_ARG
    bad = nets.tiny(2)
    bad["layers"][2]["inputs"] = [5]            # consumes a later layer
    assert status(bad) == binding.ERR_INVALID_ARG
    bad = nets.tiny(2)
    bad["layers"][0]["k"] = 99                  # window larger than the image
    assert status(bad) == binding.ERR_INVALID_ARG
    bad = nets.tiny(2)
    bad["batch"] = 0
    assert status(bad) == binding.ERR_INVALID_ARG
    bad = nets.tiny(2)
    bad["layers"][2]["inputs"] = [0]            # pool reads conv output that an in-place relu overwrites
    assert status(bad) == binding.ERR_INVALID_ARG
    assert binding.lib.vdnn_create(None, 0, None) == binding.ERR_INVALID_ARG


def test_backward_without_forward_is_a_state_error():
    n = binding.Net(nets.tiny(2), 0)
    assert binding.lib.vdnn_backward(n.h) == binding.ERR_STATE
    n.close()


def test_oversized_tensors_and_degenerate_nets():
    # a feature map with 2^31 or more elements is rejected at create (32-bit element offsets inside kernels)
    big = nets._Builder("big", 4096, 64, 224, 224)
    big.conv(64, 3, pad=1)
    big.fc(10, relu=False)
    desc, keep = binding.make_desc(big.done())
    h = C.c_void_p()
    assert binding.lib.vdnn_create(C.byref(desc), 0, C.byref(h)) == binding.ERR_UNSUPPORTED
    # smallest possible nets plan and agree with the oracle: FC only, batch 1, one-pixel images
    for mk in (lambda: _fc_only(), lambda: _one_pixel()):
        net = mk()
        n = binding.Net(net, 0)
        for pol in ("none", "conv", "all", "dyn"):
            n.set_policy(pol)
            ref = ms.simulate(net, n.stats()["effective_policy"], 1 << 50, ws=lib_ws(n, net))
            assert [t[:4] for t in n.trace()] == [tuple(t) for t in ref["trace"]]
        n.close()


def _fc_only():
    b = nets._Builder("fconly", 1, 5, 1, 1)
    b.fc(3, relu=False)
    return b.done()


def _one_pixel():
    b = nets._Builder("onepx", 1, 2, 1, 1)
    b.conv(3, 3, pad=1)
    b.maxpool(1, 1)
    b.fc(2, relu=False)
    return b.done()


def test_trace_buffer_truncation_and_null_arguments():
    n = binding.Net(nets.tiny(2), 0)
    need = C.c_size_t()
    assert binding.lib.vdnn_trace(n.h, None, 0, C.byref(need)) == binding.OK and need.value > 100
    buf = C.create_string_buffer(16)
    assert binding.lib.vdnn_trace(n.h, buf, 16, C.byref(need)) == binding.OK
    assert len(buf.value) == 15  # truncated, NUL-terminated
    assert binding.lib.vdnn_trace(n.h, None, 0, None) == binding.ERR_INVALID_ARG
    assert binding.lib.vdnn_mem_stats(n.h, None) == binding.ERR_INVALID_ARG
    assert binding.lib.vdnn_set_policy(n.h, 7) == binding.ERR_INVALID_ARG
    assert binding.lib.vdnn_set_conv_algo(n.h, 9) == binding.ERR_INVALID_ARG
    assert binding.lib.vdnn_set_winograd(None, 1) == binding.ERR_INVALID_ARG and binding.lib.vdnn_set_winograd(n.h, 0) == binding.OK
    assert binding.lib.vdnn_set_weights(n.h, 1, None, 0) == binding.ERR_INVALID_ARG
    assert binding.lib.vdnn_weight_count(n.h, 99) == 0 and binding.lib.vdnn_weight_count(n.h, 0) == 16 * 3 * 9
    assert binding.lib.vdnn_output_count(n.h, 0) == 2 * 16 * 32 * 32
    n.close()


# ---------------------------------------------------------------------------------------------------
# beyond the paper: "fit" (offload set chosen per feature map) and budget-aware transfer windows.
# No definition to equal: the contract of tests/sched_util.py instead, plus what the policy promises.
# ---------------------------------------------------------------------------------------------------
def _assert_valid_schedule(n, net, budget, chosen=None):
    """The library's planned step keeps the contract of a vDNN schedule, and its statistics are the trace's."""
    st = n.stats()
    tr = n.trace()
    chosen = n.offload_set() if chosen is None else chosen
    assert n.offload_set() == set(chosen)
    assert st["peak_bytes"] <= st["pool_extent_bytes"] <= budget
    mine = check_schedule(net, tr, st["pool_extent_bytes"], chosen, st["persistent_bytes"])
    for k in ("peak_bytes", "offloaded_bytes", "prefetched_bytes", "n_offload", "n_prefetch", "n_ondemand_fetch"):
        assert st[k] == mine[k], k
    assert abs(st["avg_bytes_layerstep"] - mine["avg_bytes_layerstep"]) <= 1e-9 * mine["avg_bytes_layerstep"]
    info = ms.analyse(net)
    assert st["offloaded_bytes"] == st["prefetched_bytes"] == sum(info["nbytes"][b] for b in chosen)
    return st, tr


FIT_CASES = [(nets.tiny, 8, 1850000, 65536), (nets.tiny, 8, 1400000, None), (nets.alexnet, 128, G, None), (nets.overfeat, 128, 2 * G, None),
             (nets.googlenet, 128, 3 * G, None), (nets.vgg16, 256, 12 * G, None), (nets.vgg16, 256, 12 * G, 0), (nets.vgg16, 256, 12 * G, 1 << 30),
             (nets.vgg16, 256, 14 * G, None), (nets.vgg16, 64, 4 * G, None), (nets.vgg16, 64, 4 * G, 16 << 20), (nets.alexnet, 128, 900 << 20, None),
             (nets.overfeat, 128, 1500 << 20, 32 << 20), (nets.googlenet, 128, 2 * G, None), (nets.googlenet, 128, 1 * G, 8 << 20),
             (nets.fork_join, 4, 0, 4096), (lambda b: nets.vgg(b, extra_per_group=20), 32, 4 * G, None), (nets.vgg16, 256, 0, None),
             (nets.vgg16, 256, 60 * G, None)]


@pytest.mark.parametrize("mk,batch,budget,part", FIT_CASES)
def test_fit_policy_keeps_the_contract(mk, batch, budget, part):
    net = mk(batch)
    probe = binding.Net(net, 0)
    ws = lib_ws(probe, net)
    probe.close()
    if mk is nets.fork_join:
        budget = ms.simulate(net, "conv", 1 << 50, ws=ws)["peak_bytes"]
    n = binding.Net(net, budget)
    if part is not None:
        n.set_window_part(part)
    s = n.try_policy("fit")
    trainable = ms.simulate(net, "all", budget or 1 << 50, "m", ws=ws)["status"] == "ok"
    if s != binding.OK:
        # fit offloads at most what vDNN_all does: where all with the memory-optimal algorithm cannot train, nothing can
        assert s == binding.ERR_OOM_DEVICE and not trainable
        n.close()
        return
    st, tr = _assert_valid_schedule(n, net, budget or 1 << 60)
    assert st["effective_policy"] == "fit"
    assert budget or st["window_fill_pm"] == st["window_fill_bwd_pm"] == 0
    cands = {b for b in ms.analyse(net)["nbytes"] if ms.selected(net, ms.analyse(net), b, "all")}
    assert n.offload_set() <= cands                                   # only what vDNN_all would offload
    # no more bytes than the paper's static policies move, whenever those fit with the same algorithms
    for pol in ("conv", "all"):
        r = ms.simulate(net, pol, budget or 1 << 50, st["conv_algo"], ws=ws)
        if r["status"] == "ok":
            assert st["offloaded_bytes"] <= r["offloaded_bytes"]
    # nothing is offloaded where nothing has to be
    if ms.simulate(net, "none", budget or 1 << 50, "p", ws=ws)["status"] == "ok" and st["conv_algo"] == "p" and st["offloaded_bytes"]:
        probe = binding.Net(net, budget)
        assert probe.try_policy("none") == binding.ERR_OOM_DEVICE and "placement" in probe.last_error()
        probe.close()
    n.close()


def _rest_and_fetches(tr):
    """A library trace without its fetches (alloc + prefetch pairs), entries without their where-label except for the
    computations (a fetch issued early carries the label of where it landed), and {tag: index in that list at which the fetch
    was issued}."""
    got = [t[:4] for t in tr if t[0] != "create"]
    rest, fetch_at = [], {}
    i = 0
    while i < len(got):
        if got[i][1] == "alloc" and i + 1 < len(got) and got[i + 1][1] in ("prefetch", "ondemand"):
            assert got[i + 1][2] == got[i][2] and got[i + 1][3] == got[i][3]
            fetch_at[got[i][2]] = len(rest)
            i += 2
            continue
        rest.append(got[i][1:] if got[i][1] != "compute" else got[i])
        i += 1
    return rest, fetch_at


def test_hand_enumerated_fit_schedule():
    """The fit policy on a net small enough to write its schedule out by hand: three 3x3 convolutions (4 channels, pad 1, no
    ReLU) on a 1x4x8x8 input, FC to 5 outputs, loss.  Blocks: the input B-1 and the conv outputs B0, B1, B2 are 1024 bytes each,
    the FC output B3 and every small block 256; weights 768 per conv and 5120 for the FC layer: persistent 2 * (3 * 768 + 5120) +
    2 * 256 = 15360.  No layer needs workspace (4 channels, reductions too short to split).
    Without offloading the transient blocks peak at 5376 in the FC layer's backward computation (B-1, B0, B1, B2, dB3, dB2).
    Candidates are what vDNN_all would offload: B-1, B0, B1 (B2 feeds the FC layer).

    (a) Budget 15360 + 4352.  Offloading B-1 alone makes the step fit (the paper's schedule for it peaks at 4352, in the FC
    layer's backward computation: B0, B1, B2, dB3, dB2), and it is the smallest candidate with the lowest id.  Windows at 100 %
    of the budget: B-1's release waits until an allocation would pass the budget.  None does in forward propagation (4352 with
    B3); the first is dB3 (256) for the loss layer's backward computation, so B-1 leaves there, in BACKWARD propagation,
    long after its copy was issued.  The paper's schedule fetches B-1 before conv 1's backward computation; it may come earlier,
    from the point where live bytes plus its 1024 stay within the budget: after dB2 is released in B2.

    (b) Budget 15360 + 4096.  No single candidate makes the step fit (the FC layer's backward computation still holds three
    feature maps, dB3 and dB2: 4352), so the largest, lowest id, joins: B-1; then the smallest that makes it fit, lowest id
    first: B0 (peak 4096).  The blocks can be placed within the budget for a forward share of 94 % (15360 + 2816 after rounding
    down to 256 bytes), not more.  B1 (1024) in F1 would make 3072, so the oldest copy, B-1, goes there, and B1 moves into its
    range; the same with B2 and B0 in F2.  Backward: B0 is fetched before conv 2's backward pass, B-1 before conv 1's, or
    earlier while live bytes plus 1024 stay within the budget and the range they return to is free."""
    b = nets._Builder("hand_fit", 1, 4, 8, 8)
    for _ in range(3):
        b.conv(4, 3, pad=1, relu=False)
    b.fc(5, relu=False)
    net = b.done()
    persistent = 2 * (3 * 768 + 5120) + 2 * 256
    n = binding.Net(net, 0)
    n.set_policy("none")
    assert n.stats()["persistent_bytes"] == persistent and n.stats()["peak_bytes"] == persistent + 5376 and n.stats()["workspace_bytes"] == 0
    n.close()

    budget = persistent + 4352
    n = binding.Net(net, budget)
    assert n.try_policy("none") == binding.ERR_OOM_DEVICE
    n.set_policy("fit")
    assert n.offload_set() == {-1}
    st, tr = _assert_valid_schedule(n, net, budget)
    assert (st["window_fill_pm"], st["window_fill_bwd_pm"]) == (1000, 1000) and st["peak_bytes"] == budget
    rest, fetch_at = _rest_and_fetches(tr)
    expect = [
        ("alloc", "B-1", 1024),
        ("alloc", "B0", 1024), ("offload", "B-1", 1024), ("F0", "compute", "conv"),
        ("alloc", "B1", 1024), ("F1", "compute", "conv"),
        ("alloc", "B2", 1024), ("F2", "compute", "conv"),
        ("alloc", "B3", 256), ("F3", "compute", "fc"),
        ("F4", "compute", "softmax_ce"),
        ("free", "B-1", 1024), ("alloc", "dB3", 256), ("B4", "compute", "softmax_ce"), ("free", "B3", 256),
        ("alloc", "dB2", 1024), ("B3", "compute", "fc"), ("free", "dB3", 256), ("free", "B2", 1024),
        ("alloc", "dB1", 1024), ("B2", "compute", "conv"), ("free", "dB2", 1024), ("free", "B1", 1024),
        ("alloc", "dB0", 1024), ("B1", "compute", "conv"), ("free", "dB1", 1024), ("free", "B0", 1024),
        ("B0", "compute", "conv"), ("free", "dB0", 1024), ("free", "B-1", 1024),
    ]
    assert rest == expect
    assert expect.index(("free", "dB2", 1024)) + 1 <= fetch_at["B-1"] <= expect.index(("alloc", "dB0", 1024))
    n.close()

    budget = persistent + 4096
    n = binding.Net(net, budget)
    assert n.try_policy("none") == binding.ERR_OOM_DEVICE
    n.set_policy("fit")
    assert n.offload_set() == {-1, 0}
    st, tr = _assert_valid_schedule(n, net, budget)
    assert (st["window_fill_pm"], st["window_fill_bwd_pm"]) == (940, 1000) and st["peak_bytes"] <= budget
    rest, fetch_at = _rest_and_fetches(tr)
    expect = [
        ("alloc", "B-1", 1024),
        ("alloc", "B0", 1024), ("offload", "B-1", 1024), ("F0", "compute", "conv"),
        ("free", "B-1", 1024), ("alloc", "B1", 1024), ("offload", "B0", 1024), ("F1", "compute", "conv"),
        ("free", "B0", 1024), ("alloc", "B2", 1024), ("F2", "compute", "conv"),
        ("alloc", "B3", 256), ("F3", "compute", "fc"),
        ("F4", "compute", "softmax_ce"),
        ("alloc", "dB3", 256), ("B4", "compute", "softmax_ce"), ("free", "B3", 256),
        ("alloc", "dB2", 1024), ("B3", "compute", "fc"), ("free", "dB3", 256), ("free", "B2", 1024),
        ("alloc", "dB1", 1024), ("B2", "compute", "conv"), ("free", "dB2", 1024), ("free", "B1", 1024),
        ("alloc", "dB0", 1024), ("B1", "compute", "conv"), ("free", "dB1", 1024), ("free", "B0", 1024),
        ("B0", "compute", "conv"), ("free", "dB0", 1024), ("free", "B-1", 1024),
    ]
    assert rest == expect
    addr = {t[2]: t[4] for t in tr if t[0][0] == "F" and t[1] == "alloc"}
    assert addr["B1"] == addr["B-1"] and addr["B2"] == addr["B0"]          # each moved into the range of the copy that had just left
    assert expect.index(("free", "dB3", 256)) + 1 <= fetch_at["B0"] <= expect.index(("alloc", "dB1", 1024))
    assert max(fetch_at["B0"], expect.index(("free", "dB2", 1024)) + 1) <= fetch_at["B-1"] <= expect.index(("alloc", "dB0", 1024))
    n.close()


def test_explicit_offload_sets_and_window_fills():
    import random
    rnd = random.Random(7)
    n_ok = n_moved = 0
    for mk, batch in ((nets.alexnet, 8), (nets.fork_join, 4), (lambda b: nets.googlenet(b, in_hw=64, modules=nets._INCEPTION[:4]), 4),
                      (lambda b: nets.vgg(b, in_hw=32), 8)):
        net = mk(batch)
        info = ms.analyse(net)
        probe = binding.Net(net, 0)
        ws = lib_ws(probe, net)
        probe.close()
        # what vDNN_all would offload, and the inputs of the classification layers (Section 3, opening)
        fc_inputs = [b for b in sorted(info["nbytes"]) if any(net["layers"][r]["type"] == "fc" for r in info["readers"][b])]
        assert fc_inputs
        cands = sorted({b for b in info["nbytes"] if ms.selected(net, info, b, "all")} | set(fc_inputs))
        peak_all = ms.simulate(net, "all", 1 << 50, ws=ws)["peak_bytes"]
        peak_none = ms.simulate(net, "none", 1 << 50, ws=ws)["peak_bytes"]
        for trial in range(12):
            chosen = set(b for b in cands if rnd.random() < (0.3, 0.6, 1.0)[trial % 3])
            base = ms.simulate(net, "none", 1 << 50, offload_set=chosen, ws=ws)
            budget = base["peak_bytes"] + rnd.choice((0, 256, (peak_none - peak_all) // 3, peak_none))
            for fill, fill_bwd in ((0, 0), (1000, 1000), (900, 700), (600, 1000), (0, 950), (1000, 0)):
                part = rnd.choice((0, 4096, 65536, 1 << 20, 128 << 20))
                n = binding.Net(net, budget)
                n.set_window_part(part)
                s = n.try_offload_set(chosen, fill, fill_bwd)
                assert s in (binding.OK, binding.ERR_OOM_DEVICE)
                if s == binding.OK:
                    st, tr = _assert_valid_schedule(n, net, budget, chosen)
                    assert st["effective_policy"] == "custom"
                    assert (st["window_fill_pm"], st["window_fill_bwd_pm"]) == (fill, fill_bwd)
                    if not fill and not fill_bwd:
                        # the paper's schedule for this set: equal to the oracle's, op for op
                        assert [t[:4] for t in tr] == [tuple(t) for t in base["trace"]]
                        assert st["peak_bytes"] == base["peak_bytes"]
                    else:
                        # windows only move releases later and fetches earlier: the same computations and copies, never fewer live bytes
                        assert sorted(t[:4] for t in tr if t[1] == "compute") == sorted(tuple(t) for t in base["trace"] if t[1] == "compute")
                        assert st["peak_bytes"] >= base["peak_bytes"]
                        n_moved += [t[:4] for t in tr] != [tuple(t) for t in base["trace"]]
                    n_ok += 1
                else:
                    assert "placement" in n.last_error() or fill == fill_bwd == 0
                n.close()
    assert n_ok > 200 and n_moved > 100, (n_ok, n_moved)   # the cases do exercise the windows
    # what is not a CONV / POOL / FC input that backward needs is refused
    net = nets.tiny(8)
    n = binding.Net(net, 0)
    fc = [i for i, l in enumerate(net["layers"]) if l["type"] == "fc"][0]
    fc_in = net["layers"][fc]["inputs"][0]
    fc_in = net["layers"][fc_in]["inputs"][0] if net["layers"][fc_in]["type"] == "relu" else fc_in
    assert n.try_offload_set({fc_in}) == binding.OK and n.offload_set() == {fc_in}
    assert n.try_offload_set({fc}) == binding.ERR_INVALID_ARG      # the logits: only the loss layer reads them
    assert n.try_offload_set({len(net["layers"])}) == binding.ERR_INVALID_ARG
    assert n.try_offload_set({-2}) == binding.ERR_INVALID_ARG
    assert n.try_offload_set(set(), 1001) == binding.ERR_INVALID_ARG
    assert n.try_offload_set(set(), 500, -1) == binding.ERR_INVALID_ARG
    assert n.try_policy("fit") == binding.OK and n.offload_set() == set()
    n.close()


@pytest.mark.parametrize("seed", list(range(16)) + ["w104", "w108", "w110", "w113", "w122", "w124", "w133", "w142"])
def test_random_graphs_all_policies(seed):
    """Fuzz: irregular graphs (forks of uneven depth, convs without ReLU, strided layers, several readers of one
    feature map).  Every static policy's plan equals the memory-schedule oracle's, dyn decides as the oracle does, fit
    keeps the contract, at budgets drawn between the peaks of all and none."""
    import random
    if isinstance(seed, str):   # "w<seed>": 128 ... 384 channels on 8 x 8 images, plans with Winograd workspaces
        seed = int(seed[1:])
        net = nets.random_net(seed, batch=2, in_hw=8, wide=True)
    else:
        net = nets.random_net(seed)
    rnd = random.Random(1000 + seed)
    peaks = {}
    ws = None
    for policy in ("none", "conv", "all"):
        n = binding.Net(net, 0)
        n.set_policy(policy)
        ws = lib_ws(n, net)
        ref = ms.simulate(net, policy, 1 << 50, ws=ws)
        st, tr = _assert_valid_schedule(n, net, 1 << 60)
        assert [t[:4] for t in tr] == [tuple(t) for t in ref["trace"]]
        peaks[policy] = ref["peak_bytes"]
        n.close()
    lo, hi = peaks["all"], peaks["none"]
    for budget in {hi, lo, lo + (hi - lo) // 2, rnd.randrange(lo, hi + 1) // 256 * 256, hi - 256}:
        pol, algo, ref = ms.dynamic(net, budget, ws)
        n = binding.Net(net, budget)
        s = n.try_policy("dyn")
        if pol is None:
            assert s == binding.ERR_OOM_DEVICE
        elif s == binding.OK:
            st = n.stats()
            if (st["effective_policy"], st["conv_algo"]) != (pol, algo):
                # the oracle counts bytes; right at a live-byte peak the library may find no placement of the blocks and
                # move on to the next pass of the sequence: the pass the oracle adopted must fail for that reason only
                probe = binding.Net(net, budget)
                probe.set_conv_algo(algo)
                assert probe.try_policy(pol) == binding.ERR_OOM_DEVICE and "placement" in probe.last_error()
                probe.close()
                ref = ms.simulate(net, st["effective_policy"], budget, st["conv_algo"], ws=ws)
                assert ref["status"] == "ok"
            st, tr = _assert_valid_schedule(n, net, budget)
            assert [t[:4] for t in tr] == [tuple(t) for t in ref["trace"]]
        else:
            assert "placement" in n.last_error()   # the byte count fits, the address range does not
        part = rnd.choice((0, 1024, 16384, 128 << 20))
        n.set_window_part(part)
        s = n.try_policy("fit")
        if s == binding.OK:
            _assert_valid_schedule(n, net, budget)
        else:
            assert ms.simulate(net, "all", budget, "m", ws=ws)["status"] == "oom" or "placement" in n.last_error()
        n.close()


# ---------------------------------------------------------------------------------------------------
# kernels and their workspaces (host side of the library: no GPU needed)
# ---------------------------------------------------------------------------------------------------
def test_every_plan_of_a_net_runs_the_same_kernels():
    """What makes "offload on = offload off, bit for bit" hold across policies and budgets: under the performance-optimal
    mode a layer's kernels do not depend on the plan."""
    for mk, batch, budget in ((nets.vgg16, 256, 12 * G), (nets.alexnet, 128, G), (nets.overfeat, 128, 2 * G), (nets.googlenet, 128, 3 * G),
                              (nets.googlenet, 128, 2 * G)):
        net = mk(batch)
        convs = [i for i, l in enumerate(net["layers"]) if l["type"] == "conv"]
        n = binding.Net(net, 0)
        n.set_policy("none")
        want = {i: n.layer_kernels(i) for i in convs}
        n.close()
        assert any(kk.startswith("winograd") for k in want.values() for kk in k) or mk is nets.googlenet
        n = binding.Net(net, budget)
        for pol in ("none", "conv", "all", "dyn", "fit"):
            if n.try_policy(pol) != binding.OK:
                continue
            if n.stats()["conv_algo"] == "p":
                assert {i: n.layer_kernels(i) for i in convs} == want, pol
            else:
                assert n.stats()["n_downgraded_convs"] > 0 or n.stats()["conv_algo"] == "m"
        n.close()


def test_workspace_sizes_by_hand():
    """The workspace rules of the kernels evaluated by hand for VGG-16 (256) layers.  Winograd F(2x2, 3x3): transformed filter
    16*C*K floats, then 16*(C + K) floats per 2x2 output tile for a chunk of images: as many as keep the whole workspace
    within 384 MiB, evened out over the chunks that takes; backward-filter: the 16 products once plus once per reduction
    split, then the same chunk.  F(4x4, 3x3): the same with 36 products per 4x4 output tile.  Packed: one copy of W (rounded
    up to 256 bytes)."""
    MiB = 1 << 20
    CHUNK = 384 * MiB
    q = binding.op_conv_workspace
    # c4_2: 512 -> 512 at 28 x 28: 196 tiles per image, 16 * 1024 * 196 * 4 = 12 845 056 bytes per image; beside the 16 MiB of
    # the transformed filter 30 images fit: 9 chunks for 256 images, 29 images each (the last one 24)
    x, w = (256, 512, 28, 28), (512, 512, 3, 3)
    U = 16 * 512 * 512 * 4
    assert q("fwd", "winograd", x, w, 1, 1) == q("bwd_data", "winograd", x, w, 1, 1) == U + 29 * 12845056
    assert U + 30 * 12845056 <= CHUNK < U + 31 * 12845056 and 8 * 30 < 256 <= 9 * 29
    assert q("fwd", "packed", x, w, 1, 1) == 512 * 512 * 9 * 4
    assert q("fwd", "gather", x, w, 1, 1) == q("bwd_filter", "gather", x, w, 1, 1) == 0
    # backward-filter of c4_2: 4 x 4 tiles of 128 x 128 per product, 16 products: 256 workgroups -> 4 splits; beside the
    # products and their partial sums (5 U) 24 images fit: 11 chunks of 24
    assert q("bwd_filter", "winograd", x, w, 1, 1) == U * (1 + 4) + 24 * 12845056
    assert 5 * U + 24 * 12845056 <= CHUNK < 5 * U + 25 * 12845056
    # c5: 14 x 14, 49 tiles: 3 211 264 bytes per image, 120 images fit: three chunks of 86; a batch smaller than the chunk: all of it
    assert q("fwd", "winograd", (256, 512, 14, 14), w, 1, 1) == U + 86 * 3211264
    assert q("fwd", "winograd", (8, 512, 14, 14), w, 1, 1) == U + 8 * 3211264
    # 13 x 13 (odd sides): 7 x 7 tiles as well
    assert q("fwd", "winograd", (8, 384, 13, 13), (256, 384, 3, 3), 1, 1) == 16 * 384 * 256 * 4 + 8 * 16 * 640 * 49 * 4
    # c3_2 backward-filter: 256 -> 256 at 56 x 56: 784 tiles, 25 690 112 bytes per image; 2 x 2 tiles x 16 = 64 workgroups -> 16
    # splits, 17 x 4 MiB; 12 images fit beside them: 22 chunks of 12
    assert q("bwd_filter", "winograd", (256, 256, 56, 56), (256, 256, 3, 3), 1, 1) == 16 * 256 * 256 * 4 * (1 + 16) + 12 * 25690112
    # F(4x4, 3x3) on c4_2: 49 tiles per image, 36 * 1024 * 49 * 4 = 7 225 344 bytes per image, 50 fit beside the 36 MiB filter:
    # 6 chunks of 43; backward-filter: 4 x 4 tiles x 36 products = 576 workgroups: up to 3 splits (2048 workgroups), 34 images fit
    # beside 4 x 36 MiB: 8 chunks of 32
    U4 = 36 * 512 * 512 * 4
    assert q("fwd", "winograd4", x, w, 1, 1) == q("bwd_data", "winograd4", x, w, 1, 1) == U4 + 43 * 7225344
    assert U4 + 50 * 7225344 <= CHUNK < U4 + 51 * 7225344 and 5 * 50 < 256 <= 6 * 43
    assert q("bwd_filter", "winograd4", x, w, 1, 1) == U4 * (1 + 3) + 32 * 7225344
    assert q("fwd", "winograd4_small", x, w, 1, 1) == U4 + 22 * 7225344
    # c5: 14 x 14 is covered by 4 x 4 tiles of 4 x 4: 2 359 296 bytes per image, two chunks of 128
    assert q("fwd", "winograd4", (256, 512, 14, 14), w, 1, 1) == U4 + 128 * 36 * 1024 * 16 * 4
    # c3_2 backward-filter: 196 tiles, 14 450 688 bytes per image; 2 x 2 x 36 = 144 workgroups -> up to 14 splits, 15 x 9 MiB; 18
    # images fit: 15 chunks of 18, whose 18 * 196 tile positions make 7 splits of at least 512
    assert q("bwd_filter", "winograd4", (256, 256, 56, 56), (256, 256, 3, 3), 1, 1) == 36 * 256 * 256 * 4 * (1 + 7) + 18 * 14450688
    # F(4x4) moves 2.25 instead of 4 times the tensor through the workspace and pays from 128 channels on (c2_2, c3_1 forward)
    assert q("fwd", "winograd4", (256, 128, 112, 112), (128, 128, 3, 3), 1, 1) is not None and q("fwd", "winograd", (256, 128, 112, 112), (128, 128, 3, 3), 1, 1) is None
    assert q("bwd_filter", "winograd4", (256, 128, 112, 112), (128, 128, 3, 3), 1, 1) is not None
    assert q("fwd", "winograd4", (256, 64, 112, 112), (128, 64, 3, 3), 1, 1) is None and q("bwd_data", "winograd4", (256, 64, 112, 112), (128, 64, 3, 3), 1, 1) is None
    # every Winograd workspace stays within the chunk size unless one image alone passes it
    for kernel in ("winograd", "winograd4"):
        for xs, ws_ in ((x, w), ((256, 256, 56, 56), (256, 256, 3, 3)), ((128, 1024, 12, 12), (1024, 1024, 3, 3)), ((256, 512, 14, 14), w)):
            for pass_ in ("fwd", "bwd_data", "bwd_filter"):
                assert q(pass_, kernel, xs, ws_, 1, 1) <= CHUNK, (kernel, xs, pass_)
    # not wide enough, not 3x3, strided, unpadded, channels not a multiple of 16: no Winograd
    for xs, ws_, st, pd in (((256, 128, 28, 28), (512, 128, 3, 3), 1, 1), ((256, 512, 28, 28), (64, 512, 3, 3), 1, 1),
                            ((256, 512, 28, 28), (512, 512, 5, 5), 1, 2), ((256, 512, 28, 28), (512, 512, 3, 3), 2, 1),
                            ((256, 512, 28, 28), (512, 512, 3, 3), 1, 0), ((256, 520, 28, 28), (512, 520, 3, 3), 1, 1)):
        assert q("fwd", "winograd", xs, ws_, st, pd) is None, (xs, ws_, st, pd)
        assert (q("fwd", "winograd4", xs, ws_, st, pd) is None) == (xs[1] != 128), (xs, ws_, st, pd)
    assert q("bwd_filter", "winograd", (256, 192, 56, 56), (256, 192, 3, 3), 1, 1) is None      # input channels not a multiple of 128
    assert q("bwd_filter", "winograd4", (256, 192, 56, 56), (256, 192, 3, 3), 1, 1) is None
    assert q("bwd_filter", "winograd", (256, 256, 56, 56), (128, 256, 3, 3), 1, 1) is None      # fewer than 256 output channels
    # the packed kernels need reduction channels in multiples of 16 (forward: C, backward-data: K; backward-filter: C in 32s
    # or a reduction worth splitting); the first layer of a net (C = 3) has only the gather kernel in forward
    assert q("fwd", "packed", (256, 3, 224, 224), (64, 3, 3, 3), 1, 1) is None
    assert q("bwd_data", "packed", (256, 64, 56, 56), (24, 64, 3, 3), 1, 1) is None
    assert q("bwd_data", "packed", (256, 64, 56, 56), (32, 64, 3, 3), 2, 1) is None             # strided backward-data
    # c1_2 backward-filter: 64 channels, three-tap column tiles: 1 row tile x 3 column tiles -> 341 splits of |W|
    assert q("bwd_filter", "packed", (256, 64, 224, 224), (64, 64, 3, 3), 1, 1) == (1024 // 3) * 64 * 64 * 9 * 4
    # the fastest-kernel queries agree with the per-kernel ones
    assert binding.op_conv_fwd_workspace(x, w, 1, 1) == q("fwd", "winograd4", x, w, 1, 1)
    assert binding.op_conv_fwd_workspace((256, 64, 56, 56), (256, 64, 3, 3), 1, 1) == q("fwd", "packed", (256, 64, 56, 56), (256, 64, 3, 3), 1, 1)


def test_a_plan_names_its_kernels():
    """The planner's choice reaches the kernels by name, not by workspace size.  For C = 1024, K = 256, 3x3, 32 images of
    8x8 the packed kernels' backward workspace (76.5 MB) is larger than the Winograd backward-filter and backward-data
    workspaces (75.5 MB, 58.7 MB): a launcher that inferred the algorithm from the bytes it was given would run Winograd
    although the plan had decided against it."""
    x, w = (32, 1024, 8, 8), (256, 1024, 3, 3)
    q = binding.op_conv_workspace
    packed = max(q("bwd_filter", "packed", x, w, 1, 1), q("bwd_data", "packed", x, w, 1, 1))
    assert packed >= q("bwd_filter", "winograd", x, w, 1, 1) and packed >= q("bwd_data", "winograd", x, w, 1, 1)
    b = nets._Builder("wide", 32, 1024, 8, 8)
    b.conv(1024, 1)
    b.conv(256, 3, pad=1)
    b.fc(10, relu=False)
    net = b.done()
    conv = 2
    assert net["layers"][conv]["type"] == "conv" and net["layers"][conv]["k"] == 3
    n = binding.Net(net, 0)
    n.set_policy("none")
    assert n.layer_kernels(conv) == ("winograd4", "winograd4", "winograd4") and n.stats()["n_winograd_convs"] == 1
    n.set_winograd(False)
    n.set_policy("none")
    assert n.layer_kernels(conv) == ("packed", "packed", "packed") and n.stats()["n_winograd_convs"] == 0
    assert n.workspace_options(conv, True)[0] == packed
    n.set_conv_algo("m")
    n.set_policy("none")
    assert n.layer_kernels(conv) == ("gather", "gather", "gather")
    n.close()


def test_a_plan_keeps_naming_its_kernels_when_the_lists_change():
    """vdnn_layer_kernels and the step-time estimate describe the CURRENT plan, also after something rebuilt the layers' lists
    (a profile put in, the Winograd kernels switched off) and before the next vdnn_set_policy."""
    net = nets.vgg(8, in_hw=32)
    n = binding.Net(net, 0)
    n.set_policy("none")
    convs = [i for i, l in enumerate(net["layers"]) if l["type"] == "conv"]
    before = {i: n.layer_kernels(i) for i in convs}
    assert any(k[0].startswith("winograd") for k in before.values())
    _uniform_profile(n, net, winograd=9.0, packed=1.0, gather=0.5)      # every list now starts with the gather kernel
    assert {i: n.layer_kernels(i) for i in convs} == before
    est = n.estimate_step_ms()
    n.set_winograd(False)                                                 # lists get shorter
    assert {i: n.layer_kernels(i) for i in convs} == before and n.estimate_step_ms() == est
    n.set_policy("none")
    assert all(k == ("gather", "gather", "gather") for k in (n.layer_kernels(i) for i in convs))
    assert n.estimate_step_ms() < est
    n.close()


def test_winograd_can_be_switched_off_and_its_workspace_must_fit():
    """Wide 3x3 layers of VGG-16 (256) run the Winograd kernels in every plan (10 layers: c2_2 ... c5_3); a
    budget that has no room for a layer's workspace fails the performance-optimal plan rather than changing the kernel
    behind the caller's back, and the greedy mode then moves that layer down its list."""
    net = nets.vgg16(256)
    n = binding.Net(net, 0)
    n.set_policy("none")
    ws = lib_ws(n, net)
    none_peak = n.stats()["peak_bytes"]
    assert n.stats()["n_winograd_convs"] == 10
    none_kernels = {i: n.layer_kernels(i) for i, l in enumerate(net["layers"]) if l["type"] == "conv"}
    n.set_winograd(2)        # only the F(2x2, 3x3) forms: c3_1 (backward only) ... c5_3
    n.set_policy("none")
    assert n.stats()["n_winograd_convs"] == 9
    assert all(not kk.startswith("winograd4") for i in none_kernels for kk in n.layer_kernels(i))
    assert n.layer_kernels(12) == ("winograd", "winograd", "winograd") and n.layer_kernels(7) == ("packed", "packed", "packed")
    assert binding.lib.vdnn_set_winograd(n.h, 3) == binding.ERR_INVALID_ARG
    n.set_winograd(False)
    n.set_policy("none")
    assert n.stats()["n_winograd_convs"] == 0 and n.stats()["peak_bytes"] < none_peak
    n.close()
    tight = none_peak - (192 << 20)
    n = binding.Net(net, tight)
    assert n.try_policy("none") == binding.ERR_OOM_DEVICE
    n.set_conv_algo("greedy")
    n.set_policy("none")
    st = n.stats()
    ref = ms.simulate(net, "none", tight, "greedy", ws=ws)
    assert 0 < st["n_downgraded_convs"] == ref["n_downgraded_convs"] and st["n_memopt_convs"] == ref["n_memopt_convs"] == 0
    assert st["peak_bytes"] == ref["peak_bytes"] <= tight
    convs = [i for i, l in enumerate(net["layers"]) if l["type"] == "conv"]
    moved = [n.layer_kernels(i) for i in convs if n.layer_kernels(i) != none_kernels[i]]
    # the next entry of a wide layer's list is the same algorithm on chunks of half the size
    assert len(moved) == st["n_downgraded_convs"] and all(any(kk not in ("winograd4", "gather") for kk in k) for k in moved)
    assert [t[:4] for t in n.trace()] == [tuple(t) for t in ref["trace"]]
    n.close()
    for chunk in (64 << 20, 0):
        binding.op_set_winograd_chunk_bytes(chunk)
        try:
            n = binding.Net(net, 0)
            n.set_policy("none")
            assert n.stats()["n_winograd_convs"] == 10
            assert (n.stats()["workspace_bytes"] < 200 << 20) == (chunk != 0)
            n.close()
        finally:
            binding.op_set_winograd_chunk_bytes(0)


# ---------------------------------------------------------------------------------------------------
# profile-driven choices (Section 3.3: vDNN_dyn decides from profiled layer times); the numbers are put in by hand here
# ---------------------------------------------------------------------------------------------------
def _hand_fit_net():
    b = nets._Builder("hand_fit", 1, 4, 8, 8)
    for _ in range(3):
        b.conv(4, 3, pad=1, relu=False)
    b.fc(5, relu=False)
    return b.done()


def test_estimated_step_time_by_hand():
    """Three convolutions, FC, loss (the net of test_hand_enumerated_fit_schedule) under vDNN_all, layer times and link rates
    given by hand: conv forward 1 ms, backward-filter and backward-data 1 ms each, FC 0.5 ms each way, loss 0.1 ms each way;
    the three 1024-byte feature maps that vDNN_all offloads take 1.024 ms to the host (1000 bytes per ms) and 0.512 ms back.
    Forward: each offload starts with its layer and the layer ends when both have (Section 3.2): three times 1.024 ms, then
    0.5 + 0.1.  Backward: the prefetch of conv 2's input is issued with the loss layer (0.1 ms of computation, 0.512 ms of
    copy: the layer ends at +0.512); FC 0.5; conv 2's backward pass (2 ms) hides the prefetch of conv 1's input, conv 1's (2 ms)
    that of the network input; conv 0 has no backward-data pass: 1 ms."""
    net = _hand_fit_net()
    n = binding.Net(net, 0)
    assert n.try_policy("none") == binding.OK
    with pytest.raises(binding.VdnnError):
        n.estimate_step_ms()                       # no profile yet
    for i in (0, 1, 2):
        for pass_ in ("fwd", "bwd_data", "bwd_filter"):
            n.set_layer_profile(i, pass_, "gather", 1.0)
    n.set_layer_profile(3, 0, 0, 0.5)
    n.set_layer_profile(3, 1, 0, 0.5)
    n.set_layer_profile(4, 0, 0, 0.1)
    n.set_layer_profile(4, 1, 0, 0.1)
    n.set_link_rate(1e-3, 2e-3)                    # GB/s: 1000 and 2000 bytes per millisecond
    assert n.link_rate() == (1e-3, 2e-3)
    assert n.layer_profile(0) == {("fwd", "gather"): 1.0, ("bwd_data", "gather"): 1.0, ("bwd_filter", "gather"): 1.0}
    assert n.layer_profile(3) == {"fwd": 0.5, "bwd": 0.5}
    n.set_policy("none")
    assert abs(n.estimate_step_ms() - (3 * 1.0 + 0.5 + 0.1 + 0.1 + 0.5 + 2.0 + 2.0 + 1.0)) < 1e-6
    n.set_policy("all")
    assert n.offload_set() == {-1, 0, 1}
    forward = 3 * 1.024 + 0.5 + 0.1
    backward = 0.512 + 0.5 + 2.0 + 2.0 + 1.0
    assert abs(n.estimate_step_ms() - (forward + backward)) < 1e-6
    # a link ten times slower: every layer that carries a transfer lasts as long as the transfer
    n.set_link_rate(1e-4, 2e-4)
    assert abs(n.estimate_step_ms() - (3 * 10.24 + 0.6 + 5.12 + 0.5 + 5.12 + 5.12 + 1.0)) < 1e-6
    n.close()


def _uniform_profile(n, net, winograd=1.0, packed=1.3, gather=4.0, other=0.1, link=50.0):
    shapes, _ = nets.shapes(net)
    for i, l in enumerate(net["layers"]):
        if l["type"] == "conv":
            src = l["inputs"][0]
            xs = (net["batch"], net["in_c"], net["in_h"], net["in_w"]) if src < 0 else shapes[src]
            for pass_ in ("fwd", "bwd_data", "bwd_filter"):
                for kernel, ms in (("winograd4", 0.8 * winograd), ("winograd4_small", 0.85 * winograd), ("winograd", winograd),
                                   ("winograd_small", 1.05 * winograd), ("packed", packed), ("gather", gather)):
                    if binding.op_conv_workspace(pass_, kernel, xs, (l["out"], xs[1], l["k"], l["k"]), l["stride"], l["pad"]) is not None:
                        n.set_layer_profile(i, pass_, kernel, ms)
        else:
            n.set_layer_profile(i, 0, 0, other)
            n.set_layer_profile(i, 1, 0, other)
    n.set_link_rate(link, link)


def test_profile_orders_the_kernel_lists():
    """Before a profile a wide 3x3 layer prefers Winograd, then the packed kernel, then the gather kernel.  Measured times
    reorder the list; a kernel that is slower than one needing less workspace drops out of it (the greedy mode would never
    pick it)."""
    b = nets._Builder("wide", 8, 256, 14, 14)
    b.conv(256, 1)
    b.conv(256, 3, pad=1)
    b.fc(10, relu=False)
    net = b.done()
    conv = 2
    n = binding.Net(net, 0)
    n.set_policy("none")
    assert n.layer_kernels(conv) == ("winograd4", "winograd4", "winograd4")
    before = n.workspace_options(conv, False)
    ws_of = lambda k: binding.op_conv_workspace("fwd", k, (8, 256, 14, 14), (256, 256, 3, 3), 1, 1)
    # expected order F(4x4), F(4x4) on half chunks, F(2x2), F(2x2) on half chunks, packed, gather; an entry that needs no less
    # workspace than one expected faster is not on the list (F(2x2) on full chunks, the packed kernel)
    assert before == [ws_of("winograd4"), ws_of("winograd4_small"), ws_of("winograd_small"), 0]
    assert ws_of("winograd") > ws_of("winograd4_small") > ws_of("winograd_small") and ws_of("packed") > ws_of("winograd_small")
    _uniform_profile(n, net, winograd=2.0, packed=1.0, gather=5.0)      # the packed kernel measured faster than Winograd
    n.set_policy("none")
    assert n.layer_kernels(conv) == ("packed", "packed", "packed")
    # the Winograd kernels on full chunks: slower and larger, gone; on half chunks they need less workspace and stay
    assert n.workspace_options(conv, False) == [ws_of("packed"), ws_of("winograd4_small"), ws_of("winograd_small"), 0]
    _uniform_profile(n, net, winograd=1.0, packed=1.0, gather=0.5)      # the gather kernel fastest: the only entry left
    n.set_policy("none")
    assert n.layer_kernels(conv) == ("gather", "gather", "gather") and n.workspace_options(conv, False) == [0]
    # naming the kernels overrides the list
    n.set_layer_kernels(conv, ("winograd", "packed", "gather"))
    n.set_policy("none")
    assert n.layer_kernels(conv) == ("winograd", "packed", "gather")
    assert n.workspace_options(conv, False) == [ws_of("winograd")]
    assert binding.lib.vdnn_set_layer_kernels(n.h, 0, (C.c_int32 * 3)(2, 0, 0)) == binding.ERR_INVALID_ARG   # 1x1: no Winograd
    assert binding.lib.vdnn_set_layer_kernels(n.h, 3, (C.c_int32 * 3)(0, 0, 0)) == binding.ERR_INVALID_ARG   # not a CONV layer
    n.set_layer_kernels(conv, None)
    n.set_policy("none")
    assert n.layer_kernels(conv) == ("gather", "gather", "gather")
    n.close()


def test_dyn_with_a_profile_chooses_by_estimated_time():
    """AlexNet-shaped, batch 128, 1 GiB.  Without a profile vDNN_dyn follows the paper's order and adopts vDNN_all with the
    performance-optimal algorithms (the first configuration of the sequence that fits).  With measured times it compares the
    configurations that fit and takes the fastest: on a link this slow relative to the layers, no offloading at all with the
    greedy downgrade of the layers whose Winograd workspace does not fit."""
    net = nets.alexnet(128)
    n = binding.Net(net, G)
    n.set_policy("dyn")
    st = n.stats()
    assert (st["effective_policy"], st["conv_algo"]) == ("all", "p")
    _uniform_profile(n, net, link=2.0)
    n.set_policy("dyn")
    st = n.stats()
    assert (st["effective_policy"], st["conv_algo"]) == ("none", "greedy") and st["offloaded_bytes"] == 0 and st["n_downgraded_convs"] > 0
    fast = n.estimate_step_ms()
    for pol, algo in (("all", "p"), ("conv", "greedy"), ("all", "greedy")):
        n.set_conv_algo(algo)
        if n.try_policy(pol) == binding.OK:
            assert n.estimate_step_ms() >= fast
    # with an (imaginary) link so fast that transfers are free, what runs every layer on its fastest kernel wins
    _uniform_profile(n, net, link=1e6)
    n.set_policy("dyn")
    st = n.stats()
    assert (st["effective_policy"], st["conv_algo"]) == ("all", "p")
    n.close()


def test_fit_with_a_profile_considers_the_greedy_mode():
    """AlexNet-shaped under 1 GiB has no room for the fastest kernels' workspaces without offloading.  On a slow link giving
    three layers a slower kernel beats moving feature maps: fit finds that plan (as dyn does) although a step that fills the
    pool to the brim takes more placement effort than a search candidate gets."""
    net = nets.alexnet(128)
    n = binding.Net(net, G)
    _uniform_profile(n, net, link=5.0, winograd=0.5, packed=0.9, gather=3.0, other=0.05)
    n.set_policy("dyn")
    assert (n.stats()["effective_policy"], n.stats()["conv_algo"]) == ("none", "greedy")
    dyn_ms = n.estimate_step_ms()
    n.set_policy("fit")
    assert n.stats()["conv_algo"] == "greedy" and n.estimate_step_ms() <= dyn_ms + 1e-9
    _assert_valid_schedule(n, net, G)
    n.close()


def test_fit_with_a_profile_never_estimates_worse():
    """The time-driven search of the offload set starts from the byte-driven choice and only takes moves that shorten the
    estimated step: the result is a valid schedule whose estimate is no worse."""
    net = nets.vgg16(64)
    budget = 4 * G
    n = binding.Net(net, budget)
    n.set_policy("fit")
    by_bytes = n.offload_set()
    assert by_bytes
    _uniform_profile(n, net, link=50.0)
    n.set_offload_set(by_bytes, n.stats()["window_fill_pm"], 1000)
    start = n.estimate_step_ms()
    n.set_policy("fit")
    assert n.estimate_step_ms() <= start + 1e-9
    _assert_valid_schedule(n, net, budget)
    n.close()
