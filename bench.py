#!/usr/bin/env python3
"""Benchmark: one training step (forward + backward) of VGG-16, batch 256, fp32, on one MI355X,
with the vDNN memory manager under a 12 GiB device budget.

  python bench.py [--gpus 1] [--steps K] [--warmup W]

Prints ONE JSON line.  `value` is images/s with vDNN_dyn, the paper's proposed policy, under 12 GiB (inputs resident
in HBM; on this machine dyn adopts conv);
the `policies` object gives the same measurement for none (unlimited budget), conv, all, dyn and for
fit (beyond the paper: per-feature-map offload set with budget-aware transfer windows), with peak pool
bytes and achieved host-link GB/s.  dyn runs after conv and all: the host link, which it runs at the pace of, has
on some machines delivered about half its rate during the first seconds of a process.  `roofline` times the dominant kernel (the
implicit-GEMM convolution) with HIP events on its own stream; `cpu_baseline` times the CPU oracle
on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GIB = 1 << 30
FP32_MFMA_PEAK_TFLOPS = 157.3
# HBM-side bytes per launch of the roofline kernel, from the rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# runs summarised in profiles/conv_fwd_vgg16_c2_1_b256.txt, each scaled by what the same counter reads
# for a plain 1 GiB copy kernel (FETCH_SIZE x 2.000, WRITE_SIZE x 1.000).  Algorithmic bytes: 2.467e9.
ROOFLINE_LAYER = "c2_1"
ROOFLINE_TRAFFIC_BYTES = 2.500e9
LINK_PEAK_GBPS = 64.0  # PCIe Gen5 x16, per direction
WINOGRAD = 1            # vdnn_set_winograd level: --no-winograd = 0 (direct kernels only), --winograd-level 2 = only F(2x2,3x3)
PROFILE = True          # --no-profile: dyn and fit decide without the profiling passes (the paper's fixed order; bytes)
PROFILE_DATA = None     # what run_profile measured; loaded into every net before its policy is set
HBM_PEAK_TBPS = 8.0
KERNEL_LETTER = {"gather": "g", "packed": "p", "winograd": "w", "winograd_small": "s", "winograd4": "W", "winograd4_small": "S"}


def conv_layers_vgg16(batch):
    """(name, N, C, H, W, K) of the 13 convolutions, 3x3 stride 1 pad 1."""
    cfg = [("c1_1", 3, 224, 64), ("c1_2", 64, 224, 64), ("c2_1", 64, 112, 128), ("c2_2", 128, 112, 128),
           ("c3_1", 128, 56, 256), ("c3_2", 256, 56, 256), ("c3_3", 256, 56, 256), ("c4_1", 256, 28, 512),
           ("c4_2", 512, 28, 512), ("c4_3", 512, 28, 512), ("c5_1", 512, 14, 512), ("c5_2", 512, 14, 512),
           ("c5_3", 512, 14, 512)]
    return [(n, batch, c, h, h, k) for n, c, h, k in cfg]


def time_kernel(fn, stream, warmup=2, iters=8):
    """Average duration (ms) of fn() launches, from HIP events recorded on the launch stream."""
    import torch
    with torch.cuda.stream(stream):
        for _ in range(warmup):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(iters):
            fn()
        e1.record(stream)
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


_STREAMS = None


def streams():
    """One (compute, memory) stream pair for the whole process."""
    global _STREAMS
    if _STREAMS is None:
        import torch
        _STREAMS = (torch.cuda.Stream(), torch.cuda.Stream())
    return _STREAMS


def conv_kernel_table(B, batch, which=("fwd", "bwd_data", "bwd_filter"), layers=None, iters=5, ramp_ms=0, kernel="auto"):
    """kernel: "auto" = the fastest kernel for each shape and pass, else that kernel (forward and backward-data).
    ramp_ms: before timing, keep the GPU busy for about that long with a kernel of another name (the
    backward-filter pass), so that the clocks have settled and a profiler's average over ALL launches of the
    timed kernel agrees with the average over the timed ones."""
    import torch
    stream = streams()[0]
    rows = []
    for name, n, c, h, w, k in conv_layers_vgg16(batch):
        if layers and name not in layers:
            continue
        x = torch.randn((n, c, h, w), device="cuda")
        wt = torch.randn((k, c, 3, 3), device="cuda") * 0.05
        y = torch.empty((n, k, h, w), device="cuda")
        flop = 2.0 * n * h * w * k * c * 9
        row = dict(layer=name, gflop=flop / 1e9)
        torch.cuda.synchronize()
        # workspace of the faster algorithm (packed W + partial sums of split tiles; ignored when it does not apply)
        kern = {p: kernel if kernel == "auto" or B.op_conv_workspace(p, kernel, x.shape, wt.shape, 1, 1) is not None else "gather"
                for p in ("fwd", "bwd_data", "bwd_filter")}   # a kernel that does not apply to the shape (C = 3): the gather kernel
        if kernel == "auto":
            nws = max(B.op_conv_fwd_workspace(x.shape, wt.shape, 1, 1), B.op_conv_bwd_data_workspace(x.shape, wt.shape, 1, 1), 4)
        else:
            nws = max([B.op_conv_workspace(p, kern[p], x.shape, wt.shape, 1, 1) or 0 for p in ("fwd", "bwd_data") if p in which and (p == "fwd" or c > 3)] + [4])
        wsp = torch.empty(nws // 4, device="cuda")
        if ramp_ms:
            nb = max(B.op_conv_bwd_filter_workspace(x.shape, wt.shape, 1, 1), B.op_conv_workspace("bwd_filter", "packed", x.shape, wt.shape, 1, 1) or 0)
            ws = torch.empty(max(nb, 4) // 4, device="cuda")
            dw = torch.empty_like(wt)
            t0 = time.perf_counter()
            while (time.perf_counter() - t0) * 1e3 < ramp_ms:
                B.op_conv_bwd_filter(x, y, dw, ws, 1, 1, stream, kernel=kern["bwd_filter"])
                stream.synchronize()
            del ws, dw
        if "fwd" in which:
            ms = time_kernel(lambda: B.op_conv_fwd(x, wt, y, 1, 1, False, stream, wsp, kern["fwd"]), stream, iters=iters)
            row["fwd_ms"], row["fwd_tflops"] = ms, flop / ms / 1e9
        if "bwd_data" in which and c > 3:
            dx = torch.empty_like(x)
            ms = time_kernel(lambda: B.op_conv_bwd_data(y, wt, dx, 1, 1, stream, wsp, kernel=kern["bwd_data"]), stream, iters=iters)
            row["bwd_data_ms"], row["bwd_data_tflops"] = ms, flop / ms / 1e9
            del dx
        if "bwd_filter" in which:
            nb = max(B.op_conv_bwd_filter_workspace(x.shape, wt.shape, 1, 1), B.op_conv_workspace("bwd_filter", "packed", x.shape, wt.shape, 1, 1) or 0)
            ws = torch.empty(max(nb, 4) // 4, device="cuda")
            dw = torch.empty_like(wt)
            ms = time_kernel(lambda: B.op_conv_bwd_filter(x, y, dw, ws, 1, 1, stream, kernel=kern["bwd_filter"]), stream, iters=iters)
            row["bwd_filter_ms"], row["bwd_filter_tflops"] = ms, flop / ms / 1e9
            del ws, dw
        rows.append(row)
        del x, wt, y
    return rows


def roofline(B, batch):
    """Dominant kernel: the 128x128 implicit-GEMM convolution tile kernel (direct convolutions and the grouped GEMMs
    of the Winograd layers), timed on the largest layer that runs it as a direct convolution in the step
    (c2_1 forward: 256 x 64 x 112 x 112 -> 128 channels, 473.5 GFLOP per launch)."""
    row = conv_kernel_table(B, batch, which=("fwd",), layers=(ROOFLINE_LAYER,), iters=20, ramp_ms=300, kernel="packed")[0]
    ach = row["fwd_tflops"]
    return dict(bound="mfma", kernel="conv_fast_kernel<128,128,2,2> (implicit-GEMM conv forward), VGG-16 %s b%d" % (ROOFLINE_LAYER, batch), achieved=ach,
                peak=FP32_MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=ach / FP32_MFMA_PEAK_TFLOPS, traffic=ROOFLINE_TRAFFIC_BYTES,
                flop_per_launch=row["gflop"] * 1e9, ms_per_launch=row["fwd_ms"])


def cpu_baseline(sample_batch):
    """The CPU oracle, as it stands, on one training step of VGG-16 at a small batch.  Its loops run in parallel over
    (image, channel) pairs or, for backward-data, over images only, so the batch has to give every core an image's worth of
    work: 8 images take most of a minute on 16 cores."""
    from oracle import net as onet
    from synth import gen, nets
    net = nets.vgg16(sample_batch)
    x, labels, weights = gen.make(net, seed=gen.seed_for("vgg16"))
    t0 = time.perf_counter()
    onet.step(net, x, labels, weights)
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", 0)) or len(os.sched_getaffinity(0))
    return dict(value=sample_batch / dt, unit="img/s", cores=cores, kind="oracle",
                sample="one fwd+bwd step of VGG-16 at batch %d in %.1f s on %d threads (the benchmark's batch is 256: the same layers, 1/%d of the images)" % (sample_batch, dt, cores, 256 // sample_batch))


def per_layer_sync_bound(trace, layer_ms, d2h_gbps, h2d_gbps):
    """Step time that the paper's end-of-layer synchronisation allows (Section 3.2): a layer cannot end before
    its own computation and the transfer issued with it have both ended.  trace: the planned step; layer_ms:
    (forward, backward) per-layer compute times measured without offloading."""
    fwd, bwd = layer_ms
    off, pre = [0] * len(fwd), [0] * len(bwd)
    for t in trace:
        if t[1] == "offload":
            off[int(t[0][1:])] += t[3]
        elif t[1] in ("prefetch", "ondemand"):
            pre[int(t[0][1:])] += t[3]
    ms = sum(max(c, b / (d2h_gbps * 1e6)) for c, b in zip(fwd, off)) + sum(max(c, b / (h2d_gbps * 1e6)) for c, b in zip(bwd, pre))
    return ms


def layer_table(B, n, net):
    """Per layer and pass of the planned step: the kernel it runs, its profiled time, its algorithmic work (FLOP of the
    direct form for CONV / FC, bytes that have to cross HBM for the others) and the fraction of the roofline that bounds it;
    and the step-weighted figures: all CONV / FC work of the step over all CONV / FC time, against the fp32 MFMA peak, by the
    direct form's operation count and by the multiplications actually executed (Winograd F(2x2,3x3): 16 per 36, F(4x4,3x3): 36 per 144)."""
    shapes, _ = nets_shapes(net)
    batch = net["batch"]
    rows = []
    tot = dict(flop=0.0, executed=0.0, mfma_ms=0.0, hbm_bytes=0.0, hbm_ms=0.0)
    for i, l in enumerate(net["layers"]):
        src = l["inputs"][0]
        xin = (batch, net["in_c"], net["in_h"], net["in_w"]) if src < 0 else shapes[src]
        out = shapes[i]
        prof = n.layer_profile(i)
        if l["type"] == "conv":
            flop = 2.0 * batch * out[2] * out[3] * out[1] * xin[1] * l["k"] * l["k"]
            kern = n.layer_kernels(i)
            for pass_, kname in zip(("fwd", "bwd_data", "bwd_filter"), kern):
                ms = prof.get((pass_, kname))
                if ms is None or (pass_ == "bwd_data" and src < 0):
                    continue
                executed = flop
                if kname.startswith("winograd"):   # (m + 2)^2 multiplications per m x m output tile instead of 9 m^2, tiles that hang over the edge included
                    m = 4 if kname.startswith("winograd4") else 2
                    tiles = -(-out[2] // m) * -(-out[3] // m)
                    executed = flop * (m + 2) ** 2 * tiles / (9.0 * out[2] * out[3])
                rows.append(dict(layer=i, type="conv", what=pass_, kernel=kname, ms=ms, gflop=flop / 1e9, tflops=flop / ms / 1e9,
                                 frac_of_mfma_peak=flop / ms / 1e9 / FP32_MFMA_PEAK_TFLOPS, executed_frac_of_mfma_peak=executed / ms / 1e9 / FP32_MFMA_PEAK_TFLOPS))
                tot["flop"] += flop; tot["executed"] += executed; tot["mfma_ms"] += ms
        elif l["type"] == "fc":
            flop = 2.0 * batch * (xin[1] * xin[2] * xin[3]) * l["out"]
            for pass_, mult in (("fwd", 1), ("bwd", 2 if src >= 0 else 1)):
                ms = prof.get(pass_)
                if ms:
                    rows.append(dict(layer=i, type="fc", what=pass_, kernel="gemm", ms=ms, gflop=mult * flop / 1e9, tflops=mult * flop / ms / 1e9,
                                     frac_of_mfma_peak=mult * flop / ms / 1e9 / FP32_MFMA_PEAK_TFLOPS))
                    tot["flop"] += mult * flop; tot["executed"] += mult * flop; tot["mfma_ms"] += ms
        elif l["type"] != "softmax_ce":
            nx, ny = 4.0 * batch * xin[1] * xin[2] * xin[3], 4.0 * batch * out[1] * out[2] * out[3]
            traffic = dict(relu=(2 * ny, 3 * ny), maxpool=(nx + ny, 2 * nx + ny), avgpool=(nx + ny, nx + ny), concat=(2 * ny, 2 * ny))[l["type"]]
            for pass_, nbytes in zip(("fwd", "bwd"), traffic):
                ms = prof.get(pass_)
                if ms:   # 0: a ReLU whose work runs inside a neighbouring kernel
                    rows.append(dict(layer=i, type=l["type"], what=pass_, kernel="hbm", ms=ms, gbytes=nbytes / 1e9, tbps=nbytes / ms / 1e9,
                                     frac_of_hbm_peak=nbytes / ms / 1e9 / HBM_PEAK_TBPS))
                    tot["hbm_bytes"] += nbytes; tot["hbm_ms"] += ms
    summary = dict(conv_fc_ms=tot["mfma_ms"], other_ms=tot["hbm_ms"],
                   conv_fc_frac_of_mfma_peak_direct_count=tot["flop"] / tot["mfma_ms"] / 1e9 / FP32_MFMA_PEAK_TFLOPS if tot["mfma_ms"] else None,
                   conv_fc_frac_of_mfma_peak_executed=tot["executed"] / tot["mfma_ms"] / 1e9 / FP32_MFMA_PEAK_TFLOPS if tot["mfma_ms"] else None,
                   other_frac_of_hbm_peak=tot["hbm_bytes"] / tot["hbm_ms"] / 1e9 / HBM_PEAK_TBPS if tot["hbm_ms"] else None)
    return rows, summary


def nets_shapes(net):
    from synth import nets
    return nets.shapes(net)


def run_profile(B, net):
    """The profiling passes of Section 3.3, once, outside every timed region: every kernel of every layer and the link, on a
    net without a budget (so that every kernel's workspace fits beside its layer's tensors)."""
    global PROFILE_DATA
    n = B.Net(net, 0)
    n.set_winograd(WINOGRAD)
    n.set_policy("none")
    n.attach_torch(streams=streams())
    t0 = time.perf_counter()
    n.profile(3)
    dt = time.perf_counter() - t0
    PROFILE_DATA = n.dump_profile()
    n.close()
    import torch
    torch.cuda.empty_cache()
    return dt


def run_policy(B, net, x_dev, lab_dev, weights, policy, budget, steps, warmup, window_part_mib=None, layer_ms=None, table=None):
    """policy: none | conv | all | dyn | fit, optionally with ":m" / ":greedy" for another convolution algorithm mode;
    or "set:<id>+<id>...:<fill>[:<fill_bwd>]" for an explicit offload set with transfer windows filling <fill> per mille.
    Every net is given the profile that run_profile measured before its policy is set."""
    import torch
    t_plan = time.perf_counter()
    n = B.Net(net, budget)
    n.set_winograd(WINOGRAD)
    if window_part_mib is not None:
        n.set_window_part(int(window_part_mib * (1 << 20)))
    if PROFILE_DATA is not None:
        n.load_profile(PROFILE_DATA)   # every policy decides from the same measured times: same kernels, comparable steps
    if policy.startswith("set:"):
        _, ids, *fills = policy.split(":")
        status = n.try_offload_set({int(v) for v in ids.split("+") if v}, *[int(f) for f in fills])
    elif policy.startswith("fit:"):     # the offload set that fit chooses, with the window shares given
        status = n.try_policy("fit")
        if status == B.OK:
            status = n.try_offload_set(n.offload_set(), *[int(f) for f in policy.split(":")[1:]])
    else:
        if ":" in policy:
            policy, algo = policy.split(":")
            n.set_conv_algo(algo)
        status = n.try_policy(policy)
    if status != B.OK:
        msg = n.last_error()
        n.close()
        return dict(status="oom" if status == B.ERR_OOM_DEVICE else "error %d" % status, detail=msg)
    print("bench: %s planned in %.1f s" % (policy, time.perf_counter() - t_plan), file=sys.stderr, flush=True)   # a long plan must not look like a hang
    n.attach_torch(streams=streams())
    for i, w in weights.items():
        n.set_weights(i, w)
    loss = None
    for _ in range(warmup):
        loss = n.forward(x_dev, lab_dev)
        n.backward()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    fwd_ms = bwd_ms = stall = d2h = h2d = 0.0
    per_step = []
    for _ in range(steps):
        loss = n.forward(x_dev, lab_dev)
        n.backward()
        st = n.stats()
        fwd_ms += st["fwd_ms"]; bwd_ms += st["bwd_ms"]; stall += st["stall_ms"]; d2h += st["d2h_gbps"]; h2d += st["h2d_gbps"]
        per_step.append(round(st["fwd_ms"] + st["bwd_ms"], 1))
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    st = n.stats()
    if policy == "none" and layer_ms is not None:   # one more step with an event per layer: per-layer compute times
        n.set_layer_timing(True)
        n.forward(x_dev, lab_dev)
        n.backward()
        layer_ms.extend(n.layer_times())
        n.set_layer_timing(False)
    print("bench: %s %.1f ms per step" % (policy, dt * 1e3), file=sys.stderr, flush=True)
    out = dict(status="ok", img_per_s=net["batch"] / dt, ms_per_step=dt * 1e3, fwd_ms=fwd_ms / steps, bwd_ms=bwd_ms / steps,
               stall_ms=stall / steps, loss=loss, effective_policy=st["effective_policy"], budget_bytes=budget,
               peak_bytes=st["peak_bytes"], pool_extent_bytes=st["pool_extent_bytes"], avg_bytes=st["avg_bytes_layerstep"],
               baseline_bytes=st["baseline_bytes"], offloaded_bytes=st["offloaded_bytes"], pinned_host_bytes=st["pinned_host_bytes"],
               n_offload=st["n_offload"], n_prefetch=st["n_prefetch"], n_ondemand_fetch=st["n_ondemand_fetch"],
               d2h_gbps=d2h / steps, h2d_gbps=h2d / steps, link_peak_gbps=LINK_PEAK_GBPS,
               conv_algo=st["conv_algo"], n_memopt_convs=st["n_memopt_convs"], window_fill_pm=st["window_fill_pm"], window_fill_bwd_pm=st["window_fill_bwd_pm"],
               offload_set=sorted(n.offload_set()), per_step_ms=per_step, n_winograd_convs=st["n_winograd_convs"], n_downgraded_convs=st["n_downgraded_convs"],
               kernels="/".join("".join(KERNEL_LETTER[k] for k in n.layer_kernels(i)) for i, l in enumerate(net["layers"]) if l["type"] == "conv"))
    if PROFILE_DATA is not None:
        out["estimated_ms"] = n.estimate_step_ms()
    if table is not None and policy == "none" and PROFILE_DATA is not None:
        rows, summary = layer_table(B, n, net)
        table["rows"], table["summary"] = rows, summary
    if st["offloaded_bytes"]:
        # the step cannot be shorter than the time the host link needs for the bytes of each pass
        link_s = (st["offloaded_bytes"] + st["prefetched_bytes"]) / (LINK_PEAK_GBPS * 1e9)
        out["link_bound_img_per_s"] = net["batch"] / link_s
        out["link_frac_of_peak"] = (st["offloaded_bytes"] + st["prefetched_bytes"]) / dt / (LINK_PEAK_GBPS * 1e9)
        if layer_ms and st["window_fill_pm"] == 0 and st["window_fill_bwd_pm"] == 0:
            ms = per_layer_sync_bound(n.trace(), layer_ms, d2h / steps, h2d / steps)
            out["per_layer_sync_bound_ms"] = ms
            out["per_layer_sync_bound_img_per_s"] = net["batch"] / (ms / 1e3)
    n.close()
    del n
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--budget-gib", type=float, default=12.0)
    ap.add_argument("--policies", default="none,conv,all,dyn,fit")
    ap.add_argument("--workload", default="vgg16", choices=["tiny", "alexnet", "overfeat", "googlenet", "vgg16", "vgg116", "vgg416"],
                    help="vgg16 is the benchmark; the others are the paper's remaining workloads (side measurements)")
    ap.add_argument("--window-part-mib", type=float, default=None, help="side workloads: piece size of the transfer windows (0 = whole blocks)")
    ap.add_argument("--kernel-only", action="store_true", help="only the roofline kernel (for rocprofv3 runs)")
    ap.add_argument("--calibrate-copy", action="store_true", help="with --kernel-only: also run a 1 GiB plain copy kernel")
    ap.add_argument("--kernel-table", action="store_true", help="also time every VGG-16 convolution, three passes each")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true", help="skip the roofline kernel (for a profile of the steps alone)")
    ap.add_argument("--no-winograd", action="store_true", help="keep every plan on the direct convolution kernels (side measurement)")
    ap.add_argument("--winograd-level", type=int, default=1, choices=[0, 1, 2], help="side measurement: 2 = only the F(2x2,3x3) Winograd kernels, 0 = none")
    ap.add_argument("--cpu-sample-batch", type=int, default=8)
    ap.add_argument("--no-profile", action="store_true", help="dyn and fit decide without the profiling passes")
    ap.add_argument("--winograd-chunk-mib", type=int, default=0, help="side measurement: chunk size of the Winograd workspace (0 = the library's default)")
    ap.add_argument("--no-layer-table", action="store_true", help="skip the per-layer table of the no-offload step")
    args = ap.parse_args()
    global WINOGRAD, PROFILE
    WINOGRAD = 0 if args.no_winograd else args.winograd_level
    PROFILE = not args.no_profile
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the vDNN step is a single-GPU method); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1602_08124_amd import binding as B
    from synth import gen, nets

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.winograd_chunk_mib:
        B.op_set_winograd_chunk_bytes(args.winograd_chunk_mib << 20)
    if args.kernel_only:
        out = dict(roofline=roofline(B, args.batch))
        if args.calibrate_copy:
            # a plain copy of known size, so that FETCH_SIZE / WRITE_SIZE readings can be scaled
            nfl = (1 << 30) // 4
            src = torch.ones(nfl, device="cuda")
            dst = torch.empty(nfl, device="cuda")
            st = streams()[0]
            for _ in range(3):
                B.op_concat_copy(src, dst, 1, 1, 1, 0, nfl, True, st)
            st.synchronize()
            out["copy_calibration"] = dict(kernel="concat_copy_kernel", read_bytes=nfl * 4, write_bytes=nfl * 4)
        print(json.dumps(out))
        return

    if args.workload != "vgg16":
        # side measurement of another workload: its own batch and budget, policies as asked; one JSON line, no roofline
        defaults = {"tiny": (8, 4 / 1024), "alexnet": (128, 1.0), "overfeat": (128, 2.0), "googlenet": (128, 3.0),
                    "vgg116": (32, 12.0), "vgg416": (32, 12.0)}   # the very deep VGGs of Section 5.5
        batch, gib = defaults[args.workload]
        if args.budget_gib != 12.0:
            gib = args.budget_gib
        deep = {"vgg116": 20, "vgg416": 80}
        net = nets.vgg(batch, extra_per_group=deep[args.workload]) if args.workload in deep else nets.CONFIGS[args.workload](batch)
        x, labels, weights = gen.make(net)
        x_dev, lab_dev = torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda()
        profile_s = run_profile(B, net) if PROFILE else None
        res = {pol: run_policy(B, net, x_dev, lab_dev, weights, pol, 0 if pol == "none" else int(gib * GIB), args.steps, args.warmup,
                               args.window_part_mib)
               for pol in args.policies.split(",")}
        print(json.dumps({"workload": args.workload, "batch": batch, "budget_gib": gib, "profile_s": profile_s, "policies": res}))
        return
    net = nets.vgg16(args.batch)
    x, labels, weights = gen.make(net)
    x_dev, lab_dev = torch.from_numpy(x).cuda(), torch.from_numpy(labels).cuda()
    budget = int(args.budget_gib * GIB)
    policies = {}
    layer_ms = []   # filled by the no-offload run; the offloading policies are compared with the bound it implies
    table = None if args.no_layer_table else {}
    profile_s = run_profile(B, net) if PROFILE else None
    for pol in args.policies.split(","):
        policies[pol] = run_policy(B, net, x_dev, lab_dev, weights, pol, 0 if pol == "none" else budget, args.steps, args.warmup,
                                   layer_ms=layer_ms, table=table)
        print("[bench] %s: %s" % (pol, json.dumps(policies[pol])), file=sys.stderr, flush=True)
    head = policies.get("dyn") or next(iter(policies.values()))
    head_name = "dyn" if "dyn" in policies else next(iter(policies))
    none = policies.get("none")
    if none and none.get("status") == "ok":
        for p in policies.values():
            if p.get("status") == "ok":
                p["vs_no_offload"] = p["img_per_s"] / none["img_per_s"]
    # offloading changes where bytes live, not their values: every policy that runs the same kernels has the same loss, bit for bit
    by_kernels = {}
    for name, p in policies.items():
        if p.get("status") == "ok":
            by_kernels.setdefault(p["kernels"], set()).add(p["loss"])
    identical = all(len(v) == 1 for v in by_kernels.values())
    assert identical, "policies that run the same kernels computed different losses: %r" % by_kernels
    rf = None if args.no_roofline else roofline(B, args.batch)
    out = {
        "metric": "img/s VGG-16 b%d fp32 under %g GiB budget (vDNN_%s)" % (args.batch, args.budget_gib, head_name),
        "value": head.get("img_per_s"), "unit": "img/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head.get("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "vgg16_b%d_fp32_fwd+bwd_vdnn_%s_%ggib" % (args.batch, head_name, args.budget_gib), "batch": args.batch,
                   "budget_bytes": budget, "policy": head_name, "effective_policy": head.get("effective_policy"),
                   "step_tflop": 23.718 * args.batch / 256},
        "step_tflops_achieved": 23.718 * args.batch / 256 / (head["ms_per_step"] / 1e3) if head.get("ms_per_step") else None,
        "peak_gpu_bytes": head.get("peak_bytes"),
        "policies": policies,
        "loss_bit_identical_across_policies_with_equal_kernels": identical,
        "roofline": rf,
    }
    if table:
        out["no_offload_step_by_layer"] = table
    if PROFILE_DATA is not None:
        out["profile"] = dict(seconds=profile_s, link_gbps=PROFILE_DATA["link"],
                              layers={str(i): {"/".join(k) if isinstance(k, tuple) else k: v for k, v in e.items()} for i, e in PROFILE_DATA["layers"].items()})
    if args.kernel_table:
        out["conv_kernels"] = conv_kernel_table(B, args.batch, kernel="auto" if WINOGRAD else "packed")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample_batch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
