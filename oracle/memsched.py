"""Memory-schedule oracle: replays the vDNN memory manager's rules on a network description
with host integers only (test infrastructure; shares no code with the library).

What it follows (Section 3, "Virtualized DNN"):
  * layer-wise sliding-window allocation from a pool of fixed size (3.1, 3.2 "Memory
    Allocation/Release");
  * forward: a layer's input feature map X is offloaded to host memory, overlapped with the same
    layer's forward computation, only when the current layer is the LAST consumer of X
    (Fig. nonlinear_dfg, Refcnt); the compute stream waits for the copy at the end of the layer
    and X is then released (3.2 "Memory Offload");
  * backward: before layer m's backward computation a search over the preceding layers, bounded
    by the next CONV layer, picks one offloaded-and-not-yet-prefetched X to copy back, overlapped
    with layer m's backward computation (3.2 "Memory Prefetch", caption of Fig. code_prefetch);
    data is released as soon as no remaining backward computation needs it (3.1 "Backward
    Propagation");
  * policies (3.3): all = every CONV/POOL input, conv = inputs that feed a CONV layer,
    none = the baseline without offloading, dyn = the profiling-pass sequence with
    out-of-memory as the signal.

Workspace (Section 2.2: convolution algorithms trade workspace for speed) is an INPUT here, not something this
file derives: `ws` maps (layer id, "fwd" | "bwd") to the workspace bytes of the ways that layer can run, fastest
first.  How many bytes an implementation's kernels want is that implementation's business; the tests pass in what
the library reports, and hand-written values in the pins.

Readings where the paper is silent are listed in the repository's design notes; the ones that
matter here: feature maps that no backward computation needs are released in forward; a
feature map is released right after its last backward use; gradient maps are allocated on
first write and released after their producer's backward computation; ReLU is in place and
shares its input's buffers; FC/loss inputs are never offloaded; sizes are rounded up to
256-byte blocks; a pass fails when the live total would pass the budget.
"""

ALIGN = 256
IN_PLACE = ("relu",)
NEEDS_X_IN_BWD = ("conv", "maxpool", "fc", "softmax_ce")


def _al(n):
    return (n + ALIGN - 1) // ALIGN * ALIGN


class OutOfMemory(Exception):
    pass


class Pool:
    """Byte accounting of the pool: a request fails when the live total would pass the budget.
    (Where blocks are placed inside the pool is the library's business; its placement is
    checked separately for overlap, not predicted here.)"""

    def __init__(self, budget):
        self.budget = budget // ALIGN * ALIGN
        self.live = 0
        self.peak = 0

    def alloc(self, nbytes):
        size = _al(max(nbytes, 1))
        if self.live + size > self.budget:
            raise OutOfMemory(nbytes)
        self.live += size
        self.peak = max(self.peak, self.live)
        return size

    def release(self, size):
        self.live -= size


def analyse(net):
    """Shapes, buffers and consumer lists of a network description."""
    n = net["batch"]
    layers = net["layers"]
    shape = []
    buf = []          # layer id -> buffer id (id of the producing non-in-place layer, -1 = input)

    def shp(i):
        return (net["in_c"], net["in_h"], net["in_w"]) if i < 0 else shape[i]

    def bufof(i):
        return -1 if i < 0 else buf[i]

    for i, l in enumerate(layers):
        c, h, w = shp(l["inputs"][0])
        t, k, st, pd = l["type"], l["k"], l["stride"], l["pad"]
        if t == "conv":
            shape.append((l["out"], (h + 2 * pd - k) // st + 1, (w + 2 * pd - k) // st + 1))
        elif t in ("maxpool", "avgpool"):
            shape.append((c, (h + 2 * pd - k) // st + 1, (w + 2 * pd - k) // st + 1))
        elif t == "fc":
            shape.append((l["out"], 1, 1))
        elif t == "concat":
            shape.append((sum(shp(j)[0] for j in l["inputs"]), h, w))
        elif t == "relu":
            shape.append((c, h, w))
        elif t == "softmax_ce":
            shape.append((0, 0, 0))
        else:
            raise ValueError(t)
        buf.append(bufof(l["inputs"][0]) if t in IN_PLACE else i)
    nbytes = {-1: 4 * n * net["in_c"] * net["in_h"] * net["in_w"]}
    for i, l in enumerate(layers):
        if buf[i] == i and l["type"] != "softmax_ce":
            c, h, w = shape[i]
            nbytes[i] = 4 * n * c * h * w
    readers = {b: [] for b in nbytes}     # non-in-place layers reading buffer b, ascending
    inplace = {b: [] for b in nbytes}     # in-place layers living in buffer b
    for i, l in enumerate(layers):
        if l["type"] in IN_PLACE:
            inplace[buf[i]].append(i)
        else:
            for j in l["inputs"]:
                readers[bufof(j)].append(i)
    return dict(shape=shape, buf=buf, bufof=bufof, nbytes=nbytes, readers=readers, inplace=inplace, shp=shp)


def layer_weight_bytes(net, info, i):
    l = net["layers"][i]
    c, h, w = info["shp"](l["inputs"][0])
    if l["type"] == "conv":
        return 4 * l["out"] * c * l["k"] * l["k"]
    if l["type"] == "fc":
        return 4 * l["out"] * c * h * w
    return 0


def bwd_users(net, info, b):
    """Layers whose backward computation reads the contents of buffer b."""
    users = [i for i in info["readers"][b] if net["layers"][i]["type"] in NEEDS_X_IN_BWD]
    return sorted(users + info["inplace"][b])


def selected(net, info, b, policy):
    types = {net["layers"][i]["type"] for i in info["readers"][b]}
    if not bwd_users(net, info, b):
        return False
    if policy == "all":
        return bool(types & {"conv", "maxpool", "avgpool"})
    if policy == "conv":
        return "conv" in types
    return False


def baseline_bytes(net, ws=None):
    """Network-wide allocation of the baseline (Fig. mem_allocation_policy_global): every feature
    map, W and dW, two gradient maps sized to the largest one, one workspace sized to the largest
    (the performance-optimal algorithm of every layer: the first entry of its list)."""
    info = analyse(net)
    fm = sum(_al(v) for v in info["nbytes"].values())
    wb = sum(2 * _al(layer_weight_bytes(net, info, i)) for i in range(len(net["layers"]))
             if layer_weight_bytes(net, info, i))
    gmax = max(_al(v) for b, v in info["nbytes"].items() if b >= 0)
    wmax = max([v[0] for v in (ws or {}).values() if v] + [0])
    return fm + wb + 2 * gmax + _al(wmax)


def simulate(net, policy, budget, algo="p", offload_set=None, ws=None):
    """One training step under a static policy ("none" | "all" | "conv") and a convolution algorithm
    mode (Section 3.3): "p" performance-optimal (every layer runs the first entry of its list), "m"
    memory-optimal (CONV layers use no workspace), "greedy" = per CONV layer the first entry whose
    workspace still fits the budget at that point of the step, the memory-optimal algorithm if none does
    (phase 3 of vDNN_dyn).
    offload_set: when given, exactly these buffers are offloaded (the policy argument is then unused).
    ws: {(layer, "fwd" | "bwd"): [workspace bytes, fastest algorithm first]}; a layer without an entry needs none.
    Returns a dict with status ("ok" | "oom"), where it failed, peak / average / final pool bytes,
    transfer counts, the number of CONV layers on the memory-optimal algorithm by decision of the mode, the number
    the greedy mode moved off their first entry, and the ordered op trace."""
    info = analyse(net)
    layers = net["layers"]
    nl = len(layers)
    pool = Pool(budget)
    trace = []
    samples = []
    st = dict(offloaded_bytes=0, prefetched_bytes=0, n_offload=0, n_prefetch=0, n_ondemand_fetch=0)
    memopt = set()      # CONV layers put on the memory-optimal algorithm in either pass
    downgraded = set()  # CONV layers the greedy mode moved off their first entry in either pass
    ws_options = ws or {}

    def layer_ws(i, phase):
        options = list(ws_options.get((i, phase), ()))
        if layers[i]["type"] != "conv":
            return options[0] if options else 0
        if algo == "m":
            memopt.add(i)
            return 0
        if algo == "p" or not options:
            return options[0] if options else 0
        for k, nbytes in enumerate(options):
            if not nbytes or pool.live + _al(nbytes) <= pool.budget:
                break
        else:
            k, nbytes = len(options), 0
        if k > 0:
            downgraded.add(i)
            if not nbytes:
                memopt.add(i)
        return nbytes

    res = {}        # buffer -> (tag, size) while resident
    grad = {}       # buffer -> (tag, size) of its gradient map
    on_host = set()
    offloaded_at = {}  # layer -> [buffers it offloaded]
    where = "create"

    def alloc(tag, nbytes):
        size = pool.alloc(nbytes)
        trace.append((where, "alloc", tag, size))
        return tag, size

    def free(tag, blk):
        pool.release(blk[1])
        trace.append((where, "free", blk[0], blk[1]))

    try:
        for i in range(nl):
            wb = layer_weight_bytes(net, info, i)
            if wb:
                alloc("W%d" % i, wb)
                alloc("dW%d" % i, wb)
        alloc("labels", 4 * net["batch"])
        alloc("loss", 4)
        persistent = pool.live

        # ---- forward ----
        where = "F-1"
        res[-1] = alloc("B-1", info["nbytes"][-1])
        for i, l in enumerate(layers):
            where = "F%d" % i
            samples.append(pool.live)
            t = l["type"]
            if t not in IN_PLACE and t != "softmax_ce":
                res[i] = alloc("B%d" % i, info["nbytes"][i])
            ws = layer_ws(i, "fwd")
            wsb = alloc("WS", ws) if ws else None
            if t not in IN_PLACE:
                for b in dict.fromkeys(info["bufof"](j) for j in l["inputs"]):
                    if info["readers"][b][-1] == i and (b in offload_set if offload_set is not None
                                                         else selected(net, info, b, policy)):
                        trace.append((where, "offload", "B%d" % b, info["nbytes"][b]))
                        st["offloaded_bytes"] += info["nbytes"][b]
                        st["n_offload"] += 1
                        offloaded_at.setdefault(i, []).append(b)
            trace.append((where, "compute", t))
            if wsb:
                free("WS", wsb)
            for b in offloaded_at.get(i, []):
                free("B%d" % b, res.pop(b))
                on_host.add(b)
            if t not in IN_PLACE:
                for b in dict.fromkeys(info["bufof"](j) for j in l["inputs"]):
                    if b in res and info["readers"][b][-1] == i and not bwd_users(net, info, b):
                        free("B%d" % b, res.pop(b))

        # ---- backward ----
        def fetch(b, kind):
            res[b] = alloc("B%d" % b, info["nbytes"][b])
            on_host.discard(b)
            trace.append((where, kind, "B%d" % b, info["nbytes"][b]))
            st["prefetched_bytes"] += info["nbytes"][b]

        for m in range(nl - 1, -1, -1):
            where = "B%d" % m
            samples.append(pool.live)
            l = layers[m]
            t = l["type"]
            # findPrefetchLayer: nearest preceding layer with an offloaded, not yet prefetched X;
            # the search stops at the first CONV layer that has nothing to prefetch.
            for j in range(m - 1, -1, -1):
                pending = [b for b in offloaded_at.get(j, []) if b in on_host]
                if pending:
                    for b in pending:
                        fetch(b, "prefetch")
                        st["n_prefetch"] += 1
                    break
                if layers[j]["type"] == "conv":
                    break
            own = info["buf"][m]
            in_bufs = list(dict.fromkeys(info["bufof"](j) for j in l["inputs"]))
            needed = [own] if t in IN_PLACE else ([b for b in in_bufs] if t in NEEDS_X_IN_BWD else [])
            for b in needed:
                if b in on_host:
                    fetch(b, "ondemand")
                    st["n_ondemand_fetch"] += 1
            temps = []
            if t not in IN_PLACE:
                for b in in_bufs:
                    if b < 0:
                        continue
                    if b not in grad:
                        grad[b] = alloc("dB%d" % b, info["nbytes"][b])
                    else:
                        temps.append(alloc("T%d" % b, info["nbytes"][b]))
            ws = layer_ws(m, "bwd")
            wsb = alloc("WS", ws) if ws else None
            trace.append((where, "compute", t))
            if wsb:
                free("WS", wsb)
            for blk in temps:
                free("T", blk)
            if t not in IN_PLACE and t != "softmax_ce":
                free("dB%d" % m, grad.pop(m))
            for b in sorted(res):
                users = bwd_users(net, info, b)
                if users and users[0] == m:
                    free("B%d" % b, res.pop(b))
        status, oom_at = "ok", None
    except OutOfMemory:
        status, oom_at = "oom", where
    out = dict(status=status, oom_at=oom_at, peak_bytes=pool.peak, cur_bytes=pool.live,
               avg_bytes_layerstep=(sum(samples) / len(samples) if samples else 0.0),
               trace=trace, budget_bytes=pool.budget)
    if status == "ok":
        out["persistent_bytes"] = persistent
    out.update(st)
    out["n_memopt_convs"] = len(memopt)
    out["n_downgraded_convs"] = len(downgraded)
    return out


def dynamic(net, budget, ws=None):
    """vDNN_dyn (Section 3.3, "Dynamic vDNN").  Pass 1: all with the memory-optimal algorithm must fit.
    Pass 2: performance-optimal algorithms with no offloading, else conv, else all - adopt the first
    that fits.  Pass 3: greedy per-layer downgrade under conv, then all; else the configuration of pass 1.
    Returns (policy or None, algorithm mode, result of the adopted pass)."""
    first = simulate(net, "all", budget, "m", ws=ws)
    if first["status"] != "ok":
        return None, None, first
    for pol in ("none", "conv", "all"):
        r = simulate(net, pol, budget, "p", ws=ws)
        if r["status"] == "ok":
            return pol, "p", r
    for pol in ("conv", "all"):
        r = simulate(net, pol, budget, "greedy", ws=ws)
        if r["status"] == "ok":
            return pol, "greedy", r
    return "all", "m", first


def trace_stats(trace):
    """Peak, final and layer-step average of the live bytes of a trace (sampled before the first entry of
    each layer of each pass), and its transfer counts."""
    live = peak = 0
    samples = []
    seen = set()
    st = dict(offloaded_bytes=0, prefetched_bytes=0, n_offload=0, n_prefetch=0, n_ondemand_fetch=0)
    for t in trace:
        if t[0] != "create" and t[0] != "F-1" and t[0] not in seen:
            seen.add(t[0])
            samples.append(live)
        if t[1] == "alloc":
            live += t[3]
            peak = max(peak, live)
        elif t[1] == "free":
            live -= t[3]
        elif t[1] == "offload":
            st["offloaded_bytes"] += t[3]
            st["n_offload"] += 1
        elif t[1] in ("prefetch", "ondemand"):
            st["prefetched_bytes"] += t[3]
            st["n_prefetch" if t[1] == "prefetch" else "n_ondemand_fetch"] += 1
    st.update(peak_bytes=peak, cur_bytes=live, avg_bytes_layerstep=sum(samples) / len(samples) if samples else 0.0)
    return st
