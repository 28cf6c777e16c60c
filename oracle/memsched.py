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

Readings where the paper is silent are listed in the repository's design notes; the ones that
matter here: feature maps that no backward computation needs are released in forward; a
feature map is released right after its last backward use; gradient maps are allocated on
first write and released after their producer's backward computation; ReLU is in place and
shares its input's buffers; FC/loss inputs are never offloaded; sizes are rounded up to
256-byte blocks; a pass fails when the live total would pass the budget.
"""

ALIGN = 256
TARGET_BLOCKS = 1024
MIN_SPLIT_LEN = 512
IN_PLACE = ("relu",)
NEEDS_X_IN_BWD = ("conv", "maxpool", "fc", "softmax_ce")


def _al(n):
    return (n + ALIGN - 1) // ALIGN * ALIGN


def _cdiv(a, b):
    return (a + b - 1) // b


def gemm_splits(m, n, kred):
    """Number of reduction splits (and hence workspace slices) of a GEMM whose output is m x n."""
    bm = 64 if m <= 64 else 128
    tiles = _cdiv(m, bm) * _cdiv(n, 128)
    return max(1, min(TARGET_BLOCKS // tiles, _cdiv(kred, MIN_SPLIT_LEN)))


def conv_slots(rows):
    """Resident workgroups of the packed-weight convolution kernel on 256 CUs: 4 per CU for every tile shape."""
    return 1024


WINOGRAD_CHUNK_BYTES = 512 << 20


def winograd_workspace(n, cred, h, w, rows, k, stride, pad):
    """Workspace of the F(2x2,3x3) Winograd algorithm where the library runs it (0 elsewhere): 3x3 / stride 1 / pad 1,
    reduction channels a multiple of 16 and at least 256, rows a multiple of 4 and at least 128.  Transformed filter (16 x cred x rows floats, rounded up to 256 bytes) plus transformed
    input and products (16 x (cred + rows) floats per 2x2 output tile) for as many images as fit the chunk size."""
    if not (k == 3 and stride == 1 and pad == 1 and cred % 16 == 0 and rows % 4 == 0
            and 256 <= cred <= 65535 and 128 <= rows <= 65535 and ((h + 1) // 2) * ((w + 1) // 2) <= 32768):
        return 0
    per_image = 16 * (cred + rows) * ((h + 1) // 2) * ((w + 1) // 2) * 4
    nb = max(1, min(n, 65535, WINOGRAD_CHUNK_BYTES // per_image))
    return _cdiv(16 * cred * rows, 64) * 64 * 4 + nb * per_image


def winograd_filter_workspace(n, c, h, w, k, ksz, stride, pad):
    """Workspace of the Winograd backward-filter pass where the library runs it (0 elsewhere): same geometry, input
    channels a multiple of 128, 256 or more output channels.  The 16 accumulated products (16 x K x C floats),
    their partial sums per reduction split, and the transformed X and dY for as many images as fit the chunk size."""
    if not (ksz == 3 and stride == 1 and pad == 1 and c % 128 == 0 and c <= 65535 and 256 <= k <= 65535
            and ((h + 1) // 2) * ((w + 1) // 2) <= 32768):
        return 0
    t = ((h + 1) // 2) * ((w + 1) // 2)
    per_image = 16 * (c + k) * t * 4
    nb = max(1, min(n, 65535, WINOGRAD_CHUNK_BYTES // per_image))
    tiles = _cdiv(k, 128) * (c // 128) * 16
    splits = max(1, min(1024 // tiles, _cdiv(nb * t, 512)))
    return 16 * k * c * 4 * (1 + splits) + nb * per_image


def conv_packed_workspace(wcount, rows, m, cred, rs):
    """Workspace of the packed-weight convolution kernel: a packed copy of W (rounded up to 256 bytes), plus
    partial sums for the tiles whose reduction is split because the last round of workgroups would be
    mostly idle (fewer than 70 % of the resident workgroups) and the job is short (under 4 full rounds)."""
    bm = 32 if rows <= 32 else (64 if rows <= 64 else 128)
    bn = 256 if rows <= 64 else 128
    tiles = _cdiv(rows, bm) * _cdiv(m, bn)
    steps = cred // 16 * rs
    CONV_SLOTS = conv_slots(rows)
    tail = tiles - tiles // CONV_SLOTS * CONV_SLOTS
    extra = 0
    if tail > 0 and tail * 10 < CONV_SLOTS * 7 and tiles - tail < 4 * CONV_SLOTS:
        s = min(CONV_SLOTS // tail, 8, steps // 8)
        if s > 1:
            per = _cdiv(steps, s)
            extra = tail * _cdiv(steps, per) * bm * bn * 4
    return _cdiv(wcount, 64) * 64 * 4 + extra


def _ws(m, n, kred):
    s = gemm_splits(m, n, kred)
    return s * m * n * 4 if s > 1 else 0


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


def workspace_bytes(net, info, i, phase, memopt=False, direct=False):
    """Transient workspace of layer i: partial sums of reduction-split GEMMs, packed weights, Winograd transforms.
    memopt: the CONV layer runs the memory-optimal algorithm, which needs X, Y and W only (Section 2.2).
    direct: a CONV layer wide enough for the Winograd algorithm is sized for the direct kernel instead."""
    l = net["layers"][i]
    n = net["batch"]
    c, h, w = info["shp"](l["inputs"][0])
    if l["type"] == "conv" and memopt:
        return 0
    if l["type"] == "conv":
        k, p, q = info["shape"][i]
        wbytes = 4 * k * c * l["k"] * l["k"]
        # packed copy of W for the faster kernel: reduction channels a multiple of 16, tensors below 4 GiB
        rs = l["k"] * l["k"]
        if phase == "fwd":
            if c % 16 == 0 and 4 * n * c * h * w < 0xfffffff0:
                return ((0 if direct else winograd_workspace(n, c, h, w, k, l["k"], l["stride"], l["pad"]))
                        or conv_packed_workspace(wbytes // 4, k, n * p * q, c, rs))
            return 0
        need_dx = info["bufof"](l["inputs"][0]) >= 0
        packed = 0
        if need_dx and l["stride"] == 1 and l["pad"] <= l["k"] - 1 and k % 16 == 0 and 4 * n * k * p * q < 0xfffffff0:
            packed = ((0 if direct else winograd_workspace(n, k, h, w, c, l["k"], l["stride"], l["pad"]))
                      or conv_packed_workspace(wbytes // 4, c, n * h * w, k, rs))
        # backward-filter: the Winograd form on wide 3x3 layers; else partial sums of the split reduction; with input
        # channels a multiple of 32 the faster kernel always stages dW through the workspace (at least one copy)
        wino_filt = 0 if direct else winograd_filter_workspace(n, c, h, w, k, l["k"], l["stride"], l["pad"])
        if wino_filt:
            return max(wino_filt, packed)
        if c % 32 == 0 and 4 * n * c * h * w < 0xfffffff0 and 4 * n * k * p * q < 0xfffffff0:
            if c == 64 and rs % 3 == 0:
                # 64-channel layers run column tiles of three taps: the split count follows from that tile count
                tiles = _cdiv(k, 64 if k <= 64 else 128) * (rs // 3)
                filt = max(1, min(TARGET_BLOCKS // tiles, _cdiv(n * p * q, MIN_SPLIT_LEN))) * wbytes
            else:
                filt = gemm_splits(k, c * l["k"] * l["k"], n * p * q) * wbytes
        else:
            filt = _ws(k, c * l["k"] * l["k"], n * p * q)
        return max(filt, packed)
    if l["type"] == "fc":
        i_feat, o = c * h * w, l["out"]
        if phase == "fwd":
            return _ws(n, o, i_feat)
        need_dx = info["bufof"](l["inputs"][0]) >= 0
        return max(_ws(o, i_feat, n), _ws(n, i_feat, o) if need_dx else 0)
    return 0


def baseline_bytes(net):
    """Network-wide allocation of the baseline (Fig. mem_allocation_policy_global): every feature
    map, W and dW, two gradient maps sized to the largest one, one workspace sized to the largest."""
    info = analyse(net)
    fm = sum(_al(v) for v in info["nbytes"].values())
    wb = sum(2 * _al(layer_weight_bytes(net, info, i)) for i in range(len(net["layers"]))
             if layer_weight_bytes(net, info, i))
    gmax = max(_al(v) for b, v in info["nbytes"].items() if b >= 0)
    wmax = max(max(workspace_bytes(net, info, i, "fwd"), workspace_bytes(net, info, i, "bwd"))
               for i in range(len(net["layers"])))
    return fm + wb + 2 * gmax + _al(wmax)


def simulate(net, policy, budget, algo="p", offload_set=None, winograd=True):
    """One training step under a static policy ("none" | "all" | "conv") and a convolution algorithm
    mode: "p" performance-optimal (workspace), "m" memory-optimal (none), "greedy" = performance-optimal
    except where that layer's workspace would overflow the budget (Section 3.3, phase 3 of vDNN_dyn).
    offload_set: when given, exactly these buffers are offloaded (the policy argument is then unused).
    winograd: False keeps every layer on the direct kernel (the library's vdnn_set_winograd(net, 0)).
    Returns a dict with status ("ok" | "oom"), where it failed, peak / average / final pool bytes,
    transfer counts, the number of CONV layers on the memory-optimal algorithm and the ordered op trace."""
    info = analyse(net)
    layers = net["layers"]
    nl = len(layers)
    pool = Pool(budget)
    trace = []
    samples = []
    st = dict(offloaded_bytes=0, prefetched_bytes=0, n_offload=0, n_prefetch=0, n_ondemand_fetch=0)
    memopt = set()  # CONV layers downgraded (or set) to the memory-optimal algorithm in either pass
    wino = set()    # CONV layers given the Winograd workspace in either pass

    def layer_ws(i, phase):
        conv = layers[i]["type"] == "conv"
        if conv and algo == "m":
            memopt.add(i)
            return 0
        ws = workspace_bytes(net, info, i, phase)
        direct = workspace_bytes(net, info, i, phase, direct=True) if conv else ws
        if conv and ws and (not winograd or (offload_set and phase == "fwd") or pool.live + _al(ws) > pool.budget):
            # the Winograd algorithm runs where its workspace fits at this point; elsewhere the direct kernel stays;
            # with an explicit, non-empty offload set the forward pass keeps the direct kernel everywhere
            ws = direct
        if conv and ws > direct:
            wino.add(i)
        if conv and algo == "greedy" and ws and pool.live + _al(ws) > pool.budget:
            memopt.add(i)
            return 0
        return ws

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
    out["n_winograd_convs"] = len(wino)
    return out


def dynamic(net, budget, winograd=True):
    """vDNN_dyn (Section 3.3, "Dynamic vDNN").  Pass 1: all with the memory-optimal algorithm must fit.
    Pass 2: performance-optimal algorithms with no offloading, else conv, else all - adopt the first
    that fits.  Pass 3: greedy per-layer downgrade under conv, then all; else the configuration of pass 1.
    Returns (policy or None, algorithm mode, result of the adopted pass)."""
    first = simulate(net, "all", budget, "m", winograd=winograd)
    if first["status"] != "ok":
        return None, None, first
    for pol in ("none", "conv", "all"):
        r = simulate(net, pol, budget, "p", winograd=winograd)
        if r["status"] == "ok":
            return pol, "p", r
    for pol in ("conv", "all"):
        r = simulate(net, pol, budget, "greedy", winograd=winograd)
        if r["status"] == "ok":
            return pol, "greedy", r
    return "all", "m", first


# ---------------------------------------------------------------------------------------------------
# Beyond the paper's three policies: "fit".
#
# Section 3.3 motivates vDNN_dyn with the observation that offloading more than needed costs
# performance, and Section 3.1 (reuse distance) with the observation that a transfer can hide behind
# whatever computation lies between the two uses of X.  On a machine whose arithmetic is fast relative
# to its host link both become the whole story: the step time is the bytes moved divided by the link
# rate.  "fit" therefore (a) offloads a set of feature maps chosen to move few bytes, and (b) keeps the
# paper's transfers but drops the layer-by-layer synchronisation wherever the budget has room: an
# offloaded X is released only when a later allocation needs its bytes, and a prefetch is issued as
# early as its destination fits.
# ---------------------------------------------------------------------------------------------------

# Share of the budget (per mille) the forward windows may fill: the library takes the largest for which the blocks
# can be placed inside the budget.
FILLS_PM = (1000, 990, 980, 970, 960, 950, 940, 930, 920, 910, 900, 880, 860, 840, 820, 800, 750, 700, 600, 500, 0)


def fit_candidates(net):
    """Buffers vDNN_all would offload, ascending id."""
    info = analyse(net)
    return [b for b in sorted(info["nbytes"]) if selected(net, info, b, "all")]


def fit_select(net, budget, algo="p", winograd=True):
    """Offload set for "fit": start empty; while the step does not fit, add the SMALLEST remaining candidate
    whose addition makes it fit, and if there is none add the LARGEST remaining one (ties: lower id) and
    repeat.  Returns the set, or None when even every candidate together does not fit."""
    info = analyse(net)
    cands = fit_candidates(net)
    chosen = set()

    def fits(s):
        return simulate(net, "none", budget, algo, offload_set=s, winograd=winograd)["status"] == "ok"

    while not fits(chosen):
        rest = [b for b in cands if b not in chosen]
        if not rest:
            return None
        by_size = sorted(rest, key=lambda b: (info["nbytes"][b], b))
        done = next((b for b in by_size if fits(chosen | {b})), None)
        if done is not None:
            chosen.add(done)
            break
        chosen.add(max(rest, key=lambda b: (info["nbytes"][b], -b)))
    return chosen


def _phase(where):
    return 0 if where == "create" else (1 if where[0] == "F" else 2)


PART_BYTES = 128 << 20   # transfers of larger blocks are cut into at most MAX_PARTS pieces of about this size
MAX_PARTS = 32


def parts_of(size, raw, part_bytes):
    """[(block bytes, bytes to copy)] of the pieces of a block of `size` (aligned) bytes holding `raw` bytes."""
    if not part_bytes or size <= part_bytes:
        return [(size, raw)]
    k = min(MAX_PARTS, _cdiv(size, part_bytes))
    step = _al(_cdiv(size, k))
    out = []
    for i in range(k):
        lo = i * step
        if lo >= size:
            break
        out.append((min(step, size - lo), max(0, min(step, raw - lo))))
    return out


def retime(trace, budget, fill_pm, part_bytes=PART_BYTES, lent=None, twins=None):
    """Budget-aware transfer windows on the op trace of a static schedule.

    Forward: the release of an offloaded X no longer follows its last consumer; released blocks queue up in
    copy order, and an allocation that would pass `soft` = budget * fill_pm / 1000 first releases the oldest
    of them until the live total fits.  The address range of X is lent out while X is away: a feature map that
    is not offloaded itself and whose allocation had to release something becomes a TENANT of the block
    released last; tenants line up from the low end of the host's range (pieces leave from the low end
    upwards), and the allocation keeps releasing until the host has room for it.  When the host runs out of
    pieces, the next block in the queue becomes the host.  Whatever is still queued at the end of forward
    propagation is released there.
    Backward: fetches keep their place in the static schedule here.  (The library issues them earlier, as soon
    as the address range a fetch will occupy is free in its placement of the blocks; that needs addresses,
    which this byte-counting model does not have: see settle_fetches.)  A fetch returns to the range its block
    had in forward propagation (it is the host's TWIN) when every tenant has left by then.
    Blocks larger than part_bytes are copied, released and fetched in pieces ("B7#2" = third piece of B7);
    forward gives the pieces up from the low end upwards, backward fetches them from the top one down.

    lent: optional dict, filled with {tenant tag: (host tag, byte offset inside the host's range)};
    twins: optional set, filled with the tags whose fetch returns to the forward range."""
    budget_al = budget // ALIGN * ALIGN
    soft = budget_al * fill_pm // 1000 // ALIGN * ALIGN
    create = [t for t in trace if _phase(t[0]) == 0]
    fwd = [t for t in trace if _phase(t[0]) == 1]
    bwd = [t for t in trace if _phase(t[0]) == 2]
    live = sum(t[3] for t in create if t[1] == "alloc")
    size_of = {}           # tag -> aligned size of the block while it is live
    offloaded = {t[2] for t in fwd if t[1] == "offload"}
    lent = {} if lent is None else lent
    twins = set() if twins is None else twins

    def pieces(tag, raw):
        ps = parts_of(size_of[tag], raw, part_bytes)
        return [(tag if len(ps) == 1 else "%s#%d" % (tag, i), sz, rw) for i, (sz, rw) in enumerate(ps)]

    # ---- forward: copies in pieces, lazy release of offloaded blocks, tenants ----
    out = list(create)
    pending = []           # (piece tag, size, block tag), oldest first
    copying = {}           # tag -> raw bytes being offloaded
    released = {}          # host tag -> bytes released so far (from the low end of its range)
    taken = {}             # host tag -> bytes lent so far
    host = None            # block released last
    for t in fwd:
        kind = t[1]
        if kind == "offload":
            copying[t[2]] = t[3]
            out.extend((t[0], "offload", tag, rw) for tag, _, rw in pieces(t[2], t[3]))
            continue
        if kind == "free" and t[2] in copying:
            pending.extend((tag, sz, t[2]) for tag, sz, _ in pieces(t[2], copying.pop(t[2])))
            continue
        if kind == "alloc":
            if live + t[3] > soft:
                rents = t[2][0] == "B" and t[2] not in offloaded

                def room():
                    return released[host] - taken[host] if host is not None else 0

                while pending and (live + t[3] > soft or (rents and room() < t[3])):
                    tag, size, host = pending.pop(0)
                    out.append((t[0], "free", tag, size))
                    live -= size
                    released[host] = released.get(host, 0) + size
                    taken.setdefault(host, 0)
                if rents and room() >= t[3]:
                    lent[t[2]] = (host, taken[host])
                    taken[host] += t[3]
            live += t[3]
            size_of[t[2]] = t[3]
        elif kind == "free":
            live -= t[3]
        out.append(t)
    last_fwd = fwd[-1][0] if fwd else "F0"
    for tag, size, _ in pending:
        out.append((last_fwd, "free", tag, size))
        live -= size

    # ---- backward: fetches in pieces, top piece first, at their place in the static schedule ----
    freed_at = {t[2]: i for i, t in enumerate(bwd) if t[1] == "free"}
    i = 0
    while i < len(bwd):
        t = bwd[i]
        if t[1] == "alloc" and i + 1 < len(bwd) and bwd[i + 1][1] in ("prefetch", "ondemand") and bwd[i + 1][2] == t[2]:
            size_of[t[2]] = t[3]
            tenants = [tn for tn, (h, _) in lent.items() if h == t[2]]
            if tenants and all(freed_at.get(tn, -1) < i for tn in tenants):   # not in freed_at: released in forward already
                twins.add(t[2])
            for tag, size, raw in reversed(pieces(t[2], bwd[i + 1][3])):
                out.append((t[0], "alloc", tag, size))
                out.append((t[0], bwd[i + 1][1], tag, raw))
            i += 2
            continue
        out.append(t)
        i += 1
    return out


def settle_fetches(trace):
    """Canonical form of a backward schedule whose fetches may have been issued early: every (alloc, prefetch |
    ondemand) pair of a fetched block or piece is taken out.  Returns (trace without them, [(tag, number of
    compute entries that precede the pair)]).  Two schedules that differ only in how early fetches are issued
    have the same first part; the second part says how early."""
    rest, fetches = [], []
    computes = 0
    i = 0
    while i < len(trace):
        t = trace[i]
        if (_phase(t[0]) == 2 and t[1] == "alloc" and i + 1 < len(trace) and trace[i + 1][1] in ("prefetch", "ondemand")
                and trace[i + 1][2] == t[2]):
            fetches.append((t[2], computes))
            i += 2
            continue
        computes += t[1] == "compute"
        rest.append(t)
        i += 1
    return rest, fetches


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


def fit(net, budget, fill_pm=1000, part_bytes=PART_BYTES, extra=0, windows=None, winograd=True):
    """The "fit" policy: offload set from fit_select (performance-optimal algorithms first, then the greedy
    downgrade, then memory-optimal everywhere), transfer windows from retime.  windows (default: fill_pm > 0)
    = False keeps the static schedule of the chosen set.  extra: that many more candidates, largest first (ties: lower id), join the
    set (what the library does when it finds no placement of the blocks inside the budget).
    Returns (offload set, algorithm mode, result dict) or (None, None, None)."""
    for algo in ("p", "greedy", "m"):
        chosen = fit_select(net, budget, algo, winograd)
        if chosen is not None:
            break
    else:
        return None, None, None
    info = analyse(net)
    for _ in range(extra):
        rest = [b for b in fit_candidates(net) if b not in chosen]
        chosen.add(max(rest, key=lambda b: (info["nbytes"][b], -b)))
    r = simulate(net, "none", budget, algo, offload_set=chosen, winograd=winograd)
    if (fill_pm > 0 if windows is None else windows) and budget:
        r["trace"] = retime(r["trace"], budget, fill_pm, part_bytes)
        r.update(trace_stats(r["trace"]))
    return chosen, algo, r
