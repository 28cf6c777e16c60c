"""Checks of a planned training step that hold whatever produced it.

The library reports its plan as an op trace (vdnn_trace): (where, kind, tag, bytes, offset) for alloc / free,
(where, kind, tag, bytes) for offload / prefetch / ondemand, (where, "compute", layer type).  For the paper's own
policies the trace has to EQUAL the memory-schedule oracle's (oracle/memsched.py).  For schedules that go beyond the
paper (transfer windows, blocks moved in pieces, fetches issued early, an offload set chosen per feature map) there is
no such definition to compare with; what there is, is the contract any valid vDNN schedule keeps (Sections 3.1, 3.2):

  1. no two live blocks share an address, and everything lies inside the pool;
  2. live bytes never pass the budget;
  3. the computations run layer by layer, forward 0 .. L-1, then backward L-1 .. 0;
  4. whatever a computation reads or writes is resident when it runs, and holds valid contents: a feature map that
     left the GPU has been copied to the host in full before any of it was released, and copied back in full before
     its first backward reader;
  5. a feature map is offloaded at most once, by its last forward consumer (Fig. nonlinear_dfg), and exactly the
     feature maps of the offload set are;
  6. every offloaded byte is fetched exactly once; feature maps come back in the reverse of the order they left in;
  7. at the end of the step only the persistent blocks (W, dW, labels, loss) are live.
"""
from oracle import memsched as ms


def lib_ws(n, net):
    """The workspace sizes the library reports for its kernels, in the form the oracle takes them as a parameter."""
    ws = {}
    for i in range(len(net["layers"])):
        for phase in ("fwd", "bwd"):
            opts = n.workspace_options(i, phase == "bwd")
            if opts:
                ws[i, phase] = opts
    return ws


def check_placement(trace, budget):
    """Every allocated range lies inside the pool and meets no live range; every release gives back ranges
    that are live under the same block tag.  A block that moves in pieces ("B3#2") is allocated whole and
    released piece by piece, or the other way round; the pieces must tile the block's range exactly.
    Returns {tag: [(offset, size)]} of what is still live."""
    live = {}
    for t in trace:
        if t[1] not in ("alloc", "free"):
            continue
        tag, size, off = t[2].split("#")[0], t[3], t[4]
        if t[1] == "alloc":
            assert off % 256 == 0 and off + size <= budget, t
            for tag2, ranges in live.items():
                for o2, s2 in ranges:
                    assert off + size <= o2 or o2 + s2 <= off, (t, tag2)
            live.setdefault(tag, []).append((off, size))
        elif t[1] == "free":
            ranges = sorted(live.pop(tag))
            assert all(a[0] + a[1] == b[0] for a, b in zip(ranges, ranges[1:])), (t, ranges)   # contiguous
            lo, hi = ranges[0][0], ranges[-1][0] + ranges[-1][1]
            assert lo <= off and off + size <= hi, (t, ranges)
            rest = [(a, b - a) for a, b in ((lo, off), (off + size, hi)) if b > a]
            # pieces are released in address order from the bottom of the block, or the block goes as a whole
            assert len(rest) <= 1, (t, ranges)
            if rest:
                live[tag] = rest
    return live


def check_schedule(net, trace, budget, offload_set, persistent_bytes):
    """Asserts properties 1-7 of the module docstring on a library trace.  Returns trace_stats(trace)."""
    info = ms.analyse(net)
    layers = net["layers"]
    nl = len(layers)
    nbytes = info["nbytes"]
    offload_set = set(offload_set)

    # 1, 7
    left = check_placement(trace, budget)
    assert sum(s for r in left.values() for _, s in r) == persistent_bytes
    assert all(not tag.startswith(("B", "dB", "T", "WS")) for tag in left), sorted(left)

    # 3
    computes = [t[0] for t in trace if t[1] == "compute"]
    assert computes == ["F%d" % i for i in range(nl)] + ["B%d" % i for i in range(nl - 1, -1, -1)]

    def buf_of_tag(tag):
        return int(tag.split("#")[0][1:])

    def in_bufs(i):
        return list(dict.fromkeys(info["bufof"](j) for j in layers[i]["inputs"]))

    live = 0
    resident = {}                      # block tag without piece suffix -> bytes currently allocated under it
    size_al = {b: ms._al(v) for b, v in nbytes.items()}
    produced = set([-1])               # feature maps whose contents exist somewhere (GPU or host)
    on_host_bytes = {}                 # buffer -> raw bytes whose offload has been issued
    away = set()                       # buffers that have (partly) left the GPU and are not back in full
    fetched_bytes = {}                 # buffer -> raw bytes whose fetch has been issued since it left
    offload_order, fetch_order = [], []
    seen_pieces = set()
    computed = set()                   # where-labels of the computations seen so far

    def full(b):
        return resident.get("B%d" % b, 0) == size_al[b]

    def readable(b):
        return b in produced and full(b) and b not in away

    for t in trace:
        where, kind = t[0], t[1]
        if kind == "alloc":
            live += t[3]
            assert live <= budget, t                                                    # 2
            base = t[2].split("#")[0]
            resident[base] = resident.get(base, 0) + t[3]
        elif kind == "free":
            live -= t[3]
            base = t[2].split("#")[0]
            resident[base] -= t[3]
            assert resident[base] >= 0, t
            if base[0] == "B" and buf_of_tag(base) in nbytes:
                b = buf_of_tag(base)
                if b in offload_set and b not in fetch_order:
                    # 4: the copy that forward propagation made leaves the pool (in forward propagation, or, with transfer
                    # windows, early in backward propagation): only once the host has all of it
                    assert on_host_bytes.get(b, 0) == nbytes[b], t
                    away.add(b)
                    fetched_bytes.setdefault(b, 0)
                elif where[0] == "F":
                    # 4: anything else released in forward propagation is something no backward computation reads
                    assert not ms.bwd_users(net, info, b), t
        elif kind == "offload":
            b = buf_of_tag(t[2])
            assert (kind, t[2]) not in seen_pieces, t                                   # 5: once
            seen_pieces.add((kind, t[2]))
            assert b in offload_set, t
            assert where == "F%d" % info["readers"][b][-1], t                           # 5: by the last forward consumer
            assert where not in computed, t                                             # ... overlapped with it: issued before it runs
            assert readable(b), t
            if b not in offload_order:
                offload_order.append(b)
            on_host_bytes[b] = on_host_bytes.get(b, 0) + t[3]
        elif kind in ("prefetch", "ondemand"):
            b = buf_of_tag(t[2])
            assert (kind if kind == "prefetch" else "prefetch", t[2]) not in seen_pieces, t   # 6: once
            seen_pieces.add(("prefetch", t[2]))
            assert b in away and where[0] == "B", t
            assert resident.get("B%d" % b, 0) <= size_al[b], t     # the forward copy has gone completely before any of it returns
            if b not in fetch_order:
                fetch_order.append(b)
            fetched_bytes[b] += t[3]
            assert fetched_bytes[b] <= nbytes[b], t
            if fetched_bytes[b] == nbytes[b]:
                assert full(b), t
                away.discard(b)
        elif kind == "compute":
            computed.add(where)
            i = int(where[1:])
            layer = layers[i]
            typ = layer["type"]
            own = info["buf"][i]
            if where[0] == "F":
                for b in in_bufs(i):
                    assert readable(b), (t, b)                                          # 4
                if typ != "softmax_ce":
                    assert full(own), t
                    produced.add(own)
            else:
                if typ in ms.IN_PLACE:
                    assert readable(own), t
                elif typ in ms.NEEDS_X_IN_BWD:
                    for b in in_bufs(i):
                        assert readable(b), (t, b)
                if typ != "softmax_ce":
                    assert resident.get("dB%d" % own, 0) == size_al[own], t            # dY
                if typ not in ms.IN_PLACE:
                    for b in in_bufs(i):
                        if b >= 0:
                            assert resident.get("dB%d" % b, 0) == size_al[b], (t, b)    # dX (or the sum it is added to)
    assert live == persistent_bytes
    assert set(offload_order) == offload_set                                            # 5: exactly the set
    assert all(on_host_bytes[b] == nbytes[b] for b in offload_set)
    assert fetch_order == offload_order[::-1]                                           # 6
    assert not away
    return ms.trace_stats([t[:4] for t in trace])
