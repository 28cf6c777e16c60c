"""What the memory-schedule oracle says a library net planned with transfer windows should look like."""
from oracle import memsched as ms


def assert_windows_match(lib_trace, ref_trace, lent=None, twins=None, hoisted=True):
    """lib_trace: the library's (where, kind, tag, bytes, offset) trace; ref_trace: the oracle's retimed trace
    (forward windows; fetches at their static place).  Everything except how early fetches are issued must be
    equal; a fetch may only move earlier, fetches keep their order, and tenants / twins sit at the address the
    host's range dictates."""
    lib_rest, lib_f = ms.settle_fetches([t[:4] for t in lib_trace])
    ref_rest, ref_f = ms.settle_fetches([tuple(t) for t in ref_trace])
    assert lib_rest == ref_rest
    assert [f[0] for f in lib_f] == [f[0] for f in ref_f]               # same fetches, same order
    assert all(a[1] <= b[1] for a, b in zip(lib_f, ref_f))              # none later than the static schedule
    if not hoisted:
        assert lib_f == ref_f
    addr = {}
    for t in lib_trace:
        if t[1] == "alloc":
            addr.setdefault(t[2], []).append(t[4])
    for tenant, (host, rel) in (lent or {}).items():
        assert addr[tenant][0] == addr[host][0] + rel, (tenant, host)
    for host in twins or ():
        first = addr[host][0]
        back = [a for tag, al in addr.items() if tag.split("#")[0] == host for a in (al[1:] if tag == host else al)]
        assert back and min(back) == first, host                           # the fetch starts where the block was
    return lib_f, ref_f


def fit_reference(n, net, budget, part=None):
    """n: a binding.Net on which set_policy("fit") succeeded.  The oracle's choice of offload set may be
    extended by the library where no placement of the blocks fits the budget (largest remaining candidates
    first); how many were added, and how far the forward windows fill the budget, is read from n.
    Returns (offload set, algorithm mode, oracle result, lent, twins)."""
    part = ms.PART_BYTES if part is None else part
    chosen, _, _ = ms.fit(net, budget or 1 << 50, 0)
    extra = len(n.offload_set()) - len(chosen)
    assert extra >= 0, (n.offload_set(), chosen)
    st = n.stats()
    assert st["window_fill_pm"] in ms.FILLS_PM and st["window_fill_bwd_pm"] in (0, 1000)
    windows = bool(budget) and (st["window_fill_pm"] > 0 or st["window_fill_bwd_pm"] > 0)
    lent, twins = {}, set()
    chosen, algo, base = ms.fit(net, budget or 1 << 50, 0, part, extra, windows=False)
    if windows:
        base["trace"] = ms.retime(base["trace"], budget, st["window_fill_pm"], part, lent, twins)
        base.update(ms.trace_stats(base["trace"]))
    return chosen, algo, base, lent, twins
