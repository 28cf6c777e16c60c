"""What the memory-schedule oracle says a library net planned under the "fit" policy should look like."""
from oracle import memsched as ms


def fit_reference(n, net, budget, part=None):
    """n: a binding.Net on which set_policy("fit") succeeded.  The oracle's choice of offload set may be
    extended by the library where no placement of the blocks fits the budget (largest remaining candidates
    first); how many were added, and how far the transfer windows fill the budget, is read from n.
    Returns (offload set, algorithm mode, oracle result)."""
    part = ms.PART_BYTES if part is None else part
    chosen, _, _ = ms.fit(net, budget or 1 << 50, 0)
    extra = len(n.offload_set()) - len(chosen)
    assert 0 <= extra <= 3, (n.offload_set(), chosen)
    st = n.stats()
    assert st["window_fill_pm"] in ms.FILLS_PM and st["window_fill_bwd_pm"] in ms.FILLS_PM
    return ms.fit(net, budget or 1 << 50, st["window_fill_pm"], part, extra, st["window_fill_bwd_pm"])
