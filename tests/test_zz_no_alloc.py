"""The entry point that allocates nothing: vdnn_op_conv_bwd_filter_static runs the backward-filter kernels on the library's
static device buffer.  Checked through the C ABI against vdnn_op_conv_bwd_filter (same kernel, caller's workspace) bit for
bit, and against the CPU oracle, on calls in a row that share the buffer, each smaller than the one before."""
import numpy as np
import pytest

from oracle import layers as L
from tests.gpu_util import TOL, host, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_1602_08124_amd import binding
    return binding


# (N, C, H, W, K, kernel the shape resolves to): a split reduction over 25 088 pixels, the Winograd form, a small packed
# case, a shape only the gather kernel takes -- in this order, so that each call finds the leftovers of a larger one
CALLS = [(8, 64, 56, 56, 64, "packed"), (4, 256, 14, 14, 256, "winograd4"), (2, 32, 14, 14, 48, "packed"), (3, 5, 9, 7, 6, "gather")]
FASTEST_FIRST = ("winograd4", "winograd4_small", "winograd", "winograd_small", "packed", "gather")


def test_static_scratch_backward_filter(B):
    import torch
    g = torch.Generator(device="cuda").manual_seed(77)
    ws = torch.empty(B.STATIC_SCRATCH_BYTES // 4, device="cuda")
    for n, c, h, w, k, kernel in CALLS:
        x = torch.randn((n, c, h, w), device="cuda", generator=g)
        dy = torch.randn((n, k, h, w), device="cuda", generator=g)
        need = B.op_conv_workspace("bwd_filter", kernel, x.shape, (k, c, 3, 3), 1, 1)
        assert need is not None and need <= B.STATIC_SCRATCH_BYTES
        for better in FASTEST_FIRST[:FASTEST_FIRST.index(kernel)]:
            assert B.op_conv_workspace("bwd_filter", better, x.shape, (k, c, 3, 3), 1, 1) is None   # `kernel` is the fastest that applies
        want = torch.full((k, c, 3, 3), float("nan"), device="cuda")
        ws.fill_(float("nan"))
        B.op_conv_bwd_filter(x, dy, want, ws, 1, 1, kernel=kernel)
        for how in ("auto", kernel):
            got = torch.full((k, c, 3, 3), float("nan"), device="cuda")
            B.op_conv_bwd_filter_static(x, dy, got, 1, 1, kernel=how)
            assert np.array_equal(host(got), host(want)), (n, c, h, w, k, how)
        ref = L.conv_bwd_filter(host(x), host(dy), (k, c, 3, 3), 1, 1)
        assert rel_err(host(got), ref) < TOL, (n, c, h, w, k)
    # a kernel whose workspace does not fit the static buffer is refused before anything is launched
    x = torch.randn((64, 512, 28, 28), device="cuda", generator=g)
    dy = torch.randn((64, 512, 28, 28), device="cuda", generator=g)
    dw = torch.zeros((512, 512, 3, 3), device="cuda")
    assert B.op_conv_workspace("bwd_filter", "winograd4", x.shape, dw.shape, 1, 1) > B.STATIC_SCRATCH_BYTES
    assert B.try_op_conv_bwd_filter_static(x, dy, dw, 1, 1) == B.ERR_INVALID_ARG
    assert "static buffer holds" in B.lib.vdnn_op_last_error().decode()
    assert float(dw.abs().max()) == 0.0
    # a kernel that does not apply to the shape, and a kernel id out of range
    small = torch.randn((3, 5, 9, 7), device="cuda", generator=g)
    assert B.try_op_conv_bwd_filter_static(small, torch.randn((3, 6, 9, 7), device="cuda", generator=g), torch.zeros((6, 5, 3, 3), device="cuda"),
                                           1, 1, kernel="winograd") == B.ERR_INVALID_ARG
    # the packed kernel fits for the large shape and is what the caller can fall back to
    assert B.op_conv_workspace("bwd_filter", "packed", x.shape, dw.shape, 1, 1) <= B.STATIC_SCRATCH_BYTES
    B.op_conv_bwd_filter_static(x, dy, dw, 1, 1, kernel="packed")
    want = torch.empty_like(dw)
    B.op_conv_bwd_filter(x, dy, want, ws, 1, 1, kernel="packed")
    assert np.array_equal(host(dw), host(want))
