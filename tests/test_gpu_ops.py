"""GPU parity, single layers: every kernel behind the C ABI against the CPU oracle, element by
element, on seeded inputs whose sizes span several tiles and leave ragged tails."""
import numpy as np
import pytest

from oracle import layers as L
from tests.gpu_util import TOL, dev, host, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_1602_08124_amd import binding
    return binding


def _t(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape).astype(np.float32)


CONV_SHAPES = [
    # N, C, H, W, K, R, stride, pad
    (2, 3, 32, 32, 16, 3, 1, 1),      # 32-row tile, K-tail (27)
    (3, 16, 17, 19, 40, 3, 1, 1),     # 64-row tile, ragged pixel count (969)
    (2, 24, 20, 20, 136, 3, 1, 1),    # 128-row tile + ragged rows, reduction 216 (not a multiple of 16)
    (2, 3, 35, 35, 96, 11, 4, 0),     # AlexNet-style first layer
    (2, 8, 14, 14, 20, 5, 1, 2),      # 5x5
    (1, 16, 9, 9, 8, 1, 1, 0),        # 1x1
    (2, 3, 30, 30, 64, 7, 2, 3),      # GoogLeNet-style stem
    (1, 130, 7, 7, 260, 3, 1, 1),     # more rows than pixels, 3 row tiles
    (5, 4, 3, 3, 4, 3, 1, 1),         # tiny image
    (2, 6, 12, 12, 10, 3, 1, 0),      # no padding
    (2, 6, 12, 12, 10, 3, 1, 2),      # padding larger than usual (output grows)
    (2, 32, 20, 20, 136, 3, 1, 1),    # channels a multiple of 16: the packed-weight kernel, ragged row tile
    (3, 64, 14, 14, 80, 5, 1, 2),     # 5x5, packed-weight kernel both ways (C and K multiples of 16)
    (1, 48, 9, 9, 32, 1, 1, 0),       # 1x1
    (2, 16, 30, 30, 64, 7, 2, 3),     # strided forward on the packed-weight kernel
    (2, 16, 33, 31, 48, 3, 1, 1),     # 64-row tile, ragged pixels
    (1, 16, 3, 3, 16, 3, 1, 1),       # tiny image: every tap but the centre hits padding somewhere
    (2, 16, 12, 12, 38, 3, 1, 1),     # packed-weight kernel, rows not a multiple of 4 (one weight row per load), 64-row tile
    (2, 32, 10, 14, 134, 3, 1, 1),    # the same on the 128-row tile; backward-data on the 32-row tile
    (1, 256, 6, 6, 256, 3, 1, 1),     # two tiles, 144 K-steps: the split-reduction path with its fix-up, both directions
    (3, 32, 5, 7, 64, 3, 1, 1),       # odd pixel count per image (35): neighbouring pixels of a lane may lie in two images
]


def _ws(nbytes):
    import torch
    return torch.empty(max(nbytes, 4) // 4, device="cuda") if nbytes else None


@pytest.mark.parametrize("shape", CONV_SHAPES)
@pytest.mark.parametrize("relu,use_ws", [(False, False), (True, False), (False, True), (True, True)])
def test_conv_fwd(B, shape, relu, use_ws):
    """use_ws=False: the no-workspace algorithm; True: the packed-weight algorithm where it applies."""
    import torch
    n, c, h, w, k, r, st, pd = shape
    x, wt = _t((n, c, h, w), 1), _t((k, c, r, r), 2)
    ref = L.conv_fwd(x, wt, st, pd)
    if relu:
        ref = L.relu_fwd(ref)
    nbytes = B.op_conv_fwd_workspace(x.shape, wt.shape, st, pd)
    assert (nbytes >= wt.size * 4) if c % 16 == 0 else (nbytes == 0)
    y = torch.full(ref.shape, float("nan"), device="cuda")
    B.op_conv_fwd(dev(x), dev(wt), y, st, pd, relu, ws=_ws(nbytes) if use_ws else None)
    assert rel_err(host(y), ref) < TOL


@pytest.mark.parametrize("shape", CONV_SHAPES)
@pytest.mark.parametrize("use_ws", [False, True])
def test_conv_bwd_data(B, shape, use_ws):
    import torch
    n, c, h, w, k, r, st, pd = shape
    wt = _t((k, c, r, r), 3)
    p, q = L.out_dim(h, r, st, pd), L.out_dim(w, r, st, pd)
    dy = _t((n, k, p, q), 4)
    ref = L.conv_bwd_data(dy, wt, (n, c, h, w), st, pd)
    nbytes = B.op_conv_bwd_data_workspace((n, c, h, w), wt.shape, st, pd)
    assert (nbytes >= wt.size * 4) if (k % 16 == 0 and st == 1 and pd <= r - 1) else (nbytes == 0)
    dx = torch.full((n, c, h, w), float("nan"), device="cuda")
    B.op_conv_bwd_data(dev(dy), dev(wt), dx, st, pd, ws=_ws(nbytes) if use_ws else None)
    assert rel_err(host(dx), ref) < TOL
    # with the backward of a preceding in-place ReLU folded into the store
    xr = np.maximum(_t((n, c, h, w), 44), 0)
    dx.fill_(float("nan"))
    B.op_conv_bwd_data(dev(dy), dev(wt), dx, st, pd, ws=_ws(nbytes) if use_ws else None, relu_mask=dev(xr))
    assert rel_err(host(dx), L.relu_bwd(xr, ref)) < TOL


BWDF_EXTRA = [
    (8, 8, 64, 64, 16, 3, 1, 1),      # long reduction, split 16 ways
    (4, 20, 40, 40, 72, 3, 1, 1),
    # input channels a multiple of 64: the tap-uniform kernel, all four tile shapes
    (2, 128, 10, 10, 72, 3, 1, 1),    # 128x128 tiles, ragged rows
    (2, 128, 9, 9, 48, 3, 1, 1),      # 64x128
    (2, 64, 12, 12, 32, 3, 1, 1),     # 64x64
    (2, 64, 14, 14, 80, 3, 1, 1),     # 128x64, ragged rows
    (1, 192, 8, 8, 130, 1, 1, 0),     # 1x1, 128x64, two row tiles
    (2, 64, 15, 15, 64, 3, 2, 1),     # strided
    (6, 64, 40, 40, 64, 3, 1, 1),     # reduction 9600: split, ragged last chunk
]


@pytest.mark.parametrize("shape", CONV_SHAPES + BWDF_EXTRA)
def test_conv_bwd_filter(B, shape):
    import torch
    n, c, h, w, k, r, st, pd = shape
    x = _t((n, c, h, w), 5)
    p, q = L.out_dim(h, r, st, pd), L.out_dim(w, r, st, pd)
    dy = _t((n, k, p, q), 6)
    ref = L.conv_bwd_filter(x, dy, (k, c, r, r), st, pd)
    nbytes = B.op_conv_bwd_filter_workspace(x.shape, (k, c, r, r), st, pd)
    ws = torch.empty(max(nbytes, 4) // 4, device="cuda") if nbytes else None
    dw = torch.full((k, c, r, r), float("nan"), device="cuda")
    B.op_conv_bwd_filter(dev(x), dev(dy), dw, ws, st, pd)
    assert rel_err(host(dw), ref) < TOL
    # memory-optimal algorithm: no workspace, the reduction is not split
    dw.fill_(float("nan"))
    B.op_conv_bwd_filter(dev(x), dev(dy), dw, None, st, pd)
    assert rel_err(host(dw), ref) < TOL


NAMED = [(2, 32, 20, 20, 136, 3, 1, 1), (1, 256, 6, 6, 256, 3, 1, 1), (2, 256, 9, 9, 128, 3, 1, 1), (3, 64, 14, 14, 80, 5, 1, 2), (2, 3, 30, 30, 64, 7, 2, 3),
         (5, 256, 12, 12, 256, 3, 1, 1), (2, 256, 14, 14, 256, 3, 1, 1), (1, 256, 95, 93, 128, 3, 1, 1),
         (1, 128, 130, 126, 128, 3, 1, 1)]   # the last: planes too large for the LDS-staged F(4x4) input transform


@pytest.mark.parametrize("shape", NAMED)
def test_conv_kernels_by_name(B, shape):
    """Every kernel that applies to a shape, named explicitly and given exactly the workspace it asks for, against the
    oracle, for all three passes; the kernel the workspace-driven choice makes (VDNN_KERNEL_AUTO) is one of them, bit for bit."""
    import torch
    n, c, h, w, k, r, st, pd = shape
    x, wt = _t((n, c, h, w), 11), _t((k, c, r, r), 12)
    p, q = L.out_dim(h, r, st, pd), L.out_dim(w, r, st, pd)
    dy = _t((n, k, p, q), 13)
    refs = dict(fwd=L.conv_fwd(x, wt, st, pd), bwd_data=L.conv_bwd_data(dy, wt, x.shape, st, pd), bwd_filter=L.conv_bwd_filter(x, dy, wt.shape, st, pd))
    xd, wd, dyd = dev(x), dev(wt), dev(dy)
    _named_kernels_body(B, shape, x, wt, dy, refs, xd, wd, dyd)
    if n == 5:
        # a chunk size that leaves room for 2 images (F(2x2) forward and backward-data: 2 + 2 + 1) or for one at a time
        B.op_set_winograd_chunk_bytes(7 << 20)
        try:
            assert B.op_conv_workspace("fwd", "winograd", x.shape, wt.shape, st, pd) == 16 * c * k * 4 + 2 * 16 * (c + k) * 36 * 4
            assert B.op_conv_workspace("fwd", "winograd4", x.shape, wt.shape, st, pd) == 36 * c * k * 4 + 1 * 36 * (c + k) * 9 * 4
            _named_kernels_body(B, shape, x, wt, dy, refs, xd, wd, dyd, chunked=True)
        finally:
            B.op_set_winograd_chunk_bytes(0)


def _named_kernels_body(B, shape, x, wt, dy, refs, xd, wd, dyd, chunked=False):
    import torch
    n, c, h, w, k, r, st, pd = shape
    ran = 0
    for pass_ in ("fwd", "bwd_data", "bwd_filter"):
        results = {}
        for kernel in ("gather", "packed", "winograd", "winograd_small", "winograd4", "winograd4_small"):
            nbytes = B.op_conv_workspace(pass_, kernel, x.shape, wt.shape, st, pd)
            out = torch.full(refs[pass_].shape, float("nan"), device="cuda")
            ws = _ws(nbytes) if nbytes else None
            if nbytes is None:   # does not apply: refused, nothing written
                big = _ws(1 << 20)
                call = dict(fwd=lambda: B.try_op_conv_fwd(xd, wd, out, st, pd, ws=big, kernel=kernel),
                            bwd_data=lambda: B.try_op_conv_bwd_data(dyd, wd, out, st, pd, ws=big, kernel=kernel),
                            bwd_filter=lambda: B.try_op_conv_bwd_filter(xd, dyd, out, big, st, pd, kernel=kernel))[pass_]
                assert call() == B.ERR_INVALID_ARG and bool(torch.isnan(out).all())
                continue
            if pass_ == "fwd":
                B.op_conv_fwd(xd, wd, out, st, pd, ws=ws, kernel=kernel)
            elif pass_ == "bwd_data":
                B.op_conv_bwd_data(dyd, wd, out, st, pd, ws=ws, kernel=kernel)
            else:
                B.op_conv_bwd_filter(xd, dyd, out, ws, st, pd, kernel=kernel)
            results[kernel] = host(out)
            assert rel_err(results[kernel], refs[pass_]) < TOL, (pass_, kernel)
            ran += 1
        # 5 images run as chunks of 3 + 2 in the small-chunk forms
        assert "gather" in results and (n != 5 or chunked or ("winograd_small" in results and "winograd4_small" in results))
        assert "winograd4" in results or "winograd" not in results    # F(4x4) applies wherever F(2x2) does, and from 128 channels on
        for full in ("winograd", "winograd4"):
            if full + "_small" in results and pass_ != "bwd_filter":   # chunking only partitions the images: same bits
                assert np.array_equal(results[full + "_small"], results[full])
        fastest = [kk for kk in ("winograd4", "winograd4_small", "winograd", "winograd_small", "packed", "gather") if kk in results][0]
        nbytes = B.op_conv_workspace(pass_, fastest, x.shape, wt.shape, st, pd)
        out = torch.full(refs[pass_].shape, float("nan"), device="cuda")
        ws = _ws(nbytes) if nbytes else None
        if pass_ == "fwd":
            B.op_conv_fwd(xd, wd, out, st, pd, ws=ws)
        elif pass_ == "bwd_data":
            B.op_conv_bwd_data(dyd, wd, out, st, pd, ws=ws)
        else:
            B.op_conv_bwd_filter(xd, dyd, out, ws, st, pd)
        assert np.array_equal(host(out), results[fastest]), (pass_, fastest)
    assert ran >= 3


def test_conv_bwd_filter_is_split_and_deterministic(B):
    import torch
    shape = (8, 8, 64, 64, 16, 3, 1, 1)
    n, c, h, w, k, r, st, pd = shape
    nbytes = B.op_conv_bwd_filter_workspace((n, c, h, w), (k, c, r, r), st, pd)
    assert nbytes == 64 * k * c * r * r * 4  # reduction of 32768 in 64 pieces of 512
    x, dy = dev(_t((n, c, h, w), 7)), dev(_t((n, k, h, w), 8))
    outs = []
    for _ in range(3):
        ws = torch.empty(nbytes // 4, device="cuda")
        dw = torch.empty((k, c, r, r), device="cuda")
        B.op_conv_bwd_filter(x, dy, dw, ws, st, pd)
        outs.append(host(dw).copy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_conv_adjoint_identities_on_gpu(B):
    """<conv(X,W),dY> = <X,bwd_data(dY,W)> = <W,bwd_filter(X,dY)> with the GPU's own tensors (fp64 inner products)."""
    import torch
    n, c, h, w, k, r, st, pd = 4, 32, 28, 28, 48, 3, 1, 1
    x, wt, dy = dev(_t((n, c, h, w), 9)), dev(_t((k, c, r, r), 10)), dev(_t((n, k, h, w), 11))
    y = torch.empty((n, k, h, w), device="cuda")
    dx = torch.empty((n, c, h, w), device="cuda")
    dw = torch.empty((k, c, r, r), device="cuda")
    nbytes = B.op_conv_bwd_filter_workspace((n, c, h, w), (k, c, r, r), st, pd)
    ws = torch.empty(max(nbytes, 4) // 4, device="cuda")
    wsp = _ws(max(B.op_conv_fwd_workspace(x.shape, wt.shape, st, pd), B.op_conv_bwd_data_workspace(x.shape, wt.shape, st, pd)))
    B.op_conv_fwd(x, wt, y, st, pd, ws=wsp)
    B.op_conv_bwd_data(dy, wt, dx, st, pd, ws=wsp)
    B.op_conv_bwd_filter(x, dy, dw, ws, st, pd)
    a = np.vdot(host(y).astype(np.float64), host(dy).astype(np.float64))
    b = np.vdot(host(x).astype(np.float64), host(dx).astype(np.float64))
    cc = np.vdot(host(wt).astype(np.float64), host(dw).astype(np.float64))
    assert abs(a - b) < 1e-5 * abs(a) and abs(a - cc) < 1e-5 * abs(a)


@pytest.mark.parametrize("nio", [(8, 2048, 10), (5, 300, 130), (64, 4096, 256), (256, 1000, 384), (130, 520, 260)])
def test_fc(B, nio):
    import torch
    n, i, o = nio
    x, w, dy = _t((n, i), 12), _t((o, i), 13), _t((n, o), 14)

    def ws(which):
        nb = B.op_fc_workspace(n, i, o, which)
        return torch.empty(nb // 4, device="cuda") if nb else None
    # without workspace the reduction is not split: same result to rounding order
    y0 = torch.full((n, o), float("nan"), device="cuda")
    B.op_fc_fwd(dev(x), dev(w), y0, None)
    assert rel_err(host(y0), L.fc_fwd(x, w)) < TOL
    y = torch.full((n, o), float("nan"), device="cuda")
    B.op_fc_fwd(dev(x), dev(w), y, ws(0))
    assert rel_err(host(y), L.fc_fwd(x, w)) < TOL
    dx = torch.full((n, i), float("nan"), device="cuda")
    B.op_fc_bwd_data(dev(dy), dev(w), dx, ws(1))
    assert rel_err(host(dx), L.fc_bwd_data(dy, w, (n, i))) < TOL
    dw = torch.full((o, i), float("nan"), device="cuda")
    B.op_fc_bwd_filter(dev(x), dev(dy), dw, ws(2))
    assert rel_err(host(dw), L.fc_bwd_filter(x, dy)) < TOL


@pytest.mark.parametrize("count", [1, 3, 4, 1023, 4096 * 33 + 2])
def test_relu(B, count):
    x = _t((count,), 15)
    x[::7] = 0.0
    y = dev(x.copy())
    B.op_relu_fwd(y)
    ref = L.relu_fwd(x)
    assert np.array_equal(host(y), ref.astype(np.float32))
    g = _t((count,), 16)
    dy = dev(g.copy())
    B.op_relu_bwd(y, dy)
    assert np.array_equal(host(dy), L.relu_bwd(ref, g).astype(np.float32))


POOLS = [(2, 3, 8, 8, 2, 2, 0), (3, 5, 12, 20, 2, 2, 0), (2, 2, 6, 10, 2, 2, 0), (1, 2, 7, 8, 2, 2, 0), (2, 5, 13, 13, 3, 2, 0), (3, 4, 14, 14, 3, 2, 1), (2, 6, 7, 9, 3, 1, 1), (1, 2, 7, 7, 7, 1, 0),
         (2, 3, 55, 55, 3, 2, 0), (1, 3, 6, 6, 2, 2, 0), (2, 3, 9, 11, 3, 2, 2), (1, 2, 5, 5, 3, 1, 0), (2, 2, 3, 3, 3, 1, 1), (1, 1, 4, 7, 3, 2, 1),
         (2, 3, 28, 28, 3, 1, 1), (2, 3, 112, 112, 3, 2, 1), (1, 2, 3, 4, 3, 1, 2), (1, 2, 6, 5, 3, 2, 0), (3, 2, 27, 27, 3, 2, 0)]


@pytest.mark.parametrize("cfg", POOLS)
def test_maxpool(B, cfg):
    import torch
    n, c, h, w, k, st, pd = cfg
    x = _t((n, c, h, w), 17)
    x = np.maximum(x, 0)  # post-ReLU style input: plenty of ties at 0, the case the tie rule is for
    ref = L.maxpool_fwd(x, k, st, pd)
    y = torch.full(ref.shape, float("nan"), device="cuda")
    B.op_maxpool_fwd(dev(x), y, k, st, pd)
    assert np.array_equal(host(y), ref.astype(np.float32))
    dy = _t(ref.shape, 18)
    dx = torch.full(x.shape, float("nan"), device="cuda")
    B.op_maxpool_bwd(dev(x), dev(dy), dx, k, st, pd)
    assert rel_err(host(dx), L.maxpool_bwd(x, dy, k, st, pd)) < 1e-6
    dx.fill_(float("nan"))
    B.op_maxpool_bwd(dev(x), dev(dy), dx, k, st, pd, relu_mask=True)
    assert rel_err(host(dx), L.relu_bwd(x, L.maxpool_bwd(x, dy, k, st, pd))) < 1e-6
    # ties everywhere (few distinct values, many zeros as after a ReLU): the first maximum of a window wins
    xt = np.maximum(np.round(x * 2.0), 0.0).astype(np.float32)
    B.op_maxpool_bwd(dev(xt), dev(dy), dx, k, st, pd)
    assert rel_err(host(dx), L.maxpool_bwd(xt, dy, k, st, pd)) < 1e-6


@pytest.mark.parametrize("cfg", POOLS)
def test_avgpool(B, cfg):
    import torch
    n, c, h, w, k, st, pd = cfg
    x = _t((n, c, h, w), 19)
    ref = L.avgpool_fwd(x, k, st, pd)
    y = torch.full(ref.shape, float("nan"), device="cuda")
    B.op_avgpool_fwd(dev(x), y, k, st, pd)
    assert rel_err(host(y), ref) < 1e-6
    dy = _t(ref.shape, 20)
    dx = torch.full(x.shape, float("nan"), device="cuda")
    B.op_avgpool_bwd(dev(dy), dx, k, st, pd)
    assert rel_err(host(dx), L.avgpool_bwd(dy, x.shape, k, st, pd)) < 1e-6


@pytest.mark.parametrize("nc", [(8, 10), (256, 1000), (3, 1000), (17, 65), (1, 2)])
def test_softmax_ce(B, nc):
    import torch
    n, classes = nc
    z = _t((n, classes), 21) * 3
    lab = np.random.default_rng(22).integers(0, classes, n).astype(np.int32)
    loss_ref, dz_ref = L.softmax_ce(z, lab)
    loss = torch.full((1,), float("nan"), device="cuda")
    B.op_softmax_ce_fwd(dev(z), dev(lab), loss)
    assert abs(host(loss)[0] - loss_ref) < TOL * abs(loss_ref)
    dz = torch.full((n, classes), float("nan"), device="cuda")
    B.op_softmax_ce_bwd(dev(z), dev(lab), dz)
    assert rel_err(host(dz), dz_ref) < TOL
    # zero logits: the loss is ln(classes)
    B.op_softmax_ce_fwd(dev(np.zeros((n, classes), np.float32)), dev(lab), loss)
    assert abs(host(loss)[0] - np.log(classes)) < 1e-6 * np.log(classes) + 1e-7


def test_concat_and_add(B):
    import torch
    n, hw = 3, 35
    parts = [_t((n, c, 5, 7), 30 + c) for c in (3, 8, 1)]
    big = torch.full((n, 12, 5, 7), float("nan"), device="cuda")
    off = 0
    for p in parts:
        B.op_concat_copy(dev(p), big, n, p.shape[1], 12, off, hw, True)
        off += p.shape[1]
    ref = np.concatenate(parts, axis=1)
    assert np.array_equal(host(big), ref)
    off = 0
    for p in parts:
        small = torch.full(p.shape, float("nan"), device="cuda")
        B.op_concat_copy(big, small, n, p.shape[1], 12, off, hw, False)
        assert np.array_equal(host(small), p)
        off += p.shape[1]
    a, b = _t((1000,), 40), _t((1000,), 41)
    acc = dev(a.copy())
    B.op_add(acc, dev(b))
    assert np.array_equal(host(acc), a + b)


def test_invalid_arguments_are_rejected(B):
    import torch
    x = torch.zeros(16, device="cuda")
    lib = B.lib
    assert lib.vdnn_op_conv_fwd(None, x.data_ptr(), x.data_ptr(), None, 0, 1, 1, 4, 4, 1, 3, 3, 1, 1, 0, -1, None) == B.ERR_INVALID_ARG
    assert lib.vdnn_op_conv_fwd(x.data_ptr(), x.data_ptr(), x.data_ptr(), None, 0, 1, 1, 2, 2, 1, 5, 5, 1, 0, 0, -1, None) == B.ERR_INVALID_ARG
    # a kernel id out of range, a kernel that does not apply to the shape (C = 1: gather only), a workspace too small for the kernel named
    assert lib.vdnn_op_conv_fwd(x.data_ptr(), x.data_ptr(), x.data_ptr(), None, 0, 1, 1, 4, 4, 1, 3, 3, 1, 1, 0, 3, None) == B.ERR_INVALID_ARG
    assert lib.vdnn_op_conv_fwd(x.data_ptr(), x.data_ptr(), x.data_ptr(), None, 0, 1, 1, 4, 4, 1, 3, 3, 1, 1, 0, B.KERNEL["packed"], None) == B.ERR_INVALID_ARG
    xs, ws = (2, 16, 8, 8), (16, 16, 3, 3)
    assert B.op_conv_workspace("fwd", "packed", xs, ws, 1, 1) > 64
    xx, wt, yy = torch.zeros(xs, device="cuda"), torch.zeros(ws, device="cuda"), torch.zeros((2, 16, 8, 8), device="cuda")
    assert B.try_op_conv_fwd(xx, wt, yy, 1, 1, ws=x, kernel="packed") == B.ERR_INVALID_ARG
    assert B.try_op_conv_bwd_data(yy, wt, xx, 1, 1, ws=x, kernel="packed") == B.ERR_INVALID_ARG
    assert B.try_op_conv_bwd_filter(xx, yy, wt, x, 1, 1, kernel="packed") == B.ERR_INVALID_ARG
    assert lib.vdnn_op_maxpool_fwd(x.data_ptr(), x.data_ptr(), 1, 1, 4, 4, 2, 0, 0, None) == B.ERR_INVALID_ARG
    assert lib.vdnn_op_conv_bwd_filter(x.data_ptr(), None, x.data_ptr(), None, 0, 8, 8, 64, 64, 16, 3, 3, 1, 1, -1, None) == B.ERR_INVALID_ARG
    # tensors of 2^31 - 1 elements or more are refused before anything is launched (kernels index with 32 bits)
    big = (64, 32, 1024, 1024)   # 2^31 elements
    p = x.data_ptr()
    assert lib.vdnn_op_conv_fwd(p, p, p, None, 0, *big, 1, 3, 3, 1, 1, 0, -1, None) == B.ERR_INVALID_ARG
    assert lib.vdnn_op_conv_bwd_data(p, p, p, None, 0, *big, 1, 3, 3, 1, 1, None, -1, None) == B.ERR_INVALID_ARG
    assert lib.vdnn_op_conv_bwd_filter(p, p, p, None, 0, *big, 1, 3, 3, 1, 1, -1, None) == B.ERR_INVALID_ARG
    assert lib.vdnn_op_conv_fwd(p, p, p, None, 0, 1, 1, 1024, 1024, 2048, 3, 3, 1, 1, 0, -1, None) == B.ERR_INVALID_ARG   # the output is what is too large
    assert lib.vdnn_op_maxpool_fwd(p, p, *big, 2, 2, 0, None) == B.ERR_INVALID_ARG
    assert lib.vdnn_op_maxpool_bwd(p, p, p, *big, 2, 2, 0, 0, None) == B.ERR_INVALID_ARG


def _random_conv_shapes(count, seed, wide=False):
    """wide: windows up to 11, stride up to 4, images up to 39 pixels a side, channel counts up to 384 on either side,
    at most 3e9 multiply-adds per pass."""
    r = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        k_sz = int(r.choice([1, 2, 3, 3, 3, 3, 4, 5, 7, 11] if wide else [1, 2, 3, 3, 3, 5, 7]))
        st = int(r.choice([1, 1, 1, 2, 3, 4] if wide else [1, 1, 1, 2, 3]))
        pd = int(r.integers(0, k_sz))
        c = int(r.choice([1, 2, 3, 4, 8, 15, 16, 17, 32, 48, 64, 96, 100, 128, 160, 256, 272, 384] if wide else [1, 3, 5, 16, 24, 32, 48, 64, 80, 128]))
        k = int(r.choice([1, 2, 4, 7, 16, 31, 32, 33, 64, 65, 96, 128, 130, 256, 260, 384] if wide else [1, 7, 16, 33, 64, 96, 130]))
        h, w = (int(r.integers(1, 40)), int(r.integers(1, 40))) if wide else (int(r.integers(1, 25)), int(r.integers(1, 25)))
        n = int(r.integers(1, 6 if wide else 5))
        if h + 2 * pd < k_sz or w + 2 * pd < k_sz:
            continue
        if wide and n * c * h * w * k * k_sz * k_sz > 3e9:
            continue
        out.append((n, c, h, w, k, k_sz, st, pd))
    return out


@pytest.mark.parametrize("shape", _random_conv_shapes(48, 20260101) + _random_conv_shapes(64, 20260102, wide=True), ids=lambda s: "x".join(map(str, s)))
def test_conv_random_shapes(B, shape):
    """Seeded random geometry (odd sizes, one-pixel images, even windows, stride 3, channel counts on both sides of
    every tile and algorithm boundary): all three convolution passes, with and without workspace."""
    import torch
    n, c, h, w, k, r, st, pd = shape
    x, wt = _t((n, c, h, w), 51), _t((k, c, r, r), 52)
    p, q = L.out_dim(h, r, st, pd), L.out_dim(w, r, st, pd)
    dy = _t((n, k, p, q), 53)
    ref_y = L.conv_fwd(x, wt, st, pd)
    ref_dx = L.conv_bwd_data(dy, wt, x.shape, st, pd)
    ref_dw = L.conv_bwd_filter(x, dy, wt.shape, st, pd)
    xd, wd, dyd = dev(x), dev(wt), dev(dy)
    for use_ws in (False, True):
        y = torch.full(ref_y.shape, float("nan"), device="cuda")
        B.op_conv_fwd(xd, wd, y, st, pd, False, ws=_ws(B.op_conv_fwd_workspace(x.shape, wt.shape, st, pd)) if use_ws else None)
        assert rel_err(host(y), ref_y) < TOL
        dx = torch.full(x.shape, float("nan"), device="cuda")
        B.op_conv_bwd_data(dyd, wd, dx, st, pd, ws=_ws(B.op_conv_bwd_data_workspace(x.shape, wt.shape, st, pd)) if use_ws else None)
        assert rel_err(host(dx), ref_dx) < TOL
        dw = torch.full(wt.shape, float("nan"), device="cuda")
        B.op_conv_bwd_filter(xd, dyd, dw, _ws(B.op_conv_bwd_filter_workspace(x.shape, wt.shape, st, pd)) if use_ws else None, st, pd)
        assert rel_err(host(dw), ref_dw) < TOL


# ---- Winograd F(2x2,3x3): layers wide enough for the library to choose it (256 or more channels on both sides) ----
WINO_SHAPES = [
    # N, C, H, W, K
    (2, 256, 8, 8, 512),     # forward: 256 -> 512; backward-data: 512 -> 256
    (1, 512, 6, 10, 256),    # 15 tiles per image (odd), non-square image
    (3, 512, 4, 4, 512),     # four tiles per image
    (2, 272, 2, 2, 512),     # one tile per image; backward-data has a ragged row tile (272 rows); channels not a multiple of 32
    (2, 256, 13, 13, 384),   # odd sides (AlexNet's last layers): the last tile row and column hang over the edge
    (1, 384, 7, 10, 256),    # odd height, even width
    (2, 256, 6, 5, 256),     # even height, odd width
    (1, 256, 1, 1, 256),     # a single pixel: one tile, three of its four outputs dropped
]


def _wino_case(B, shape, chunk_bytes=0):
    import torch
    n, c, h, w, k = shape
    x, wt = _t((n, c, h, w), 61), _t((k, c, 3, 3), 62)
    dy = _t((n, k, h, w), 63)
    xr = np.maximum(_t((n, c, h, w), 64), 0)
    ref_y = L.conv_fwd(x, wt, 1, 1)
    ref_dx = L.conv_bwd_data(dy, wt, x.shape, 1, 1)
    ref_dw = L.conv_bwd_filter(x, dy, wt.shape, 1, 1)
    B.op_set_winograd_chunk_bytes(chunk_bytes)
    try:
        nf = B.op_conv_fwd_workspace(x.shape, wt.shape, 1, 1)
        nb = B.op_conv_bwd_data_workspace(x.shape, wt.shape, 1, 1)
        # the transformed filter alone is 16/9 of W: the Winograd workspace, not the packed-weight one
        assert nf > 16 * wt.size * 4 // 9 and (nb > 16 * wt.size * 4 // 9 or k < 256)
        for relu in (False, True):
            y = torch.full(ref_y.shape, float("nan"), device="cuda")
            B.op_conv_fwd(dev(x), dev(wt), y, 1, 1, relu, ws=_ws(nf))
            assert rel_err(host(y), np.maximum(ref_y, 0) if relu else ref_y) < TOL
        dx = torch.full(x.shape, float("nan"), device="cuda")
        B.op_conv_bwd_data(dev(dy), dev(wt), dx, 1, 1, ws=_ws(nb))
        assert rel_err(host(dx), ref_dx) < TOL
        dx.fill_(float("nan"))
        B.op_conv_bwd_data(dev(dy), dev(wt), dx, 1, 1, ws=_ws(nb), relu_mask=dev(xr))
        assert rel_err(host(dx), L.relu_bwd(xr, ref_dx)) < TOL
        nw = B.op_conv_bwd_filter_workspace(x.shape, wt.shape, 1, 1)
        if c % 128 == 0 and k >= 256:
            assert nw > 2 * 16 * wt.size * 4 // 9   # the 16 products and at least one copy of partial sums
        dw = torch.full(wt.shape, float("nan"), device="cuda")
        B.op_conv_bwd_filter(dev(x), dev(dy), dw, _ws(nw), 1, 1)
        assert rel_err(host(dw), ref_dw) < TOL
        return nf, nb
    finally:
        B.op_set_winograd_chunk_bytes(0)


@pytest.mark.parametrize("shape", WINO_SHAPES)
def test_conv_winograd(B, shape):
    _wino_case(B, shape)


def test_conv_winograd_in_chunks(B):
    """A chunk size that leaves room for two images of five beside the transformed filter (chunks of 2, 2 and 1) and one that
    holds a single image (F(4x4, 3x3), the fastest kernel for the shape: 2 x 2 tiles of 36 products per image)."""
    shape = (5, 256, 8, 8, 512)
    per_image = 36 * (256 + 512) * 4 * 4
    whole, _ = _wino_case(B, shape)
    assert whole == 36 * 256 * 512 * 4 + 5 * per_image
    two, _ = _wino_case(B, shape, chunk_bytes=36 * 256 * 512 * 4 + 2 * per_image + 100)
    one, _ = _wino_case(B, shape, chunk_bytes=per_image // 2)   # smaller than one image: still one image per chunk
    assert whole - two == 3 * per_image and two - one == per_image


def test_conv_workspace_levels(B):
    """With room for the packed weights only, a Winograd-sized layer runs the packed-weight kernel; with less, the
    no-workspace kernel: all three agree with the oracle."""
    import torch
    n, c, h, w, k = 2, 256, 8, 8, 512
    x, wt = _t((n, c, h, w), 71), _t((k, c, 3, 3), 72)
    ref = L.conv_fwd(x, wt, 1, 1)
    full = B.op_conv_fwd_workspace(x.shape, wt.shape, 1, 1)
    outs = []
    assert full > 9 << 20  # 8.4 MB of transformed filter + 0.8 MB per image
    for nbytes in (full, 8 << 20, 1024):  # 8 MiB: room for the packed weights (4.7 MB) and the split tiles' partial sums (2 MB)
        y = torch.full(ref.shape, float("nan"), device="cuda")
        B.op_conv_fwd(dev(x), dev(wt), y, 1, 1, False, ws=_ws(nbytes))
        assert rel_err(host(y), ref) < TOL
        outs.append(host(y))
    assert not np.array_equal(outs[0], outs[1])  # different algorithms, different rounding


def test_conv_winograd_is_deterministic(B):
    """No atomics anywhere in the Winograd path (partial sums and image chunks are added in a fixed order): two runs of
    each pass give the same bits, chunked or not."""
    import torch
    n, c, h, w, k = 5, 256, 8, 8, 384
    x, wt, dy = dev(_t((n, c, h, w), 81)), dev(_t((k, c, 3, 3), 82)), dev(_t((n, k, h, w), 83))
    for chunk in (0, 2 * 16 * (c + k) * 16 * 4 + 64):
        B.op_set_winograd_chunk_bytes(chunk)
        try:
            runs = []
            for _ in range(2):
                y = torch.empty((n, k, h, w), device="cuda")
                dx = torch.empty((n, c, h, w), device="cuda")
                dw = torch.empty((k, c, 3, 3), device="cuda")
                B.op_conv_fwd(x, wt, y, 1, 1, True, ws=_ws(B.op_conv_fwd_workspace(x.shape, wt.shape, 1, 1)))
                B.op_conv_bwd_data(dy, wt, dx, 1, 1, ws=_ws(B.op_conv_bwd_data_workspace(x.shape, wt.shape, 1, 1)))
                B.op_conv_bwd_filter(x, dy, dw, _ws(B.op_conv_bwd_filter_workspace(x.shape, wt.shape, 1, 1)), 1, 1)
                runs.append((host(y), host(dx), host(dw)))
            for a, b in zip(*runs):
                assert np.array_equal(a, b)
        finally:
            B.op_set_winograd_chunk_bytes(0)
