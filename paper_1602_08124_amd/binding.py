"""Thin ctypes binding over include/vdnn.h: same names, argument marshalling only.

PyTorch is used for device memory and streams (the pool tensor and two torch streams that the
library borrows); every computation runs in the library's own kernels.  There is no fallback:
if libvdnn.so is missing, importing this module raises.
"""
import ctypes as C
import os

# PyTorch ships its own copy of the HIP runtime (same SONAME as the system one).  It has to be in the
# process BEFORE libvdnn.so is loaded, so that the library binds to that same runtime instance; in the
# other order the process ends up with two runtimes and the pool and streams borrowed from torch
# would belong to a different one than the library's kernels are launched with.
try:
    import torch  # noqa: F401
except ImportError:  # a pure C / ctypes user without torch: the system runtime is the only one
    torch = None

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libvdnn.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libvdnn.so is not built: run `python -m paper_1602_08124_amd.build` first (%s)" % LIB_PATH)
lib = C.CDLL(LIB_PATH)

OK, ERR_INVALID_ARG, ERR_OOM_DEVICE, ERR_OOM_HOST, ERR_HIP, ERR_STATE, ERR_UNSUPPORTED = range(7)
POLICY = {"none": 0, "all": 1, "conv": 2, "dyn": 3, "fit": 4}
POLICY_NAME = {v: k for k, v in POLICY.items()}
POLICY_NAME[5] = "custom"
ALGO = {"p": 0, "m": 1, "greedy": 2}
ALGO_NAME = {v: k for k, v in ALGO.items()}
LAYER_TYPE = {"conv": 0, "relu": 1, "maxpool": 2, "avgpool": 3, "fc": 4, "concat": 5, "softmax_ce": 6}
MAX_INPUTS = 8


class LayerDesc(C.Structure):
    _fields_ = [("type", C.c_int32), ("n_inputs", C.c_int32), ("inputs", C.c_int32 * MAX_INPUTS),
                ("out_channels", C.c_int32), ("kernel", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32)]


class NetDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("n_layers", C.c_int32), ("layers", C.POINTER(LayerDesc))]


class MemStats(C.Structure):
    _fields_ = [("budget_bytes", C.c_uint64), ("cur_bytes", C.c_uint64), ("peak_bytes", C.c_uint64),
                ("pool_extent_bytes", C.c_uint64), ("baseline_bytes", C.c_uint64), ("persistent_bytes", C.c_uint64),
                ("avg_bytes_layerstep", C.c_double), ("offloaded_bytes", C.c_uint64), ("prefetched_bytes", C.c_uint64),
                ("pinned_host_bytes", C.c_uint64), ("workspace_bytes", C.c_uint64),
                ("n_offload", C.c_int32), ("n_prefetch", C.c_int32), ("n_ondemand_fetch", C.c_int32),
                ("effective_policy", C.c_int32), ("conv_algo", C.c_int32), ("n_memopt_convs", C.c_int32),
                ("window_fill_pm", C.c_int32), ("window_fill_bwd_pm", C.c_int32),
                ("n_winograd_convs", C.c_int32), ("n_downgraded_convs", C.c_int32),
                ("fwd_ms", C.c_double), ("bwd_ms", C.c_double), ("stall_ms", C.c_double), ("d2h_ms", C.c_double),
                ("h2d_ms", C.c_double), ("d2h_gbps", C.c_double), ("h2d_gbps", C.c_double)]


_vp = C.c_void_p
_i = C.c_int
_sz = C.c_size_t

EXPORTS = {
    "vdnn_create": ([C.POINTER(NetDesc), _sz, C.POINTER(_vp)], _i),
    "vdnn_set_policy": ([_vp, _i], _i),
    "vdnn_set_conv_algo": ([_vp, _i], _i),
    "vdnn_set_winograd": ([_vp, C.c_int32], _i),
    "vdnn_layer_workspace_options": ([_vp, _i, C.c_int32, C.POINTER(C.c_uint64), _sz, C.POINTER(_sz)], _i),
    "vdnn_layer_kernels": ([_vp, _i, C.POINTER(C.c_int32)], _i),
    "vdnn_set_layer_kernels": ([_vp, _i, C.POINTER(C.c_int32)], _i),
    "vdnn_set_offload_set": ([_vp, C.POINTER(C.c_int32), _sz, C.c_int32, C.c_int32], _i),
    "vdnn_get_offload_set": ([_vp, C.POINTER(C.c_int32), _sz, C.POINTER(_sz)], _i),
    "vdnn_set_window_part": ([_vp, _sz], _i),
    "vdnn_profile": ([_vp, C.c_int32], _i),
    "vdnn_set_layer_profile": ([_vp, _i, C.c_int32, C.c_int32, C.c_float], _i),
    "vdnn_get_layer_profile": ([_vp, _i, C.c_int32, C.c_int32, C.POINTER(C.c_float)], _i),
    "vdnn_estimate_step_ms": ([_vp, C.POINTER(C.c_double)], _i),
    "vdnn_set_link_rate": ([_vp, C.c_double, C.c_double], _i),
    "vdnn_get_link_rate": ([_vp, C.POINTER(C.c_double), C.POINTER(C.c_double)], _i),
    "vdnn_set_layer_timing": ([_vp, C.c_int32], _i),
    "vdnn_layer_times": ([_vp, C.POINTER(C.c_float), C.POINTER(C.c_float), _sz], _i),
    "vdnn_forward": ([_vp, _vp, _vp, C.POINTER(C.c_float)], _i),
    "vdnn_backward": ([_vp], _i),
    "vdnn_mem_stats": ([_vp, C.POINTER(MemStats)], _i),
    "vdnn_attach_device": ([_vp, _vp, _sz, _vp, _vp], _i),
    "vdnn_set_weights": ([_vp, _i, _vp, _sz], _i),
    "vdnn_get_weight_grad": ([_vp, _i, _vp, _sz], _i),
    "vdnn_get_weights": ([_vp, _i, _vp, _sz], _i),
    "vdnn_sgd_step": ([_vp, C.c_float], _i),
    "vdnn_weight_count": ([_vp, _i], _sz),
    "vdnn_output_count": ([_vp, _i], _sz),
    "vdnn_get_output": ([_vp, _i, _vp, _sz], _i),
    "vdnn_capture_output": ([_vp, _i, _vp], _i),
    "vdnn_capture_grad": ([_vp, _i, _vp], _i),
    "vdnn_trace": ([_vp, C.c_char_p, _sz, C.POINTER(_sz)], _i),
    "vdnn_last_error": ([_vp], C.c_char_p),
    "vdnn_destroy": ([_vp], None),
    "vdnn_op_last_error": ([], C.c_char_p),
    "vdnn_op_set_winograd_chunk_bytes": ([_sz], None),
    "vdnn_op_conv_fwd_workspace": ([_i] * 9, _sz),
    "vdnn_op_conv_bwd_data_workspace": ([_i] * 9, _sz),
    "vdnn_op_conv_workspace": ([_i] * 11, _sz),
    "vdnn_op_conv_fwd": ([_vp] * 4 + [_sz] + [_i] * 11 + [_vp], _i),
    "vdnn_op_conv_bwd_data": ([_vp] * 4 + [_sz] + [_i] * 9 + [_vp, _i, _vp], _i),
    "vdnn_op_conv_bwd_filter_workspace": ([_i] * 9, _sz),
    "vdnn_op_conv_bwd_filter": ([_vp] * 4 + [_sz] + [_i] * 10 + [_vp], _i),
    "vdnn_op_conv_bwd_filter_static": ([_vp] * 3 + [_i] * 10 + [_vp], _i),
    "vdnn_op_fc_workspace": ([_i] * 4, _sz),
    "vdnn_op_fc_fwd": ([_vp] * 4 + [_sz] + [_i] * 3 + [_vp], _i),
    "vdnn_op_fc_bwd_data": ([_vp] * 4 + [_sz] + [_i] * 3 + [_vp], _i),
    "vdnn_op_fc_bwd_filter": ([_vp] * 4 + [_sz] + [_i] * 3 + [_vp], _i),
    "vdnn_op_relu_fwd": ([_vp, _sz, _vp], _i),
    "vdnn_op_relu_bwd": ([_vp, _vp, _sz, _vp], _i),
    "vdnn_op_maxpool_fwd": ([_vp] * 2 + [_i] * 7 + [_vp], _i),
    "vdnn_op_maxpool_bwd": ([_vp] * 3 + [_i] * 8 + [_vp], _i),
    "vdnn_op_avgpool_fwd": ([_vp] * 2 + [_i] * 7 + [_vp], _i),
    "vdnn_op_avgpool_bwd": ([_vp] * 2 + [_i] * 7 + [_vp], _i),
    "vdnn_op_softmax_ce_fwd": ([_vp] * 3 + [_i] * 2 + [_vp], _i),
    "vdnn_op_softmax_ce_bwd": ([_vp] * 3 + [_i] * 2 + [_vp], _i),
    "vdnn_op_concat_copy": ([_vp] * 2 + [_i] * 6 + [_vp], _i),
    "vdnn_op_add": ([_vp, _vp, _sz, _vp], _i),
}
for _name, (_args, _res) in EXPORTS.items():
    _f = getattr(lib, _name)
    _f.argtypes = _args
    _f.restype = _res


class VdnnError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("vdnn status %d: %s" % (status, msg))
        self.status = status


def make_desc(net):
    """net: a workload dict (see synth/nets.py).  Returns (NetDesc, keepalive)."""
    layers = (LayerDesc * len(net["layers"]))()
    for d, l in zip(layers, net["layers"]):
        d.type = LAYER_TYPE[l["type"]]
        d.n_inputs = len(l["inputs"])
        for j, s in enumerate(l["inputs"]):
            d.inputs[j] = s
        d.out_channels, d.kernel, d.stride, d.pad = l["out"], l["k"], l["stride"], l["pad"]
    desc = NetDesc(net["batch"], net["in_c"], net["in_h"], net["in_w"], len(net["layers"]), layers)
    return desc, layers


class Net:
    """vdnn_create / vdnn_set_policy / vdnn_forward / vdnn_backward / vdnn_mem_stats."""

    def __init__(self, net, budget_bytes=0):
        desc, keep = make_desc(net)
        h = _vp()
        s = lib.vdnn_create(C.byref(desc), budget_bytes, C.byref(h))
        if s != OK:
            raise VdnnError(s, "vdnn_create failed (invalid network description)")
        self.h = h
        self.net = net
        self._pool = None
        self._streams = None

    def _chk(self, s):
        if s != OK:
            raise VdnnError(s, lib.vdnn_last_error(self.h).decode())

    def close(self):
        if self.h:
            lib.vdnn_destroy(self.h)
            self.h = None
            self._pool = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_policy(self, policy):
        self._chk(lib.vdnn_set_policy(self.h, POLICY[policy]))

    def set_winograd(self, enabled):
        """True / 1: every Winograd kernel; 2: only the F(2x2,3x3) forms; False / 0: none (see vdnn_set_winograd)."""
        self._chk(lib.vdnn_set_winograd(self.h, int(enabled)))

    def workspace_options(self, layer, bwd):
        """Workspace bytes of the ways a layer can run, performance-optimal first (see vdnn_layer_workspace_options)."""
        k = _sz(0)
        self._chk(lib.vdnn_layer_workspace_options(self.h, layer, int(bwd), None, 0, C.byref(k)))
        arr = (C.c_uint64 * max(k.value, 1))()
        self._chk(lib.vdnn_layer_workspace_options(self.h, layer, int(bwd), arr, k.value, C.byref(k)))
        return list(arr[:k.value])

    def layer_kernels(self, layer):
        """(forward, backward-data, backward-filter) kernel names of a CONV layer in the current plan."""
        arr = (C.c_int32 * 3)()
        self._chk(lib.vdnn_layer_kernels(self.h, layer, arr))
        return tuple(KERNEL_NAME[v] for v in arr)

    def set_layer_kernels(self, layer, names):
        """names: (forward, backward-data, backward-filter) kernel names, or None to give the layer its list back."""
        arr = None if names is None else (C.c_int32 * 3)(*[KERNEL[v] for v in names])
        self._chk(lib.vdnn_set_layer_kernels(self.h, layer, arr))

    def set_conv_algo(self, algo):
        """"p" (performance-optimal, workspace), "m" (memory-optimal) or "greedy"; applies at the next set_policy."""
        self._chk(lib.vdnn_set_conv_algo(self.h, ALGO[algo]))

    def try_policy(self, policy):
        """Returns the status instead of raising (OOM is an expected outcome)."""
        return lib.vdnn_set_policy(self.h, POLICY[policy])

    def set_offload_set(self, buffers, window_fill_pm=0, window_fill_bwd_pm=None):
        """Offload exactly these feature maps (-1 = network input, else producing layer id)."""
        self._chk(self.try_offload_set(buffers, window_fill_pm, window_fill_bwd_pm))

    def try_offload_set(self, buffers, window_fill_pm=0, window_fill_bwd_pm=None):
        ids = sorted(buffers)
        arr = (C.c_int32 * max(len(ids), 1))(*ids)
        fb = window_fill_pm if window_fill_bwd_pm is None else window_fill_bwd_pm
        return lib.vdnn_set_offload_set(self.h, arr, len(ids), window_fill_pm, fb)

    def profile(self, repeats=2):
        """The profiling passes of vDNN_dyn (needs a plan that fits and a GPU)."""
        self._chk(lib.vdnn_profile(self.h, repeats))

    def set_layer_profile(self, layer, pass_, kernel, ms):
        self._chk(lib.vdnn_set_layer_profile(self.h, layer, PASS[pass_] if isinstance(pass_, str) else pass_,
                                             KERNEL[kernel] if isinstance(kernel, str) else kernel, ms))

    def layer_profile(self, layer):
        """CONV: {(pass, kernel): ms} of what was measured; other layers: {"fwd": ms, "bwd": ms}."""
        v = C.c_float()
        out = {}
        if self.net["layers"][layer]["type"] == "conv":
            for pn, p in PASS.items():
                for kn, k in KERNEL.items():
                    if k >= 0:
                        self._chk(lib.vdnn_get_layer_profile(self.h, layer, p, k, C.byref(v)))
                        if v.value >= 0:
                            out[pn, kn] = v.value
        else:
            for pn, p in (("fwd", 0), ("bwd", 1)):
                self._chk(lib.vdnn_get_layer_profile(self.h, layer, p, 0, C.byref(v)))
                if v.value >= 0:
                    out[pn] = v.value
        return out

    def estimate_step_ms(self):
        v = C.c_double()
        self._chk(lib.vdnn_estimate_step_ms(self.h, C.byref(v)))
        return v.value

    def dump_profile(self):
        """Everything the profiling passes measured, as plain data: {"layers": {id: {...}}, "link": (d2h, h2d)}."""
        return dict(layers={i: self.layer_profile(i) for i in range(len(self.net["layers"]))}, link=self.link_rate())

    def load_profile(self, prof):
        """Puts a profile measured on another net of the same shape in (vdnn_set_layer_profile, vdnn_set_link_rate)."""
        for i, entries in prof["layers"].items():
            for key, ms in entries.items():
                if isinstance(key, tuple):
                    self.set_layer_profile(int(i), key[0], key[1], ms)
                else:
                    self.set_layer_profile(int(i), 0 if key == "fwd" else 1, 0, ms)
        if prof["link"][0] > 0 and prof["link"][1] > 0:
            self.set_link_rate(*prof["link"])

    def set_link_rate(self, d2h_gbps, h2d_gbps):
        self._chk(lib.vdnn_set_link_rate(self.h, d2h_gbps, h2d_gbps))

    def link_rate(self):
        a, b = C.c_double(), C.c_double()
        self._chk(lib.vdnn_get_link_rate(self.h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def set_layer_timing(self, on=True):
        self._chk(lib.vdnn_set_layer_timing(self.h, int(on)))

    def layer_times(self):
        """(forward ms, backward ms) per layer of the last timed step."""
        k = len(self.net["layers"])
        f, b = (C.c_float * k)(), (C.c_float * k)()
        self._chk(lib.vdnn_layer_times(self.h, f, b, k))
        return list(f), list(b)

    def set_window_part(self, part_bytes):
        self._chk(lib.vdnn_set_window_part(self.h, part_bytes))

    def offload_set(self):
        k = _sz(0)
        self._chk(lib.vdnn_get_offload_set(self.h, None, 0, C.byref(k)))
        arr = (C.c_int32 * max(k.value, 1))()
        self._chk(lib.vdnn_get_offload_set(self.h, arr, k.value, C.byref(k)))
        return set(arr[:k.value])

    def last_error(self):
        return lib.vdnn_last_error(self.h).decode()

    def stats(self):
        st = MemStats()
        self._chk(lib.vdnn_mem_stats(self.h, C.byref(st)))
        d = {k: getattr(st, k) for k, _ in MemStats._fields_}
        d["effective_policy"] = POLICY_NAME[d["effective_policy"]]
        d["conv_algo"] = ALGO_NAME[d["conv_algo"]]
        return d

    def trace(self):
        need = _sz()
        self._chk(lib.vdnn_trace(self.h, None, 0, C.byref(need)))
        buf = C.create_string_buffer(need.value)
        self._chk(lib.vdnn_trace(self.h, buf, need.value, C.byref(need)))
        out = []
        for line in buf.value.decode().splitlines():
            t = line.split()
            out.append(tuple(t[:3]) + tuple(int(v) for v in t[3:]))
        return out

    def attach_torch(self, pool_bytes=None, streams=None):
        """Allocates the pool as a torch uint8 tensor and lends it to the library together with two
        torch streams (compute, memory).  Pass `streams` to reuse a pair: a process that keeps
        creating streams ends up with several of them on one hardware queue, where a copy and
        a kernel from different streams no longer overlap."""
        import torch
        st = self.stats()
        nbytes = int(pool_bytes if pool_bytes is not None else (st["budget_bytes"] or st["pool_extent_bytes"]))
        self._pool = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self._streams = tuple(streams) if streams is not None else (torch.cuda.Stream(), torch.cuda.Stream())
        self._chk(lib.vdnn_attach_device(self.h, self._pool.data_ptr(), nbytes, self._streams[0].cuda_stream,
                                         self._streams[1].cuda_stream))

    def weight_count(self, layer):
        return lib.vdnn_weight_count(self.h, layer)

    def output_count(self, layer):
        return lib.vdnn_output_count(self.h, layer)

    def set_weights(self, layer, w):
        import numpy as np
        w = np.ascontiguousarray(w, dtype=np.float32)
        self._chk(lib.vdnn_set_weights(self.h, layer, w.ctypes.data, w.size))

    def get_weight_grad(self, layer, shape=None):
        import numpy as np
        out = np.empty(self.weight_count(layer), np.float32)
        self._chk(lib.vdnn_get_weight_grad(self.h, layer, out.ctypes.data, out.size))
        return out.reshape(shape) if shape is not None else out

    def get_weights(self, layer, shape=None):
        import numpy as np
        out = np.empty(self.weight_count(layer), np.float32)
        self._chk(lib.vdnn_get_weights(self.h, layer, out.ctypes.data, out.size))
        return out.reshape(shape) if shape is not None else out

    def sgd_step(self, lr):
        self._chk(lib.vdnn_sgd_step(self.h, lr))

    def get_output(self, layer=-1):
        """A layer's output at the end of forward propagation (-1: the logits), as a flat fp32 array."""
        import numpy as np
        src = self.net["layers"][-1]["inputs"][0] if layer == -1 else layer
        out = np.empty(self.output_count(src), np.float32)
        self._chk(lib.vdnn_get_output(self.h, layer, out.ctypes.data, out.size))
        return out

    def capture_output(self, layer, arr):
        self._chk(lib.vdnn_capture_output(self.h, layer, arr.ctypes.data if arr is not None else None))

    def capture_grad(self, layer, arr):
        self._chk(lib.vdnn_capture_grad(self.h, layer, arr.ctypes.data if arr is not None else None))

    def forward(self, x_dev, labels_dev):
        """x_dev: torch float32 CUDA tensor (NCHW), labels_dev: torch int32 CUDA tensor.  Returns the loss."""
        import torch
        assert x_dev.is_cuda and x_dev.dtype == torch.float32 and x_dev.is_contiguous()
        assert labels_dev.is_cuda and labels_dev.dtype == torch.int32
        torch.cuda.current_stream().synchronize()
        loss = C.c_float()
        self._chk(lib.vdnn_forward(self.h, x_dev.data_ptr(), labels_dev.data_ptr(), C.byref(loss)))
        return loss.value

    def backward(self):
        self._chk(lib.vdnn_backward(self.h))


def _stream_ptr(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream


def _ck(s, what):
    if s != OK:
        raise VdnnError(s, what + ": " + lib.vdnn_op_last_error().decode())


# ---- single-layer entry points on torch CUDA tensors (marshalling only) -------------------------
def _ws_args(ws):
    return (ws.data_ptr() if ws is not None else None, ws.numel() * ws.element_size() if ws is not None else 0)


def op_set_winograd_chunk_bytes(nbytes):
    lib.vdnn_op_set_winograd_chunk_bytes(int(nbytes))


def op_conv_fwd_workspace(x_shape, w_shape, stride, pad):
    n, c, h, wd = x_shape
    k, _, r, s = w_shape
    return lib.vdnn_op_conv_fwd_workspace(n, c, h, wd, k, r, s, stride, pad)


def op_conv_bwd_data_workspace(x_shape, w_shape, stride, pad):
    n, c, h, wd = x_shape
    k, _, r, s = w_shape
    return lib.vdnn_op_conv_bwd_data_workspace(n, c, h, wd, k, r, s, stride, pad)


KERNEL = {"auto": -1, "gather": 0, "packed": 1, "winograd": 2, "winograd_small": 3, "winograd4": 4, "winograd4_small": 5}
KERNEL_NAME = {v: k for k, v in KERNEL.items()}
PASS = {"fwd": 0, "bwd_data": 1, "bwd_filter": 2}
NO_KERNEL = C.c_size_t(-1).value


def op_conv_workspace(pass_, kernel, x_shape, w_shape, stride, pad):
    """Workspace bytes of one kernel for one pass, or None where the kernel does not apply to the shape."""
    n, c, h, wd = x_shape
    k, _, r, s = w_shape
    v = lib.vdnn_op_conv_workspace(PASS[pass_], KERNEL[kernel], n, c, h, wd, k, r, s, stride, pad)
    return None if v == NO_KERNEL else v


def try_op_conv_fwd(x, w, y, stride, pad, relu=False, stream=None, ws=None, kernel="auto"):
    n, c, h, wd = x.shape
    k, _, r, s = w.shape
    return lib.vdnn_op_conv_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), *_ws_args(ws), n, c, h, wd, k, r, s, stride, pad,
                                int(relu), KERNEL[kernel], _stream_ptr(stream))


def op_conv_fwd(x, w, y, stride, pad, relu=False, stream=None, ws=None, kernel="auto"):
    _ck(try_op_conv_fwd(x, w, y, stride, pad, relu, stream, ws, kernel), "conv_fwd")


def try_op_conv_bwd_data(dy, w, dx, stride, pad, stream=None, ws=None, relu_mask=None, kernel="auto"):
    n, c, h, wd = dx.shape
    k, _, r, s = w.shape
    return lib.vdnn_op_conv_bwd_data(dy.data_ptr(), w.data_ptr(), dx.data_ptr(), *_ws_args(ws), n, c, h, wd, k, r, s, stride,
                                     pad, relu_mask.data_ptr() if relu_mask is not None else None, KERNEL[kernel], _stream_ptr(stream))


def op_conv_bwd_data(dy, w, dx, stride, pad, stream=None, ws=None, relu_mask=None, kernel="auto"):
    _ck(try_op_conv_bwd_data(dy, w, dx, stride, pad, stream, ws, relu_mask, kernel), "conv_bwd_data")


def op_conv_bwd_filter_workspace(x_shape, w_shape, stride, pad):
    n, c, h, wd = x_shape
    k, _, r, s = w_shape
    return lib.vdnn_op_conv_bwd_filter_workspace(n, c, h, wd, k, r, s, stride, pad)


def try_op_conv_bwd_filter(x, dy, dw, ws, stride, pad, stream=None, kernel="auto"):
    n, c, h, wd = x.shape
    k, _, r, s = dw.shape
    return lib.vdnn_op_conv_bwd_filter(x.data_ptr(), dy.data_ptr(), dw.data_ptr(), *_ws_args(ws), n, c, h, wd, k, r, s, stride,
                                       pad, KERNEL[kernel], _stream_ptr(stream))


def op_conv_bwd_filter(x, dy, dw, ws, stride, pad, stream=None, kernel="auto"):
    _ck(try_op_conv_bwd_filter(x, dy, dw, ws, stride, pad, stream, kernel), "conv_bwd_filter")


STATIC_SCRATCH_BYTES = 64 << 20


def try_op_conv_bwd_filter_static(x, dy, dw, stride, pad, stream=None, kernel="auto"):
    n, c, h, wd = x.shape
    k, _, r, s = dw.shape
    return lib.vdnn_op_conv_bwd_filter_static(x.data_ptr(), dy.data_ptr(), dw.data_ptr(), n, c, h, wd, k, r, s, stride, pad,
                                              KERNEL[kernel], _stream_ptr(stream))


def op_conv_bwd_filter_static(x, dy, dw, stride, pad, stream=None, kernel="auto"):
    _ck(try_op_conv_bwd_filter_static(x, dy, dw, stride, pad, stream, kernel), "conv_bwd_filter_static")


def op_fc_workspace(n, i, o, which):
    return lib.vdnn_op_fc_workspace(n, i, o, which)


def op_fc_fwd(x, w, y, ws, stream=None):
    o, i = w.shape
    _ck(lib.vdnn_op_fc_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), *_ws_args(ws), x.shape[0], i, o, _stream_ptr(stream)), "fc_fwd")


def op_fc_bwd_data(dy, w, dx, ws, stream=None):
    o, i = w.shape
    _ck(lib.vdnn_op_fc_bwd_data(dy.data_ptr(), w.data_ptr(), dx.data_ptr(), *_ws_args(ws), dy.shape[0], i, o, _stream_ptr(stream)), "fc_bwd_data")


def op_fc_bwd_filter(x, dy, dw, ws, stream=None):
    o, i = dw.shape
    _ck(lib.vdnn_op_fc_bwd_filter(x.data_ptr(), dy.data_ptr(), dw.data_ptr(), *_ws_args(ws), dy.shape[0], i, o, _stream_ptr(stream)), "fc_bwd_filter")


def op_relu_fwd(y, stream=None):
    _ck(lib.vdnn_op_relu_fwd(y.data_ptr(), y.numel(), _stream_ptr(stream)), "relu_fwd")


def op_relu_bwd(y, dy, stream=None):
    _ck(lib.vdnn_op_relu_bwd(y.data_ptr(), dy.data_ptr(), y.numel(), _stream_ptr(stream)), "relu_bwd")


def op_maxpool_fwd(x, y, k, stride, pad, stream=None):
    _ck(lib.vdnn_op_maxpool_fwd(x.data_ptr(), y.data_ptr(), *x.shape, k, stride, pad, _stream_ptr(stream)), "maxpool_fwd")


def op_maxpool_bwd(x, dy, dx, k, stride, pad, stream=None, relu_mask=False):
    _ck(lib.vdnn_op_maxpool_bwd(x.data_ptr(), dy.data_ptr(), dx.data_ptr(), *x.shape, k, stride, pad, int(relu_mask),
                                _stream_ptr(stream)), "maxpool_bwd")


def op_avgpool_fwd(x, y, k, stride, pad, stream=None):
    _ck(lib.vdnn_op_avgpool_fwd(x.data_ptr(), y.data_ptr(), *x.shape, k, stride, pad, _stream_ptr(stream)), "avgpool_fwd")


def op_avgpool_bwd(dy, dx, k, stride, pad, stream=None):
    _ck(lib.vdnn_op_avgpool_bwd(dy.data_ptr(), dx.data_ptr(), *dx.shape, k, stride, pad, _stream_ptr(stream)), "avgpool_bwd")


def op_softmax_ce_fwd(z, labels, loss, stream=None):
    _ck(lib.vdnn_op_softmax_ce_fwd(z.data_ptr(), labels.data_ptr(), loss.data_ptr(), z.shape[0], z.shape[1], _stream_ptr(stream)), "softmax_ce_fwd")


def op_softmax_ce_bwd(z, labels, dz, stream=None):
    _ck(lib.vdnn_op_softmax_ce_bwd(z.data_ptr(), labels.data_ptr(), dz.data_ptr(), z.shape[0], z.shape[1], _stream_ptr(stream)), "softmax_ce_bwd")


def op_concat_copy(src, dst, n, c_small, c_big, c_off, hw, to_big, stream=None):
    _ck(lib.vdnn_op_concat_copy(src.data_ptr(), dst.data_ptr(), n, c_small, c_big, c_off, hw, int(to_big), _stream_ptr(stream)), "concat_copy")


def op_add(acc, src, stream=None):
    _ck(lib.vdnn_op_add(acc.data_ptr(), src.data_ptr(), acc.numel(), _stream_ptr(stream)), "add")
