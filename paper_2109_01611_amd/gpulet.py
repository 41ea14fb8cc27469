"""ctypes binding of ``libgpulet.so`` (declared in ``include/gpulet.h``).

Argument marshalling only: every step of the forward pass runs in the HIP
library.  The module-level functions carry the C names without the prefix
(``conv2d_fwd`` is ``gpulet_conv2d_fwd`` ...).  Tensors are torch tensors on
the GPU (torch is used for device memory only) or raw device addresses.

Loading fails loudly if the library has not been built
(``python -m paper_2109_01611_amd.build``); there is no CPU fallback.
"""

import ctypes
import os
from ctypes import POINTER, byref, c_double, c_float, c_int, c_int32, c_size_t, c_uint32, c_uint64, c_void_p

# torch ships its own copy of the HIP runtime.  It must be the first one loaded
# so that the library below binds to the same runtime instance; two runtimes in
# one process do not both see the GPU.
import torch  # noqa: F401  (device memory provider)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgpulet.so")

OK, EINVAL, EOVERSUB, EHIP, ENOMEM = 0, -1, -2, -3, -4
POOL_MAX, POOL_AVG, POOL_GLOBAL_AVG = 0, 1, 2
OP_CONV, OP_POOL, OP_FC, OP_DWCONV = 0, 1, 2, 3
CONV_TILES = 14  # GPULET_CONV_TILES: set_conv_tile takes -1 .. CONV_TILES - 1


class GpuletError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        msg = "%s: %s" % (what, lib.gpulet_status_string(status).decode())
        if status == EHIP:
            msg += " (hipError_t %d)" % lib.gpulet_last_hip_error()
        super().__init__(msg)


class Layer(ctypes.Structure):
    """Mirror of ``gpulet_layer``."""
    _fields_ = [(n, c_int32) for n in (
        "op", "in_buf", "out_buf", "res_buf", "C", "K", "R", "S", "stride", "pad", "relu", "mode",
        "out_ch_total", "out_ch_offset", "out_fp32", "pre_pool", "in_ch_total", "in_ch_offset", "K2", "out2_buf",
        "out2_ch_total", "out2_ch_offset", "side_pool", "pool_buf",
        "group_next")] + [("w", c_void_p), ("b", c_void_p)]


class ConvDesc(ctypes.Structure):
    """Mirror of ``gpulet_conv_desc``."""
    _fields_ = [("x", c_void_p), ("w", c_void_p), ("b", c_void_p), ("y", c_void_p), ("residual", c_void_p)] + \
               [(n, c_int32) for n in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad", "relu",
                                       "x_ch_stride", "x_ch_offset", "y_ch_stride", "y_ch_offset")]


class SchedModel(ctypes.Structure):
    """Mirror of ``gpulet_sched_model``."""
    _fields_ = [("rate", c_double), ("slo_ms", c_double), ("latency_ms", POINTER(c_double))]


class SchedProblem(ctypes.Structure):
    """Mirror of ``gpulet_sched_problem``."""
    _fields_ = [("n_model", c_int), ("n_size", c_int), ("n_batch", c_int), ("n_gpu", c_int),
                ("size", POINTER(c_int)), ("batch", POINTER(c_int)), ("model", POINTER(SchedModel)),
                ("slowdown", POINTER(c_double)), ("merge", c_int)]


class SchedEntry(ctypes.Structure):
    """Mirror of ``gpulet_sched_entry``."""
    _fields_ = [("gpu", c_int), ("size", c_int), ("which", c_int), ("model", c_int), ("batch", c_int),
                ("rate", c_double), ("duty_ms", c_double)]


class ModelDesc(ctypes.Structure):
    """Mirror of ``gpulet_model_desc``."""
    _fields_ = [(n, c_int32) for n in (
        "n_layers", "n_bufs", "in_C", "in_H", "in_W", "in_buf", "out_buf", "reserved")] + [
        ("layers", POINTER(Layer))]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libgpulet.so is not built: run `python -m paper_2109_01611_amd.build` "
                          "(needs hipcc; there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    I, P, FP = c_int, c_void_p, POINTER(c_float)
    IP, DP = POINTER(c_int), POINTER(c_double)
    sig = {
        "gpulet_status_string": ([c_int32], ctypes.c_char_p),
        "gpulet_last_hip_error": ([], c_int),
        "gpulet_mask_for_pct": ([I, I, I, I, POINTER(c_uint32), I, POINTER(I), POINTER(I)], c_int32),
        "gpulet_partition_create": ([I, I, I, POINTER(P)], c_int32),
        "gpulet_partition_destroy": ([P], c_int32),
        "gpulet_partition_info": ([P, POINTER(I), POINTER(I), POINTER(I), POINTER(I), POINTER(I),
                                   POINTER(c_uint32), POINTER(I), POINTER(P)], c_int32),
        "gpulet_partition_query_mask": ([P, POINTER(c_uint32), POINTER(I)], c_int32),
        "gpulet_partition_counters": ([P, POINTER(c_uint64), POINTER(c_uint64)], c_int32),
        "gpulet_partition_kernel_launches": ([P, POINTER(c_uint64)], c_int32),
        "gpulet_partition_sync": ([P], c_int32),
        "gpulet_partition_probe": ([P, P, I], c_int32),
        "gpulet_partition_probe_ex": ([P, P, I, I], c_int32),
        "gpulet_partition_mfma_rate": ([P, I, I, I, I, FP, DP], c_int32),
        "gpulet_model_graph_create": ([POINTER(ModelDesc), I, P, P, P, P, c_size_t, POINTER(P)], c_int32),
        "gpulet_model_graph_launch": ([P, FP], c_int32),
        "gpulet_model_graph_profile": ([P, I, I, FP, FP], c_int32),
        "gpulet_model_graph_destroy": ([P], c_int32),
        "gpulet_conv2d_fwd": ([P, P, P, P] + [I] * 10 + [P], c_int32),
        "gpulet_conv2d_fwd_ex": ([P, P, P, P] + [I] * 10 + [P, I, I, P], c_int32),
        "gpulet_conv2d_fwd_slices": ([P, P, P, P] + [I] * 10 + [P, I, I, I, I, P], c_int32),
        "gpulet_conv1x1_fwd_two_outputs": ([P, P, P, P, P] + [I] * 14 + [P], c_int32),
        "gpulet_conv1x1_maxpool3_fwd": ([P, P, P, P, P, P] + [I] * 11 + [P], c_int32),
        "gpulet_conv2d_group_fwd": ([POINTER(ConvDesc), I, P], c_int32),
        "gpulet_set_conv_tile": ([I], c_int32),
        "gpulet_set_conv_split_k": ([I], c_int32),
        "gpulet_depthwise_conv2d_fwd": ([P, P, P, P] + [I] * 9 + [P], c_int32),
        "gpulet_maxpool3_conv1x1_fwd": ([P, P, P, P] + [I] * 8 + [P], c_int32),
        "gpulet_conv3x3_maxpool2_fwd": ([P, P, P, P] + [I] * 7 + [P], c_int32),
        "gpulet_set_conv_pool_fusion": ([I], c_int32),
        "gpulet_conv2d_timeline": ([P, P, P, P] + [I] * 10 + [P, I, POINTER(ctypes.c_int64), IP], c_int32),
        "gpulet_pool": ([P, P] + [I] * 8 + [P], c_int32),
        "gpulet_fc": ([P, P, P, P] + [I] * 5 + [P], c_int32),
        "gpulet_fc_static_scratch": ([P, P, P, P] + [I] * 5 + [P], c_int32),
        "gpulet_set_model_lanes": ([I], c_int32),
        "gpulet_model_schedule": ([POINTER(ModelDesc), I, I, IP, IP, IP, I, IP], c_int32),
        "gpulet_model_workspace_bytes": ([POINTER(ModelDesc), I, POINTER(c_size_t)], c_int32),
        "gpulet_model_buffer_info": ([POINTER(ModelDesc), I, I, POINTER(I), POINTER(I), POINTER(I),
                                      POINTER(I), POINTER(c_size_t)], c_int32),
        "gpulet_run_model": ([POINTER(ModelDesc), I, P, P, P, P, c_size_t, FP], c_int32),
        "gpulet_profile_model": ([POINTER(ModelDesc), I, P, P, P, P, c_size_t, I, I, I, FP, FP], c_int32),
        "gpulet_profile_corun": ([POINTER(ModelDesc), I, P, P, P, P, c_size_t,
                                  POINTER(ModelDesc), I, P, P, P, P, c_size_t,
                                  I, c_double, FP, I, POINTER(I), FP, I, POINTER(I)], c_int32),
        "gpulet_latency_stats": ([FP, I, POINTER(c_double), POINTER(c_double), POINTER(c_double)], c_int32),
        "gpulet_time_conv2d": ([P, P, P, P] + [I] * 10 + [P, I, I, P, I, I, FP], c_int32),
        "gpulet_affordable_rate": ([IP, DP, I, c_double, c_double, DP, IP], c_int32),
        "gpulet_rate_curve": ([IP, I, I, DP, c_double, DP], c_int32),
        "gpulet_max_efficient_partition": ([IP, DP, I, IP, DP], c_int32),
        "gpulet_min_required_partition": ([IP, DP, I, c_double, IP], c_int32),
        "gpulet_elastic_partitioning": ([POINTER(SchedProblem), POINTER(SchedEntry), I, IP, IP], c_int32),
        "gpulet_interference_fit": ([DP, DP, I, DP], c_int32),
        "gpulet_interference_predict": ([DP, DP, I, DP], c_int32),
        "gpulet_interference_error": ([DP, DP, DP, I, DP, I, DP], c_int32),
        "gpulet_interference_utilisation": ([c_double] * 6 + [DP, DP], c_int32),
        "gpulet_interference_factor": ([DP, DP, I, DP], c_int32),
        "gpulet_interference_split": ([DP, I, IP, IP], c_int32),
        "gpulet_interference_worst_slowdown": ([DP, DP, I, DP], c_int32),
        "gpulet_interference_overhead": ([DP, I, DP, I, DP, c_double, DP], c_int32),
    }
    for name, (argtypes, restype) in sig.items():
        fn = getattr(L, name)
        fn.argtypes = argtypes
        fn.restype = restype
    return L, tuple(sig)


lib, EXPORTS = _load()


def _check(status, what):
    if status != OK:
        raise GpuletError(status, what)


def ptr(t):
    """Device address of a torch tensor (must be contiguous), an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def status_string(status):
    return lib.gpulet_status_string(status).decode()


def mask_for_pct(n_cu_total, n_xcd, pct, which):
    """-> (mask words, n_cu).  Pure host arithmetic."""
    words = (c_uint32 * 8)()
    n_words, n_cu = c_int(), c_int()
    _check(lib.gpulet_mask_for_pct(n_cu_total, n_xcd, pct, which, words, 8, byref(n_words), byref(n_cu)),
           "gpulet_mask_for_pct")
    return list(words[:n_words.value]), n_cu.value


class Partition:
    """A live gpu-let: ``partition_create`` .. ``partition_destroy``."""

    def __init__(self, device, pct, which=0):
        h = c_void_p()
        _check(lib.gpulet_partition_create(device, pct, which, byref(h)), "gpulet_partition_create")
        self.handle = h
        dev, p, w, n_cu, tot, nw, st = c_int(), c_int(), c_int(), c_int(), c_int(), c_int(), c_void_p()
        words = (c_uint32 * 8)()
        _check(lib.gpulet_partition_info(h, byref(dev), byref(p), byref(w), byref(n_cu), byref(tot), words,
                                         byref(nw), byref(st)), "gpulet_partition_info")
        self.device, self.pct, self.which = dev.value, p.value, w.value
        self.n_cu, self.n_cu_total = n_cu.value, tot.value
        self.mask = list(words[:nw.value])
        self.stream = st.value

    def query_mask(self):
        words, nw = (c_uint32 * 8)(), c_int()
        _check(lib.gpulet_partition_query_mask(self.handle, words, byref(nw)), "gpulet_partition_query_mask")
        return list(words[:nw.value])

    def counters(self):
        b, i = c_uint64(), c_uint64()
        _check(lib.gpulet_partition_counters(self.handle, byref(b), byref(i)), "gpulet_partition_counters")
        return b.value, i.value

    def kernel_launches(self):
        n = c_uint64()
        _check(lib.gpulet_partition_kernel_launches(self.handle, byref(n)), "gpulet_partition_kernel_launches")
        return n.value

    def sync(self):
        _check(lib.gpulet_partition_sync(self.handle), "gpulet_partition_sync")

    def probe(self, out, n_blocks, via_graph=False):
        _check(lib.gpulet_partition_probe_ex(self.handle, ptr(out), n_blocks, int(via_graph)),
               "gpulet_partition_probe_ex")

    def mfma_rate(self, dense, waves_per_cu=8, iters=2000, launches=20):
        """(milliseconds per launch, TFLOP/s) of the matrix-instruction-only probe on this gpu-let."""
        ms, tf = c_float(), c_double()
        _check(lib.gpulet_partition_mfma_rate(self.handle, int(bool(dense)), waves_per_cu, iters, launches,
                                              ctypes.byref(ms), ctypes.byref(tf)), "gpulet_partition_mfma_rate")
        return ms.value, tf.value

    def destroy(self):
        if self.handle is not None:
            h, self.handle = self.handle, None
            _check(lib.gpulet_partition_destroy(h), "gpulet_partition_destroy")

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()


def conv2d_fwd(x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, stream=None):
    _check(lib.gpulet_conv2d_fwd(ptr(x), ptr(w), ptr(b), ptr(y), N, C, H, W, K, R, S, stride, pad,
                                 int(relu), stream), "gpulet_conv2d_fwd")


def conv2d_fwd_ex(x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, residual=None, y_ch_stride=0,
                  y_ch_offset=0, stream=None):
    _check(lib.gpulet_conv2d_fwd_ex(ptr(x), ptr(w), ptr(b), ptr(y), N, C, H, W, K, R, S, stride, pad,
                                    int(relu), ptr(residual), y_ch_stride, y_ch_offset, stream),
           "gpulet_conv2d_fwd_ex")


def conv2d_fwd_slices(x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, residual=None, x_ch_stride=0,
                      x_ch_offset=0, y_ch_stride=0, y_ch_offset=0, stream=None):
    _check(lib.gpulet_conv2d_fwd_slices(ptr(x), ptr(w), ptr(b), ptr(y), N, C, H, W, K, R, S, stride, pad,
                                        int(relu), ptr(residual), x_ch_stride, x_ch_offset, y_ch_stride,
                                        y_ch_offset, stream), "gpulet_conv2d_fwd_slices")


def conv1x1_fwd_two_outputs(x, w, b, y, y2, N, C, H, W, K, k2, stride, relu, x_ch_stride=0, x_ch_offset=0,
                            y_ch_stride=0, y_ch_offset=0, y2_ch_stride=0, y2_ch_offset=0, stream=None):
    _check(lib.gpulet_conv1x1_fwd_two_outputs(ptr(x), ptr(w), ptr(b), ptr(y), ptr(y2), N, C, H, W, K, k2, stride,
                                              int(relu), x_ch_stride, x_ch_offset, y_ch_stride, y_ch_offset,
                                              y2_ch_stride, y2_ch_offset, stream), "gpulet_conv1x1_fwd_two_outputs")


def conv1x1_maxpool3_fwd(x, w, b, y, y2, pool_y, N, C, H, W, K, k2, relu, y_ch_stride=0, y_ch_offset=0,
                         y2_ch_stride=0, y2_ch_offset=0, stream=None):
    _check(lib.gpulet_conv1x1_maxpool3_fwd(ptr(x), ptr(w), ptr(b), ptr(y), ptr(y2), ptr(pool_y), N, C, H, W, K, k2,
                                           int(relu), y_ch_stride, y_ch_offset, y2_ch_stride, y2_ch_offset, stream),
           "gpulet_conv1x1_maxpool3_fwd")


def conv2d_group_fwd(layers, stream=None):
    """``layers``: dicts with the fields of ``gpulet_conv_desc`` (tensors or addresses for the pointers;
    residual, b and the slice fields optional)."""
    arr = (ConvDesc * len(layers))()
    for d, kw in zip(arr, layers):
        for k, v in kw.items():
            setattr(d, k, ptr(v) if k in ("x", "w", "b", "y", "residual") else int(v))
    _check(lib.gpulet_conv2d_group_fwd(arr, len(layers), stream), "gpulet_conv2d_group_fwd")


def set_conv_tile(tile):
    _check(lib.gpulet_set_conv_tile(tile), "gpulet_set_conv_tile")


def set_conv_split_k(max_split):
    _check(lib.gpulet_set_conv_split_k(max_split), "gpulet_set_conv_split_k")


def depthwise_conv2d_fwd(x, w, b, y, N, C, H, W, R, S, stride, pad, relu, stream=None):
    _check(lib.gpulet_depthwise_conv2d_fwd(ptr(x), ptr(w), ptr(b), ptr(y), N, C, H, W, R, S, stride, pad,
                                           int(relu), stream), "gpulet_depthwise_conv2d_fwd")


def maxpool3_conv1x1_fwd(x, w, b, y, N, C, H, W, K, relu, ch_total=0, ch_offset=0, stream=None):
    _check(lib.gpulet_maxpool3_conv1x1_fwd(ptr(x), ptr(w), ptr(b), ptr(y), N, C, H, W, K, int(relu), ch_total,
                                           ch_offset, stream), "gpulet_maxpool3_conv1x1_fwd")


def conv3x3_maxpool2_fwd(x, w, b, y, N, C, H, W, K, ch_total=0, ch_offset=0, stream=None):
    _check(lib.gpulet_conv3x3_maxpool2_fwd(ptr(x), ptr(w), ptr(b), ptr(y), N, C, H, W, K, ch_total, ch_offset,
                                           stream), "gpulet_conv3x3_maxpool2_fwd")


def conv2d_timeline(x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, stream=None, warmup=100):
    """Wall-clock stamps (10 ns units) of the first workgroups of one launch: list of rows of 8 integers,
    empty when the kernel that runs the layer records none."""
    buf = (ctypes.c_int64 * 64)()
    n = c_int()
    _check(lib.gpulet_conv2d_timeline(ptr(x), ptr(w), ptr(b), ptr(y), N, C, H, W, K, R, S, stride, pad, int(relu), stream,
                                      warmup, buf, byref(n)), "gpulet_conv2d_timeline")
    return [list(buf[i * 8:i * 8 + 8]) for i in range(n.value)]


def set_conv_pool_fusion(on):
    _check(lib.gpulet_set_conv_pool_fusion(int(bool(on))), "gpulet_set_conv_pool_fusion")


def pool(x, y, N, C, H, W, mode, k=1, stride=1, pad=0, stream=None):
    _check(lib.gpulet_pool(ptr(x), ptr(y), N, C, H, W, mode, k, stride, pad, stream), "gpulet_pool")


def fc(x, w, b, y, N, In, Out, relu, out_fp32=False, stream=None):
    _check(lib.gpulet_fc(ptr(x), ptr(w), ptr(b), ptr(y), N, In, Out, int(relu), int(out_fp32), stream),
           "gpulet_fc")


def fc_static_scratch(x, w, b, y, N, In, Out, relu, out_fp32=False, stream=None):
    _check(lib.gpulet_fc_static_scratch(ptr(x), ptr(w), ptr(b), ptr(y), N, In, Out, int(relu), int(out_fp32),
                                        stream), "gpulet_fc_static_scratch")


def time_conv2d(x, w, b, y, N, C, H, W, K, R, S, stride, pad, relu, residual=None, y_ch_stride=0,
                y_ch_offset=0, stream=None, warmup=10, iters=100):
    """Average milliseconds per launch over ``iters`` back-to-back launches."""
    ms = c_float()
    _check(lib.gpulet_time_conv2d(ptr(x), ptr(w), ptr(b), ptr(y), N, C, H, W, K, R, S, stride, pad,
                                  int(relu), ptr(residual), y_ch_stride, y_ch_offset, stream, warmup,
                                  iters, byref(ms)), "gpulet_time_conv2d")
    return ms.value


def set_model_lanes(lanes):
    _check(lib.gpulet_set_model_lanes(lanes), "gpulet_set_model_lanes")


def model_schedule(desc, batch, lanes=2):
    """-> (lane per layer, [(from, to)] cross-lane waits) for ``lanes`` lanes (host-only analysis)."""
    n = desc.n_layers
    lane = (c_int * n)()
    cap = 4 * n + 8
    wf, wt, nw = (c_int * cap)(), (c_int * cap)(), c_int()
    _check(lib.gpulet_model_schedule(byref(desc), batch, lanes, lane, wf, wt, cap, byref(nw)), "gpulet_model_schedule")
    return list(lane), [(wf[i], wt[i]) for i in range(nw.value)]


def model_workspace_bytes(desc, batch):
    n = c_size_t()
    _check(lib.gpulet_model_workspace_bytes(byref(desc), batch, byref(n)), "gpulet_model_workspace_bytes")
    return n.value


def model_buffer_info(desc, batch, buf):
    """-> (C, H, W, element bytes, workspace offset or None)."""
    C, H, W, e, off = c_int(), c_int(), c_int(), c_int(), c_size_t()
    _check(lib.gpulet_model_buffer_info(byref(desc), batch, buf, byref(C), byref(H), byref(W), byref(e),
                                        byref(off)), "gpulet_model_buffer_info")
    return C.value, H.value, W.value, e.value, (None if off.value == c_size_t(-1).value else off.value)


def run_model(desc, batch, partition, x, y, workspace, workspace_bytes, timed=False):
    """Enqueues one batch; with ``timed`` waits and returns its milliseconds."""
    ms = c_float()
    _check(lib.gpulet_run_model(byref(desc), batch, partition.handle, ptr(x), ptr(y), ptr(workspace),
                                workspace_bytes, byref(ms) if timed else None), "gpulet_run_model")
    return ms.value if timed else None


class ModelGraph:
    """A forward pass captured as a HIP graph: ``model_graph_create`` .. ``model_graph_destroy``.
    Keeps references to the tensors it is bound to."""

    def __init__(self, desc, batch, partition, x, y, workspace, workspace_bytes):
        h = c_void_p()
        _check(lib.gpulet_model_graph_create(byref(desc), batch, partition.handle, ptr(x), ptr(y), ptr(workspace),
                                             workspace_bytes, byref(h)), "gpulet_model_graph_create")
        self.handle = h
        self._keep = (desc, partition, x, y, workspace)

    def launch(self, timed=False):
        ms = c_float()
        _check(lib.gpulet_model_graph_launch(self.handle, byref(ms) if timed else None), "gpulet_model_graph_launch")
        return ms.value if timed else None

    def profile(self, warmup, iters):
        lat = (c_float * iters)()
        total = c_float()
        _check(lib.gpulet_model_graph_profile(self.handle, warmup, iters, lat, byref(total)),
               "gpulet_model_graph_profile")
        return list(lat), total.value

    def destroy(self):
        if self.handle is not None:
            h, self.handle = self.handle, None
            _check(lib.gpulet_model_graph_destroy(h), "gpulet_model_graph_destroy")

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()


def profile_model(desc, batch, partition, x, y, workspace, workspace_bytes, warmup, iters,
                  sync_each=False):
    """-> (list of per-batch milliseconds, total milliseconds).  ``sync_each`` False / True / 2:
    back to back / one batch in flight / back to back inside a single event pair."""
    lat = (c_float * iters)()
    total = c_float()
    _check(lib.gpulet_profile_model(byref(desc), batch, partition.handle, ptr(x), ptr(y), ptr(workspace),
                                    workspace_bytes, warmup, iters, int(sync_each), lat, byref(total)),
           "gpulet_profile_model")
    return list(lat), total.value


def profile_corun(a, b, warmup, window_ms, cap=100000):
    """``a`` and ``b`` are (desc, batch, partition, x, y, workspace, workspace_bytes).
    -> (latencies of a, latencies of b) in milliseconds."""
    la, lb = (c_float * cap)(), (c_float * cap)()
    na, nb = c_int(), c_int()

    def side(s):
        desc, batch, part, x, y, ws, nbytes = s
        return [byref(desc), batch, part.handle, ptr(x), ptr(y), ptr(ws), nbytes]
    _check(lib.gpulet_profile_corun(*(side(a) + side(b) + [warmup, float(window_ms), la, cap, byref(na),
                                                           lb, cap, byref(nb)])), "gpulet_profile_corun")
    return list(la[:na.value]), list(lb[:nb.value])


def latency_stats(lat):
    """-> (mean, median, nearest-rank p99) of a list of milliseconds."""
    n = len(lat)
    arr = (c_float * n)(*lat)
    mean, p50, p99 = c_double(), c_double(), c_double()
    _check(lib.gpulet_latency_stats(arr, n, byref(mean), byref(p50), byref(p99)), "gpulet_latency_stats")
    return mean.value, p50.value, p99.value
