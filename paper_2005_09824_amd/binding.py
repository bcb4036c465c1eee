"""Thin ctypes binding of liblfmmi.so (include/lfmmi.h): argument marshalling
only. Every step of the forward-backward runs in the library's HIP kernels;
there is no CPU fallback, and a missing library is an error.

Functions carry the names of the C entry points. Device arrays are torch
tensors on the GPU (PyTorch only provides device memory and the stream).
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblfmmi.so")

ORD_FWD, ORD_BWD, ORD_OCC = 0, 1, 2

EXPORTS = [
    "lfmmi_graph_create", "lfmmi_graph_pack", "lfmmi_graph_create_batch",
    "lfmmi_graph_pack_batch", "lfmmi_graph_upload", "lfmmi_graph_destroy",
    "lfmmi_forward_backward", "lfmmi_forward_backward_static", "lfmmi_loss", "lfmmi_last_error",
    "lfmmi_graph_info",
    "lfmmi_graph_ordering_info", "lfmmi_graph_ordering_copy",
    "lfmmi_profile_enable", "lfmmi_profile_read",
]

_lib = None


class LfmmiError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("lfmmi status %d: %s" % (code, message))
        self.code = code


def load_library():
    """Loads the built library; builds it first only if nothing is built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    pp = ctypes.POINTER(vp)
    single = [i32, i32, i64, vp, vp, vp, vp, vp, vp, pp]
    batch = [i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, pp]
    lib.lfmmi_graph_create.argtypes = single
    lib.lfmmi_graph_pack.argtypes = single
    lib.lfmmi_graph_create_batch.argtypes = batch
    lib.lfmmi_graph_pack_batch.argtypes = batch
    lib.lfmmi_graph_upload.argtypes = [vp]
    lib.lfmmi_graph_destroy.argtypes = [vp]
    lib.lfmmi_graph_destroy.restype = None
    lib.lfmmi_forward_backward.argtypes = [vp, vp, vp, i32, i32, i32, f32, f32,
                                           ctypes.c_int, vp, vp, vp, vp]
    lib.lfmmi_forward_backward_static.argtypes = lib.lfmmi_forward_backward.argtypes
    lib.lfmmi_loss.argtypes = [vp, vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, vp]
    lib.lfmmi_last_error.argtypes = []
    lib.lfmmi_last_error.restype = ctypes.c_char_p
    lib.lfmmi_graph_info.argtypes = [vp, vp]
    lib.lfmmi_graph_ordering_info.argtypes = [vp, i32, i32, vp]
    lib.lfmmi_graph_ordering_copy.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.lfmmi_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.lfmmi_profile_read.argtypes = [vp, vp, vp, vp]
    for name in EXPORTS:
        if name not in ("lfmmi_graph_destroy", "lfmmi_last_error"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(code):
    if code != 0:
        raise LfmmiError(code, lfmmi_last_error())


def lfmmi_last_error():
    return load_library().lfmmi_last_error().decode("utf-8", "replace")


def _host(arr, dtype):
    return np.ascontiguousarray(arr, dtype=dtype)


def _hp(arr):
    return ctypes.c_void_p(arr.ctypes.data) if arr is not None and arr.size else None


class Graph:
    """Owner of an lfmmi_graph handle."""

    def __init__(self, handle, num_graphs, num_pdfs):
        self.handle = handle
        self.num_graphs = num_graphs
        self.num_pdfs = num_pdfs

    def close(self):
        if self.handle:
            lfmmi_graph_destroy(self)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _single(fn_name, g):
    lib = load_library()
    src, dst, pdf = (_host(g[k], np.int32) for k in ("src", "dst", "pdf"))
    logw = _host(g["logw"], np.float32)
    pi = _host(g["init_prob"], np.float32)
    fin = _host(g["final_prob"], np.float32)
    S, P = int(g["num_states"]), int(g["num_pdfs"])
    if not (len(src) == len(dst) == len(pdf) == len(logw)):
        raise ValueError("arc arrays differ in length")
    if len(pi) != S or len(fin) != S:
        raise ValueError("init_prob / final_prob must have num_states entries")
    out = ctypes.c_void_p()
    _check(getattr(lib, fn_name)(S, P, len(src), _hp(src), _hp(dst), _hp(pdf), _hp(logw),
                                 _hp(pi), _hp(fin), ctypes.byref(out)))
    return Graph(out.value, 1, P)


def _batch(fn_name, graphs):
    lib = load_library()
    n = len(graphs)
    P = int(graphs[0]["num_pdfs"])
    for g in graphs:
        if int(g["num_pdfs"]) != P:
            raise ValueError("graphs of a batch must share num_pdfs")
        if len(g["init_prob"]) != int(g["num_states"]) or \
                len(g["final_prob"]) != int(g["num_states"]):
            raise ValueError("init_prob / final_prob must have num_states entries")
    state_off = np.zeros(n + 1, dtype=np.int64)
    arc_off = np.zeros(n + 1, dtype=np.int64)
    for i, g in enumerate(graphs):
        state_off[i + 1] = state_off[i] + int(g["num_states"])
        arc_off[i + 1] = arc_off[i] + len(g["src"])
    cat = lambda k, dt: _host(np.concatenate([np.asarray(g[k]) for g in graphs]), dt)
    src, dst, pdf = cat("src", np.int32), cat("dst", np.int32), cat("pdf", np.int32)
    logw = cat("logw", np.float32)
    pi, fin = cat("init_prob", np.float32), cat("final_prob", np.float32)
    out = ctypes.c_void_p()
    _check(getattr(lib, fn_name)(n, P, _hp(state_off), _hp(arc_off), _hp(src), _hp(dst),
                                 _hp(pdf), _hp(logw), _hp(pi), _hp(fin), ctypes.byref(out)))
    return Graph(out.value, n, P)


def lfmmi_graph_create(graph):
    """Pack one graph (dict of arrays) and upload it to the current device."""
    return _single("lfmmi_graph_create", graph)


def lfmmi_graph_pack(graph):
    """Host-only packing, for inspection."""
    return _single("lfmmi_graph_pack", graph)


def lfmmi_graph_create_batch(graphs):
    return _batch("lfmmi_graph_create_batch", graphs)


def lfmmi_graph_pack_batch(graphs):
    return _batch("lfmmi_graph_pack_batch", graphs)


def lfmmi_graph_upload(graph):
    _check(load_library().lfmmi_graph_upload(graph.handle))


def lfmmi_graph_destroy(graph):
    if graph.handle:
        load_library().lfmmi_graph_destroy(graph.handle)
        graph.handle = None


def lfmmi_graph_info(graph):
    info = np.zeros(8, dtype=np.int64)
    _check(load_library().lfmmi_graph_info(graph.handle, _hp(info)))
    keys = ("num_graphs", "num_pdfs", "total_states", "total_arcs", "rec_waves",
            "occ_waves", "flags", "workspace_bytes")
    out = dict(zip(keys, (int(v) for v in info)))
    out["uploaded"] = out["flags"] & 1
    out["fp64"] = (out["flags"] >> 1) & 1
    out["emission_by_state"] = (out["flags"] >> 2) & 1
    return out


def lfmmi_graph_ordering_info(graph, g, ord_):
    info = np.zeros(12, dtype=np.int64)
    _check(load_library().lfmmi_graph_ordering_info(graph.handle, g, ord_, _hp(info)))
    keys = ("rows", "slices", "waves", "total_slots", "max_wave_slots", "register_slots",
            "emission_replicated", "per_arc_leak", "gather_cycles", "closing_slots", "hub_slices",
            "lds_vector_rows")
    return dict(zip(keys, (int(v) for v in info)))


def lfmmi_graph_ordering_copy(graph, g, ord_):
    info = lfmmi_graph_ordering_info(graph, g, ord_)
    slice_off = np.zeros(info["slices"] + 1, dtype=np.int32)
    wave_first = np.zeros(info["waves"] + 1, dtype=np.int32)
    key = np.zeros(info["total_slots"] * 64, dtype=np.uint32)
    w = np.zeros(info["total_slots"] * 64, dtype=np.float32)
    row_id = np.zeros(info["slices"] * 64, dtype=np.int32)
    slice_hub = np.zeros(info["slices"], dtype=np.int32)
    _check(load_library().lfmmi_graph_ordering_copy(
        graph.handle, g, ord_, _hp(slice_off), _hp(wave_first), _hp(key), _hp(w), _hp(row_id),
        _hp(slice_hub)))
    return dict(info, slice_off=slice_off, wave_first=wave_first, key=key, w=w, row_id=row_id,
                slice_hub=slice_hub)


STATIC_WORKSPACE_BYTES = 64 << 20   # LFMMI_STATIC_WORKSPACE_BYTES
STATIC_MAX_BATCH = 256              # LFMMI_STATIC_MAX_BATCH


def lfmmi_forward_backward_static(graph, logits, lengths, leak, grad_scale, accumulate,
                                  objf, grad, status, stream=None):
    """The entry point that allocates nothing: as lfmmi_forward_backward, with the
    outputs passed in (this wrapper allocates nothing either) and the workspace
    in the library's static device array."""
    return lfmmi_forward_backward(graph, logits, lengths, leak, grad_scale, accumulate,
                                  objf, grad, status, stream,
                                  _entry="lfmmi_forward_backward_static")


def lfmmi_forward_backward(graph, logits, lengths, leak, grad_scale=1.0, accumulate=False,
                           objf=None, grad=None, status=None, stream=None,
                           _entry="lfmmi_forward_backward"):
    """logits: torch float32 CUDA tensor [B, T, P]; lengths: host int array [B].
    Returns (objf [B], grad [B, T, P], status [B]) device tensors (allocated here
    unless passed in). Enqueues on `stream` (default: torch's current stream)."""
    import torch
    if not logits.is_cuda or logits.dtype != torch.float32 or not logits.is_contiguous():
        raise ValueError("logits must be a contiguous float32 CUDA tensor")
    B, T, P = logits.shape
    lens = _host(lengths, np.int32)
    if len(lens) != B:
        raise ValueError("lengths must have B entries")
    dev = logits.device
    if objf is None:
        if accumulate:
            raise ValueError("accumulate needs existing objf / grad")
        objf = torch.empty(B, dtype=torch.float32, device=dev)
    if grad is None:
        if accumulate:
            raise ValueError("accumulate needs existing objf / grad")
        grad = torch.empty((B, T, P), dtype=torch.float32, device=dev)
    if status is None:
        status = torch.zeros(B, dtype=torch.int32, device=dev)
    for t, shape, dt in ((objf, (B,), torch.float32), (grad, (B, T, P), torch.float32),
                         (status, (B,), torch.int32)):
        if tuple(t.shape) != shape or t.dtype != dt or not t.is_contiguous() or t.device != dev:
            raise ValueError("output tensor has the wrong shape, dtype, layout or device")
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    with torch.cuda.device(dev):
        _check(getattr(load_library(), _entry)(
            graph.handle, ctypes.c_void_p(logits.data_ptr()), _hp(lens), B, T, P,
            float(leak), float(grad_scale), 1 if accumulate else 0,
            ctypes.c_void_p(objf.data_ptr()), ctypes.c_void_p(grad.data_ptr()),
            ctypes.c_void_p(status.data_ptr()), ctypes.c_void_p(stream)))
    return objf, grad, status


def lfmmi_loss(num, den, logits, lengths, leak, objf=None, grad=None, status=None, stream=None):
    """Eq. 2 / Eq. 3 in one call: objf = log p(num) - log p(den) per sequence and its
    gradient with respect to `logits` (torch float32 CUDA tensor [B, T, P]).
    Returns (objf [B], grad [B, T, P], status [B]) device tensors."""
    import torch
    if not logits.is_cuda or logits.dtype != torch.float32 or not logits.is_contiguous():
        raise ValueError("logits must be a contiguous float32 CUDA tensor")
    B, T, P = logits.shape
    lens = _host(lengths, np.int32)
    if len(lens) != B:
        raise ValueError("lengths must have B entries")
    dev = logits.device
    if objf is None:
        objf = torch.empty(B, dtype=torch.float32, device=dev)
    if grad is None:
        grad = torch.empty((B, T, P), dtype=torch.float32, device=dev)
    if status is None:
        status = torch.zeros(B, dtype=torch.int32, device=dev)
    for t, shape, dt in ((objf, (B,), torch.float32), (grad, (B, T, P), torch.float32),
                         (status, (B,), torch.int32)):
        if tuple(t.shape) != shape or t.dtype != dt or not t.is_contiguous() or t.device != dev:
            raise ValueError("output tensor has the wrong shape, dtype, layout or device")
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    with torch.cuda.device(dev):
        _check(load_library().lfmmi_loss(
            num.handle, den.handle, ctypes.c_void_p(logits.data_ptr()), _hp(lens), B, T, P,
            float(leak), ctypes.c_void_p(objf.data_ptr()), ctypes.c_void_p(grad.data_ptr()),
            ctypes.c_void_p(status.data_ptr()), ctypes.c_void_p(stream)))
    return objf, grad, status


def lfmmi_profile_enable(graph, enable=True):
    """enable: False / 0 off, True / 1 every kernel, 2 the recursion launches only."""
    _check(load_library().lfmmi_profile_enable(graph.handle, int(enable)))


def lfmmi_profile_read(graph):
    ms = np.zeros(4, dtype=np.float32)
    calls = np.zeros(1, dtype=np.int32)
    launches = np.zeros(1, dtype=np.int32)
    _check(load_library().lfmmi_profile_read(graph.handle, _hp(ms), _hp(calls), _hp(launches)))
    out = dict(zip(("emit", "rec", "scan", "occ"), (float(v) for v in ms)))
    out["calls"] = int(calls[0])
    out["launches"] = int(launches[0])
    return out
