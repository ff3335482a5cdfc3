"""Thin ctypes binding of libevconv.so (the C ABI of include/evconv.h).

Argument marshalling only: every step of the incremental path runs inside the HIP library.
PyTorch appears solely as the owner of device memory (the workspace, inputs) and of the stream.
There is no CPU fallback: if the library is missing, importing the entry points raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libevconv.so")

ABI_VERSION = 2
OK = 0
STATUS_NAMES = ["OK", "ERR_INVALID_ARG", "ERR_BAD_DESC", "ERR_SHAPE", "ERR_STATE", "ERR_WORKSPACE",
                "ERR_HIP", "ERR_UNSUPPORTED"]
(ERR_INVALID_ARG, ERR_BAD_DESC, ERR_SHAPE, ERR_STATE, ERR_WORKSPACE, ERR_HIP, ERR_UNSUPPORTED) = range(1, 8)
MODE_INCREMENTAL, MODE_DENSE_RECOMPUTE, MODE_AUTO = 0, 1, 2
FLAG_NO_FUSION, FLAG_NO_FOLD, FLAG_FORCE_VALU = 1, 2, 4
(STATE_Z, STATE_DY, STATE_IDX, STATE_COUNT, STATE_BITMAP, STATE_OCC, STATE_OCC_TOUCHED,
 STATE_X_PREV, STATE_STEP, STATE_Z2) = range(10)

EXPORTS = ["evconv_query_workspace", "evconv_create", "evconv_num_outputs", "evconv_reset", "evconv_step",
           "evconv_step_frame", "evconv_destroy", "evconv_set_mode", "evconv_node_shape", "evconv_get_state",
           "evconv_get_stats", "evconv_node_kernel", "evconv_last_error", "evconv_profile_begin",
           "evconv_profile_end", "evconv_get_node_time", "evconv_set_refresh_period", "evconv_get_state_stream",
           "evconv_stream_stride", "evconv_current_mode", "evconv_create_static", "evconv_debug_chip_probes",
           "evconv_debug_phase_stamps"]
STATIC_WORKSPACE_BYTES = 32 << 20


class NodeDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("op", "act", "in0", "in1", "c_in", "c_out", "kh", "kw", "stride", "pad", "wdtype", "is_output")] + \
               [("weight_off", ctypes.c_int64), ("bias_off", ctypes.c_int64)]


class NetDesc(ctypes.Structure):
    _fields_ = [("abi_version", ctypes.c_int32), ("n_nodes", ctypes.c_int32),
                ("nodes", ctypes.POINTER(NodeDesc)),
                ("in_c", ctypes.c_int32), ("in_h", ctypes.c_int32), ("in_w", ctypes.c_int32),
                ("flags", ctypes.c_uint32),
                ("sparsify_tp", ctypes.c_float), ("n_streams", ctypes.c_int32)]


class Out(ctypes.Structure):
    _fields_ = [("node", ctypes.c_int32), ("c", ctypes.c_int32), ("h", ctypes.c_int32), ("w", ctypes.c_int32),
                ("y", ctypes.c_void_p), ("dy", ctypes.c_void_p), ("dy_idx", ctypes.c_void_p),
                ("dy_count", ctypes.c_void_p)]


class LayerStats(ctypes.Structure):
    _fields_ = [("n_sites", ctypes.c_int32), ("n_tiles", ctypes.c_int32), ("n_touched", ctypes.c_int32),
                ("n_active", ctypes.c_int32), ("n_touched_tiles", ctypes.c_int32),
                ("flops_executed", ctypes.c_double), ("flops_dense", ctypes.c_double)]


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libevconv.so.  Raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2303_04670_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.evconv_query_workspace.argtypes = [ctypes.POINTER(NetDesc), ctypes.POINTER(ctypes.c_size_t)]
        L.evconv_create.argtypes = [ctypes.POINTER(NetDesc), vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp,
                                    ctypes.POINTER(vp)]
        L.evconv_create_static.argtypes = [ctypes.POINTER(NetDesc), vp, ctypes.c_size_t, vp, ctypes.POINTER(vp)]
        L.evconv_num_outputs.argtypes = [vp]
        L.evconv_reset.argtypes = [vp, vp, ctypes.POINTER(Out)]
        L.evconv_step.argtypes = [vp, vp, ctypes.POINTER(Out)]
        L.evconv_step_frame.argtypes = [vp, vp, ctypes.POINTER(Out)]
        L.evconv_destroy.argtypes = [vp]
        L.evconv_set_mode.argtypes = [vp, i32]
        L.evconv_current_mode.argtypes = [vp]
        L.evconv_set_refresh_period.argtypes = [vp, i32]
        L.evconv_node_shape.argtypes = [vp, i32, ctypes.POINTER(i32)]
        L.evconv_get_state.argtypes = [vp, i32, i32, vp, ctypes.c_size_t]
        L.evconv_get_state_stream.argtypes = [vp, i32, i32, i32, vp, ctypes.c_size_t]
        L.evconv_stream_stride.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(i32)]
        L.evconv_get_stats.argtypes = [vp, i32, ctypes.POINTER(LayerStats)]
        L.evconv_node_kernel.argtypes = [vp, i32]
        L.evconv_node_kernel.restype = ctypes.c_char_p
        L.evconv_last_error.argtypes = [vp]
        L.evconv_last_error.restype = ctypes.c_char_p
        L.evconv_profile_begin.argtypes = [vp, i32]
        L.evconv_profile_end.argtypes = [vp]
        L.evconv_get_node_time.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(ctypes.c_int64)]
        L.evconv_debug_chip_probes.argtypes = [vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_float), i32]
        L.evconv_debug_phase_stamps.argtypes = [i32, vp, i32, i32, ctypes.POINTER(i32)]
        _lib = L
    return _lib


def use_library(path):
    """Load another build of the library (the one with phase stamps) instead of libevconv.so; to
    be called before anything else of this module."""
    global LIB_PATH, _lib
    assert _lib is None, "the library is already loaded"
    LIB_PATH = path


def phase_stamps(operand_mode, reset=True, max_records=1 << 15):
    """evconv_debug_phase_stamps: (records as a uint64 array [n][32], number of workgroups that wrote
    one).  Raises EvConvError(UNSUPPORTED) on a library built without phase stamps."""
    buf = np.zeros((max_records, 32), np.uint64)
    n = ctypes.c_int32(0)
    st = lib().evconv_debug_phase_stamps(operand_mode, buf.ctypes.data, max_records, 1 if reset else 0, ctypes.byref(n))
    if st != 0:
        raise EvConvError(st, "evconv_debug_phase_stamps (library built without --phase-stamps?)")
    return buf[:min(n.value, max_records)], n.value


CHIP_PROBE_VALUES = 23
CHIP_PROBE_SCRATCH_BYTES = 1 << 20


def chip_probes(device="cuda:0"):
    """evconv_debug_chip_probes on a scratch tensor of its own: the list of probe values."""
    import torch
    scratch = torch.empty(CHIP_PROBE_SCRATCH_BYTES, dtype=torch.uint8, device=device)
    out = (ctypes.c_float * CHIP_PROBE_VALUES)()
    with torch.cuda.device(scratch.device):
        st = lib().evconv_debug_chip_probes(scratch.data_ptr(), scratch.numel(), torch.cuda.current_stream().cuda_stream,
                                            out, CHIP_PROBE_VALUES)
    if st != 0:
        raise EvConvError(st, "evconv_debug_chip_probes failed")
    return list(out)


class EvConvError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"evconv {STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {text}")
        self.status = status


def marshal_desc(net, flags=0, sparsify_tp=None, n_streams=1):
    """workloads.Net -> (NetDesc, keep-alive node array).  Element offsets become byte offsets."""
    nodes = (NodeDesc * len(net.nodes))()
    for i, nd in enumerate(net.nodes):
        n = nodes[i]
        n.op, n.act, n.in0, n.in1 = nd.op, nd.act, nd.in0, max(nd.in1, -1)
        n.c_in, n.c_out, n.kh, n.kw, n.stride, n.pad = nd.c_in, nd.c_out, nd.k, nd.k, nd.stride, nd.pad
        n.wdtype, n.is_output = nd.wdtype, nd.is_output
        n.weight_off = nd.w_off * 4 if nd.w_off >= 0 else -1
        n.bias_off = nd.b_off * 4 if nd.b_off >= 0 else -1
    if sparsify_tp is None:
        sparsify_tp = float(getattr(net, "sparsify_tp", 0.0))
    d = NetDesc(ABI_VERSION, len(net.nodes), nodes, net.in_c, net.in_h, net.in_w, flags,
                sparsify_tp, n_streams)
    return d, nodes


def evconv_query_workspace(desc: NetDesc) -> int:
    n = ctypes.c_size_t(0)
    st = lib().evconv_query_workspace(ctypes.byref(desc), ctypes.byref(n))
    if st != OK:
        raise EvConvError(st, lib().evconv_last_error(None).decode())
    return n.value


class _DeviceBytes:
    """A span of device memory owned by somebody else, for torch.as_tensor (no copy)."""

    def __init__(self, ptr, nbytes):
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False), "version": 2}


class EvConvNet:
    """Owns one evconv_net handle plus the torch tensors that back it.  static_workspace=True
    builds the net in the library's own per-GPU array (evconv_create_static): no workspace tensor
    is allocated."""

    def __init__(self, net, device="cuda:0", stream=None, static_workspace=False, **desc_kw):
        import torch
        self.torch = torch
        self.net = net
        self.device = torch.device(device)
        desc, self._nodes_keep = marshal_desc(net, **desc_kw)
        self._desc = desc
        nbytes = evconv_query_workspace(desc)
        self.workspace_bytes = nbytes
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        w = np.ascontiguousarray(net.weights, dtype=np.float32)
        h = ctypes.c_void_p()
        with torch.cuda.device(self.device):
            if static_workspace:
                self.workspace = None
                st = lib().evconv_create_static(ctypes.byref(desc), w.ctypes.data_as(ctypes.c_void_p), w.nbytes,
                                                ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(h))
            else:
                self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
                ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
                st = lib().evconv_create(ctypes.byref(desc), w.ctypes.data_as(ctypes.c_void_p), w.nbytes,
                                         ctypes.c_void_p(ws_ptr), nbytes,
                                         ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(h))
        if st != OK:
            raise EvConvError(st, lib().evconv_last_error(None).decode())
        self._h = h
        self.n_outputs = lib().evconv_num_outputs(self._h)
        self._outs = (Out * self.n_outputs)()
        stride, n = ctypes.c_size_t(0), ctypes.c_int32(0)
        self._check(lib().evconv_stream_stride(self._h, ctypes.byref(stride), ctypes.byref(n)))
        self.stream_stride, self.n_streams = stride.value, n.value

    # ---- the four calls
    def _check(self, st):
        if st != OK:
            raise EvConvError(st, lib().evconv_last_error(self._h).decode())

    def _dev_ptr(self, t):
        torch = self.torch
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
        want = (self.net.in_c, self.net.in_h, self.net.in_w)
        assert tuple(t.shape) == (want if self.n_streams == 1 else (self.n_streams,) + want)
        return ctypes.c_void_p(t.data_ptr())

    def reset(self, x0):
        self._check(lib().evconv_reset(self._h, self._dev_ptr(x0), self._outs))

    def step(self, increment):
        self._check(lib().evconv_step(self._h, self._dev_ptr(increment), self._outs))

    def step_frame(self, x_t):
        self._check(lib().evconv_step_frame(self._h, self._dev_ptr(x_t), self._outs))

    def destroy(self):
        if getattr(self, "_h", None):
            lib().evconv_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def set_mode(self, mode):
        self._check(lib().evconv_set_mode(self._h, mode))

    def current_mode(self) -> int:
        return lib().evconv_current_mode(self._h)

    def set_refresh_period(self, period):
        self._check(lib().evconv_set_refresh_period(self._h, int(period)))

    # ---- observability
    def shape(self, node):
        s = (ctypes.c_int32 * 3)()
        self._check(lib().evconv_node_shape(self._h, node, s))
        return int(s[0]), int(s[1]), int(s[2])

    def state(self, node, kind, stream=0) -> np.ndarray:
        c, h, w = self.shape(node)
        tiles = (-(-h // 8)) * (-(-w // 8))
        if kind in (STATE_Z, STATE_DY, STATE_Z2):
            a = np.empty((h, w, c), np.float32)
        elif kind == STATE_X_PREV:
            a = np.empty((c, h, w), np.float32)
        elif kind == STATE_IDX:
            a = np.empty(h * w, np.int32)
        elif kind == STATE_COUNT:
            a = np.empty(1, np.int32)
        elif kind == STATE_STEP:
            a = np.empty(1, np.float32)
        elif kind == STATE_BITMAP:
            a = np.empty(-(-tiles // 64), np.uint64)
        else:
            a = np.empty(tiles, np.uint64)
        self._check(lib().evconv_get_state_stream(self._h, stream, node, kind, a.ctypes.data_as(ctypes.c_void_p),
                                                  a.nbytes))
        return a

    def site_list(self, node, stream=0) -> np.ndarray:
        n = int(self.state(node, STATE_COUNT, stream)[0])
        return self.state(node, STATE_IDX, stream)[:n].copy()

    def stats(self, node) -> LayerStats:
        s = LayerStats()
        self._check(lib().evconv_get_stats(self._h, node, ctypes.byref(s)))
        return s

    def profile_begin(self, max_records):
        self._check(lib().evconv_profile_begin(self._h, max_records))

    def profile_end(self):
        self._check(lib().evconv_profile_end(self._h))

    def node_time(self, node):
        """(total milliseconds, launches) of a node's kernels since profile_begin."""
        ms, n = ctypes.c_double(), ctypes.c_int64()
        self._check(lib().evconv_get_node_time(self._h, node, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def kernel_name(self, node) -> str:
        return lib().evconv_node_kernel(self._h, node).decode()

    def outputs(self, stream=0):
        """Per output node: dict of torch views (y, dy as C x H x W; idx; count) of one stream, valid
        until the next call on this net.  The caller synchronises the stream before reading."""
        torch = self.torch
        res = []

        def view(ptr, nbytes, dtype, shape):
            span = _DeviceBytes(ptr + stream * self.stream_stride, nbytes)
            return torch.as_tensor(span, device=self.device).view(dtype).view(*shape)
        for j in range(self.n_outputs):
            o = self._outs[j]
            n = o.c * o.h * o.w
            res.append(dict(node=o.node,
                            y=view(o.y, n * 4, torch.float32, (o.c, o.h, o.w)),
                            dy=view(o.dy, n * 4, torch.float32, (o.c, o.h, o.w)),
                            idx=view(o.dy_idx, o.h * o.w * 4, torch.int32, (o.h * o.w,)),
                            count=view(o.dy_count, 4, torch.int32, (1,))))
        return res
