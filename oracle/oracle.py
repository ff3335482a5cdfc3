"""ctypes front end of the CPU oracle (oracle/evconv_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg.  Nothing in the product package imports this module.

Besides marshalling it derives, from the oracle's per-site byte masks, the integer
products the HIP path must reproduce bit for bit: ascending site lists, per-tile
occupancy words and the tile bitmap ("Implementation of Increment Layers": a mask element
says whether a region of the tensor is entirely zero).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libevconv_oracle.so")
_SRC = os.path.join(_HERE, "evconv_oracle.cpp")

KIND_Z, KIND_DY, KIND_Y, KIND_DENSE_Z, KIND_DENSE_A, KIND_POOL_IN = range(6)
SET_ACTIVE, SET_TOUCHED = 0, 1


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with g++ (no fast-math, no FMA contraction, OpenMP)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O3", "-march=x86-64-v3", "-fopenmp", "-ffp-contract=off", "-std=c++17",
               "-shared", "-fPIC", "-o", _SO, _SRC]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        L = ctypes.CDLL(_SO)
        L.evo_create.restype = ctypes.c_void_p
        L.evo_create.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_longlong,
                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double]
        L.evo_get_step.restype = ctypes.c_float
        L.evo_get_step.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.evo_destroy.argtypes = [ctypes.c_void_p]
        for f in (L.evo_dense_forward, L.evo_reset, L.evo_refresh, L.evo_step_frame, L.evo_step_increment):
            f.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
            f.restype = None
        L.evo_get_tensor.restype = ctypes.c_longlong
        L.evo_get_tensor.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.evo_get_set.restype = ctypes.c_longlong
        L.evo_get_set.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        L.evo_get_shape.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.evo_get_x_prev.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        L.evo_get_macs.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        _lib = L
    return _lib


def _f32(x):
    a = np.ascontiguousarray(x, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


class Oracle:
    """One network instance.  `net` is a workloads.Net (plain data).  fp32_state=True runs every
    operation in binary32 instead of binary64."""

    def __init__(self, net, fp32_state: bool = False):
        L = _load()
        self.net = net
        desc = np.zeros((len(net.nodes), 12), np.int32)
        for i, nd in enumerate(net.nodes):
            desc[i] = [nd.op, nd.act, nd.in0, nd.in1, nd.c_in, nd.c_out, nd.k, nd.stride, nd.pad,
                       nd.w_off, nd.b_off, nd.is_output]
        w = np.ascontiguousarray(net.weights, dtype=np.float64)
        self._h = L.evo_create(len(net.nodes), desc.ctypes.data_as(ctypes.c_void_p),
                               w.ctypes.data_as(ctypes.c_void_p), w.size,
                               net.in_c, net.in_h, net.in_w, int(fp32_state),
                               float(getattr(net, "sparsify_tp", 0.0)))
        if not self._h:
            raise ValueError("oracle rejected the network description")
        self.n_nodes = len(net.nodes)
        self.outputs = [i for i, nd in enumerate(net.nodes) if nd.is_output]

    def __del__(self):
        if getattr(self, "_h", None):
            _load().evo_destroy(self._h)
            self._h = None

    # ---- driving
    def dense_forward(self, x):
        a, p = _f32(x)
        _load().evo_dense_forward(self._h, p)

    def reset(self, x0):
        a, p = _f32(x0)
        _load().evo_reset(self._h, p)

    def refresh(self, x):
        """A regular forward pass in mid-stream: every accumulated tensor is recomputed, the
        recurrent state (DELAY nodes) is kept."""
        p = np.ascontiguousarray(x, dtype=np.float32).ctypes.data_as(ctypes.c_void_p)
        _load().evo_refresh(self._h, p)

    def step_frame(self, xt):
        a, p = _f32(xt)
        _load().evo_step_frame(self._h, p)

    def step_increment(self, inc):
        a, p = _f32(inc)
        _load().evo_step_increment(self._h, p)

    # ---- reading
    def shape(self, node):
        s = np.zeros(3, np.int32)
        _load().evo_get_shape(self._h, node, s.ctypes.data_as(ctypes.c_void_p))
        return int(s[0]), int(s[1]), int(s[2])

    def tensor(self, node, kind) -> np.ndarray:
        """H x W x C float64 array of the requested kind."""
        L = _load()
        n = L.evo_get_tensor(self._h, node, kind, None)
        if n < 0:
            raise ValueError("no such tensor")
        out = np.zeros(n, np.float64)
        L.evo_get_tensor(self._h, node, kind, out.ctypes.data_as(ctypes.c_void_p))
        c, h, w = self.shape(node)
        if kind == KIND_POOL_IN:
            c, h, w = self.shape(self.net.nodes[node].in0)
        return out.reshape(h, w, c) if n else out

    def z(self, node): return self.tensor(node, KIND_Z)
    def z2(self, node): return self.tensor(node, 6)   # elementwise multiply: accumulated second input
    def dy(self, node): return self.tensor(node, KIND_DY)
    def y(self, node): return self.tensor(node, KIND_Y)
    def dense_z(self, node): return self.tensor(node, KIND_DENSE_Z)
    def dense_value(self, node): return self.tensor(node, KIND_DENSE_A)

    def x_prev(self):
        out = np.zeros((self.net.in_c, self.net.in_h, self.net.in_w), np.float32)
        _load().evo_get_x_prev(self._h, out.ctypes.data_as(ctypes.c_void_p))
        return out

    def mask(self, node, kind=SET_ACTIVE) -> np.ndarray:
        """H x W uint8 mask of the active (kind 0) or touched (kind 1) set; node -1 = input."""
        L = _load()
        n = L.evo_get_set(self._h, node, kind, None)
        out = np.zeros(n, np.uint8)
        L.evo_get_set(self._h, node, kind, out.ctypes.data_as(ctypes.c_void_p))
        _, h, w = self.shape(node)
        return out.reshape(h, w)

    def site_list(self, node, kind=SET_ACTIVE) -> np.ndarray:
        """Strictly ascending int32 linear indices y*W + x of the set."""
        return np.flatnonzero(self.mask(node, kind).ravel()).astype(np.int32)

    def step_size(self, node) -> float:
        """Rounding step k of a sparsification node after the last refresh."""
        return float(_load().evo_get_step(self._h, node))

    def macs(self, node, tile=(8, 8)) -> dict:
        """Multiply-accumulate counts of a conv / linear node: `site` and `tile` = executed by the
        last step at site and at mask-tile granularity, `dense` = a regular forward pass without
        the padding taps, `dense_nominal` = outputs * k * k * c_in * c_out."""
        out = np.zeros(4, np.float64)
        _load().evo_get_macs(self._h, node, int(tile[0]), int(tile[1]), out.ctypes.data_as(ctypes.c_void_p))
        return dict(site=float(out[0]), tile=float(out[1]), dense=float(out[2]), dense_nominal=float(out[3]))


def tile_words(mask: np.ndarray, th: int = 8, tw: int = 8):
    """From an H x W mask: (occ, bitmap).  occ[t] is the 64-bit occupancy word of tile t (tiles
    row-major, tiles_x = ceil(W/tw)), bit (y % th) * tw + (x % tw); bitmap bit t % 64 of word
    t // 64 says that tile t holds at least one active site."""
    assert th * tw <= 64
    h, w = mask.shape
    ty, tx = -(-h // th), -(-w // tw)
    occ = np.zeros(ty * tx, np.uint64)
    ys, xs = np.nonzero(mask)
    t = (ys // th) * tx + xs // tw
    bit = ((ys % th) * tw + xs % tw).astype(np.uint64)
    np.bitwise_or.at(occ, t, np.uint64(1) << bit)
    bitmap = np.zeros(-(-occ.size // 64), np.uint64)
    nz = np.flatnonzero(occ)
    np.bitwise_or.at(bitmap, nz // 64, np.uint64(1) << (nz % 64).astype(np.uint64))
    return occ, bitmap
