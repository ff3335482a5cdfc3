"""Seeded synthetic workloads: network descriptions, weights and event streams.

This module is the only code shared by the CPU oracle's tests and the HIP path's
binding.  It holds *inputs only*: graph descriptions (plain data), random weights
and synthetic event streams.  None of the method's arithmetic (increments,
convolutions, masks, compaction) lives here.

The five workloads stand in for the paper's evaluation data (Experiments section:
346x260 / 240x180 sensors, voxel-grid, event-count and latest-timestamp encodings,
windows shifted by a small step), which is not available; only shapes and
increment densities are reproduced.

Network description = list of `Node`.  A node reads earlier nodes (`in0`, `in1`;
-1 is the network input).  Weight layout is `[c_out][c_in][k][k]` row-major fp32 in
one flat array; `w_off` / `b_off` are element offsets into it (-1: no bias).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Iterator, List, Optional, Tuple

import numpy as np

# op / activation codes: plain data shared by both marshalling layers
(OP_CONV2D, OP_ADD, OP_CONCAT, OP_UPSAMPLE2X, OP_MAXPOOL, OP_GAP, OP_LINEAR, OP_ACT, OP_SPARSIFY,
 OP_MUL, OP_DELAY) = range(11)   # OP_DELAY: in0 = the LATER node whose previous-step value it is, in1 = an
#                                  earlier node (or -1) with its height and width, c_out = its channels
ACT_NONE, ACT_RELU, ACT_SIGMOID, ACT_TANH, ACT_ONE_MINUS = range(5)   # ONE_MINUS: 1 - z
WD_F32, WD_BF16, WD_F32_SPLIT = 0, 1, 2   # WD_F32_SPLIT: fp32 weights, contraction through bf16 high/low parts


@dataclasses.dataclass
class Node:
    op: int
    act: int = ACT_NONE
    in0: int = -1
    in1: int = -2          # -2: unused
    c_in: int = 0
    c_out: int = 0
    k: int = 1
    stride: int = 1
    pad: int = 0
    w_off: int = -1
    b_off: int = -1
    is_output: int = 0
    wdtype: int = WD_F32


@dataclasses.dataclass
class Net:
    name: str
    in_c: int
    in_h: int
    in_w: int
    nodes: List[Node]
    weights: np.ndarray      # flat float32
    sparsify_tp: float = 0.0  # threshold parameter t_p of the sparsification layers (0: none)

    def node_shapes(self) -> List[Tuple[int, int, int]]:
        """(C, H, W) of every node's output (pure shape bookkeeping)."""
        out = []
        for nd in self.nodes:
            def shp(i):
                return (self.in_c, self.in_h, self.in_w) if i == -1 else out[i]
            if nd.op == OP_DELAY:
                _, h, w = shp(nd.in1)
                out.append((nd.c_out, h, w))
                continue
            c, h, w = shp(nd.in0)
            if nd.op in (OP_CONV2D, OP_MAXPOOL):
                ho = (h + 2 * nd.pad - nd.k) // nd.stride + 1
                wo = (w + 2 * nd.pad - nd.k) // nd.stride + 1
                out.append((nd.c_out if nd.op == OP_CONV2D else c, ho, wo))
            elif nd.op in (OP_ADD, OP_ACT, OP_SPARSIFY, OP_MUL):
                out.append((c, h, w))
            elif nd.op == OP_CONCAT:
                c2, _, _ = shp(nd.in1)
                out.append((c + c2, h, w))
            elif nd.op == OP_UPSAMPLE2X:
                out.append((c, 2 * h, 2 * w))
            elif nd.op == OP_GAP:
                out.append((c, 1, 1))
            elif nd.op == OP_LINEAR:
                out.append((nd.c_out, 1, 1))
            else:
                raise ValueError(nd.op)
        return out


class _NetBuilder:
    """Appends nodes and draws He-initialised weights N(0, 2/(k*k*c_in))."""

    def __init__(self, name, in_c, in_h, in_w, seed, bf16=False, bias=False, sparsify=False, sparsify_k=None,
                 sparsify_input=False):
        """sparsify: put a sparsification layer ahead of every convolution whose input is not the
        network input (sparsify_input: ahead of those as well, for streams whose input increments
        are dense but small); sparsify_k: fixed rounding step for all of them (None: the library
        derives it from the net's threshold parameter and the layer input at refresh time)."""
        self.sparsify, self.sparsify_k, self.sparsify_input = sparsify, sparsify_k, sparsify_input
        self.name, self.in_c, self.in_h, self.in_w = name, in_c, in_h, in_w
        self.rng = np.random.Generator(np.random.PCG64(seed))
        self.nodes: List[Node] = []
        self.chunks: List[np.ndarray] = []
        self.n_w = 0
        self.bf16 = bf16
        self.bias = bias

    def _chan(self, i):
        if i == -1:
            return self.in_c
        nd = self.nodes[i]
        if nd.op in (OP_CONV2D, OP_LINEAR, OP_DELAY):
            return nd.c_out
        if nd.op == OP_SPARSIFY:
            return self._chan(nd.in0)
        if nd.op == OP_CONCAT:
            return self._chan(nd.in0) + self._chan(nd.in1)
        return self._chan(nd.in0)

    def _push(self, arr):
        off = self.n_w
        self.chunks.append(arr.astype(np.float32).ravel())
        self.n_w += arr.size
        return off

    def sparsify_node(self, src):
        """A sparsification layer on node `src` (if this builder places such layers at all)."""
        if not self.sparsify:
            return src
        c_in = self._chan(src)
        k_off = -1
        if self.sparsify_k is not None:
            k_off = self._push(np.asarray([self.sparsify_k], np.float32))
        self.nodes.append(Node(OP_SPARSIFY, ACT_NONE, src, -2, c_in, c_in, 1, 1, 0, k_off, -1, 0))
        return len(self.nodes) - 1

    def conv(self, src, c_out, k, stride=1, pad=None, act=ACT_RELU, out=0, op=OP_CONV2D, sparsify_input=True):
        """sparsify_input=False: the caller has placed this conv's sparsification layer itself."""
        c_in = self._chan(src)
        if sparsify_input and (src >= 0 or self.sparsify_input) and op == OP_CONV2D:
            src = self.sparsify_node(src)
        pad = k // 2 if pad is None else pad
        std = math.sqrt(2.0 / (k * k * c_in))
        w = self.rng.standard_normal((c_out, c_in, k, k)) * std
        w = w.astype(np.float32)
        if self.bf16:
            w = round_to_bf16(w)
        w_off = self._push(w)
        b_off = -1
        if self.bias:
            b_off = self._push((self.rng.standard_normal(c_out) * 0.1).astype(np.float32))
        self.nodes.append(Node(op, act, src, -2, c_in, c_out, k, stride, pad, w_off, b_off, out,
                               WD_BF16 if self.bf16 else WD_F32))
        return len(self.nodes) - 1

    def linear(self, src, c_out, act=ACT_NONE, out=0):
        return self.conv(src, c_out, 1, 1, 0, act, out, op=OP_LINEAR)

    def simple(self, op, a, b=-2, act=ACT_NONE, k=1, stride=1, pad=0, out=0):
        c = self._chan(a)
        c_out = c + (self._chan(b) if op == OP_CONCAT else 0)
        self.nodes.append(Node(op, act, a, b, c, c_out, k, stride, pad, -1, -1, out))
        return len(self.nodes) - 1

    def delay(self, c, like=-1):
        """A recurrent state of c channels with the height and width of node `like`; the node it
        delays is set afterwards with close_delay()."""
        self.nodes.append(Node(OP_DELAY, ACT_NONE, -3, like, c, c, 1, 1, 0, -1, -1, 0))
        return len(self.nodes) - 1

    def close_delay(self, d, src):
        self.nodes[d].in0 = src

    def finish(self) -> Net:
        w = np.concatenate(self.chunks) if self.chunks else np.zeros(0, np.float32)
        return Net(self.name, self.in_c, self.in_h, self.in_w, self.nodes, w)


def with_weight_dtype(net: Net, wdtype: int) -> Net:
    """The same network and fp32 weight values with another declared contraction dtype on every
    conv / linear node (plain data; WD_BF16 here does not round the values)."""
    nodes = [dataclasses.replace(nd, wdtype=wdtype) if nd.op in (OP_CONV2D, OP_LINEAR) else nd for nd in net.nodes]
    return dataclasses.replace(net, nodes=nodes, name=net.name + f"_wd{wdtype}")


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 -> nearest-even bf16, returned as fp32 (an input transformation only)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


# --------------------------------------------------------------------------- networks

def net_single_conv(seed=1001, c=16, h=64, w=64) -> Net:
    """Workload 1: one 3x3 conv c->c, stride 1, pad 1, then ReLU."""
    b = _NetBuilder("single_conv3x3", c, h, w, seed)
    b.conv(-1, c, 3, 1, 1, ACT_RELU, out=1)
    return b.finish()


def net_conv_stack(seed=1002, h=180, w=240, sparsify=False, sparsify_k=None) -> Net:
    """Workload 2: 4 conv3x3 layers 5->32 s1, 32->32 s2, 32->64 s2, 64->64 s1, ReLU each."""
    b = _NetBuilder("conv_stack4" + ("_sp" if sparsify else ""), 5, h, w, seed, sparsify=sparsify,
                    sparsify_k=sparsify_k)
    x = b.conv(-1, 32, 3, 1)
    x = b.conv(x, 32, 3, 2)
    x = b.conv(x, 64, 3, 2)
    b.conv(x, 64, 3, 1, out=1)
    return b.finish()


def net_unet_depth(seed=1003, h=256, w=352, bf16=False, width=32, sparsify=False, sparsify_k=None,
                   sparsify_input=False) -> Net:
    """Workload 3: UNet depth net.  head 5x5 -> 3 strided 5x5 encoders -> 2 residual blocks
    -> 3 x (skip-add, bilinear x2, conv5x5) -> skip-add with head -> 1x1 conv + sigmoid."""
    b = _NetBuilder("unet_depth" + ("_bf16" if bf16 else "") + ("_sp" if sparsify else ""), 5, h, w, seed,
                    bf16=bf16, sparsify=sparsify, sparsify_k=sparsify_k, sparsify_input=sparsify_input)
    head = b.conv(-1, width, 5)
    e1 = b.conv(head, 2 * width, 5, 2)
    e2 = b.conv(e1, 4 * width, 5, 2)
    e3 = b.conv(e2, 8 * width, 5, 2)
    x = e3
    for _ in range(2):
        r = b.conv(x, 8 * width, 3)
        r = b.conv(r, 8 * width, 3, act=ACT_NONE)
        x = b.simple(OP_ADD, x, r, act=ACT_RELU)
    for skip, c_out in ((e3, 4 * width), (e2, 2 * width), (e1, width)):
        x = b.simple(OP_ADD, x, skip)
        # (the decoder conv's sparsification layer sits ahead of the up-sampling: conv o up-sampling
        # is one linear operator, and its input is the tensor at the lower resolution)
        x = b.sparsify_node(x)
        x = b.simple(OP_UPSAMPLE2X, x)
        x = b.conv(x, c_out, 5, sparsify_input=False)
    x = b.simple(OP_ADD, x, head)
    b.conv(x, 1, 1, 1, 0, ACT_SIGMOID, out=1)
    return b.finish()


def net_resnet18(seed=1004, h=224, w=224, n_classes=101, bf16=False, width=64) -> Net:
    """Workload 4: ResNet-18-style classifier on a 2-channel event histogram (BN folded away,
    1x1 stride-2 projection shortcuts)."""
    b = _NetBuilder("resnet18" + ("_bf16" if bf16 else ""), 2, h, w, seed, bf16=bf16)
    x = b.conv(-1, width, 7, 2, 3)
    x = b.simple(OP_MAXPOOL, x, k=3, stride=2, pad=1)
    c = width
    for stage in range(4):
        c_out = width << stage
        for blk in range(2):
            s = 2 if (stage > 0 and blk == 0) else 1
            r = b.conv(x, c_out, 3, s)
            r = b.conv(r, c_out, 3, 1, act=ACT_NONE)
            sc = x if (s == 1 and c == c_out) else b.conv(x, c_out, 1, s, 0, act=ACT_NONE)
            x = b.simple(OP_ADD, r, sc, act=ACT_RELU)
            c = c_out
    g = b.simple(OP_GAP, x)
    b.linear(g, n_classes, out=1)
    return b.finish()


def net_flow(seed=1005, h=256, w=256, width=64) -> Net:
    """Workload 5: optical-flow encoder-decoder, skip concat, a 2-channel flow head per scale."""
    b = _NetBuilder("flow_encdec", 4, h, w, seed)
    enc = []
    x = -1
    for i in range(4):
        x = b.conv(x, width << i, 3, 2)
        enc.append(x)
    for _ in range(2):
        r = b.conv(x, width << 3, 3)
        r = b.conv(r, width << 3, 3, act=ACT_NONE)
        x = b.simple(OP_ADD, x, r, act=ACT_RELU)
    skips = [enc[2], enc[1], enc[0], -1]
    outs = [width << 2, width << 1, width, width >> 1]
    for skip, c_out in zip(skips, outs):
        u = b.simple(OP_UPSAMPLE2X, x)
        cat = b.simple(OP_CONCAT, u, skip)
        x = b.conv(cat, c_out, 3)
        b.conv(x, 2, 1, 1, 0, ACT_NONE, out=1)
    return b.finish()


def net_flow_delayed(seed=1006, h=256, w=256, width=64, d_width=32) -> Net:
    """Delayed-integration variant of the optical-flow encoder-decoder ("Mitigating Reduced
    Sparsity on Upsampling"): same encoders and residual blocks as `net_flow`; a decoder no
    longer receives the previous decoder's output, only its skip (the first one still gets the
    bottleneck); every decoder output D and its 2-channel prediction P is upsampled to full
    resolution, all are concatenated, and two convolutions produce the final prediction.

    Own choices (the figures are not available): every decoder emits `d_width` channels so that
    the full-resolution tensors stay small; the first of the two final convolutions (3x3 over
    the concatenation of all D' and all P') is applied as two partial convolutions, over the D'
    channels and over the P' channels, whose outputs are added before the ReLU - the same
    function by linearity (Eq.9), and it keeps the wide part a multiple of 32 channels.
    """
    b = _NetBuilder("flow_delayed", 4, h, w, seed)
    enc = []
    x = -1
    for i in range(4):
        x = b.conv(x, width << i, 3, 2)
        enc.append(x)
    for _ in range(2):
        r = b.conv(x, width << 3, 3)
        r = b.conv(r, width << 3, 3, act=ACT_NONE)
        x = b.simple(OP_ADD, x, r, act=ACT_RELU)
    u = b.simple(OP_UPSAMPLE2X, x)
    dec_in = [b.simple(OP_CONCAT, u, enc[2]), enc[1], enc[0], -1]   # resolutions 1/8, 1/4, 1/2, 1
    d_full, p_full = [], []
    for level, src in enumerate(dec_in):
        d = b.conv(src, d_width, 3)
        p = b.conv(d, 2, 1, 1, 0, ACT_NONE, out=1)
        for _ in range(3 - level):
            d = b.simple(OP_UPSAMPLE2X, d)
            p = b.simple(OP_UPSAMPLE2X, p)
        d_full.append(d)
        p_full.append(p)
    dc, pc = d_full[0], p_full[0]
    for d, p in zip(d_full[1:], p_full[1:]):
        dc = b.simple(OP_CONCAT, dc, d)
        pc = b.simple(OP_CONCAT, pc, p)
    fd = b.conv(dc, d_width, 3, act=ACT_NONE)
    fp = b.conv(pc, d_width, 3, act=ACT_NONE)
    f = b.simple(OP_ADD, fd, fp, act=ACT_RELU)
    b.conv(f, 2, 1, 1, 0, ACT_NONE, out=1)
    return b.finish()


def net_gated(seed=1007, in_c=5, h=64, w=96, width=32, bias=False) -> Net:
    """Gated convolution blocks: the gate structure of ConvLSTM / ConvGRU cells (a sigmoid gate
    times a tanh candidate, an update gate blending the block input with the candidate), without
    the recurrence.  Exercises the elementwise-multiply increment (Eq.15-17) with both operands
    changing, one operand constant over a step, and a product of products."""
    b = _NetBuilder("gated", in_c, h, w, seed, bias=bias)
    x = b.conv(-1, width, 3)
    for _ in range(2):
        g = b.conv(x, width, 3, act=ACT_SIGMOID)          # gate in (0, 1)
        c = b.conv(x, width, 3, act=ACT_TANH)             # candidate in (-1, 1)
        gc = b.simple(OP_MUL, g, c)                       # g * c
        u = b.conv(x, width, 1, 1, 0, act=ACT_SIGMOID)    # update gate
        ux = b.simple(OP_MUL, u, x)                       # u * x
        x = b.simple(OP_ADD, gc, ux, act=ACT_RELU)
    sq = b.simple(OP_MUL, x, x)                           # both operands the same node
    b.conv(sq, 2, 1, 1, 0, ACT_NONE, out=1)
    return b.finish()


def net_random_small(seed, in_c=3, h=13, w=11, bias=True) -> Net:
    """A tiny graph touching every op, odd sizes, K in {1,3,5,7}, strides 1 and 2 (tests only)."""
    b = _NetBuilder("random_small", in_c, h, w, seed, bias=bias)
    a = b.conv(-1, 6, 3, 1)
    c = b.conv(a, 6, 5, 1, act=ACT_NONE)
    d = b.simple(OP_ADD, a, c, act=ACT_RELU)
    e = b.conv(d, 8, 7, 2)
    f = b.simple(OP_UPSAMPLE2X, e)
    g = b.conv(f, 6, 3, 1, act=ACT_RELU)
    # upsample of ceil(h/2) may overshoot h by one: crop by a stride-1 valid 1x1/2x? keep
    # sizes consistent by pooling both branches instead
    p1 = b.simple(OP_MAXPOOL, d, k=3, stride=2, pad=1)
    p2 = b.simple(OP_MAXPOOL, g, k=3, stride=2, pad=1)
    p2 = b.simple(OP_MAXPOOL, p2, k=3, stride=2, pad=1)
    p1b = b.simple(OP_MAXPOOL, p1, k=3, stride=2, pad=1)
    cat = b.simple(OP_CONCAT, p1b, p2)
    s = b.conv(cat, 4, 1, 1, 0, ACT_SIGMOID, out=1)
    q = b.simple(OP_ACT, cat, act=ACT_RELU)
    gp = b.simple(OP_GAP, q)
    b.linear(gp, 5, out=1)
    return b.finish()


# --------------------------------------------------------------------------- streams

def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _raster_segment(x0, y0, x1, y1):
    """Integer pixels on the segment (dense sampling, deduplicated by caller)."""
    n = int(max(abs(x1 - x0), abs(y1 - y0)) * 2) + 2
    t = np.linspace(0.0, 1.0, n)
    return np.rint(x0 + (x1 - x0) * t).astype(np.int64), np.rint(y0 + (y1 - y0) * t).astype(np.int64)


class _Primitive:
    """A moving edge (segment) or blob (circle outline) that reflects at the borders."""

    def __init__(self, rng, h, w, vmin, vmax, kinds=("edge", "blob")):
        self.h, self.w = h, w
        self.kind = kinds[int(rng.integers(len(kinds)))]
        self.cx = rng.uniform(0, w)
        self.cy = rng.uniform(0, h)
        sp = rng.uniform(vmin, vmax)
        ang = rng.uniform(0, 2 * math.pi)
        self.vx, self.vy = sp * math.cos(ang), sp * math.sin(ang)
        if self.kind == "edge":
            self.len = rng.uniform(20, 80)
            self.theta = rng.uniform(0, math.pi)
        else:
            self.r = rng.uniform(3, 8)

    def advance(self):
        self.cx += self.vx
        self.cy += self.vy
        if self.cx < 0 or self.cx > self.w - 1:
            self.vx = -self.vx
            self.cx = min(max(self.cx, 0), self.w - 1)
        if self.cy < 0 or self.cy > self.h - 1:
            self.vy = -self.vy
            self.cy = min(max(self.cy, 0), self.h - 1)

    def pixels(self):
        if self.kind == "edge":
            dx, dy = 0.5 * self.len * math.cos(self.theta), 0.5 * self.len * math.sin(self.theta)
            xs, ys = _raster_segment(self.cx - dx, self.cy - dy, self.cx + dx, self.cy + dy)
        else:
            n = int(2 * math.pi * self.r * 2) + 4
            a = np.linspace(0, 2 * math.pi, n, endpoint=False)
            xs = np.rint(self.cx + self.r * np.cos(a)).astype(np.int64)
            ys = np.rint(self.cy + self.r * np.sin(a)).astype(np.int64)
        ok = (xs >= 0) & (xs < self.w) & (ys >= 0) & (ys < self.h)
        return np.unique(ys[ok] * self.w + xs[ok])


class _Scene:
    """Moving primitives; each step yields candidate event pixels (newly covered: polarity +1,
    newly uncovered: polarity -1), topped up with uniform background-activity pixels and
    thinned to hit a requested number of event pixels."""

    def __init__(self, rng, h, w, n_prim, vmin=0.5, vmax=2.0):
        self.rng, self.h, self.w = rng, h, w
        self.prims = [_Primitive(rng, h, w, vmin, vmax) for _ in range(n_prim)]
        self.cover = [p.pixels() for p in self.prims]

    def step_events(self, n_target: int):
        on, off = [], []
        for i, p in enumerate(self.prims):
            p.advance()
            new = p.pixels()
            on.append(np.setdiff1d(new, self.cover[i], assume_unique=True))
            off.append(np.setdiff1d(self.cover[i], new, assume_unique=True))
            self.cover[i] = new
        on = np.unique(np.concatenate(on))
        off = np.setdiff1d(np.unique(np.concatenate(off)), on, assume_unique=True)
        pix = np.concatenate([on, off])
        pol = np.concatenate([np.ones(on.size), -np.ones(off.size)])
        if pix.size > n_target:
            keep = np.sort(self.rng.choice(pix.size, n_target, replace=False))
            pix, pol = pix[keep], pol[keep]
        elif pix.size < n_target:
            extra = self.rng.choice(self.h * self.w, n_target - pix.size, replace=False)
            extra = np.setdiff1d(extra, pix)
            pix = np.concatenate([pix, extra])
            pol = np.concatenate([pol, self.rng.choice([-1.0, 1.0], extra.size)])
        return pix, pol


def stream_line_increments(seed=1001, c=16, h=64, w=64, steps=10, density=0.02, n_seg=3):
    """Workload 1.  Returns (x0, [dx_1 .. dx_steps]) as C x H x W fp32.  x0 ~ U(-1,1); each
    increment is nonzero on `n_seg` one-pixel-wide moving segments (all channels ~ N(0, 0.5^2)
    there, exactly 0 elsewhere) covering about `density` of the pixels."""
    rng = _rng(seed)
    x0 = rng.uniform(-1.0, 1.0, (c, h, w)).astype(np.float32)
    target = max(1, int(round(density * h * w)))
    seg_len = target / n_seg
    segs = []
    for _ in range(n_seg):
        segs.append(dict(cx=rng.uniform(0, w), cy=rng.uniform(0, h), th=rng.uniform(0, math.pi),
                         vx=rng.uniform(-2, 2), vy=rng.uniform(-2, 2)))
    incs = []
    for _ in range(steps):
        pix = []
        for s in segs:
            s["cx"] += s["vx"]
            s["cy"] += s["vy"]
            if s["cx"] < 0 or s["cx"] > w - 1:
                s["vx"] = -s["vx"]
                s["cx"] = min(max(s["cx"], 0), w - 1)
            if s["cy"] < 0 or s["cy"] > h - 1:
                s["vy"] = -s["vy"]
                s["cy"] = min(max(s["cy"], 0), h - 1)
            dx, dy = 0.5 * seg_len * math.cos(s["th"]), 0.5 * seg_len * math.sin(s["th"])
            xs, ys = _raster_segment(s["cx"] - dx, s["cy"] - dy, s["cx"] + dx, s["cy"] + dy)
            ok = (xs >= 0) & (xs < w) & (ys >= 0) & (ys < h)
            pix.append(ys[ok] * w + xs[ok])
        pix = np.unique(np.concatenate(pix))
        if pix.size > target:
            pix = np.sort(rng.choice(pix, target, replace=False))
        elif pix.size < target:
            extra = np.setdiff1d(rng.choice(h * w, target - pix.size, replace=False), pix)
            pix = np.sort(np.concatenate([pix, extra]))
        d = np.zeros((c, h * w), np.float32)
        d[:, pix] = (rng.standard_normal((c, pix.size)) * 0.5).astype(np.float32)
        incs.append(d.reshape(c, h, w))
    return x0, incs


class VoxelStream:
    """Workloads 2 and 3: frames of a B-bin event voxel grid over a sliding window.

    Own definition (the paper names the encoding but gives no formula): time is cut into
    absolute slots of `slot` steps; an event at absolute slot-time tau adds
    polarity * max(0, 1 - |k - tau|) to slots k = floor(tau), floor(tau)+1, stored in channel
    k mod B (a ring), so an event's contribution never changes while it is inside the window.
    Frame t holds the events of the last `window` steps; consecutive frames therefore differ
    only at pixels with entering or leaving events.  `density(t)` is the requested fraction of
    changed pixels per step (entering + leaving).
    """

    def __init__(self, seed, h, w, bins=5, n_prim=20, slot=4, window=12, density=0.02):
        assert window + slot <= (bins - 1) * slot, "ring would alias"
        self.rng = _rng(seed)
        self.h, self.w, self.bins, self.slot, self.window = h, w, bins, slot, window
        self.scene = _Scene(self.rng, h, w, n_prim)
        self.density = density if callable(density) else (lambda t, d=density: d)
        self.t = 0
        self.events = []    # per step: (pix, pol, tau)

    def _emit(self):
        n_changed = self.density(self.t) * self.h * self.w
        pix, pol = self.scene.step_events(max(1, int(round(n_changed / 2))))
        tau = (self.t + self.rng.integers(0, 8, pix.size) / 8.0) / self.slot
        self.events.append((pix, pol, tau))
        self.t += 1

    def frame(self) -> np.ndarray:
        """Advance one step and return the C x H x W fp32 frame of the current window."""
        self._emit()
        acc = np.zeros((self.bins, self.h * self.w), np.float64)
        for pix, pol, tau in self.events[-self.window:]:
            k0 = np.floor(tau).astype(np.int64)
            f = tau - k0
            np.add.at(acc, (k0 % self.bins, pix), pol * (1.0 - f))
            np.add.at(acc, ((k0 + 1) % self.bins, pix), pol * f)
        if len(self.events) > self.window:
            self.events = self.events[-self.window:]
        return acc.astype(np.float32).reshape(self.bins, self.h, self.w)


def stream_voxel(seed, h, w, steps, density=0.02, warm=None, **kw) -> Iterator[np.ndarray]:
    """Yields steps+1 frames: x0 (after `warm` warm-up steps that fill the window) then one
    frame per step."""
    vs = VoxelStream(seed, h, w, density=density, **kw)
    warm = vs.window if warm is None else warm
    for _ in range(warm):
        vs._emit()
    for _ in range(steps + 1):
        yield vs.frame()


def drifting_background(frames, amplitude=0.5, drift=1e-3, event_scale=0.05):
    """The given frames, scaled by `event_scale`, on top of a smooth background of amplitude
    `amplitude` (the same in every channel) whose phase moves a little per step: every pixel
    changes by at most `drift` at every step and event pixels change by `event_scale`, both small
    against the values themselves.  Increments that are dense but tiny almost everywhere: the
    situation the sparsification layer is made for ("Forward pass with increment tensors": the
    difference of consecutive inputs is sparse *and* many of its elements have small absolute
    values)."""
    phase = None
    for t, f in enumerate(frames):
        if phase is None:
            h, w = f.shape[-2:]
            yy, xx = np.mgrid[0:h, 0:w]
            phase = 2.0 * math.pi * (3.0 * xx / w + 2.0 * yy / h)
        bg = amplitude * np.sin(phase + t * drift / amplitude)
        yield (event_scale * f + bg[None].astype(np.float32)).astype(np.float32)


def stream_voxel_drifting_background(seed, h, w, steps, density=0.02, amplitude=0.5, drift=1e-3, event_scale=0.05, **kw):
    """Workload-3 event frames under drifting_background()."""
    return drifting_background(stream_voxel(seed, h, w, steps, density, **kw), amplitude, drift, event_scale)


def density_sweep_1_5(t, period=50):
    """1 % .. 5 % changed pixels, slow sinusoid (workload 2)."""
    return 0.03 + 0.02 * math.sin(2 * math.pi * t / period)


def stream_histogram(seed=1004, h=224, w=224, steps=100, d_lo=0.005, d_hi=0.05):
    """Workload 4: 2-channel on/off event-count histogram; each step a moving-contour pixel set
    gets Poisson(lambda in [1,3]) new counts; changed-pixel density ramps d_lo -> d_hi."""
    rng = _rng(seed)
    scene = _Scene(rng, h, w, 20)
    x = np.zeros((2, h * w), np.float32)
    for t in range(steps + 1):
        dens = d_lo + (d_hi - d_lo) * (t / max(1, steps))
        pix, pol = scene.step_events(max(1, int(round(dens * h * w))))
        lam = rng.uniform(1.0, 3.0)
        cnt = np.maximum(1, rng.poisson(lam, pix.size)).astype(np.float32)
        ch = (pol < 0).astype(np.int64)
        x = x.copy()
        x[ch, pix] += cnt
        yield x.reshape(2, h, w)


def stream_count_timestamp(seed=1005, h=256, w=256, densities=None, steps_per=100):
    """Workload 5: 4 channels = per-polarity counts (0,1) and latest normalised timestamps
    (2,3).  `densities` log-spaced 0.1 % .. 20 %, `steps_per` steps at each."""
    rng = _rng(seed)
    if densities is None:
        densities = np.geomspace(0.001, 0.2, 10)
    scene = _Scene(rng, h, w, 20)
    total = len(densities) * steps_per
    x = np.zeros((4, h * w), np.float32)
    yield x.reshape(4, h, w).copy()
    t = 0
    for dens in densities:
        for _ in range(steps_per):
            t += 1
            pix, pol = scene.step_events(max(1, int(round(dens * h * w))))
            ch = (pol < 0).astype(np.int64)
            x = x.copy()
            x[ch, pix] += 1.0
            x[2 + ch, pix] = np.float32(t / total)
            yield x.reshape(4, h, w)


def changed_fraction(a: np.ndarray, b: np.ndarray) -> float:
    """Fraction of pixels at which two C x H x W frames differ (diagnostic for recipes)."""
    return float(np.any(a != b, axis=0).mean())


def net_random_wide(seed, h=24, w=40) -> Net:
    """A random encoder-decoder-like graph over the ops of the matrix-core paths (tests only):
    channel counts that are multiples of 4 including ragged ones (20, 36, 68), kernels 1/3/5,
    strides 1/2, residual and skip adds, x2 up-sampling straight into a convolution, concat,
    gates (sigmoid x tanh), a prediction head."""
    rng = np.random.Generator(np.random.PCG64(seed))
    b = _NetBuilder(f"random_wide_{seed}", int(rng.choice([3, 4, 5])), h, w, seed + 1000, bias=bool(rng.integers(0, 2)))
    chans = [16, 20, 32, 36, 48, 64, 68]
    c0 = 32 * int(rng.integers(1, 3))
    x = b.conv(-1, c0, int(rng.choice([3, 5])), 1)                      # narrow-input layer
    full = [x]
    c1 = 32 * int(rng.integers(1, 4))
    y = b.conv(x, c1, int(rng.choice([3, 5])), 2)                       # down
    for _ in range(int(rng.integers(1, 3))):                            # residual blocks at half resolution
        r = b.conv(y, c1, 3, 1)
        r = b.conv(r, c1, int(rng.choice([1, 3])), 1, act=ACT_NONE)
        y = b.simple(OP_ADD, y, r, act=ACT_RELU)
    if rng.integers(0, 2):                                              # a gate
        g = b.conv(y, c1, 1, 1, 0, act=ACT_SIGMOID)
        t = b.conv(y, c1, 3, 1, act=ACT_TANH)
        y = b.simple(OP_MUL, g, t)
    cm = int(rng.choice(chans))
    if cm % 32:                                                         # ragged channel count into the matrix cores
        y = b.conv(y, 32, 3, 1)
        cat = b.simple(OP_CONCAT, y, b.conv(y, cm - 32 if cm > 32 else 4, 1, 1, 0))
        y = b.conv(cat, c1, 3, 1)
    u = b.simple(OP_UPSAMPLE2X, y)                                      # straight into a conv: folded into its gather
    d = b.conv(u, c0, int(rng.choice([3, 5])), 1, act=ACT_NONE)
    d = b.simple(OP_ADD, d, full[0], act=ACT_RELU)                      # skip add in the conv epilogue
    b.conv(d, int(rng.choice([1, 2, 3])), 1, 1, 0, int(rng.choice([ACT_NONE, ACT_SIGMOID])), out=1)
    return b.finish()


def net_convlstm(seed=1008, in_c=4, h=64, w=96, hidden=28, out_c=2, k=3, bias=True) -> Net:
    """A ConvLSTM cell on the event tensor followed by a 1 x 1 prediction head (tests and a
    benchmark leg; random weights): i, f, o = sigmoid(conv([x, h'])), g = tanh(conv([x, h'])),
    c = f * c' + i * g, h = o * tanh(c), with h', c' the cell's own h, c of the previous step."""
    b = _NetBuilder(f"convlstm_{hidden}", in_c, h, w, seed, bias=bias)
    h_prev = b.delay(hidden)
    c_prev = b.delay(hidden)
    xh = b.simple(OP_CONCAT, -1, h_prev)
    gi = b.conv(xh, hidden, k, 1, act=ACT_SIGMOID)
    gf = b.conv(xh, hidden, k, 1, act=ACT_SIGMOID)
    go = b.conv(xh, hidden, k, 1, act=ACT_SIGMOID)
    gg = b.conv(xh, hidden, k, 1, act=ACT_TANH)
    fc = b.simple(OP_MUL, gf, c_prev)
    ig = b.simple(OP_MUL, gi, gg)
    c_new = b.simple(OP_ADD, fc, ig)
    tc = b.simple(OP_ACT, c_new, act=ACT_TANH)
    h_new = b.simple(OP_MUL, go, tc)
    b.close_delay(h_prev, h_new)
    b.close_delay(c_prev, c_new)
    b.conv(h_new, out_c, 1, 1, 0, ACT_NONE, out=1)
    return b.finish()


def net_convgru(seed=1009, in_c=4, h=64, w=96, hidden=32, out_c=2, k=3, bias=True) -> Net:
    """A ConvGRU cell and a 1 x 1 head (tests; random weights): z, r = sigmoid(conv([x, h'])),
    c = tanh(conv([x, r * h'])), h = (1 - z) * h' + z * c, with h' the cell's own h of the previous
    step."""
    b = _NetBuilder(f"convgru_{hidden}", in_c, h, w, seed, bias=bias)
    h_prev = b.delay(hidden)
    xh = b.simple(OP_CONCAT, -1, h_prev)
    gz = b.conv(xh, hidden, k, 1, act=ACT_SIGMOID)
    gr = b.conv(xh, hidden, k, 1, act=ACT_SIGMOID)
    rh = b.simple(OP_MUL, gr, h_prev)
    xrh = b.simple(OP_CONCAT, -1, rh)
    cand = b.conv(xrh, hidden, k, 1, act=ACT_TANH)
    omz = b.simple(OP_ACT, gz, act=ACT_ONE_MINUS)
    keep = b.simple(OP_MUL, omz, h_prev)
    new = b.simple(OP_MUL, gz, cand)
    h_new = b.simple(OP_ADD, keep, new)
    b.close_delay(h_prev, h_new)
    b.conv(h_new, out_c, 1, 1, 0, ACT_NONE, out=1)
    return b.finish()
