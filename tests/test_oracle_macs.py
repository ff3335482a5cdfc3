"""Pins for the oracle's multiply-accumulate counters (the paper's "MFLOPs" columns, Tables I-III,
under an explicit counting rule).  Every expected number is a hand count: a (tap, output) pair of a
convolution costs c_in * c_out multiply-accumulates, and

  * at site granularity a pair is executed when its input site is inside the image and active,
  * at tile granularity every tile of th x tw outputs that holds a touched output is computed in
    full, all k * k taps ("Convolution on Sparse Inputs": filter applications are skipped per
    all-zero section of the mask),
  * a regular forward pass executes every pair whose input site is inside the image.
"""
import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2303_04670_amd import workloads as wl


def _conv_net(c_in, c_out, k, stride, h, w, pad=None):
    b = wl._NetBuilder("one_conv", c_in, h, w, 5)
    b.conv(-1, c_out, k, stride, pad=pad, act=wl.ACT_RELU, out=1)
    return b.finish()


def _one_pixel_step(net, pixels):
    o = Oracle(net)
    o.reset(np.zeros((net.in_c, net.in_h, net.in_w), np.float32))
    inc = np.zeros((net.in_c, net.in_h, net.in_w), np.float32)
    for (y, x) in pixels:
        inc[0, y, x] = 1.0
    o.step_increment(inc)
    return o


# (k, stride, h, w, active pixels) -> number of executed (tap, output) pairs, counted by hand:
#  3x3 s1 pad 1, interior pixel: the 9 outputs around it, one tap each
#  corner pixel (0,0): outputs (0..1, 0..1) only
#  last-row pixel: 2 x 3 outputs
#  two horizontally adjacent pixels: 9 pairs each (3 x 4 outputs, the middle six hit by two taps)
#  5x5 s2 pad 2: output o reads input 2o - 2 + t, so an even input coordinate is read through taps
#  {0, 2, 4} (3 outputs) and an odd one through taps {1, 3} (2 outputs): (4,4) -> 9, (5,4) -> 6,
#  (5,5) -> 4; at the first row / column one of the three falls off: (0,0) -> 2 x 2
#  1x1: the site itself
PAIR_CASES = [
    (3, 1, 12, 10, [(4, 4)], 9),
    (3, 1, 12, 10, [(0, 0)], 4),
    (3, 1, 12, 10, [(11, 5)], 6),
    (3, 1, 12, 10, [(4, 4), (4, 5)], 18),
    (5, 2, 16, 16, [(4, 4)], 9),
    (5, 2, 16, 16, [(5, 4)], 6),
    (5, 2, 16, 16, [(5, 5)], 4),
    (5, 2, 16, 16, [(0, 0)], 4),
    (1, 1, 7, 9, [(3, 3), (6, 8)], 2),
]


@pytest.mark.parametrize("k,stride,h,w,pixels,pairs", PAIR_CASES)
def test_site_level_macs_are_the_hand_counted_pairs(k, stride, h, w, pixels, pairs):
    c_in, c_out = 3, 5
    o = _one_pixel_step(_conv_net(c_in, c_out, k, stride, h, w), pixels)
    assert o.macs(0)["site"] == pairs * c_in * c_out


def test_site_level_macs_follow_the_previous_layers_active_set():
    """Second layer: its executed pairs are counted over the first layer's value-pruned active
    set, not over the touched set.  Layer 1 = 1x1 conv with weight -1 and ReLU on an input that is
    0 after reset: a positive increment gives relu(-1) - relu(0) = 0 (site pruned), a negative one
    gives 1 (site kept).  Layer 2 = 3x3: 9 pairs for the kept interior site only."""
    nodes = [wl.Node(wl.OP_CONV2D, wl.ACT_RELU, -1, -2, 1, 1, 1, 1, 0, 0, -1, 0),
             wl.Node(wl.OP_CONV2D, wl.ACT_NONE, 0, -2, 1, 2, 3, 1, 1, 1, -1, 1)]
    net = wl.Net("two", 1, 9, 9, nodes, np.concatenate([[-1.0], np.ones(18)]).astype(np.float32))
    o = Oracle(net)
    o.reset(np.zeros((1, 9, 9), np.float32))
    inc = np.zeros((1, 9, 9), np.float32)
    inc[0, 2, 2] = 1.0    # pruned by the ReLU
    inc[0, 6, 6] = -1.0   # kept
    o.step_increment(inc)
    assert o.macs(0)["site"] == 2 * 1 * 1
    assert o.site_list(0).tolist() == [6 * 9 + 6]
    assert o.macs(1)["site"] == 9 * 1 * 2


def test_tile_level_macs_count_whole_tiles_with_all_taps():
    c_in, c_out, k = 3, 5, 3
    net = _conv_net(c_in, c_out, k, 1, 20, 20)
    per_out = k * k * c_in * c_out
    # pixel (4,4): touched outputs rows/cols 3..5 -> inside tile (0,0) of an 8x8 grid
    o = _one_pixel_step(net, [(4, 4)])
    assert o.macs(0, (8, 8))["tile"] == 1 * 64 * per_out
    # 4x4 tiles: rows 3..5 straddle tiles 0 and 1 in both directions -> 4 tiles of 16 outputs
    assert o.macs(0, (4, 4))["tile"] == 4 * 16 * per_out
    # 1x1 tiles = touched outputs, every tap counted (also the ones on inactive inputs)
    assert o.macs(0, (1, 1))["tile"] == 9 * per_out
    # pixel (7,7): outputs 6..8 -> four 8x8 tiles
    o = _one_pixel_step(net, [(7, 7)])
    assert o.macs(0, (8, 8))["tile"] == 4 * 64 * per_out
    # a ragged last tile still counts as a whole tile (20 = 2.5 tiles): pixel (18,18) -> tile (2,2)
    o = _one_pixel_step(net, [(18, 18)])
    assert o.macs(0, (8, 8))["tile"] == 1 * 64 * per_out
    # nothing active: nothing executed
    o = _one_pixel_step(net, [])
    assert o.macs(0)["site"] == 0 and o.macs(0)["tile"] == 0


@pytest.mark.parametrize("k,stride,pad,h,w", [(3, 1, 1, 12, 10), (5, 2, 2, 16, 16), (5, 2, 2, 15, 17), (7, 2, 3, 14, 14),
                                              (1, 1, 0, 6, 5), (3, 1, 0, 9, 9)])
def test_dense_macs_closed_form_with_border_cuts(k, stride, pad, h, w):
    """Separable closed form: the in-image taps of output row oy are those t with
    0 <= oy * stride - pad + t < h; the pair count is (sum over rows) * (sum over columns)."""
    c_in, c_out = 3, 5
    o = Oracle(_conv_net(c_in, c_out, k, stride, h, w, pad=pad))
    ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    rows = sum(sum(1 for t in range(k) if 0 <= oy * stride - pad + t < h) for oy in range(ho))
    cols = sum(sum(1 for t in range(k) if 0 <= ox * stride - pad + t < w) for ox in range(wo))
    m = o.macs(0)
    assert m["dense"] == rows * cols * c_in * c_out
    assert m["dense_nominal"] == ho * wo * k * k * c_in * c_out
    if pad == 0:
        assert m["dense"] == m["dense_nominal"]
    if (k, stride, pad) == (3, 1, 1):
        assert m["dense"] == (3 * h - 2) * (3 * w - 2) * c_in * c_out   # each border row / column loses one tap


def test_all_sites_active_executes_the_dense_count():
    """With every input site active the site-level count of a step equals the regular pass's."""
    net = _conv_net(2, 3, 5, 2, 13, 11)
    o = Oracle(net)
    o.reset(np.zeros((2, 13, 11), np.float32))
    o.step_increment(np.ones((2, 13, 11), np.float32))
    m = o.macs(0)
    assert m["site"] == m["dense"]
    ho, wo = 7, 6
    assert m["tile"] == 1 * 64 * 25 * 2 * 3   # 7 x 6 outputs sit in one 8 x 8 tile
    assert o.macs(0, (4, 4))["tile"] == 2 * 2 * 16 * 25 * 2 * 3
