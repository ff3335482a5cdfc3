"""Pins for the oracle's elementwise-multiply increment (Eq.15-17) and tanh activation: exact
hand-computed cases, the telescoping identity against PyTorch's regular forward pass, the OR
mask (Eq.16).  A dropped cross term, swapped accumulators or an accumulator advanced before
use each fail at least one of them."""
import numpy as np

from oracle.oracle import Oracle
from paper_2303_04670_amd import workloads as wl
from torch_ref import torch_forward


def two_selectors_times():
    """2-channel input; node 0 picks channel 0, node 1 picks 3 x channel 1, node 2 multiplies."""
    w = np.asarray([1.0, 0.0, 0.0, 3.0], np.float32)
    nodes = [
        wl.Node(wl.OP_CONV2D, wl.ACT_NONE, -1, -2, 2, 1, 1, 1, 0, 0, -1, 0),
        wl.Node(wl.OP_CONV2D, wl.ACT_NONE, -1, -2, 2, 1, 1, 1, 0, 2, -1, 0),
        wl.Node(wl.OP_MUL, wl.ACT_NONE, 0, 1, 1, 1, 1, 1, 0, -1, -1, 1),
    ]
    return wl.Net("mul_pin", 2, 1, 4, nodes, w)


def test_hand_computed_products():
    net = two_selectors_times()
    o = Oracle(net)
    x0 = np.asarray([[[2.0, 2.0, 2.0, 1.0]], [[4.0, 4.0, 4.0, 5.0]]], np.float32)      # C x 1 x 4
    o.reset(x0)
    np.testing.assert_array_equal(o.y(2).ravel(), [24.0, 24.0, 24.0, 15.0])
    # site 0: only the first factor moves; site 1: only the second; site 2: both; site 3: none
    x1 = np.asarray([[[2.5, 2.0, 2.5, 1.0]], [[4.0, 4.5, 4.5, 5.0]]], np.float32)
    o.step_frame(x1)
    # Eq.15: (x1acc + d1) * d2 + x2acc * d1 with x1acc = 2, x2acc = 12, d1 = 0.5, d2 = 1.5
    np.testing.assert_array_equal(o.dy(2).ravel(), [12 * 0.5, 2 * 1.5, 2.5 * 1.5 + 12 * 0.5, 0.0])
    np.testing.assert_array_equal(o.mask(2).ravel(), [1, 1, 1, 0])                    # Eq.16
    np.testing.assert_array_equal(o.z(2).ravel(), [2.5, 2.0, 2.5, 1.0])               # Eq.17
    np.testing.assert_array_equal(o.z2(2).ravel(), [12.0, 13.5, 13.5, 15.0])
    np.testing.assert_array_equal(o.y(2).ravel(), [2.5 * 12, 2 * 13.5, 2.5 * 13.5, 15.0])
    # a second step uses the advanced accumulators
    x2 = np.asarray([[[3.0, 2.0, 2.5, 1.0]], [[4.0, 4.5, 4.0, 5.0]]], np.float32)
    o.step_frame(x2)
    np.testing.assert_array_equal(o.dy(2).ravel(), [12 * 0.5, 0.0, 2.5 * -1.5, 0.0])
    np.testing.assert_array_equal(o.mask(2).ravel(), [1, 0, 1, 0])


def test_gated_net_state_equals_regular_forward_pass():
    """Eq.2 through sigmoid x tanh gates, u * x and x * x: after every step the accumulated
    output equals PyTorch's forward pass of the current frame."""
    net = wl.net_gated(21, in_c=3, h=10, w=12, width=4, bias=True)
    rng = np.random.default_rng(0)
    x = (np.rint(rng.standard_normal((3, 10, 12)) * 256) / 256).astype(np.float32)
    o = Oracle(net)
    o.reset(x)
    out = o.outputs[0]
    for step in range(6):
        m = rng.random((1, 10, 12)) < 0.15
        x = (x + (np.rint(rng.standard_normal(x.shape) * 128) / 256).astype(np.float32) * m).astype(np.float32)
        o.step_frame(x)
        ref = torch_forward(net, x)
        np.testing.assert_allclose(o.y(out), ref[out][1], atol=1e-11)
        for i, nd in enumerate(net.nodes):
            if nd.op == wl.OP_MUL:
                np.testing.assert_allclose(o.z(i), ref[nd.in0][1], atol=1e-12)
                np.testing.assert_allclose(o.z2(i), ref[nd.in1][1], atol=1e-12)
    # tanh candidates really are in use and saturate nowhere near exactly
    tanh_nodes = [i for i, nd in enumerate(net.nodes) if nd.act == wl.ACT_TANH]
    assert tanh_nodes and all(np.abs(ref[i][1]).max() < 1 for i in tanh_nodes)


def test_fp32_product_increment_is_single_rounded_ops():
    """binary32 mode: t = fl(x1acc + d1); y = fl(fl(t * d2) + fl(x2acc * d1)), no fused
    multiply-add."""
    net = two_selectors_times()
    o = Oracle(net, fp32_state=True)
    rng = np.random.default_rng(1)
    f32 = np.float32
    x0 = rng.standard_normal((2, 1, 4)).astype(f32)
    o.reset(x0)
    a, b = x0[0].ravel().copy(), (f32(3) * x0[1].ravel()).astype(f32)
    x = x0
    for _ in range(5):
        xn = (x + rng.standard_normal(x.shape).astype(f32)).astype(f32)
        o.step_frame(xn)
        d1 = (xn[0] - x[0]).ravel().astype(f32)
        d2 = (f32(3) * (xn[1] - x[1]).ravel().astype(f32)).astype(f32)
        want = ((a + d1).astype(f32) * d2).astype(f32) + (b * d1).astype(f32)
        np.testing.assert_array_equal(o.dy(2).ravel().astype(f32), want.astype(f32))
        a, b = (a + d1).astype(f32), (b + d2).astype(f32)
        x = xn
