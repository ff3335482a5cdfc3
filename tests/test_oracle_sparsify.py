"""Pins for the oracle's sparsification layer (Eq.3-8 of "Sparsification layer", under the
reading stated in the oracle header).  The paper prints no worked example, so the pins are the
properties its text demands of the layer plus exact hand-computed cases."""
import numpy as np
import pytest

from oracle.oracle import Oracle
from paper_2303_04670_amd import workloads as wl
from torch_ref import torch_forward


def sp_only_net(c=3, h=6, w=7, k=None):
    """network input -> sparsification layer -> output (no conv, so x_inc is known exactly)"""
    w_arr = np.zeros(0, np.float32)
    k_off = -1
    if k is not None:
        w_arr = np.asarray([k], np.float32)
        k_off = 0
    nodes = [wl.Node(wl.OP_SPARSIFY, wl.ACT_NONE, -1, -2, c, c, 1, 1, 0, k_off, -1, 1)]
    return wl.Net("sp_only", c, h, w, nodes, w_arr)


def test_hand_computed_rounding_cases():
    """k = 0.5: y_inc = k * floor(0.5 + x_corr / k).  Half-way values round up (0.25 -> 0.5,
    -0.25 -> 0), values inside [-k/2, k/2) vanish and are carried in delta."""
    net = sp_only_net(c=1, h=1, w=8, k=0.5)
    o = Oracle(net)
    o.reset(np.zeros((1, 1, 8), np.float32))
    x = np.asarray([0.25, -0.25, 0.2, -0.2, 0.74, 0.75, -0.76, 1.3], np.float32).reshape(1, 1, 8)
    o.step_increment(x)
    y = o.dy(0).ravel()
    d = o.z(0).ravel()
    np.testing.assert_array_equal(y, [0.5, 0.0, 0.0, 0.0, 0.5, 1.0, -1.0, 1.5])
    np.testing.assert_allclose(d, x.ravel().astype(np.float64) - y, atol=1e-7)
    assert list(o.site_list(0)) == [0, 4, 5, 6, 7]           # all-zero outputs are dropped
    # the residual is added to the next increment (error feedback): 0.2 + 0.2 = 0.4 -> 0.5
    o.step_increment(np.asarray([0, 0, 0.2, -0.2, 0, 0, 0, 0], np.float32).reshape(1, 1, 8))
    np.testing.assert_array_equal(o.dy(0).ravel(), [0, 0, 0.5, -0.5, 0, 0, 0, 0])
    np.testing.assert_allclose(o.z(0).ravel()[2:4], [-0.1, 0.1], atol=1e-7)


def test_conservation_and_residual_bound():
    """What the text requires of delta: it stays small (-k/2 <= delta < k/2) and nothing is lost:
    sum of emitted increments + delta == sum of input increments, elementwise."""
    net = sp_only_net(c=3, h=9, w=8, k=0.3)
    k = float(np.float32(0.3))
    o = Oracle(net)
    rng = np.random.default_rng(0)
    x0 = rng.standard_normal((3, 9, 8)).astype(np.float32)
    o.reset(x0)
    sum_in = np.zeros((9, 8, 3))
    sum_out = np.zeros((9, 8, 3))
    for step in range(40):
        m = rng.random((9, 8)) < 0.5
        inc = (rng.standard_normal((3, 9, 8)) * 0.2).astype(np.float32) * m[None]
        o.step_increment(inc)
        sum_in += np.transpose(inc, (1, 2, 0)).astype(np.float64)
        sum_out += o.dy(0)
        d = o.z(0)
        assert d.min() >= -k / 2 - 1e-9 and d.max() < k / 2 + 1e-9
        np.testing.assert_allclose(sum_out + d, sum_in, atol=1e-9)
        np.testing.assert_allclose(o.dy(0) / k, np.rint(o.dy(0) / k), atol=1e-6)   # multiples of k
        # the output node's running sum (Eq.2) is the refresh value plus everything emitted
        np.testing.assert_allclose(o.y(0), np.transpose(x0, (1, 2, 0)) + sum_out, atol=1e-9)


def test_zero_threshold_is_the_lossless_network():
    """t_p = 0 gives k = 0: the layers are the identity and every tensor equals the network
    without them."""
    base = wl.net_conv_stack(5, h=17, w=20)
    sp = wl.net_conv_stack(5, h=17, w=20, sparsify=True)
    sp.sparsify_tp = 0.0
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 17, 20)).astype(np.float32)
    a, b = Oracle(base), Oracle(sp)
    a.reset(x)
    b.reset(x)
    for _ in range(4):
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * (rng.random((1, 17, 20)) < 0.1)).astype(np.float32)
        a.step_frame(x)
        b.step_frame(x)
    conv_b = [i for i, nd in enumerate(sp.nodes) if nd.op == wl.OP_CONV2D]
    for ia, ib in enumerate(conv_b):
        np.testing.assert_allclose(a.z(ia), b.z(ib), atol=1e-12)
        np.testing.assert_array_equal(a.mask(ia), b.mask(ib))
    np.testing.assert_allclose(a.y(a.outputs[0]), b.y(b.outputs[0]), atol=1e-12)


def test_step_is_tp_times_rms_of_layer_input_at_refresh():
    net = wl.net_conv_stack(6, h=12, w=14, sparsify=True)
    net.sparsify_tp = 0.1
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 12, 14)).astype(np.float32)
    o = Oracle(net)
    o.reset(x)
    ref = torch_forward_sp(net, x)
    for i, nd in enumerate(net.nodes):
        if nd.op == wl.OP_SPARSIFY:
            rms = np.sqrt(np.mean(ref[nd.in0] ** 2))
            k = o.step_size(i)
            assert abs(k - 0.1 * rms) <= 0.1 * rms * 2.0 ** -8        # kept to 8 fraction bits
            assert (np.float32(k).view(np.uint32) & 0x7fff) == 0


def test_step_size_closed_forms_and_a_hand_quantised_value():
    """k = t_p * sqrt(mean(x^2)) over the layer input at the reset, kept to the nine leading bits of
    its significand (round to nearest at the 16th fraction bit).  Inputs whose root mean square is
    known without arithmetic: a constant, +-c, a 6-8-0 pattern (36 + 64 over 100 elements: mean
    square 1); and 0.3 quantised by hand: 0.3f = 0x3e99999a -> + 0x4000 -> 0x3e99d99a -> low 15 bits
    cleared -> 0x3e998000 = 0.2998046875."""
    def k_of(x, tp):
        net = sp_only_net(c=x.shape[0], h=x.shape[1], w=x.shape[2])
        net.sparsify_tp = tp
        o = Oracle(net)
        o.reset(x.astype(np.float32))
        return o.step_size(0)
    assert k_of(np.full((3, 6, 7), 2.0), 0.25) == 0.5
    pm = np.where((np.arange(3 * 6 * 7) % 2) == 0, 3.0, -3.0).reshape(3, 6, 7)
    assert k_of(pm, 0.5) == 1.5
    x = np.zeros((1, 10, 10))
    x[0, 2, 3], x[0, 7, 1] = 6.0, -8.0
    assert k_of(x, 0.125) == 0.125
    assert k_of(np.ones((2, 5, 5)), 0.3) == 0.2998046875
    assert np.float32(0.2998046875).view(np.uint32) == 0x3e998000
    # zero input: k = 0, the layer is the identity
    assert k_of(np.zeros((2, 5, 5)), 0.3) == 0.0


def torch_forward_sp(net, x):
    """values of every node of a net with sparsification layers in a regular forward pass
    (the layers are the identity there): run the PyTorch reference on the net without them."""
    import copy
    plain = copy.deepcopy(net)
    for nd in plain.nodes:
        if nd.op == wl.OP_SPARSIFY:
            nd.op = wl.OP_ACT
            nd.w_off = -1
    return [v for _, v in torch_forward(plain, x)]


def test_refresh_is_a_regular_forward_pass_and_clears_the_residual():
    net = wl.net_conv_stack(7, h=12, w=14, sparsify=True)
    net.sparsify_tp = 0.2
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 12, 14)).astype(np.float32)
    o = Oracle(net)
    o.reset(x)
    for _ in range(5):
        x = (x + 0.3 * rng.standard_normal(x.shape).astype(np.float32) * (rng.random((1, 12, 14)) < 0.3)).astype(np.float32)
        o.step_frame(x)
    out = o.outputs[0]
    assert any(np.abs(o.z(i)).max() > 0 for i, nd in enumerate(net.nodes) if nd.op == wl.OP_SPARSIFY)
    lossy = o.y(out).copy()
    o.reset(x)
    ref = torch_forward_sp(net, x)
    np.testing.assert_allclose(o.y(out), ref[out], atol=1e-11)
    for i, nd in enumerate(net.nodes):
        if nd.op == wl.OP_SPARSIFY:
            assert not o.z(i).any()
    # and the lossy running output was a bounded approximation of it
    assert 0 < np.abs(lossy - ref[out]).max() < 0.5 * np.abs(ref[out]).max()


def test_sparsification_reduces_downstream_activity():
    """The purpose of the layer (Fig. 1b, qualitative): with a threshold the deeper layers see
    fewer active sites than without."""
    rng = np.random.default_rng(4)
    x = rng.standard_normal((5, 40, 48)).astype(np.float32)
    counts = {}
    for tp in (0.0, 0.3):
        net = wl.net_conv_stack(8, h=40, w=48, sparsify=True)
        net.sparsify_tp = tp
        o = Oracle(net)
        o.reset(x)
        xs = x
        r = np.random.default_rng(5)
        tot = 0
        for _ in range(6):
            xs = (xs + 0.05 * r.standard_normal(x.shape).astype(np.float32) * (r.random((1, 40, 48)) < 0.02)).astype(np.float32)
            o.step_frame(xs)
            tot += sum(int(o.mask(i).sum()) for i, nd in enumerate(net.nodes) if nd.op == wl.OP_CONV2D)
        counts[tp] = tot
    assert counts[0.3] < 0.7 * counts[0.0], counts
