"""Pins for the CPU oracle against things other than itself (all CPU, no GPU needed).

Each test names what fixes the expected value: a library routine (PyTorch CPU fp64), an
identity from the paper (Eq.2 telescoping sum, Eq.9 linearity, Eq.12 with a zero increment,
refresh == regular forward pass), a closed form, or brute force with exact integer arithmetic.
"""
import numpy as np
import pytest

from oracle.oracle import Oracle, tile_words, SET_ACTIVE, SET_TOUCHED
from paper_2303_04670_amd import workloads as wl
from torch_ref import torch_forward


def small_nets():
    return [
        wl.net_random_small(7),
        wl.net_random_small(8, in_c=2, h=9, w=16, bias=False),
        wl.net_single_conv(11, c=4, h=12, w=10),
        wl.net_conv_stack(12, h=21, w=30),
        wl.net_unet_depth(13, h=16, w=24, width=4),
        wl.net_resnet18(14, h=40, w=40, n_classes=7, width=4),
        wl.net_flow(15, h=32, w=32, width=4),
        wl.net_flow_delayed(16, h=32, w=48, width=4, d_width=4),
        wl.net_gated(17, in_c=3, h=11, w=13, width=4, bias=True),
    ]


def _dyadic(a):
    """Round to multiples of 2^-10 so that fp32 sums and differences of frames are exact (the
    telescoping identities then hold without the rounding of Eq.1's subtraction)."""
    return (np.rint(np.clip(a, -8, 8) * 1024.0) / 1024.0).astype(np.float32)


def rand_frame(rng, net, scale=1.0):
    return _dyadic(rng.standard_normal((net.in_c, net.in_h, net.in_w)) * scale)


def sparse_increment(rng, net, density=0.05):
    m = rng.random((net.in_h, net.in_w)) < density
    d = _dyadic(rng.standard_normal((net.in_c, net.in_h, net.in_w)) * 0.5)
    return d * m[None]


@pytest.mark.parametrize("net", small_nets(), ids=lambda n: f"{n.name}_{n.in_h}x{n.in_w}")
def test_dense_pass_matches_torch_fp64(net):
    """Library pin: every node of the oracle's regular forward pass equals PyTorch CPU fp64
    conv2d / relu / sigmoid / max_pool2d / interpolate(bilinear, align_corners=False) / mean."""
    rng = np.random.default_rng(1)
    x = rand_frame(rng, net)
    o = Oracle(net)
    o.dense_forward(x)
    ref = torch_forward(net, x)
    for i, (z_ref, v_ref) in enumerate(ref):
        np.testing.assert_allclose(o.dense_z(i), z_ref, rtol=1e-11, atol=1e-11, err_msg=f"node {i} z")
        np.testing.assert_allclose(o.dense_value(i), v_ref, rtol=1e-11, atol=1e-11, err_msg=f"node {i} value")


@pytest.mark.parametrize("net", small_nets(), ids=lambda n: f"{n.name}_{n.in_h}x{n.in_w}")
def test_eq2_incremental_state_equals_dense_forward(net):
    """Eq.2: after k incremental steps every accumulated tensor and the summed output equal a
    regular forward pass of x_t (checked against PyTorch, not against the oracle's own dense
    half), both when frames are diffed (Eq.1) and when increments are supplied."""
    rng = np.random.default_rng(2)
    x = rand_frame(rng, net)
    o = Oracle(net)
    o.reset(x)
    for step in range(6):
        inc = sparse_increment(rng, net, density=0.03 + 0.03 * step)
        if step % 2 == 0:
            x = (x + inc).astype(np.float32)
            o.step_frame(x)
        else:
            o.step_increment(inc)
            x = (x + inc).astype(np.float32)
        np.testing.assert_array_equal(o.x_prev(), x)
    ref = torch_forward(net, x)
    for i, nd in enumerate(net.nodes):
        z_ref, v_ref = ref[i]
        scale = max(1.0, np.abs(z_ref).max())
        keeps_z = (nd.op in (wl.OP_CONV2D, wl.OP_LINEAR, wl.OP_GAP, wl.OP_ACT) or nd.act != wl.ACT_NONE) \
            and nd.op != wl.OP_MAXPOOL
        if keeps_z:
            np.testing.assert_allclose(o.z(i), z_ref, atol=1e-11 * scale, rtol=0, err_msg=f"node {i} z")
        if nd.is_output:
            np.testing.assert_allclose(o.y(i), v_ref, atol=1e-11 * scale, rtol=0, err_msg=f"node {i} y")


def test_refresh_equals_stepped_state():
    """Drift Errors section: a refresh is a regular forward pass, so reset(x_t) must reproduce
    the state reached by stepping."""
    net = wl.net_unet_depth(21, h=16, w=16, width=4)
    rng = np.random.default_rng(3)
    x = rand_frame(rng, net)
    a, b = Oracle(net), Oracle(net)
    a.reset(x)
    for _ in range(5):
        x = (x + sparse_increment(rng, net, 0.1)).astype(np.float32)
        a.step_frame(x)
    b.reset(x)
    for i, nd in enumerate(net.nodes):
        if nd.op == wl.OP_CONV2D or nd.act != wl.ACT_NONE:
            np.testing.assert_allclose(a.z(i), b.z(i), atol=1e-11, rtol=0)
    out = a.outputs[0]
    np.testing.assert_allclose(a.y(out), b.y(out), atol=1e-12, rtol=0)


def test_eq9_linearity_of_conv_increment():
    """Eq.9: theta_L(a + b) = theta_L(a) + theta_L(b) for a conv without activation."""
    net = wl.net_single_conv(31, c=3, h=10, w=9)
    net.nodes[0].act = wl.ACT_NONE
    rng = np.random.default_rng(4)
    x0 = rand_frame(rng, net)
    da, db = sparse_increment(rng, net, 0.2), sparse_increment(rng, net, 0.2)
    outs = []
    for inc in (da, db, (da.astype(np.float64) + db).astype(np.float32)):
        o = Oracle(net)
        o.reset(x0)
        o.step_increment(inc)
        outs.append(o.dy(0))
    np.testing.assert_allclose(outs[0] + outs[1], outs[2], atol=1e-6, rtol=0)


@pytest.mark.parametrize("net", small_nets()[:5], ids=lambda n: n.name)
def test_zero_increment_gives_empty_lists_and_keeps_state(net):
    """Eq.12 with x_inc = 0: the output increment is zero, lists are empty, state untouched."""
    rng = np.random.default_rng(5)
    x = rand_frame(rng, net)
    o = Oracle(net)
    o.reset(x)
    o.step_frame((x + sparse_increment(rng, net, 0.2)).astype(np.float32))
    z_before = [o.z(i) if o.tensor(i, 0).size else None for i in range(o.n_nodes)]
    y_before = [o.y(i) for i in o.outputs]
    o.step_increment(np.zeros_like(x))
    assert o.site_list(-1).size == 0
    for i in range(o.n_nodes):
        assert o.site_list(i, SET_ACTIVE).size == 0
        assert o.site_list(i, SET_TOUCHED).size == 0
        assert not o.dy(i).any()
        if z_before[i] is not None:
            np.testing.assert_array_equal(o.z(i), z_before[i])
    for yb, i in zip(y_before, o.outputs):
        np.testing.assert_array_equal(o.y(i), yb)


@pytest.mark.parametrize("k,s,pad", [(1, 1, 0), (3, 1, 1), (3, 2, 1), (5, 1, 2), (5, 2, 2), (7, 2, 3), (3, 2, 0)])
def test_touched_set_closed_form_single_pixel(k, s, pad):
    """Closed form: one active input pixel (iy, ix) touches exactly R(iy) x R(ix) with
    R(i) = {(i + pad - t)/s : t in [0,K), (i + pad - t) mod s == 0, result in [0, H_out)}."""
    h, w = 11, 14
    net = wl.net_single_conv(41, c=2, h=h, w=w)
    nd = net.nodes[0]
    nd.k, nd.stride, nd.pad = k, s, pad
    rng = np.random.default_rng(k * 10 + s)
    net.weights = rng.standard_normal(nd.c_out * nd.c_in * k * k).astype(np.float32)
    o = Oracle(net)
    _, ho, wo = o.shape(0)
    pts = [(0, 0), (0, w - 1), (h - 1, 0), (h - 1, w - 1), (5, 7), (4, 6), (1, 12)]
    for iy, ix in pts:
        o.reset(np.zeros((2, h, w), np.float32))
        inc = np.zeros((2, h, w), np.float32)
        inc[1, iy, ix] = 1.5
        o.step_increment(inc)

        def R(i, n_out):
            return {(i + pad - t) // s for t in range(k) if (i + pad - t) >= 0 and (i + pad - t) % s == 0
                    and (i + pad - t) // s < n_out}
        expect = np.zeros((ho, wo), np.uint8)
        for oy in R(iy, ho):
            for ox in R(ix, wo):
                expect[oy, ox] = 1
        np.testing.assert_array_equal(o.mask(0, SET_TOUCHED), expect)
        assert list(o.site_list(-1)) == [iy * w + ix]


def test_lists_brute_force_exact_integer_arithmetic():
    """Brute force: with integer-valued weights and inputs all sums are exact, so the pruned
    active set of a ReLU layer must equal the support of relu(z(x_t)) - relu(z(x_{t-1}))
    computed from two regular forward passes (PyTorch), with no rounding ambiguity."""
    net = wl.net_conv_stack(51, h=19, w=22)
    rng = np.random.default_rng(6)
    net.weights = rng.integers(-3, 4, net.weights.size).astype(np.float32)
    x = rng.integers(-4, 5, (net.in_c, net.in_h, net.in_w)).astype(np.float32)
    o = Oracle(net)
    o.reset(x)
    for _ in range(4):
        m = rng.random((net.in_h, net.in_w)) < 0.04
        inc = rng.integers(-2, 3, x.shape).astype(np.float32) * m[None]
        x_new = x + inc
        prev, cur = torch_forward(net, x), torch_forward(net, x_new)
        o.step_frame(x_new)
        np.testing.assert_array_equal(o.mask(-1), np.any(inc != 0, axis=0).astype(np.uint8))
        for i in range(len(net.nodes)):
            diff = cur[i][1] - prev[i][1]
            np.testing.assert_array_equal(o.mask(i, SET_ACTIVE), np.any(diff != 0, axis=2).astype(np.uint8))
            np.testing.assert_array_equal(o.dy(i), diff)
            assert np.all(o.mask(i, SET_ACTIVE) <= o.mask(i, SET_TOUCHED))
        x = x_new


def test_structural_sets_of_add_concat_upsample():
    """Eq.11b: the mask of a sum (and of a concat) is the OR of the input masks; an upsampled
    site is touched iff one of its (up to four) bilinear source sites is active."""
    net = wl.net_flow(61, h=32, w=32, width=4)
    rng = np.random.default_rng(7)
    x = rand_frame(rng, net)
    o = Oracle(net)
    o.reset(x)
    o.step_frame((x + sparse_increment(rng, net, 0.02)).astype(np.float32))
    for i, nd in enumerate(net.nodes):
        if nd.op == wl.OP_CONCAT or (nd.op == wl.OP_ADD and nd.act == wl.ACT_NONE):
            np.testing.assert_array_equal(o.mask(i), o.mask(nd.in0) | o.mask(nd.in1))
        if nd.op == wl.OP_UPSAMPLE2X:
            src = o.mask(nd.in0)
            h, w = src.shape
            exp = np.zeros((2 * h, 2 * w), np.uint8)
            for oy in range(2 * h):
                ys = {max(oy // 2 - 1, 0), oy // 2} if oy % 2 == 0 else {oy // 2, min(oy // 2 + 1, h - 1)}
                for ox in range(2 * w):
                    xs = {max(ox // 2 - 1, 0), ox // 2} if ox % 2 == 0 else {ox // 2, min(ox // 2 + 1, w - 1)}
                    exp[oy, ox] = max(src[y_, x_] for y_ in ys for x_ in xs)
            np.testing.assert_array_equal(o.mask(i), exp)


def test_masks_skip_only_zeros():
    """Implementation of Increment Layers: a mask may only mark all-zero regions, so spelling
    the zeros out (every site made active by an increment that cancels in the next step)
    must not change any accumulated value beyond rounding."""
    net = wl.net_unet_depth(71, h=16, w=16, width=4)
    rng = np.random.default_rng(8)
    x = rand_frame(rng, net)
    inc = sparse_increment(rng, net, 0.05)
    a, b = Oracle(net), Oracle(net)
    a.reset(x)
    a.step_increment(inc)
    noise = np.full_like(x, 2.0 ** -3)             # every site active, exactly representable
    b.reset(x)
    b.step_increment(inc + noise)
    b.step_increment(-noise)
    assert b.site_list(-1).size == net.in_h * net.in_w
    out = a.outputs[0]
    np.testing.assert_allclose(a.y(out), b.y(out), atol=1e-12, rtol=0)
    for i, nd in enumerate(net.nodes):
        if nd.op == wl.OP_CONV2D:
            np.testing.assert_allclose(a.z(i), b.z(i), atol=1e-11, rtol=0)


@pytest.mark.parametrize("tile", [(1, 1), (4, 4), (6, 6), (8, 8), (4, 16)])
def test_tile_words_consistent_with_lists(tile):
    """Tile occupancy words / bitmap are a re-encoding of the site set for any tile size."""
    th, tw = tile
    rng = np.random.default_rng(9)
    m = (rng.random((21, 30)) < 0.1).astype(np.uint8)
    occ, bitmap = tile_words(m, th, tw)
    tx = -(-30 // tw)
    rec = np.zeros_like(m)
    for t, word in enumerate(occ):
        for bit in range(th * tw):
            if (int(word) >> bit) & 1:
                rec[(t // tx) * th + bit // tw, (t % tx) * tw + bit % tw] = 1
    np.testing.assert_array_equal(rec, m)
    for t, word in enumerate(occ):
        assert bool((int(bitmap[t // 64]) >> (t % 64)) & 1) == (word != 0)


def test_fp32_state_drifts_and_refresh_removes_it():
    """Drift Errors section (qualitative; the figure is not available): with binary32 state the
    incremental output drifts away from the regular forward pass as steps accumulate, and a
    refresh brings the error back to the single-pass level."""
    net = wl.net_single_conv(81, c=4, h=16, w=16)
    rng = np.random.default_rng(10)
    x = rng.standard_normal((4, 16, 16)).astype(np.float32)
    f = Oracle(net, fp32_state=True)
    f.reset(x)
    err_first = None
    for step in range(1000):
        m = rng.random((1, 16, 16)) < 0.5          # half the pixels get fresh values: |x| stays O(1)
        x = np.where(m, rng.standard_normal(x.shape), x).astype(np.float32)
        f.step_frame(x)
        if step == 0:
            err_first = np.abs(f.y(0) - torch_forward(net, x)[0][1]).max()
    err_last = np.abs(f.y(0) - torch_forward(net, x)[0][1]).max()
    f.reset(x)
    err_refresh = np.abs(f.y(0) - torch_forward(net, x)[0][1]).max()
    print(err_first, err_last, err_refresh)
    assert err_last > 3 * err_first > 0
    assert err_last > 3 * err_refresh


def test_fp32_activation_increment_is_single_rounded_ops():
    """Eq.12-14 in binary32 (the mode used for bit-exact checks of elementwise GPU kernels):
    x_acc += x_inc; y_inc = relu(x_acc_new) - relu(x_acc_old), each one IEEE binary32 op."""
    net = wl.Net("act", 3, 8, 8, [wl.Node(wl.OP_ACT, wl.ACT_RELU, -1, -2, 3, 3, is_output=1)], np.zeros(0, np.float32))
    rng = np.random.default_rng(11)
    x = rand_frame(rng, net)
    f = Oracle(net, fp32_state=True)
    f.reset(x)
    acc = np.transpose(x, (1, 2, 0)).copy()
    for _ in range(5):
        inc = sparse_increment(rng, net, 0.4)
        f.step_increment(inc)
        d = np.transpose(inc, (1, 2, 0))
        new = (acc + d).astype(np.float32)
        exp = (np.maximum(new, np.float32(0)) - np.maximum(acc, np.float32(0))).astype(np.float32)
        exp = exp * np.any(d != 0, axis=2, keepdims=True)
        np.testing.assert_array_equal(f.dy(0).astype(np.float32), exp)
        acc = np.where(np.any(d != 0, axis=2, keepdims=True), new, acc)
        np.testing.assert_array_equal(f.z(0).astype(np.float32), acc)
