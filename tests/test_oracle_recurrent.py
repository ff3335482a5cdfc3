"""Pins for the oracle's recurrent state (DELAY nodes; the evaluation networks of the paper's
"Experiments" section are recurrent): a hand-computed running sum, a ConvLSTM cell against
PyTorch's regular forward passes run frame after frame from the zero state, a refresh in
mid-stream that keeps the state.  A delay of the wrong step, a state that is not zero before
the first frame, a mask taken from the wrong step or a refresh that clears the state each fail
at least one of them."""
import numpy as np

from oracle.oracle import Oracle
from paper_2303_04670_amd import workloads as wl
from torch_ref import torch_recurrent


def running_sum_net():
    """s(n) = x(n) + s(n-1): node 0 delays node 1, node 1 adds the input and node 0."""
    nodes = [
        wl.Node(wl.OP_DELAY, wl.ACT_NONE, 1, -1, 1, 1, 1, 1, 0, -1, -1, 0),
        wl.Node(wl.OP_ADD, wl.ACT_NONE, -1, 0, 1, 1, 1, 1, 0, -1, -1, 1),
    ]
    return wl.Net("running_sum", 1, 1, 4, nodes, np.zeros(0, np.float32))


def test_hand_computed_running_sum():
    o = Oracle(running_sum_net())
    x0 = np.asarray([[[1.0, 2.0, 3.0, 0.0]]], np.float32)
    o.reset(x0)                                   # zero state: s(0) = x(0)
    np.testing.assert_array_equal(o.y(1).ravel(), [1, 2, 3, 0])
    np.testing.assert_array_equal(o.z(0).ravel(), [0, 0, 0, 0])
    # same frame again: the input increment is zero, the state's increment is s(0) at every site
    o.step_frame(x0)
    np.testing.assert_array_equal(o.dy(0).ravel(), [1, 2, 3, 0])
    np.testing.assert_array_equal(o.mask(0).ravel(), [1, 1, 1, 1])
    np.testing.assert_array_equal(o.y(1).ravel(), [2, 4, 6, 0])         # s(1) = x + s(0)
    # one pixel moves: the state's increment is s(1) - s(0), its mask that of node 1 at step 1
    x2 = np.asarray([[[1.0, 2.0, 3.5, 0.0]]], np.float32)
    o.step_frame(x2)
    np.testing.assert_array_equal(o.dy(0).ravel(), [1, 2, 3, 0])
    np.testing.assert_array_equal(o.z(0).ravel(), [2, 4, 6, 0])         # = s(1)
    np.testing.assert_array_equal(o.y(1).ravel(), [3, 6, 9.5, 0])       # s(2) = x(2) + s(1)
    np.testing.assert_array_equal(o.mask(1).ravel(), [1, 1, 1, 1])      # OR of the input's and the state's masks
    o.step_frame(x2)
    np.testing.assert_array_equal(o.dy(0).ravel(), [1, 2, 3.5, 0])      # s(2) - s(1)
    np.testing.assert_array_equal(o.y(1).ravel(), [4, 8, 13, 0])


def _frames(rng, c, h, w, n, p=0.1):
    x = (np.rint(rng.standard_normal((c, h, w)) * 256) / 256).astype(np.float32)
    out = [x]
    for _ in range(n):
        m = rng.random((1, h, w)) < p
        x = (x + (np.rint(rng.standard_normal(x.shape) * 128) / 256).astype(np.float32) * m).astype(np.float32)
        out.append(x)
    return out


def test_convlstm_equals_regular_forward_passes_frame_after_frame():
    net = wl.net_convlstm(31, in_c=3, h=9, w=11, hidden=5, out_c=2)
    frames = _frames(np.random.default_rng(1), 3, 9, 11, 6)
    ref = torch_recurrent(net, frames)
    o = Oracle(net)
    out = o.outputs[0]
    h_prev, c_prev = 0, 1
    for n, x in enumerate(frames):
        (o.reset if n == 0 else o.step_frame)(x)
        np.testing.assert_allclose(o.y(out), ref[n][out][1], atol=1e-11, err_msg=f"frame {n}")
        # the state nodes have emitted the cell's h and c of the previous frame
        for d in (h_prev, c_prev):
            want = ref[n - 1][net.nodes[d].in0][1] if n else np.zeros_like(ref[0][d][1])
            np.testing.assert_allclose(o.z(d), want, atol=1e-11, err_msg=f"frame {n} state {d}")
        if n:
            for i, nd in enumerate(net.nodes):   # every accumulated pre-activation (Eq.2 per layer)
                if nd.op == wl.OP_CONV2D:
                    np.testing.assert_allclose(o.z(i), ref[n][i][0], atol=1e-11)


def test_state_moves_without_input_events():
    """A recurrent net's output changes from step to step on a constant input (the state is one
    more input), and so do the masks of everything behind the state."""
    net = wl.net_convlstm(32, in_c=2, h=6, w=7, hidden=4, out_c=1)
    x = _frames(np.random.default_rng(2), 2, 6, 7, 0)[0]
    ref = torch_recurrent(net, [x, x, x])
    o = Oracle(net)
    o.reset(x)
    for n in (1, 2):
        o.step_frame(x)
        np.testing.assert_allclose(o.y(o.outputs[0]), ref[n][o.outputs[0]][1], atol=1e-12)
        assert o.mask(0).all() and o.mask(o.outputs[0]).any()
    assert np.abs(ref[2][o.outputs[0]][1] - ref[1][o.outputs[0]][1]).max() > 1e-4


def test_refresh_in_mid_stream_keeps_the_state():
    net = wl.net_convlstm(33, in_c=3, h=8, w=8, hidden=4, out_c=2)
    frames = _frames(np.random.default_rng(3), 3, 8, 8, 7)
    ref = torch_recurrent(net, frames)
    a, b = Oracle(net), Oracle(net)
    out = a.outputs[0]
    for n, x in enumerate(frames):
        (a.reset if n == 0 else a.step_frame)(x)
        if n == 0:
            b.reset(x)
        elif n in (3, 4):       # two regular passes in a row, then incremental steps again
            b.refresh(x)
        else:
            b.step_frame(x)
        np.testing.assert_allclose(b.y(out), ref[n][out][1], atol=1e-11, err_msg=f"frame {n}")
        np.testing.assert_allclose(b.y(out), a.y(out), atol=1e-11)
        np.testing.assert_allclose(b.z(0), a.z(0), atol=1e-11)


def test_convgru_equals_regular_forward_passes_frame_after_frame():
    """The gated recurrent unit needs 1 - z: an activation whose increment is -x_inc."""
    net = wl.net_convgru(34, in_c=3, h=8, w=10, hidden=5, out_c=2)
    frames = _frames(np.random.default_rng(4), 3, 8, 10, 6)
    ref = torch_recurrent(net, frames)
    o = Oracle(net)
    out = o.outputs[0]
    omz = next(i for i, nd in enumerate(net.nodes) if nd.act == wl.ACT_ONE_MINUS)
    for n, x in enumerate(frames):
        (o.reset if n == 0 else o.step_frame)(x)
        np.testing.assert_allclose(o.y(out), ref[n][out][1], atol=1e-11, err_msg=f"frame {n}")
        want = ref[n - 1][net.nodes[0].in0][1] if n else np.zeros_like(ref[0][0][1])
        np.testing.assert_allclose(o.z(0), want, atol=1e-11)
        if n:   # the ONE_MINUS node: accumulated input z, increment -(z's increment)
            np.testing.assert_allclose(o.z(omz), ref[n][net.nodes[omz].in0][1], atol=1e-11)
            np.testing.assert_allclose(o.dy(omz), -o.dy(net.nodes[omz].in0), atol=1e-12)
