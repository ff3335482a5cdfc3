"""Independent library reference for the oracle's dense pass: PyTorch CPU fp64 routines
(conv2d, relu, sigmoid, max_pool2d, bilinear interpolate, mean, linear).  Test-only."""
import numpy as np
import torch
import torch.nn.functional as F

from paper_2303_04670_amd import workloads as wl


def torch_forward(net, x_chw, upto=None, state=None):
    """Returns per node (pre_activation, value) as H x W x C float64 numpy arrays.  state: for
    recurrent nets, {index of a DELAY node: 1 x C x H x W tensor, its value in this pass} (a
    missing entry is the zero state)."""
    w = torch.from_numpy(np.asarray(net.weights, dtype=np.float64))
    x = torch.from_numpy(np.asarray(x_chw, dtype=np.float64))[None]
    vals, outs = [], []

    def src(i):
        return x if i == -1 else vals[i]

    shapes = net.node_shapes()
    for idx, nd in enumerate(net.nodes):
        if nd.op == wl.OP_DELAY:
            z = state[idx] if state and idx in state else torch.zeros((1,) + tuple(shapes[idx]), dtype=torch.float64)
            vals.append(z)
            outs.append((z[0].permute(1, 2, 0).numpy(), z[0].permute(1, 2, 0).numpy()))
            continue
        a = src(nd.in0)
        if nd.op in (wl.OP_CONV2D, wl.OP_LINEAR):
            wt = w[nd.w_off: nd.w_off + nd.c_out * nd.c_in * nd.k * nd.k].reshape(nd.c_out, nd.c_in, nd.k, nd.k)
            b = w[nd.b_off: nd.b_off + nd.c_out] if nd.b_off >= 0 else None
            z = F.conv2d(a, wt, b, stride=nd.stride, padding=nd.pad)
        elif nd.op == wl.OP_ADD:
            z = a + src(nd.in1)
        elif nd.op == wl.OP_MUL:
            z = a * src(nd.in1)
        elif nd.op in (wl.OP_ACT, wl.OP_SPARSIFY):
            z = a
        elif nd.op == wl.OP_CONCAT:
            z = torch.cat([a, src(nd.in1)], dim=1)
        elif nd.op == wl.OP_UPSAMPLE2X:
            z = F.interpolate(a, scale_factor=2, mode="bilinear", align_corners=False)
        elif nd.op == wl.OP_MAXPOOL:
            z = F.max_pool2d(a, nd.k, nd.stride, nd.pad)
        elif nd.op == wl.OP_GAP:
            z = a.mean(dim=(2, 3), keepdim=True)
        else:
            raise ValueError(nd.op)
        v = z
        if nd.act == wl.ACT_RELU:
            v = F.relu(z)
        elif nd.act == wl.ACT_SIGMOID:
            v = torch.sigmoid(z)
        elif nd.act == wl.ACT_TANH:
            v = torch.tanh(z)
        elif nd.act == wl.ACT_ONE_MINUS:
            v = 1.0 - z
        vals.append(v)
        outs.append((z[0].permute(1, 2, 0).numpy(), v[0].permute(1, 2, 0).numpy()))
    return outs


def torch_recurrent(net, frames):
    """Runs a recurrent net over a list of C x H x W frames from the zero state.  Returns, per
    frame, torch_forward's per-node list."""
    delays = [i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_DELAY]
    state, res = {}, []
    for x in frames:
        outs = torch_forward(net, x, state=state)
        res.append(outs)
        state = {d: torch.from_numpy(np.ascontiguousarray(outs[net.nodes[d].in0][1].transpose(2, 0, 1)))[None] for d in delays}
    return res
