"""The oracle against the hand-evaluated fixtures under tests/golden/ (each file cites the
equations it evaluates)."""
import os

import numpy as np

from oracle.oracle import Oracle
from paper_2303_04670_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    out = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#")[0].strip()
        if line:
            out.append([float(t) for t in line.split()])
    return np.asarray(out)


def test_sparsification_rounding_fixture():
    rows = _rows("eq3_8_sparsification_rounding.txt")
    n_sites = int(rows[:, 1].max()) + 1
    nodes = [wl.Node(wl.OP_SPARSIFY, wl.ACT_NONE, -1, -2, 1, 1, 1, 1, 0, 0, -1, 1)]
    net = wl.Net("sp_golden", 1, 1, n_sites, nodes, np.asarray([0.5], np.float32))
    o = Oracle(net)
    o.reset(np.zeros((1, 1, n_sites), np.float32))
    for step in sorted(set(rows[:, 0])):
        r = rows[rows[:, 0] == step]
        r = r[np.argsort(r[:, 1])]
        o.step_increment(r[:, 2].astype(np.float32).reshape(1, 1, n_sites))
        np.testing.assert_array_equal(o.dy(0).ravel(), r[:, 3], err_msg=f"step {step}: y_inc")
        np.testing.assert_allclose(o.z(0).ravel(), r[:, 4], atol=1e-7, err_msg=f"step {step}: delta")


def test_multiply_increment_fixture():
    rows = _rows("eq15_17_multiply_increment.txt")
    n_sites = int(rows[:, 1].max()) + 1
    # node 0 = channel 0, node 1 = channel 1 (exact 1x1 selectors), node 2 = their product
    w = np.asarray([1.0, 0.0, 0.0, 1.0], np.float32)
    nodes = [wl.Node(wl.OP_CONV2D, wl.ACT_NONE, -1, -2, 2, 1, 1, 1, 0, 0, -1, 0),
             wl.Node(wl.OP_CONV2D, wl.ACT_NONE, -1, -2, 2, 1, 1, 1, 0, 2, -1, 0),
             wl.Node(wl.OP_MUL, wl.ACT_NONE, 0, 1, 1, 1, 1, 1, 0, -1, -1, 1)]
    net = wl.Net("mul_golden", 2, 1, n_sites, nodes, w)
    first = rows[rows[:, 0] == rows[:, 0].min()]
    first = first[np.argsort(first[:, 1])]
    o = Oracle(net)
    o.reset(np.stack([first[:, 2], first[:, 3]]).astype(np.float32).reshape(2, 1, n_sites))
    for step in sorted(set(rows[:, 0])):
        r = rows[rows[:, 0] == step]
        r = r[np.argsort(r[:, 1])]
        np.testing.assert_array_equal(o.z(2).ravel(), r[:, 2], err_msg=f"step {step}: x1acc")
        np.testing.assert_array_equal(o.z2(2).ravel(), r[:, 3], err_msg=f"step {step}: x2acc")
        o.step_increment(np.stack([r[:, 4], r[:, 5]]).astype(np.float32).reshape(2, 1, n_sites))
        np.testing.assert_array_equal(o.dy(2).ravel(), r[:, 6], err_msg=f"step {step}: y_inc")
        np.testing.assert_array_equal(o.y(2).ravel(), r[:, 7], err_msg=f"step {step}: running output")
