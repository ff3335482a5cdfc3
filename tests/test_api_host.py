"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes workspaces, and rejects bad descriptions before any GPU work."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2303_04670_amd import evconv as ev
from paper_2303_04670_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "evconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(evconv_[a-z_]+)\s*\(", text))
    assert declared == set(ev.EXPORTS)
    L = ev.lib()
    for name in sorted(declared):
        assert hasattr(L, name), name


@pytest.mark.parametrize("make", [wl.net_single_conv, wl.net_conv_stack, wl.net_unet_depth, wl.net_resnet18,
                                  wl.net_flow, wl.net_convlstm], ids=lambda f: f.__name__)
def test_query_workspace_all_workloads(make):
    net = make()
    desc, keep = ev.marshal_desc(net)
    n = ev.evconv_query_workspace(desc)
    shapes = net.node_shapes()
    lower = sum(c * h * w * 4 for c, h, w in shapes)   # at least one increment buffer per node
    assert lower < n < 40 * lower + (64 << 20)


def _status(desc):
    n = ctypes.c_size_t(0)
    return ev.lib().evconv_query_workspace(ctypes.byref(desc), ctypes.byref(n))


def test_bad_descriptions_are_rejected():
    net = wl.net_conv_stack(1, h=16, w=16)
    desc, nodes = ev.marshal_desc(net)
    assert _status(desc) == ev.OK
    desc.abi_version = 99
    assert _status(desc) == ev.ERR_BAD_DESC
    desc.abi_version = ev.ABI_VERSION
    nodes[1].in0 = 3                       # forward reference
    assert _status(desc) == ev.ERR_BAD_DESC
    nodes[1].in0 = 0
    nodes[1].c_in = 7                      # channel mismatch
    assert _status(desc) == ev.ERR_SHAPE
    nodes[1].c_in = 32
    nodes[2].kh = 9
    assert _status(desc) == ev.ERR_UNSUPPORTED
    nodes[2].kh = 3
    nodes[0].op = 42
    assert _status(desc) == ev.ERR_INVALID_ARG
    nodes[0].op = wl.OP_CONV2D
    nodes[0].act = 5                       # one past the last activation
    assert _status(desc) == ev.ERR_INVALID_ARG
    nodes[0].act = wl.ACT_TANH
    assert _status(desc) == ev.OK
    nodes[0].act = wl.ACT_RELU
    nodes[3].op, nodes[3].in1 = wl.OP_MUL, 1       # 64 x 4 x 4 times 32 x 8 x 8
    assert _status(desc) == ev.ERR_SHAPE
    nodes[3].op, nodes[3].in1 = wl.OP_CONV2D, -2
    desc.sparsify_tp = -0.1
    assert _status(desc) == ev.ERR_INVALID_ARG
    desc.sparsify_tp = 0.0
    desc.flags = 8                         # not a planner switch
    assert _status(desc) == ev.ERR_INVALID_ARG
    desc.flags = ev.FLAG_NO_FUSION | ev.FLAG_NO_FOLD | ev.FLAG_FORCE_VALU
    assert _status(desc) == ev.OK
    desc.abi_version = 1                   # a description laid out for the previous ABI is refused
    assert _status(desc) == ev.ERR_BAD_DESC
    desc.abi_version = ev.ABI_VERSION
    assert ev.lib().evconv_query_workspace(None, None) == ev.ERR_INVALID_ARG
    assert b"" != ev.lib().evconv_last_error(None)


def test_recurrent_descriptions():
    """DELAY: in0 must name a later node of the same shape, in1 an earlier node of its size."""
    net = wl.net_convlstm(h=16, w=16, hidden=8)
    desc, nodes = ev.marshal_desc(net)
    assert _status(desc) == ev.OK
    src = nodes[0].in0
    nodes[0].in0 = 0                       # itself
    assert _status(desc) == ev.ERR_BAD_DESC
    nodes[0].in0 = len(net.nodes)          # past the end
    assert _status(desc) == ev.ERR_BAD_DESC
    nodes[0].in0 = len(net.nodes) - 1      # the 2-channel head: shape differs
    assert _status(desc) == ev.ERR_SHAPE
    nodes[0].in0 = src
    nodes[0].act = wl.ACT_RELU
    assert _status(desc) == ev.ERR_UNSUPPORTED
    nodes[0].act = wl.ACT_NONE
    nodes[1].in1 = 5                       # the size reference must be an earlier node
    assert _status(desc) == ev.ERR_BAD_DESC
    nodes[1].in1 = -1
    assert _status(desc) == ev.OK


def test_null_handles():
    L = ev.lib()
    assert L.evconv_destroy(None) == ev.OK
    assert L.evconv_num_outputs(None) == 0
    assert L.evconv_reset(None, None, None) == ev.ERR_INVALID_ARG
    assert L.evconv_step(None, None, None) == ev.ERR_INVALID_ARG
    assert L.evconv_set_mode(None, 0) == ev.ERR_INVALID_ARG
    assert L.evconv_current_mode(None) == -1


def test_measurement_aids_reject_bad_arguments_before_any_gpu_work():
    L = ev.lib()
    out = (ctypes.c_float * ev.CHIP_PROBE_VALUES)()
    INVALID, UNSUPPORTED = ev.STATUS_NAMES.index("ERR_INVALID_ARG"), ev.STATUS_NAMES.index("ERR_UNSUPPORTED")
    assert L.evconv_debug_chip_probes(None, ev.CHIP_PROBE_SCRATCH_BYTES, None, out, ev.CHIP_PROBE_VALUES) == INVALID
    dummy = ctypes.c_void_p(4096)  # (never dereferenced: the size check comes first)
    assert L.evconv_debug_chip_probes(dummy, ev.CHIP_PROBE_SCRATCH_BYTES - 1, None, out, ev.CHIP_PROBE_VALUES) == INVALID
    assert L.evconv_debug_chip_probes(dummy, ev.CHIP_PROBE_SCRATCH_BYTES, None, out, ev.CHIP_PROBE_VALUES - 1) == INVALID
    # phase stamps exist only in the measurement build; the product library says so
    n = ctypes.c_int32(-5)
    for mode in (0, 1, 2):
        assert L.evconv_debug_phase_stamps(mode, None, 0, 0, ctypes.byref(n)) == UNSUPPORTED
    assert L.evconv_debug_phase_stamps(3, None, 0, 0, ctypes.byref(n)) == INVALID
    assert L.evconv_debug_phase_stamps(0, None, 0, 0, None) == INVALID
    assert L.evconv_debug_phase_stamps(0, None, 8, 0, ctypes.byref(n)) == INVALID
    assert n.value == -5


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2303_04670_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith(".py"):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle", src, flags=re.M), f
                assert "libevconv_oracle" not in src, f
