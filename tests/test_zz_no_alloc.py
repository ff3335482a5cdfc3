"""evconv_create_static: a net built in the library's own per-GPU array must behave exactly like
one built in a caller's workspace (same kernels, same layout: bit-identical), on two nets in a
row, the second smaller than the first, whose state must not see what the first left behind."""
import numpy as np
import pytest

from paper_2303_04670_amd import evconv as ev
from paper_2303_04670_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _same_bits(a, b, what):
    np.testing.assert_array_equal(np.ascontiguousarray(a).view(np.uint8), np.ascontiguousarray(b).view(np.uint8), err_msg=what)


def _run_pair(net, frames, label):
    import torch
    print(f"no-alloc entry point: {label}, workspace {ev.evconv_query_workspace(ev.marshal_desc(net)[0]) / 2**20:.1f} MiB", flush=True)
    ref = ev.EvConvNet(net)
    before = torch.cuda.memory_allocated()
    st = ev.EvConvNet(net, static_workspace=True)
    assert st.workspace is None and torch.cuda.memory_allocated() == before   # no workspace tensor
    for t, f in enumerate(frames):
        x = _dev(f)
        for g in (ref, st):
            (g.reset if t == 0 else g.step_frame)(x)
        torch.cuda.synchronize()
        for a, b in zip(ref.outputs(), st.outputs()):
            for key in ("y", "dy", "count"):
                _same_bits(a[key].cpu().numpy(), b[key].cpu().numpy(), f"{label} step {t} output {key}")
            n = int(a["count"].cpu()[0])
            _same_bits(a["idx"].cpu().numpy()[:n], b["idx"].cpu().numpy()[:n], f"{label} step {t} output list")
        for i in range(len(net.nodes)):
            if ref.kernel_name(i).endswith(("_gather", "_weights")):
                continue
            for kind in (ev.STATE_DY, ev.STATE_OCC, ev.STATE_OCC_TOUCHED, ev.STATE_BITMAP):
                _same_bits(ref.state(i, kind), st.state(i, kind), f"{label} step {t} node {i} state {kind}")
            if net.nodes[i].op == wl.OP_CONV2D:
                _same_bits(ref.state(i, ev.STATE_Z), st.state(i, ev.STATE_Z), f"{label} step {t} node {i} z")
            _same_bits(ref.site_list(i), st.site_list(i), f"{label} step {t} node {i} list")
    # the array belongs to one net at a time
    with pytest.raises(ev.EvConvError) as e:
        ev.EvConvNet(net, static_workspace=True)
    assert e.value.status == ev.ERR_STATE
    ref.destroy()
    st.destroy()


def test_static_workspace_net_equals_a_net_in_a_caller_workspace_twice_in_a_row():
    big = wl.net_conv_stack(1002, h=180, w=240)                 # 19.6 MiB of the 32 MiB array
    frames_big = list(wl.stream_voxel(1002, 180, 240, 6, 0.03))
    _run_pair(big, frames_big, "conv stack 5x180x240")
    small = wl.net_unet_depth(1003, h=40, w=56, width=8)         # every op of the UNet, a few MiB
    frames_small = list(wl.stream_voxel(1003, 40, 56, 6, 0.05, n_prim=4))
    _run_pair(small, frames_small, "reduced UNet 5x40x56")
    # a description that does not fit is refused with both sizes in the message
    with pytest.raises(ev.EvConvError) as e:
        ev.EvConvNet(wl.net_unet_depth(), static_workspace=True)
    assert e.value.status == ev.ERR_WORKSPACE and str(ev.STATIC_WORKSPACE_BYTES) in str(e.value)
