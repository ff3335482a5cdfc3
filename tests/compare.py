"""Element-by-element comparison of the HIP path's state with the oracle's (test infrastructure).

Integer products (site lists, occupancy words, tile bitmaps, counts) must be bit-identical.  The
one licensed exception: a value-pruned set may differ at a site whose increment is at rounding
level on the side that kept it (a pre-activation within rounding distance of zero decides
differently in fp32 and fp64); such "flips" are counted and bounded, and sets derived from a
flipped set are compared under the same rule.  Floating-point tensors are compared with
max-abs error <= tol * max|reference tensor|.
"""
from __future__ import annotations

import dataclasses

import numpy as np

from oracle.oracle import Oracle, tile_words, SET_ACTIVE, SET_TOUCHED


def words_to_mask(occ: np.ndarray, h: int, w: int) -> np.ndarray:
    """Inverse of tile_words for 8 x 8 tiles."""
    ty, tx = -(-h // 8), -(-w // 8)
    bits = np.unpackbits(occ.view(np.uint8).reshape(ty, tx, 8, 1), axis=3, bitorder="little")  # [ty,tx,row,col]
    full = bits.transpose(0, 2, 1, 3).reshape(ty * 8, tx * 8)
    assert not full[h:].any() and not full[:, w:].any(), "occupancy bit outside the image"
    return full[:h, :w].astype(np.uint8)


@dataclasses.dataclass
class Report:
    flips: int = 0
    max_rel_z: float = 0.0
    max_rel_y: float = 0.0
    max_rel_inc: float = 0.0   # frobenius mode: largest ||increment error|| / ||increment|| on the common support
    nodes_checked: int = 0
    flips_by_node: dict = dataclasses.field(default_factory=dict)


def _check_set(name, gpu_mask, ref_mask, gpu_mag, ref_mag, tol_abs, rep: Report):
    """gpu_mag / ref_mag: per-site max |increment| on each side (H x W)."""
    if np.array_equal(gpu_mask, ref_mask):
        return
    only_gpu = (gpu_mask == 1) & (ref_mask == 0)
    only_ref = (ref_mask == 1) & (gpu_mask == 0)
    bad_g = only_gpu & (gpu_mag > tol_abs)
    bad_r = only_ref & (ref_mag > tol_abs)
    assert not bad_g.any() and not bad_r.any(), (
        f"{name}: active sets differ at sites carrying non-negligible increments "
        f"(gpu-only {int(bad_g.sum())}, oracle-only {int(bad_r.sum())}, tol {tol_abs:g})")
    n = int(only_gpu.sum() + only_ref.sum())
    rep.flips += n
    rep.flips_by_node[name] = rep.flips_by_node.get(name, 0) + n


def _accumulated_scale(ora: Oracle, i: int) -> float:
    """max |accumulated tensor| of node i, or of the nodes feeding it if it keeps none."""
    if i < 0:
        return float(np.abs(ora.x_prev()).max())
    z = ora.tensor(i, 0)
    if z.size:
        return float(np.abs(z).max())
    nd = ora.net.nodes[i]
    return max(_accumulated_scale(ora, j) for j in (nd.in0, nd.in1) if j >= -1)


def compare_input_stage(gpu, ora: Oracle, rep: Report):
    """Increment builder: everything is a function of the input bits => bit-exact."""
    from paper_2303_04670_amd import evconv as ev
    c, h, w = ora.shape(-1)
    mask = ora.mask(-1)
    occ_ref, bitmap_ref = tile_words(mask)
    np.testing.assert_array_equal(gpu.state(-1, ev.STATE_OCC), occ_ref, err_msg="input occupancy words")
    np.testing.assert_array_equal(gpu.state(-1, ev.STATE_BITMAP), bitmap_ref, err_msg="input tile bitmap")
    np.testing.assert_array_equal(gpu.site_list(-1), ora.site_list(-1), err_msg="input site list")
    dx_ref = ora.tensor(-1, 1).astype(np.float32)
    dx = gpu.state(-1, ev.STATE_DY)
    np.testing.assert_array_equal(dx.view(np.uint32), dx_ref.view(np.uint32), err_msg="input increment bits")
    np.testing.assert_array_equal(gpu.state(-1, ev.STATE_X_PREV).view(np.uint32), ora.x_prev().view(np.uint32))


def compare_node(gpu, ora: Oracle, i: int, rep: Report, tol=1e-4, act_scale=None, exact_sets=False, frobenius=False,
                 inc_rel_tol=6e-2):
    """frobenius=True: accumulated tensors are compared by relative Frobenius error <= tol (used
    for the bf16 contraction, tol = 2e-2) instead of max-abs error; increments element-wise
    against tol times the accumulated tensor's scale, and in Frobenius norm against inc_rel_tol
    times their own norm (an increment behind L bf16 layers carries each layer's 2^-8 product
    error relative to itself, plus the sites where a ReLU's argument changes sign on one side
    only; measured 3e-3 for a single layer, 3.4e-2 at the end of the 21-node UNet after 100 steps)."""
    from paper_2303_04670_amd import evconv as ev
    c, h, w = ora.shape(i)
    assert gpu.shape(i) == (c, h, w)
    if gpu.kernel_name(i) in ("fused_into_conv_gather", "fused_into_conv_weights", "fused_into_concat_gather"):
        return  # never materialised: the consuming conv, which is compared, reads it through its gather
    s_ref, t_ref = ora.mask(i, SET_ACTIVE), ora.mask(i, SET_TOUCHED)
    occ = gpu.state(i, ev.STATE_OCC)
    s_gpu = words_to_mask(occ, h, w)
    t_gpu = words_to_mask(gpu.state(i, ev.STATE_OCC_TOUCHED), h, w)
    dy_ref = ora.dy(i)
    dy_gpu = gpu.state(i, ev.STATE_DY).astype(np.float64)
    # the list, count and bitmap must re-encode the GPU's own occupancy words exactly
    np.testing.assert_array_equal(gpu.site_list(i), np.flatnonzero(s_gpu.ravel()).astype(np.int32),
                                  err_msg=f"node {i}: list is not the ascending encoding of the occupancy words")
    np.testing.assert_array_equal(gpu.state(i, ev.STATE_BITMAP), tile_words(s_gpu)[1], err_msg=f"node {i} bitmap")
    assert np.all(s_gpu <= t_gpu), f"node {i}: active set not inside touched set"

    scale = act_scale if act_scale is not None else max(np.abs(dy_ref).max(), 1e-30)
    tol_abs = tol * scale
    if exact_sets:
        np.testing.assert_array_equal(s_gpu, s_ref, err_msg=f"node {i} active set")
        np.testing.assert_array_equal(t_gpu, t_ref, err_msg=f"node {i} touched set")
    else:
        gm = np.abs(dy_gpu).max(axis=2) * (t_gpu == 1)
        rm = np.abs(dy_ref).max(axis=2)
        _check_set(f"node {i} touched", t_gpu, t_ref, gm, rm, tol_abs, rep)
        _check_set(f"node {i} active", s_gpu, s_ref, gm * (s_gpu == 1), rm, tol_abs, rep)
    # increments on the common support
    both = (s_gpu == 1) & (s_ref == 1)
    if both.any():
        if frobenius:
            # an increment is a small difference of accumulated values that each carry the bf16
            # error, so it is bounded against the scale of the accumulated tensor, not its own
            ref_scale = max(_accumulated_scale(ora, i), np.abs(dy_ref).max(), 1e-30)
            err = np.abs(dy_gpu[both] - dy_ref[both]).max()
            assert err <= tol * ref_scale, f"node {i}: increment error {err:g} > {tol:g} * {ref_scale:g}"
            rel = np.linalg.norm(dy_gpu[both] - dy_ref[both]) / max(np.linalg.norm(dy_ref[both]), 1e-30)
            rep.max_rel_inc = max(rep.max_rel_inc, rel)
            assert rel <= inc_rel_tol, f"node {i}: increment error {rel:g} of its own norm > {inc_rel_tol:g}"
        else:
            err = np.abs(dy_gpu[both] - dy_ref[both]).max()
            assert err <= tol_abs, f"node {i}: increment error {err:g} > {tol_abs:g}"
    # accumulated tensor
    nd = ora.net.nodes[i]
    z_ref = ora.tensor(i, 0)
    if z_ref.size:
        z_gpu = gpu.state(i, ev.STATE_Z).astype(np.float64)
        if frobenius:
            zs = max(np.linalg.norm(z_ref), 1e-30)
            err = np.linalg.norm(z_gpu - z_ref)
        else:
            zs = max(np.abs(z_ref).max(), 1e-30)
            err = np.abs(z_gpu - z_ref).max()
        rep.max_rel_z = max(rep.max_rel_z, err / zs)
        assert err <= tol * zs, f"node {i} (op {nd.op}): accumulated tensor error {err:g} > {tol:g} * {zs:g}"
    rep.nodes_checked += 1


def compare_outputs_value_only(gpu, ora: Oracle, rep: Report, tol=1e-4):
    """Only y(n): for steps run as regular forward passes, whose dy is y(n) - y(n-1) at every
    site instead of the oracle's sparse increment."""
    gpu.torch.cuda.synchronize()
    for o in gpu.outputs():
        y_ref = np.transpose(ora.y(o["node"]), (2, 0, 1))
        y = o["y"].cpu().numpy().astype(np.float64)
        scale = max(np.abs(y_ref).max(), 1e-30)
        err = np.abs(y - y_ref).max()
        rep.max_rel_y = max(rep.max_rel_y, err / scale)
        assert err <= tol * scale, f"output node {o['node']}: y error {err:g} > {tol:g} * {scale:g}"


def compare_outputs(gpu, ora: Oracle, rep: Report, tol=1e-4):
    gpu.torch.cuda.synchronize()
    for o in gpu.outputs():
        i = o["node"]
        y_ref = np.transpose(ora.y(i), (2, 0, 1))
        dy_ref = np.transpose(ora.dy(i), (2, 0, 1))
        y = o["y"].cpu().numpy().astype(np.float64)
        dy = o["dy"].cpu().numpy().astype(np.float64)
        scale = max(np.abs(y_ref).max(), 1e-30)
        err = np.abs(y - y_ref).max()
        rep.max_rel_y = max(rep.max_rel_y, err / scale)
        assert err <= tol * scale, f"output node {i}: y error {err:g} > {tol:g} * {scale:g}"
        assert np.abs(dy - dy_ref).max() <= tol * scale, f"output node {i}: y_inc error"
        n = int(o["count"].cpu()[0])
        idx = o["idx"].cpu().numpy()[:n]
        assert np.all(np.diff(idx) > 0), "output list not strictly ascending"
        support = np.flatnonzero(np.any(dy != 0, axis=0).ravel())
        assert np.all(np.isin(support, idx)), "output increment nonzero outside its list"
