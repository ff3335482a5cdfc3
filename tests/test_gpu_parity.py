"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  Integer products bit-exact (with counted rounding flips of value-pruned
sets, see compare.py); fp32 tensors within 1e-4 * max|tensor| of the fp64 oracle."""
import dataclasses
import sys

import numpy as np
import pytest

import compare as cmp
from oracle.oracle import Oracle
from paper_2303_04670_amd import evconv as ev
from paper_2303_04670_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def run_stream(net, x0, inputs, kind, check_nodes_at=None, tol=TOL, exact_sets=False, max_flips=0,
               fp32_oracle=False, label="", frobenius=False):
    """kind: 'frame' or 'increment'.  check_nodes_at: steps (1-based) at which every node is
    compared (None = every step); outputs and the input stage are compared at every step."""
    gpu = ev.EvConvNet(net)
    ora = Oracle(net, fp32_state=fp32_oracle)
    rep = cmp.Report()
    gpu.reset(_dev(x0))
    ora.reset(x0)
    cmp.compare_outputs(gpu, ora, rep, tol)
    for i in range(len(net.nodes)):
        if ora.tensor(i, 0).size:
            z = gpu.state(i, ev.STATE_Z).astype(np.float64)
            zr = ora.z(i)
            assert np.abs(z - zr).max() <= tol * max(np.abs(zr).max(), 1e-30), f"reset: node {i} z"
    for step, inp in enumerate(inputs, 1):
        if kind == "frame":
            gpu.step_frame(_dev(inp))
            ora.step_frame(inp)
        else:
            gpu.step(_dev(inp))
            ora.step_increment(inp)
        cmp.compare_input_stage(gpu, ora, rep)
        cmp.compare_outputs(gpu, ora, rep, tol)
        if check_nodes_at is None or step in check_nodes_at:
            for i in range(len(net.nodes)):
                cmp.compare_node(gpu, ora, i, rep, tol=tol, exact_sets=exact_sets, frobenius=frobenius)
        if step % 10 == 0:
            _say(f"[{label}] step {step}: flips {rep.flips} max rel z err {rep.max_rel_z:.2e} y err {rep.max_rel_y:.2e}")
    _say(f"[{label}] done: flips {rep.flips} (allowed {max_flips}) max rel z err {rep.max_rel_z:.2e} y err {rep.max_rel_y:.2e}"
         + (f" increment err (own norm) {rep.max_rel_inc:.2e}" if frobenius else ""))
    assert rep.flips <= max_flips, f"{rep.flips} rounding flips of value-pruned sets: {rep.flips_by_node}"
    gpu.destroy()
    return rep


def test_workload1_single_conv_10_steps():
    _say("workload 1: single conv3x3 16->16 on 16x64x64, 10 increments at 2 %")
    net = wl.net_single_conv()
    x0, incs = wl.stream_line_increments()
    rep = run_stream(net, x0, incs, "increment", label="w1", max_flips=2)
    assert rep.nodes_checked == 10


def test_workload2_conv_stack_100_steps():
    _say("workload 2: 4-layer conv stack on 5x180x240, 100 frames at 1-5 %")
    net = wl.net_conv_stack()
    frames = list(wl.stream_voxel(1002, 180, 240, 100, wl.density_sweep_1_5))
    run_stream(net, frames[0], frames[1:], "frame", check_nodes_at={1, 2, 3, 25, 50, 75, 100}, label="w2",
               max_flips=8)


@pytest.mark.parametrize("seed", [7, 8, 9])
def test_every_op_small_ragged_graph(seed):
    _say(f"small graph touching every op, seed {seed}")
    kw = {} if seed == 7 else dict(in_c=2, h=9, w=19, bias=(seed == 8))
    net = wl.net_random_small(seed, **kw)
    rng = np.random.default_rng(seed)
    x0 = rng.standard_normal((net.in_c, net.in_h, net.in_w)).astype(np.float32)
    frames, x = [], x0
    for t in range(12):
        m = rng.random((net.in_h, net.in_w)) < (0.02 + 0.08 * (t % 4))
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m[None]).astype(np.float32)
        frames.append(x)
    run_stream(net, x0, frames, "frame", label=f"small{seed}", max_flips=4)


def test_unet_reduced_all_nodes_every_step():
    _say("UNet depth net, reduced 5x64x96 width 8, 30 frames, all nodes every step")
    net = wl.net_unet_depth(1003, h=64, w=96, width=8)
    frames = list(wl.stream_voxel(1003, 64, 96, 30, 0.02, n_prim=6))
    run_stream(net, frames[0], frames[1:], "frame", label="unet-small", max_flips=40)


def test_unet_full_width_reduced_size_matrix_core_layers():
    _say("UNet depth net, full width (32..256 channels) on 5x64x96: matrix-core conv layers, all nodes every step")
    net = wl.net_unet_depth(1003, h=64, w=96)
    g = ev.EvConvNet(net)
    names = [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    assert names.count("conv_mfma_f32") == 10 and names[0] == "conv_narrow_mfma_f32" and names[-1] == "conv_pointwise_f32", names
    assert names.count("fused_into_conv_epilogue") == 6, names   # 2 residual adds + 4 skip adds
    # the three x2 up-samplings: only the last one's stored tensor (32 x 48) has tiles away from the border
    assert names.count("fused_into_conv_gather") == 2 and names.count("fused_into_conv_weights") == 1, names
    frames = list(wl.stream_voxel(1003, 64, 96, 20, 0.02, n_prim=6))
    run_stream(net, frames[0], frames[1:], "frame", label="unet-wide", max_flips=40)


def test_unet_full_width_without_epilogue_fusion():
    """The same graph with ADD nodes run by their own kernels instead of the conv epilogues."""
    _say("UNet depth net, full width on 5x64x96, ADD nodes unfused")
    net = wl.net_unet_depth(1003, h=64, w=96)
    g = ev.EvConvNet(net, flags=ev.FLAG_NO_FUSION)
    names = [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    assert not any(nm.startswith("fused_into_") for nm in names), names
    frames = list(wl.stream_voxel(1003, 64, 96, 8, 0.02, n_prim=6))
    run_stream(net, frames[0], frames[1:], "frame", label="unet-wide-unfused", max_flips=40)


def test_unet_bf16_matrix_core_variant_reduced():
    """bf16-weight variant: increments are rounded to bf16 in the gather, weights are bf16, fp32
    accumulation.  Oracle: the same bf16-rounded weights held exactly in fp64, unrounded
    increments.  Bar: 2e-2 relative (Frobenius) per accumulated tensor and increment."""
    _say("UNet depth net bf16 variant, full width on 5x64x96, 20 frames")
    net = wl.net_unet_depth(1003, h=64, w=96, bf16=True)
    g = ev.EvConvNet(net)
    names = [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    assert names.count("conv_mfma_bf16") == 10, names
    frames = list(wl.stream_voxel(1003, 64, 96, 20, 0.02, n_prim=6))
    run_stream(net, frames[0], frames[1:], "frame", label="unet-bf16", tol=2e-2, frobenius=True, max_flips=200)


def test_matrix_core_conv_shapes_bf16():
    _say("bf16 matrix-core conv variants")
    for k, s, ci, co in [(3, 1, 32, 32), (3, 2, 16, 64), (5, 1, 64, 32), (5, 2, 48, 96), (7, 2, 16, 32), (1, 1, 32, 64), (3, 1, 68, 32), (5, 2, 20, 32),
                         (3, 1, 69, 32), (5, 2, 21, 32), (3, 1, 18, 64), (5, 1, 35, 64),   # c_in % 4 != 0
                         (3, 1, 32, 16), (3, 1, 37, 28)]:                                   # c_out % 32 != 0
        b = wl._NetBuilder(f"conv{k}s{s}", ci, 21, 27, 100 + k * 10 + s, bf16=True, bias=True)
        b.conv(-1, co, k, s, act=wl.ACT_RELU, out=1)
        net = b.finish()
        rng = np.random.default_rng(k + s)
        x0 = rng.standard_normal((ci, 21, 27)).astype(np.float32)
        incs = []
        for t in range(4):
            m = rng.random((21, 27)) < (0.03 if t < 3 else 1.0)
            incs.append(rng.standard_normal(x0.shape).astype(np.float32) * m[None])
        g = ev.EvConvNet(net)
        assert g.kernel_name(0) == "conv_mfma_bf16"
        g.destroy()
        run_stream(net, x0, incs, "increment", label=f"bf16 k{k}s{s}", tol=2e-2, frobenius=True, max_flips=20)


def test_narrow_input_conv_shapes():
    """First-layer kernel (2-8 input channels, taps x channels <= 128): strides, tap counts, one or
    two blocks of output channels, output channel counts that are not multiples of 32."""
    _say("narrow-input conv variants")
    for k, s, ci, co in [(5, 1, 5, 32), (3, 2, 4, 64), (7, 2, 2, 64), (3, 1, 8, 96), (1, 1, 3, 32),
                         (5, 1, 5, 16), (3, 1, 4, 48), (3, 2, 6, 100), (5, 2, 3, 24)]:
        b = wl._NetBuilder(f"narrow{k}s{s}", ci, 21, 27, 200 + k * 10 + s, bias=True)
        b.conv(-1, co, k, s, act=wl.ACT_RELU, out=1)
        net = b.finish()
        rng = np.random.default_rng(k + s + ci)
        x0 = rng.standard_normal((ci, 21, 27)).astype(np.float32)
        incs = []
        for t in range(4):
            m = rng.random((21, 27)) < (0.03 if t < 3 else 1.0)
            incs.append(rng.standard_normal(x0.shape).astype(np.float32) * m[None])
        g = ev.EvConvNet(net)
        assert g.kernel_name(0) == "conv_narrow_mfma_f32", (k, s, ci, co, g.kernel_name(0))
        g.destroy()
        run_stream(net, x0, incs, "increment", label=f"narrow k{k}s{s} {ci}->{co}", max_flips=2)


def test_matrix_core_conv_shapes():
    """Every (kernel, stride, channel-chunk) variant of the matrix-core conv on ragged sizes, with
    bias, dense and sparse increments."""
    _say("matrix-core conv variants: k in {1,3,5,7}, stride {1,2}, c_in in {16,32,48,64}")
    for k, s, ci, co in [(3, 1, 32, 32), (3, 2, 16, 64), (5, 1, 64, 32), (5, 2, 48, 96), (7, 2, 16, 32), (1, 1, 32, 64),
                         (3, 1, 68, 32), (5, 1, 20, 32), (3, 2, 36, 64),      # ragged channel chunks
                         (3, 1, 69, 32), (5, 2, 21, 32), (3, 1, 18, 64), (5, 1, 35, 64), (1, 1, 17, 32),  # c_in % 4 != 0
                         (3, 1, 32, 16), (5, 2, 16, 48), (3, 1, 37, 28), (3, 2, 64, 100),    # c_out % 32 != 0
                         (3, 1, 12, 32), (5, 1, 9, 64), (3, 2, 10, 20)]:                      # fewer than 16 input channels
        b = wl._NetBuilder(f"conv{k}s{s}", ci, 21, 27, 100 + k * 10 + s, bias=True)
        b.conv(-1, co, k, s, act=wl.ACT_RELU, out=1)
        net = b.finish()
        rng = np.random.default_rng(k + s)
        x0 = rng.standard_normal((ci, 21, 27)).astype(np.float32)
        incs = []
        for t in range(4):
            m = rng.random((21, 27)) < (0.03 if t < 3 else 1.0)
            incs.append(rng.standard_normal(x0.shape).astype(np.float32) * m[None])
        g = ev.EvConvNet(net)
        assert g.kernel_name(0) == "conv_mfma_f32"
        g.destroy()
        run_stream(net, x0, incs, "increment", label=f"mfma k{k}s{s}", max_flips=2)


def test_flow_net_reduced_concat_upsample():
    _say("flow encoder-decoder, reduced 4x64x64 width 8, density sweep, all nodes every step")
    net = wl.net_flow(1005, h=64, w=64, width=8)
    g = ev.EvConvNet(net)
    names = [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    # every decoder's up-sampling is read by its concatenation alone: interpolated there, never stored
    ups = [i for i, n in enumerate(net.nodes) if n.op == wl.OP_UPSAMPLE2X]
    assert ups and all(names[i] == "fused_into_concat_gather" for i in ups), names
    frames = list(wl.stream_count_timestamp(1005, 64, 64, densities=[0.001, 0.01, 0.05, 0.2], steps_per=4))
    run_stream(net, frames[0], frames[1:], "frame", label="flow-small", max_flips=8)


def test_delayed_flow_net_reduced():
    """Delayed-integration encoder-decoder: decoders fed by skips only, upsampled decoder outputs
    and predictions concatenated at full resolution, two final convolutions."""
    _say("delayed-integration flow net, reduced 4x64x96 width 8, all nodes every step")
    net = wl.net_flow_delayed(1006, h=64, w=96, width=8, d_width=32)
    frames = list(wl.stream_count_timestamp(1006, 64, 96, densities=[0.001, 0.01, 0.05, 0.2], steps_per=4))
    run_stream(net, frames[0], frames[1:], "frame", label="delayed-small", max_flips=8)


def test_resnet_reduced_pool_gap_linear():
    _say("ResNet-18-style classifier, reduced 2x64x64 width 8")
    net = wl.net_resnet18(1004, h=64, w=64, n_classes=11, width=8)
    frames = list(wl.stream_histogram(1004, 64, 64, steps=16))
    run_stream(net, frames[0], frames[1:], "frame", label="resnet-small", max_flips=8)


def test_edge_cases_zero_full_corner_special_values():
    _say("edge cases: zero increment, every site active, corner pixels, -0.0, denormal, NaN-free inf-free")
    net = wl.net_conv_stack(77, h=21, w=27)
    rng = np.random.default_rng(77)
    x0 = rng.standard_normal((5, 21, 27)).astype(np.float32)
    incs = []
    incs.append(np.zeros_like(x0))                                   # nothing changes
    incs.append(rng.standard_normal(x0.shape).astype(np.float32))    # everything changes
    for (y, x) in [(0, 0), (0, 26), (20, 0), (20, 26)]:              # single corner pixels
        d = np.zeros_like(x0)
        d[2, y, x] = 1.25
        incs.append(d)
    d = np.zeros_like(x0)
    d[:, 3, 3] = -0.0                                                 # negative zero: inactive
    d[1, 10, 10] = np.float32(1e-42)                                  # denormal: active
    incs.append(d)
    incs.append(np.zeros_like(x0))
    rep = run_stream(net, x0, incs, "increment", label="edge", exact_sets=False, max_flips=4)
    # explicit expectations on the input stage for the special values
    gpu = ev.EvConvNet(net)
    gpu.reset(_dev(x0))
    gpu.step(_dev(d))
    assert list(gpu.site_list(-1)) == [10 * 27 + 10]
    gpu.step(_dev(np.zeros_like(x0)))
    assert gpu.site_list(-1).size == 0
    for i in range(4):
        assert gpu.site_list(i).size == 0
        assert not gpu.state(i, ev.STATE_OCC_TOUCHED).any()
    gpu.destroy()


def _nan_aware_compare(gpu, ora, net, tol=TOL):
    """Sets bit-exact; NaN and infinite elements at the same places with the same sign; finite
    elements within tol of the tensor's largest finite magnitude."""
    for i in range(len(net.nodes)):
        c, h, w = ora.shape(i)
        s_gpu = cmp.words_to_mask(gpu.state(i, ev.STATE_OCC), h, w)
        t_gpu = cmp.words_to_mask(gpu.state(i, ev.STATE_OCC_TOUCHED), h, w)
        np.testing.assert_array_equal(s_gpu, ora.mask(i, cmp.SET_ACTIVE), err_msg=f"node {i} active set")
        np.testing.assert_array_equal(t_gpu, ora.mask(i, cmp.SET_TOUCHED), err_msg=f"node {i} touched set")
        np.testing.assert_array_equal(gpu.site_list(i), ora.site_list(i))
        pairs = [(gpu.state(i, ev.STATE_DY).astype(np.float64), ora.dy(i), "increment")]
        if ora.z(i).size:
            pairs.append((gpu.state(i, ev.STATE_Z).astype(np.float64), ora.z(i), "accumulated tensor"))
        for got, ref, what in pairs:
            with np.errstate(invalid="ignore"):
                got = np.where(s_gpu[:, :, None] == 1, got, 0.0) if what == "increment" else got
                np.testing.assert_array_equal(np.isnan(got), np.isnan(ref), err_msg=f"node {i} {what}: NaN positions")
                inf = np.isinf(ref)
                np.testing.assert_array_equal(np.isinf(got), inf, err_msg=f"node {i} {what}: infinities")
                np.testing.assert_array_equal(got[inf], ref[inf], err_msg=f"node {i} {what}: sign of infinities")
                fin = np.isfinite(ref)
                scale = max(np.abs(ref[fin]).max(), 1e-30)
                assert np.abs(got[fin] - ref[fin]).max() <= tol * scale, f"node {i} {what}"


@pytest.mark.parametrize("acts", ["relu", "linear"])
def test_nan_and_inf_increments_are_active_and_propagate(acts):
    """The zero test is `!= 0` on the fp32 value, so a NaN or an infinite increment makes its site
    active; the values then follow IEEE arithmetic through the layers: a conv output that reads
    the site becomes NaN / +-inf (a sum of opposite infinities: NaN), relu(NaN) = 0 on both sides,
    so behind a ReLU the increment is 0 - relu(z_old) and the accumulated tensor stays NaN until a
    refresh; without activation the NaN reaches the output.  Narrow-input, matrix-core and
    vector kernels (5 -> 32 -> 32 -> 64 -> 64 channels, strides 1, 2, 2, 1)."""
    _say(f"edge case: NaN and +-inf increments, {acts} stack")
    net = wl.net_conv_stack(78, h=21, w=27)
    if acts == "linear":
        for nd in net.nodes:
            nd.act = wl.ACT_NONE
    rng = np.random.default_rng(78)
    x0 = rng.standard_normal((5, 21, 27)).astype(np.float32)
    d1 = np.zeros_like(x0)
    d1[1, 4, 5] = np.nan
    d1[3, 15, 20] = np.inf
    d1[0, 15, 2] = -np.inf
    d1[2, 9, 9] = 0.5                       # an ordinary change beside them
    d2 = (rng.standard_normal(x0.shape) * (rng.random((1, 21, 27)) < 0.05)).astype(np.float32)
    gpu, ora = ev.EvConvNet(net), Oracle(net)
    gpu.reset(_dev(x0))
    ora.reset(x0)
    for t, d in enumerate((d1, d2, np.zeros_like(x0))):
        gpu.step(_dev(d))
        ora.step_increment(d)
        np.testing.assert_array_equal(gpu.site_list(-1), ora.site_list(-1), err_msg=f"step {t}: input list")
        if t == 0:
            assert {4 * 27 + 5, 15 * 27 + 20, 15 * 27 + 2, 9 * 27 + 9} == set(gpu.site_list(-1).tolist())
        _nan_aware_compare(gpu, ora, net)
    z0 = gpu.state(0, ev.STATE_Z)
    assert np.isnan(z0[4, 5]).all() and np.isinf(z0[15, 20]).any()
    if acts == "linear":
        import torch
        torch.cuda.synchronize()
        assert torch.isnan(gpu.outputs()[0]["y"]).any()
    # a refresh (regular forward pass of the cached frame, which now holds the NaN) is not a cure
    # for the input; a reset on a clean frame is
    gpu.reset(_dev(x0))
    ora.reset(x0)
    gpu.step(_dev(d2))
    ora.step_increment(d2)
    _nan_aware_compare(gpu, ora, net)
    gpu.destroy()


def test_layer_statistics_equal_the_oracles_counters():
    """evconv_get_stats against the oracle: sizes of the touched and active sets, touched tiles,
    and the executed / dense operation counts (2 x the oracle's tile-level and nominal dense
    multiply-accumulate counts, which tests/test_oracle_macs.py pins against hand counts)."""
    _say("layer statistics (set sizes, touched tiles, executed and dense FLOPs) vs the oracle's counters")
    cases = [(wl.net_single_conv(), None), (wl.net_unet_depth(1003, h=64, w=96), list(wl.stream_voxel(1003, 64, 96, 4, 0.02, n_prim=6)))]
    for net, frames in cases:
        gpu, ora = ev.EvConvNet(net), Oracle(net)
        if frames is None:
            x0, incs = wl.stream_line_increments()
            steps = [("increment", d) for d in incs[:4]]
        else:
            x0, steps = frames[0], [("frame", f) for f in frames[1:]]
        gpu.reset(_dev(x0))
        ora.reset(x0)
        checked = 0
        for kind, a in steps:
            (gpu.step_frame if kind == "frame" else gpu.step)(_dev(a))
            (ora.step_frame if kind == "frame" else ora.step_increment)(a)
            for i, nd in enumerate(net.nodes):
                if gpu.kernel_name(i) in ("fused_into_conv_gather", "fused_into_conv_weights", "fused_into_concat_gather"):
                    continue
                st = gpu.stats(i)
                c, h, w = ora.shape(i)
                s_ref, t_ref = ora.mask(i, cmp.SET_ACTIVE), ora.mask(i, cmp.SET_TOUCHED)
                assert (st.n_sites, st.n_tiles) == (h * w, -(-h // 8) * -(-w // 8))
                assert st.n_touched == int(t_ref.sum()), f"node {i} touched"
                # (the value-pruned set may differ by a flip where fp32 summation order decides whether a
                # saturating sigmoid moves at all; the other counters are integer functions of the input set)
                assert abs(st.n_active - int(s_ref.sum())) <= (2 if nd.act == wl.ACT_SIGMOID else 0), f"node {i} active"
                assert st.n_touched_tiles == int(np.count_nonzero(cmp.tile_words(t_ref)[0])), f"node {i} touched tiles"
                if nd.op in (wl.OP_CONV2D, wl.OP_LINEAR):
                    m = ora.macs(i, (8, 8))
                    assert st.flops_executed == 2.0 * m["tile"], f"node {i} executed"
                    assert st.flops_dense == 2.0 * m["dense_nominal"], f"node {i} dense"
                    assert m["site"] <= m["tile"] and m["site"] <= m["dense"] <= m["dense_nominal"]
                    checked += 1
        assert checked >= 4
        gpu.destroy()


def test_delay_of_an_add_that_follows_its_conv_is_not_fused():
    """0 convA(x), 1 convB(x), 2 DELAY of node 3, 3 ADD(0, 1), 4 ADD(3, 2) -> output.  The ADD
    could run in convB's epilogue, but the DELAY between them must see the ADD's buffers as the
    previous step left them; the planner therefore leaves this ADD to its own kernel.  Checked
    against the oracle with the default plan and with every fusion switched off."""
    _say("DELAY of a later ADD placed between the ADD and the conv that could host it")
    b = wl._NetBuilder("delay_add", 16, 24, 40, 41)
    ca = b.conv(-1, 32, 3, act=wl.ACT_NONE)
    cb = b.conv(-1, 32, 3, act=wl.ACT_NONE)
    d = b.delay(32, like=ca)
    add = b.simple(wl.OP_ADD, ca, cb)
    b.close_delay(d, add)
    b.simple(wl.OP_ADD, add, d, out=1)
    net = b.finish()
    rng = np.random.default_rng(41)
    x = rng.standard_normal((16, 24, 40)).astype(np.float32)
    frames = [x]
    for t in range(6):
        m = rng.random((1, 24, 40)) < 0.05
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    g = ev.EvConvNet(net)
    assert g.kernel_name(cb) == "conv_mfma_f32" and g.kernel_name(add) == "elementwise", \
        [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    for flags in (0, ev.FLAG_NO_FUSION):
        gpu, ora, rep = ev.EvConvNet(net, flags=flags), Oracle(net), cmp.Report()
        gpu.reset(_dev(frames[0]))
        ora.reset(frames[0])
        for f in frames[1:]:
            gpu.step_frame(_dev(f))
            ora.step_frame(f)
            cmp.compare_outputs(gpu, ora, rep)
            for i in range(len(net.nodes)):
                cmp.compare_node(gpu, ora, i, rep)
        assert rep.flips <= 4
        gpu.destroy()


def test_pooling_windows_other_than_3x3_and_a_global_mean_over_many_ragged_tiles():
    """Max-pool with 2 x 2 / stride 2 / no padding and with 5 x 5 / stride 1 / padding 2 windows
    (the kernel has a path of its own for 3 x 3), and a global mean over a 27 x 43 map (4 x 6 tiles,
    ragged last row and column, most of them inactive at any step) feeding a linear layer; sparse
    and dense steps, a refresh in between."""
    _say("max-pool 2x2 / 5x5 and a global mean over ragged tiles")
    b = wl._NetBuilder("pools", 6, 27, 43, 57)
    c0 = b.conv(-1, 32, 3, act=wl.ACT_RELU)
    p5 = b.simple(wl.OP_MAXPOOL, c0, k=5, stride=1, pad=2)
    g = b.simple(wl.OP_GAP, p5)
    b.linear(g, 10, out=1)
    p2 = b.simple(wl.OP_MAXPOOL, c0, k=2, stride=2, pad=0)
    b.conv(p2, 16, 3, act=wl.ACT_RELU, out=1)
    net = b.finish()
    rng = np.random.default_rng(57)
    x = rng.standard_normal((6, 27, 43)).astype(np.float32)
    frames = [x]
    for t in range(8):
        dens = 1.0 if t == 4 else 0.02
        m = rng.random((1, 27, 43)) < dens
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    gpu, ora, rep = ev.EvConvNet(net), Oracle(net), cmp.Report()
    assert gpu.kernel_name(g) == "global_avgpool" and gpu.kernel_name(p2) == "maxpool"
    gpu.reset(_dev(frames[0]))
    ora.reset(frames[0])
    for t, f in enumerate(frames[1:]):
        if t == 6:
            gpu.reset(_dev(f))
            ora.reset(f)
        else:
            gpu.step_frame(_dev(f))
            ora.step_frame(f)
        cmp.compare_outputs(gpu, ora, rep)
        for i in range(len(net.nodes)):
            cmp.compare_node(gpu, ora, i, rep)
    assert rep.flips <= 4
    gpu.destroy()


@pytest.mark.parametrize("hw", [(20, 28), (40, 56)], ids=["few_workgroups_8_waves", "more_workgroups_4_waves"])
def test_fp32_blocks_of_16_output_channels_with_ragged_channel_counts(hw):
    """Small maps make the fp32 matrix-core conv take blocks of 16 output channels (eight waves
    per workgroup on the smaller map, four on the larger).  Output channel counts that are not
    multiples of 16, a residual ADD + ReLU folded into the epilogue, a stride-2 layer and a 1 x 1
    layer; sparse steps, one dense step, a refresh."""
    _say(f"16-channel blocks of the fp32 matrix-core conv, {hw[0]} x {hw[1]}")
    h, w = hw
    b = wl._NetBuilder("nb16", 12, h, w, 77)
    c0 = b.conv(-1, 40, 3, act=wl.ACT_RELU)
    c1 = b.conv(c0, 40, 3, act=wl.ACT_NONE)
    r = b.simple(wl.OP_ADD, c1, c0, act=wl.ACT_RELU)
    c2 = b.conv(r, 24, 5, stride=2, act=wl.ACT_RELU)
    c3 = b.conv(c2, 72, 1, pad=0, act=wl.ACT_RELU)
    b.conv(c3, 16, 3, act=wl.ACT_NONE, out=1)
    net = b.finish()
    rng = np.random.default_rng(77)
    x = rng.standard_normal((12, h, w)).astype(np.float32)
    frames = [x]
    for t in range(7):
        m = rng.random((1, h, w)) < (1.0 if t == 3 else 0.03)
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    gpu, ora, rep = ev.EvConvNet(net), Oracle(net), cmp.Report()
    assert all(gpu.kernel_name(i) == "conv_mfma_f32" for i in (c0, c1, c2, c3)), [gpu.kernel_name(i) for i in range(len(net.nodes))]
    assert gpu.kernel_name(r) == "fused_into_conv_epilogue"
    gpu.reset(_dev(frames[0]))
    ora.reset(frames[0])
    for t, f in enumerate(frames[1:]):
        if t == 5:
            gpu.reset(_dev(f))
            ora.reset(f)
        else:
            gpu.step_frame(_dev(f))
            ora.step_frame(f)
        cmp.compare_outputs(gpu, ora, rep)
        for i in range(len(net.nodes)):
            cmp.compare_node(gpu, ora, i, rep)
    assert rep.flips <= 4
    gpu.destroy()


def test_auto_mode_times_both_modes_and_keeps_the_state():
    """AUTO runs windows of incremental and of dense-recompute steps, then holds the faster mode;
    whatever it picks, the state follows the same frames (Eq.2), so outputs and accumulated
    tensors stay within the fp32 bar of the oracle at every step; a net with an active
    sparsification layer stays incremental."""
    _say("AUTO mode: state parity through the mode switches")
    net = wl.net_unet_depth(1003, h=64, w=96)
    frames = list(wl.stream_voxel(1003, 64, 96, 16, 0.02, n_prim=6))
    gpu, ora, rep = ev.EvConvNet(net), Oracle(net), cmp.Report()
    gpu.set_mode(ev.MODE_AUTO)
    gpu.reset(_dev(frames[0]))
    ora.reset(frames[0])
    seen = []
    for f in frames[1:]:
        seen.append(gpu.current_mode())
        gpu.step_frame(_dev(f))
        ora.step_frame(f)
        cmp.compare_outputs_value_only(gpu, ora, rep)
        for i, nd in enumerate(net.nodes):
            if nd.op == wl.OP_CONV2D:
                z, zr = gpu.state(i, ev.STATE_Z).astype(np.float64), ora.z(i)
                assert np.abs(z - zr).max() <= TOL * np.abs(zr).max(), f"node {i}"
    assert seen[:8] == [ev.MODE_INCREMENTAL] * 4 + [ev.MODE_DENSE_RECOMPUTE] * 4, seen
    assert all(m in (ev.MODE_INCREMENTAL, ev.MODE_DENSE_RECOMPUTE) for m in seen[8:])
    with pytest.raises(ev.EvConvError):
        gpu.set_mode(3)
    gpu.destroy()
    sp = wl.net_unet_depth(1003, h=32, w=48, width=8, sparsify=True)
    sp.sparsify_tp = 0.1
    g = ev.EvConvNet(sp)
    g.set_mode(ev.MODE_AUTO)
    g.reset(_dev(frames[0][:, :32, :48].copy()))
    for f in frames[1:10]:
        assert g.current_mode() == ev.MODE_INCREMENTAL
        g.step_frame(_dev(f[:, :32, :48].copy()))
    g.destroy()


def test_fixed_step_of_a_first_node_sparsification_layer_survives_create_on_a_side_stream():
    """evconv_create clears the workspace on the net's stream and uploads a fixed rounding step
    with a blocking copy; on a non-blocking stream the two must still be ordered."""
    import torch
    net = _sp_only_net(8, 64, 96, k=0.375)
    side = torch.cuda.Stream()
    for _ in range(3):
        with torch.cuda.stream(side):
            g = ev.EvConvNet(net, stream=side)
        assert float(g.state(0, ev.STATE_STEP)[0]) == 0.375
        g.destroy()


def test_elementwise_kernels_bit_exact_against_fp32_oracle():
    """Activation increment (Eq.12-14) and addition (Eq.11) are single-rounded fp32 operations, so
    the GPU must match the oracle's binary32 mode bit for bit (tol = 0, exact sets)."""
    _say("bit-exact elementwise: ACT(relu) and ADD+relu nets against the binary32 oracle")
    nodes = [wl.Node(wl.OP_ACT, wl.ACT_RELU, -1, -2, 4, 4),
             wl.Node(wl.OP_ADD, wl.ACT_RELU, 0, -1, 4, 4),
             wl.Node(wl.OP_ADD, wl.ACT_NONE, 1, 0, 4, 4, is_output=1)]
    net = wl.Net("elementwise", 4, 19, 23, nodes, np.zeros(0, np.float32))
    rng = np.random.default_rng(5)
    x0 = rng.standard_normal((4, 19, 23)).astype(np.float32)
    frames, x = [], x0
    for t in range(8):
        m = rng.random((19, 23)) < 0.2
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m[None]).astype(np.float32)
        frames.append(x)
    run_stream(net, x0, frames, "frame", tol=0.0, exact_sets=True, fp32_oracle=True, label="ew-bits")


def test_reset_equals_stepped_state_and_dense_recompute_mode():
    """Refresh equivalence on the GPU: after k steps, reset(x_t) and DENSE_RECOMPUTE give the same
    accumulated tensors and output as the incremental path (within fp32 tolerance)."""
    _say("refresh equivalence and dense-recompute mode")
    net = wl.net_unet_depth(21, h=32, w=48, width=8)
    frames = list(wl.stream_voxel(21, 32, 48, 12, 0.05, n_prim=4))
    a, b, c = ev.EvConvNet(net), ev.EvConvNet(net), ev.EvConvNet(net)
    a.reset(_dev(frames[0]))
    c.reset(_dev(frames[0]))
    c.set_mode(ev.MODE_DENSE_RECOMPUTE)
    for f in frames[1:]:
        a.step_frame(_dev(f))
        c.step_frame(_dev(f))
    b.reset(_dev(frames[-1]))
    import torch
    torch.cuda.synchronize()
    for i, nd in enumerate(net.nodes):
        if nd.op == wl.OP_CONV2D or nd.act != wl.ACT_NONE:
            za, zb, zc = (n.state(i, ev.STATE_Z) for n in (a, b, c))
            s = np.abs(zb).max()
            assert np.abs(za - zb).max() <= TOL * s, f"node {i}"
            np.testing.assert_array_equal(zb, zc)
    ya, yb, yc = (n.outputs()[0]["y"].cpu().numpy() for n in (a, b, c))
    assert np.abs(ya - yb).max() <= TOL
    np.testing.assert_array_equal(yb, yc)


@pytest.mark.parametrize("width,h,w", [(8, 40, 56), (32, 64, 96)])
def test_run_to_run_bit_reproducible(width, h, w):
    """width 8: the vector-ALU kernels; width 32: the matrix-core kernels (partial sums of up to
    eight waves, fused epilogue adds, folded up-sampling, occupancy words OR-ed by several
    workgroups)."""
    _say(f"determinism: the same stream twice gives identical bits (width {width})")
    net = wl.net_unet_depth(31, h=h, w=w, width=width)
    frames = list(wl.stream_voxel(31, h, w, 10, 0.03, n_prim=4))
    res = []
    for _ in range(2):
        g = ev.EvConvNet(net)
        g.reset(_dev(frames[0]))
        for f in frames[1:]:
            g.step_frame(_dev(f))
        import torch
        torch.cuda.synchronize()
        stored = [i for i in range(len(net.nodes)) if not g.kernel_name(i).endswith(("_gather", "_weights"))]
        res.append([g.state(i, ev.STATE_DY).copy() for i in stored] +
                   [g.outputs()[0]["y"].cpu().numpy()] + [g.site_list(i) for i in stored])
        g.destroy()
    for u, v in zip(*res):
        np.testing.assert_array_equal(u, v)


def test_step_before_reset_is_an_error():
    net = wl.net_single_conv(3, c=4, h=8, w=8)
    g = ev.EvConvNet(net)
    with pytest.raises(ev.EvConvError) as e:
        g.step(_dev(np.zeros((4, 8, 8), np.float32)))
    assert e.value.status == ev.ERR_STATE
    # a node index out of range is refused by the C ABI itself (called directly, past the binding)
    import ctypes
    buf = np.zeros(64, np.float32)
    for node in (1, 7, -2):
        st = ev.lib().evconv_get_state_stream(g._h, 0, node, ev.STATE_Z, buf.ctypes.data_as(ctypes.c_void_p), buf.nbytes)
        assert st != 0, node
    g.destroy()


@pytest.mark.timeout(600)
def test_workload4_resnet18_full_size():
    """Full-size ResNet-18-style classifier on 2x224x224 event histograms, density ramp 0.5-5 %:
    max-pool, strided convs with 1x1 projection shortcuts, global mean, linear head."""
    _say("workload 4: ResNet-18 2x224x224, 100 frames, density 0.5 -> 5 %")
    net = wl.net_resnet18()
    gen = wl.stream_histogram(1004, 224, 224, steps=100)
    x0 = next(gen)
    run_stream(net, x0, gen, "frame", check_nodes_at={1, 2, 50, 100}, label="w4", max_flips=64)


@pytest.mark.timeout(900)
def test_workload5_flow_net_full_size_density_sweep():
    """Full-size optical-flow encoder-decoder on 4x256x256 (concat skips, flow head per scale):
    100 consecutive steps, ten at each of ten log-spaced increment densities between 0.1 % and
    20 % (the GPU alone runs the 1000-step sweep in bench.py --sweep; the oracle takes 0.6 s per
    step of this net).  Outputs and the input stage at every step, every node at one step per
    density."""
    _say("workload 5: flow encoder-decoder 4x256x256, 10 densities 0.1 .. 20 %, 10 steps each")
    net = wl.net_flow()
    dens = [float(d) for d in np.geomspace(0.001, 0.2, 10)]
    gen = wl.stream_count_timestamp(1005, 256, 256, densities=dens, steps_per=10)
    x0 = next(gen)
    run_stream(net, x0, gen, "frame", check_nodes_at=set(range(5, 101, 10)) | {1, 100}, label="w5", max_flips=64)


@pytest.mark.timeout(600)
def test_delayed_flow_net_full_size():
    _say("delayed-integration flow net 4x256x256, densities 0.1 / 1 / 5 %, 4 steps each")
    net = wl.net_flow_delayed()
    gen = wl.stream_count_timestamp(1006, 256, 256, densities=[0.001, 0.01, 0.05], steps_per=4)
    x0 = next(gen)
    run_stream(net, x0, gen, "frame", check_nodes_at={1, 6, 11}, label="delayed-full", max_flips=64)


@pytest.mark.timeout(900)
def test_workload3_unet_bf16_full_size_100_steps():
    """Workload 3, bf16-weight variant, full size, 100 consecutive frames: 2e-2 relative."""
    _say("workload 3 (bf16 weights): UNet depth net 5x256x352, 100 frames at 2 %")
    net = wl.net_unet_depth(bf16=True)
    gen = wl.stream_voxel(1003, 256, 352, 100, 0.02)
    x0 = next(gen)
    run_stream(net, x0, gen, "frame", check_nodes_at={1, 50, 100}, label="w3-bf16", tol=2e-2, frobenius=True,
               max_flips=800)   # (measured: 378, all at the 1-channel sigmoid head and behind ReLU zero crossings)


@pytest.mark.timeout(900)
def test_workload3_unet_full_size_100_steps():
    """Full-size UNet depth net (5x256x352), 100 consecutive frames at 2 % changed pixels, in the
    configuration bench.py times.  Outputs and the input stage are compared at every step, every
    node at steps 1, 2, 50 and 100."""
    _say("workload 3: UNet depth net 5x256x352, 100 frames at 2 %")
    net = wl.net_unet_depth()
    gen = wl.stream_voxel(1003, 256, 352, 100, 0.02)
    x0 = next(gen)
    # The 1-channel sigmoid head decides "increment == 0" on differences of saturating values of
    # the order 1e-8; fp32 drift against the fp64 oracle flips that decision at a few sites per
    # thousand.  Every other node must agree on every site.
    rep = run_stream(net, x0, gen, "frame", check_nodes_at={1, 2, 50, 100}, label="w3",
                     max_flips=600)   # (measured: 170 over the 100 steps)
    assert set(rep.flips_by_node) <= {"node 20 active"}, rep.flips_by_node


# --------------------------------------------------------------------------- sparsification layer

def _sp_only_net(c, h, w, k=None, tp=0.0):
    w_arr = np.zeros(0, np.float32)
    k_off = -1
    if k is not None:
        w_arr, k_off = np.asarray([k], np.float32), 0
    nodes = [wl.Node(wl.OP_SPARSIFY, wl.ACT_NONE, -1, -2, c, c, 1, 1, 0, k_off, -1, 1)]
    return wl.Net("sp_only", c, h, w, nodes, w_arr, sparsify_tp=tp)


@pytest.mark.parametrize("k,tp", [(0.3, 0.0), (None, 0.25)])
def test_sparsification_layer_bit_exact_against_fp32_oracle(k, tp):
    """Eq.3-8 are single-rounded fp32 operations on an input both sides see bit-identically, so
    the residual, the emitted increments and the lists must match the binary32 oracle exactly;
    with k = t_p * RMS both sides must also arrive at the identical 8-bit step."""
    _say(f"sparsification layer alone, k={k} tp={tp}: bit-exact vs the binary32 oracle")
    net = _sp_only_net(8, 21, 27, k=k, tp=tp)
    rng = np.random.default_rng(3)
    x0 = rng.standard_normal((8, 21, 27)).astype(np.float32)
    frames, x = [], x0
    for t in range(12):
        m = rng.random((21, 27)) < 0.3
        x = (x + 0.2 * rng.standard_normal(x.shape).astype(np.float32) * m[None]).astype(np.float32)
        frames.append(x)
    g, o = ev.EvConvNet(net), Oracle(net, fp32_state=True)
    g.reset(_dev(x0))
    o.reset(x0)
    assert float(g.state(0, ev.STATE_STEP)[0]) == o.step_size(0) > 0
    g.destroy()
    run_stream(net, x0, frames, "frame", tol=0.0, exact_sets=True, fp32_oracle=True, label="sp-bits")


def test_sparsified_conv_net_exact_arithmetic():
    """Two convolutions with a sparsification layer between them, on values chosen so that every
    sum is exact in binary32 (dyadic weights and inputs, k = 0.5): the rounding decisions cannot
    differ, so the GPU must equal the fp64 oracle on every tensor and every list."""
    _say("conv -> sparsify -> conv with exact arithmetic")
    b = wl._NetBuilder("sp_exact", 4, 19, 23, 5, sparsify=True, sparsify_k=0.5)
    x = b.conv(-1, 32, 3, 1)
    b.conv(x, 32, 3, 1, out=1)
    net = b.finish()
    rng = np.random.default_rng(6)
    wts = net.weights.copy()
    for nd in net.nodes:
        if nd.op == wl.OP_CONV2D:
            n = nd.c_out * nd.c_in * 9
            wts[nd.w_off:nd.w_off + n] = rng.integers(-2, 3, n) / 4.0
    net.weights = wts
    x0 = (rng.integers(-8, 9, (4, 19, 23)) / 4.0).astype(np.float32)
    incs = [((rng.integers(-4, 5, x0.shape) / 4.0) * (rng.random((1, 19, 23)) < 0.1)).astype(np.float32)
            for _ in range(8)]
    g = ev.EvConvNet(net)
    assert g.kernel_name(2) == "conv_mfma_f32"
    g.destroy()
    rep = run_stream(net, x0, incs, "increment", tol=1e-7, exact_sets=True, label="sp-exact")
    assert rep.flips == 0


def test_sparsification_layers_folded_into_conv_epilogues_exact_arithmetic():
    """Sparsification layers whose input comes from a matrix-core conv, directly or through an ADD
    folded into that conv, run inside its epilogue.  Exact arithmetic again (dyadic weights and
    inputs, k = 0.5), so the GPU must equal the fp64 oracle on every tensor and every list, with
    the layers folded and with every fusion switched off."""
    _say("sparsification layers inside conv epilogues (behind the conv and behind a folded ADD), exact arithmetic")
    b = wl._NetBuilder("sp_fused_exact", 16, 21, 27, 5, sparsify=True, sparsify_k=0.5)
    c1 = b.conv(-1, 32, 3)
    c2 = b.conv(c1, 32, 3)                       # its layer reads c1: behind the conv stage
    c3 = b.conv(c2, 32, 3, act=wl.ACT_NONE)      # its layer reads c2
    a = b.simple(wl.OP_ADD, c1, c3, act=wl.ACT_RELU)   # folded into c3's epilogue
    b.conv(a, 32, 3, out=1)                      # its layer reads the ADD: behind the folded ADD stage
    net = b.finish()
    rng = np.random.default_rng(8)
    wts = net.weights.copy()
    for nd in net.nodes:
        if nd.op == wl.OP_CONV2D:
            n = nd.c_out * nd.c_in * 9
            wts[nd.w_off:nd.w_off + n] = rng.integers(-1, 2, n) / 8.0
    net.weights = wts
    x0 = (rng.integers(-8, 9, (16, 21, 27)) / 4.0).astype(np.float32)
    incs = [((rng.integers(-4, 5, x0.shape) / 4.0) * (rng.random((1, 21, 27)) < 0.1)).astype(np.float32)
            for _ in range(8)]
    incs.append(np.zeros_like(x0))
    sp_nodes = [i for i, nd in enumerate(net.nodes) if nd.op == wl.OP_SPARSIFY]
    assert len(sp_nodes) == 3
    g = ev.EvConvNet(net)
    names = [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    assert all(names[i] == "fused_into_conv_epilogue" for i in sp_nodes), names
    assert names[a] == "fused_into_conv_epilogue"
    for flags in (0, ev.FLAG_NO_FUSION):
        gpu, ora, rep = ev.EvConvNet(net, flags=flags), Oracle(net), cmp.Report()
        gpu.reset(_dev(x0))
        ora.reset(x0)
        for d in incs:
            gpu.step(_dev(d))
            ora.step_increment(d)
            cmp.compare_outputs(gpu, ora, rep, 1e-7)
            for i in range(len(net.nodes)):
                cmp.compare_node(gpu, ora, i, rep, tol=1e-7, exact_sets=True)
        # a refresh clears the residuals and leaves the layers' buffers holding values
        gpu.set_refresh_period(1)
        gpu.step(_dev(incs[0]))
        for i in sp_nodes:
            assert not gpu.state(i, ev.STATE_Z).any(), f"residual of node {i} after a refresh"
        assert rep.flips == 0
        gpu.destroy()


def test_sparsified_unet_properties_and_speed_of_convergence():
    """Lossy path on a reduced UNet with t_p = 0.3: what must hold whatever the rounding
    decisions were - residual bounded by k/2, emitted increments multiples of k, fewer active
    sites than the lossless run, output a bounded approximation of the regular forward pass,
    and a refresh returns to the regular forward pass."""
    _say("sparsified UNet (t_p = 0.3): residual bound, quantised increments, sparsity, refresh")
    base = wl.net_unet_depth(1003, h=64, w=96)
    sp = wl.net_unet_depth(1003, h=64, w=96, sparsify=True)
    sp.sparsify_tp = 0.3
    # small-valued increments (what the layer is for): a dense frame plus faint changes at 2 % of
    # the pixels per step
    rng = np.random.default_rng(11)
    frames = [rng.standard_normal((5, 64, 96)).astype(np.float32)]
    for _ in range(12):
        m = rng.random((1, 64, 96)) < 0.02
        frames.append((frames[-1] + 0.05 * rng.standard_normal(frames[0].shape).astype(np.float32) * m).astype(np.float32))
    ga, gs = ev.EvConvNet(base), ev.EvConvNet(sp)
    ga.reset(_dev(frames[0]))
    gs.reset(_dev(frames[0]))
    act_a = act_s = 0
    for f in frames[1:]:
        ga.step_frame(_dev(f))
        gs.step_frame(_dev(f))
        act_a += sum(ga.stats(i).n_active for i, nd in enumerate(base.nodes) if nd.op == wl.OP_CONV2D)
        act_s += sum(gs.stats(i).n_active for i, nd in enumerate(sp.nodes) if nd.op == wl.OP_CONV2D)
        for i, nd in enumerate(sp.nodes):
            if nd.op != wl.OP_SPARSIFY:
                continue
            k = float(gs.state(i, ev.STATE_STEP)[0])
            assert k > 0
            d = gs.state(i, ev.STATE_Z)
            assert d.min() >= -0.5 * k * (1 + 1e-5) and d.max() <= 0.5 * k * (1 + 1e-5), f"node {i}"
            m = cmp.words_to_mask(gs.state(i, ev.STATE_OCC), *gs.shape(i)[1:]).astype(bool)
            y = gs.state(i, ev.STATE_DY)[m]
            if y.size:
                assert np.abs(y / k - np.rint(y / k)).max() < 1e-3, f"node {i}: increments not multiples of k"
    assert act_s < 0.8 * act_a, (act_s, act_a)
    import torch
    torch.cuda.synchronize()
    ya = ga.outputs()[0]["y"].cpu().numpy()
    ys = gs.outputs()[0]["y"].cpu().numpy()
    assert 0 < np.abs(ya - ys).max() < 0.2          # sigmoid output in (0, 1)
    gs.reset(_dev(frames[-1]))
    ga.reset(_dev(frames[-1]))
    torch.cuda.synchronize()
    # a refresh is a regular forward pass, the layer is the identity there: the same function.  (Not
    # the same roundings: the plain net's up-sampling convs run with folded weights, this net's
    # convs read a sparsification layer and do not.)
    np.testing.assert_allclose(ga.outputs()[0]["y"].cpu().numpy(), gs.outputs()[0]["y"].cpu().numpy(), rtol=0, atol=1e-5)
    ga.destroy()
    gs.destroy()


# --------------------------------------------------------------------------- elementwise multiply

def test_multiply_increment_bit_exact_against_fp32_oracle():
    """Eq.15-17 as single-rounded binary32 operations: two 1x1 selector convolutions (exact: weights
    1, 0 and 0, 3) feed the product, so its inputs are bit-identical on both sides and the product
    increments, both accumulators and the OR-ed sets must match bit for bit."""
    _say("bit-exact elementwise multiply against the binary32 oracle")
    w = np.asarray([1.0, 0.0, 0.0, 3.0], np.float32)
    nodes = [wl.Node(wl.OP_CONV2D, wl.ACT_NONE, -1, -2, 2, 1, 1, 1, 0, 0, -1, 0),
             wl.Node(wl.OP_CONV2D, wl.ACT_NONE, -1, -2, 2, 1, 1, 1, 0, 2, -1, 0),
             wl.Node(wl.OP_MUL, wl.ACT_NONE, 0, 1, 1, 1, 1, 1, 0, -1, -1, 1),
             wl.Node(wl.OP_MUL, wl.ACT_NONE, 2, 2, 1, 1, 1, 1, 0, -1, -1, 1)]
    net = wl.Net("mul_bits", 2, 21, 27, nodes, w)
    rng = np.random.default_rng(8)
    x0 = rng.standard_normal((2, 21, 27)).astype(np.float32)
    frames, x = [], x0
    for t in range(10):
        m = rng.random((2, 21, 27)) < 0.2          # channels change independently
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    run_stream(net, x0, frames, "frame", tol=0.0, exact_sets=True, fp32_oracle=True, label="mul-bits")
    g, o = ev.EvConvNet(net), Oracle(net, fp32_state=True)
    g.reset(_dev(x0))
    o.reset(x0)
    for f in frames[:4]:
        g.step_frame(_dev(f))
        o.step_frame(f)
    for i in (2, 3):
        np.testing.assert_array_equal(g.state(i, ev.STATE_Z2), o.z2(i).astype(np.float32))
        np.testing.assert_array_equal(g.state(i, ev.STATE_Z), o.z(i).astype(np.float32))
    g.destroy()


@pytest.mark.parametrize("width,h,w", [(8, 37, 45), (32, 64, 96)])
def test_gated_network_sigmoid_tanh_products(width, h, w):
    """Gate structure of ConvLSTM / ConvGRU cells (sigmoid gate x tanh candidate, update gate x
    block input, a square) against the fp64 oracle; width 32 runs the matrix-core convolutions."""
    _say(f"gated network width {width} on 5x{h}x{w}: multiply increments, tanh, all nodes every step")
    net = wl.net_gated(1007, in_c=5, h=h, w=w, width=width)
    frames = list(wl.stream_voxel(1007, h, w, 12, 0.03, n_prim=6))
    run_stream(net, frames[0], frames[1:], "frame", label=f"gated-{width}", max_flips=16)


# --------------------------------------------------------------------------- refresh policy

@pytest.mark.parametrize("kind", ["frame", "increment"])
def test_refresh_period_runs_a_regular_forward_pass_every_nth_step(kind):
    """"Drift Errors": with period 3 the 3rd and 6th step are regular forward passes.  The net
    with the policy must be bit-identical to one that is reset by hand at those steps, and equal
    to the oracle's forward pass of the same frame."""
    _say(f"refresh period 3, {kind} input")
    net = wl.net_unet_depth(1003, h=32, w=48, width=8)
    frames = list(wl.stream_voxel(5, 32, 48, 7, 0.05, n_prim=4))
    a, b = ev.EvConvNet(net), ev.EvConvNet(net)
    a.set_refresh_period(3)
    a.reset(_dev(frames[0]))
    b.reset(_dev(frames[0]))
    ora = Oracle(net)
    out = ora.outputs[0]
    import torch
    torch.cuda.synchronize()
    y_before = a.outputs()[0]["y"].cpu().numpy()
    for t in range(1, 8):
        inp = frames[t] if kind == "frame" else (frames[t] - frames[t - 1]).astype(np.float32)
        (a.step_frame if kind == "frame" else a.step)(_dev(inp))
        if t % 3 == 0:
            cur = b.state(-1, ev.STATE_X_PREV) + inp if kind == "increment" else frames[t]
            b.reset(_dev(cur.astype(np.float32)))
        else:
            (b.step_frame if kind == "frame" else b.step)(_dev(inp))
        import torch
        torch.cuda.synchronize()
        ya, yb = a.outputs()[0]["y"].cpu().numpy(), b.outputs()[0]["y"].cpu().numpy()
        np.testing.assert_array_equal(ya, yb, err_msg=f"step {t}")
        for i in (3, 12, 18):
            np.testing.assert_array_equal(a.state(i, ev.STATE_Z), b.state(i, ev.STATE_Z), err_msg=f"step {t} node {i}")
        dya = a.outputs()[0]["dy"].cpu().numpy()
        if t % 3 == 0:
            # internal sets are empty after a refresh; the output increment is y(n) - y(n-1) at every
            # site (one fp32 subtraction), listed in full, so that Eq.2 holds across the refresh
            assert a.site_list(-1).size == 0 and a.site_list(3).size == 0
            np.testing.assert_array_equal(dya, ya - y_before, err_msg=f"step {t}: dy of a refresh step")
            np.testing.assert_array_equal(a.site_list(out), np.arange(ya[0].size, dtype=np.int32))
            ora.reset(a.state(-1, ev.STATE_X_PREV))
            ref = np.transpose(ora.y(out), (2, 0, 1))
            assert np.abs(ya - ref).max() <= TOL * np.abs(ref).max()
        else:
            np.testing.assert_array_equal(ya, y_before + dya, err_msg=f"step {t}: Eq.2")
        y_before = ya
    with pytest.raises(ev.EvConvError):
        a.set_refresh_period(-1)
    a.destroy()
    b.destroy()


# --------------------------------------------------------------------------- fp32 through bf16 high/low parts

def test_split_bf16_conv_shapes_meet_the_fp32_bar():
    """EVCONV_F32_SPLIT: fp32 weights and increments contracted as three bf16 products.  Every
    kernel variant on ragged sizes, against the fp64 oracle with the unrounded fp32 weights, at
    the fp32 tolerance."""
    _say("split-bf16 matrix-core conv variants at the fp32 tolerance")
    worst = 0.0
    for k, s, ci, co in [(3, 1, 32, 32), (3, 2, 16, 64), (5, 1, 64, 32), (5, 2, 48, 96), (7, 2, 16, 32), (1, 1, 32, 64),
                         (3, 1, 128, 64), (3, 1, 68, 32), (5, 2, 20, 32),
                         (3, 1, 69, 32), (5, 2, 21, 32), (3, 1, 18, 64), (5, 1, 35, 64),   # c_in % 4 != 0
                         (3, 1, 32, 16), (3, 1, 37, 28)]:                                   # c_out % 32 != 0
        b = wl._NetBuilder(f"conv{k}s{s}", ci, 21, 27, 100 + k * 10 + s, bias=True)
        b.conv(-1, co, k, s, act=wl.ACT_RELU, out=1)
        net = wl.with_weight_dtype(b.finish(), wl.WD_F32_SPLIT)
        rng = np.random.default_rng(k + s)
        x0 = rng.standard_normal((ci, 21, 27)).astype(np.float32)
        incs = []
        for t in range(4):
            m = rng.random((21, 27)) < (0.03 if t < 3 else 1.0)
            incs.append(rng.standard_normal(x0.shape).astype(np.float32) * m[None])
        g = ev.EvConvNet(net)
        assert g.kernel_name(0) == "conv_mfma_f32_split_bf16x3"
        g.destroy()
        rep = run_stream(net, x0, incs, "increment", label=f"split k{k}s{s}", max_flips=2)
        worst = max(worst, rep.max_rel_z, rep.max_rel_y)
    _say(f"split-bf16: worst relative error {worst:.2e} (bar {TOL:.0e})")


def test_split_bf16_unet_reduced():
    _say("UNet depth net, full width on 5x64x96, split-bf16 contraction, fp32 tolerance")
    net = wl.with_weight_dtype(wl.net_unet_depth(1003, h=64, w=96), wl.WD_F32_SPLIT)
    g = ev.EvConvNet(net)
    names = [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    assert names.count("conv_mfma_f32_split_bf16x3") == 10, names
    frames = list(wl.stream_voxel(1003, 64, 96, 20, 0.02, n_prim=6))
    rep = run_stream(net, frames[0], frames[1:], "frame", label="unet-split", max_flips=40)
    _say(f"split-bf16 UNet: max rel z err {rep.max_rel_z:.2e}, y err {rep.max_rel_y:.2e}")


@pytest.mark.timeout(900)
def test_workload3_unet_split_bf16_full_size_100_steps():
    """The bench configuration with the split-bf16 contraction: 100 frames, fp32 tolerance."""
    _say("workload 3, split-bf16 contraction: UNet depth net 5x256x352, 100 frames at 2 %")
    net = wl.with_weight_dtype(wl.net_unet_depth(), wl.WD_F32_SPLIT)
    gen = wl.stream_voxel(1003, 256, 352, 100, 0.02)
    x0 = next(gen)
    rep = run_stream(net, x0, gen, "frame", check_nodes_at={1, 2, 50, 100}, label="w3-split",
                     max_flips=600)   # (measured: 170 over the 100 steps)
    assert set(rep.flips_by_node) <= {"node 20 active"}, rep.flips_by_node
    _say(f"split-bf16 w3: max rel z err {rep.max_rel_z:.2e}, y err {rep.max_rel_y:.2e}")


# --------------------------------------------------------------------------- several streams per net

@pytest.mark.parametrize("which", ["unet", "mixed_ops", "sparsified", "recurrent"])
def test_streams_stepped_together_equal_single_stream_nets(which):
    """n_streams = 3: three independent event streams share the weights and are stepped by one
    call.  Every stream must equal a single-stream net fed the same frames, and stream 1 is also
    checked against the oracle."""
    _say(f"three streams in one net ({which}) against three single-stream nets")
    import torch
    if which == "unet":
        net = wl.net_unet_depth(1003, h=64, w=96)
        gens = [list(wl.stream_voxel(40 + s, 64, 96, 6, 0.01 * (s + 1), n_prim=5)) for s in range(3)]
    elif which == "recurrent":
        net = wl.net_convlstm(44, in_c=4, h=16, w=24, hidden=32, out_c=2)
        rng = np.random.default_rng(4)
        gens = []
        for s in range(3):
            x = rng.standard_normal((4, 16, 24)).astype(np.float32)
            fr = [x]
            for _ in range(6):
                x = (x + rng.standard_normal(x.shape).astype(np.float32) * (rng.random((1, 16, 24)) < 0.1)).astype(np.float32)
                fr.append(x)
            gens.append(fr)
    elif which == "mixed_ops":
        net = wl.net_random_small(7)
        rng = np.random.default_rng(3)
        gens = []
        for s in range(3):
            x = rng.standard_normal((3, 13, 11)).astype(np.float32)
            fr = [x]
            for _ in range(6):
                x = (x + rng.standard_normal(x.shape).astype(np.float32) * (rng.random((1, 13, 11)) < 0.2)).astype(np.float32)
                fr.append(x)
            gens.append(fr)
    else:
        net = wl.net_conv_stack(1002, h=40, w=56, sparsify=True)
        net.sparsify_tp = 0.2
        gens = [list(wl.stream_voxel(50 + s, 40, 56, 6, 0.03, n_prim=4)) for s in range(3)]
    multi = ev.EvConvNet(net, n_streams=3)
    singles = [ev.EvConvNet(net) for _ in range(3)]
    assert multi.n_streams == 3 and multi.stream_stride % 256 == 0
    ora = Oracle(net)
    keeps = [i for i in range(len(net.nodes)) if not multi.kernel_name(i).startswith("fused_into_")]
    for t in range(7):
        batch = _dev(np.stack([gens[s][t] for s in range(3)]))
        if t == 0:
            multi.reset(batch)
            ora.reset(gens[1][0])
        else:
            multi.step_frame(batch)
            ora.step_frame(gens[1][t])
        for s in range(3):
            (singles[s].reset if t == 0 else singles[s].step_frame)(_dev(gens[s][t]))
        torch.cuda.synchronize()
        # The matrix-core convolutions pick their launch shape (and with it the order of the partial
        # sums) from the number of workgroups, which grows with the number of streams: those nets
        # agree to rounding, the net without matrix-core layers bit for bit.  With sparsification
        # layers a last-bit difference can flip a rounding decision, which moves an element by one
        # rounding step k (and the sets behind it): those outputs are compared at a bar that a
        # stream mix-up would still miss by two orders of magnitude.
        exact = which == "mixed_ops"
        loose = which == "sparsified"
        for s in range(3):
            for a, b in zip(multi.outputs(s), singles[s].outputs()):
                if exact:
                    assert torch.equal(a["y"], b["y"]) and torch.equal(a["dy"], b["dy"]), f"step {t} stream {s}"
                    assert int(a["count"]) == int(b["count"])
                else:
                    scale = float(b["y"].abs().max())
                    assert float((a["y"] - b["y"]).abs().max()) <= (2e-2 if loose else 1e-5) * scale, f"step {t} stream {s}"
            for i in keeps[:: max(1, len(keeps) // 6)]:
                if exact:
                    np.testing.assert_array_equal(multi.state(i, ev.STATE_OCC, s), singles[s].state(i, ev.STATE_OCC))
                    np.testing.assert_array_equal(multi.site_list(i, s), singles[s].site_list(i))
                    np.testing.assert_array_equal(multi.state(i, ev.STATE_DY, s), singles[s].state(i, ev.STATE_DY))
                elif not loose:
                    np.testing.assert_array_equal(multi.state(i, ev.STATE_OCC_TOUCHED, s),
                                                  singles[s].state(i, ev.STATE_OCC_TOUCHED))
            np.testing.assert_array_equal(multi.state(-1, ev.STATE_X_PREV, s), gens[s][t])
        if which != "sparsified":
            out = ora.outputs[0]
            y1 = multi.outputs(1)[[o["node"] for o in multi.outputs(1)].index(out)]["y"].cpu().numpy()
            ref = np.transpose(ora.y(out), (2, 0, 1))
            assert np.abs(y1 - ref).max() <= TOL * max(np.abs(ref).max(), 1e-30)
    with pytest.raises(ev.EvConvError):
        multi.state(0, ev.STATE_DY, stream=3)
    multi.destroy()
    for g in singles:
        g.destroy()


# --------------------------------------------------------------------------- HIP graph replay

@pytest.mark.parametrize("which", ["unet", "recurrent"])
def test_step_captured_in_a_hip_graph_replays_bit_identically(which):
    """A step is a fixed sequence of kernel launches on the caller's stream (no allocation, no
    synchronisation, no memset), so the caller may capture it once and replay it.  Every replay,
    with eager work and synchronisations in between, must equal the eager net bit for bit."""
    _say("one step captured in a HIP graph, replayed 8 times against an eager net")
    import torch
    if which == "unet":
        net = wl.net_unet_depth(1003, h=64, w=96)
        frames = list(wl.stream_voxel(77, 64, 96, 9, 0.03, n_prim=5))
        watch = (0, 5, 12, 18)
    else:
        # a net with DELAY nodes is captured after an incremental step, as the header asks: the
        # kernels take "the previous pass was a regular one" as an argument
        net = wl.net_convlstm(45, in_c=5, h=32, w=48, hidden=32, out_c=1)
        frames = list(wl.stream_voxel(78, 32, 48, 9, 0.03, n_prim=5))
        watch = (0, 1, 7, 11)
    side = torch.cuda.Stream()
    eager = ev.EvConvNet(net)
    with torch.cuda.stream(side):
        captured = ev.EvConvNet(net, stream=side)
        static_in = torch.empty_like(_dev(frames[0]))
        static_in.copy_(_dev(frames[0]))
        captured.reset(static_in)
        static_in.copy_(_dev(frames[1]))
        captured.step_frame(static_in)          # one eager step first (warm-up outside the capture)
    side.synchronize()
    eager.reset(_dev(frames[0]))
    eager.step_frame(_dev(frames[1]))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        captured.step_frame(static_in)
    # capture does not execute: the state is still that of frame 1
    for t in range(2, 10):
        eager.step_frame(_dev(frames[t]))
        with torch.cuda.stream(side):
            static_in.copy_(_dev(frames[t]))
        side.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        a, b = eager.outputs()[0], captured.outputs()[0]
        assert torch.equal(a["y"], b["y"]) and torch.equal(a["dy"], b["dy"]), f"replay {t - 1}"
        assert int(a["count"]) == int(b["count"])
        for i in watch:
            np.testing.assert_array_equal(eager.state(i, ev.STATE_Z), captured.state(i, ev.STATE_Z))
    del graph
    eager.destroy()
    captured.destroy()


# --------------------------------------------------------------------------- random graphs

@pytest.mark.parametrize("seed", range(9))
def test_random_wide_graphs_all_contraction_modes(seed):
    """Random graphs over the matrix-core paths (ragged channel counts, fused epilogue adds, fused
    up-sampling gather, gates, heads), each in one of the three contraction modes, all nodes at
    every step against the oracle."""
    rng = np.random.default_rng(100 + seed)
    mode = ["f32", "split", "bf16"][seed % 3]
    net = wl.net_random_wide(seed)
    if mode == "bf16":
        net = wl.with_weight_dtype(dataclasses.replace(net, weights=wl.round_to_bf16(net.weights)), wl.WD_BF16)
    elif mode == "split":
        net = wl.with_weight_dtype(net, wl.WD_F32_SPLIT)
    _say(f"random wide graph {seed}: {len(net.nodes)} nodes, {mode}")
    g = ev.EvConvNet(net)
    names = [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    want = {"f32": "conv_mfma_f32", "split": "conv_mfma_f32_split_bf16x3", "bf16": "conv_mfma_bf16"}[mode]
    # (the up-sampling is folded into the gather of 32-channel-chunk convs only: some seeds keep it apart)
    assert names.count(want) >= 4 and "fused_into_conv_epilogue" in names, names
    x = rng.standard_normal((net.in_c, net.in_h, net.in_w)).astype(np.float32)
    frames = [x]
    for t in range(6):
        m = rng.random((1, net.in_h, net.in_w)) < (0.04 if t != 3 else 0.6)
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    if mode == "bf16":
        run_stream(net, frames[0], frames[1:], "frame", tol=2e-2, label=f"wide{seed}", max_flips=40, frobenius=True)
    else:
        run_stream(net, frames[0], frames[1:], "frame", label=f"wide{seed}", max_flips=40)


@pytest.mark.parametrize("seed,h,w", [(0, 84, 108), (6, 84, 108), (7, 72, 136), (19, 100, 92), (2, 84, 108)])
def test_upsampling_folded_into_conv_weights(seed, h, w):
    """A 5 x 5 conv reading a x2 up-sampling at sizes where the stored tensor has tiles away from
    the border: those run per output phase with folded 4 x 4 weights, the border tiles through the
    interpolating gather (ragged tile rows and columns, one or two output-channel blocks, 32-96
    input channels, fp32 and split products; bf16-declared weights must not fold).  All nodes at
    every step against the oracle; then the same frames with folding switched off: identical
    touched sets, values apart by rounding only."""
    rng = np.random.default_rng(300 + seed)
    mode = ["f32", "split", "bf16"][seed % 3]
    net = wl.net_random_wide(seed, h, w)
    if mode == "bf16":
        net = wl.with_weight_dtype(dataclasses.replace(net, weights=wl.round_to_bf16(net.weights)), wl.WD_BF16)
    elif mode == "split":
        net = wl.with_weight_dtype(net, wl.WD_F32_SPLIT)
    _say(f"folded up-sampling, random wide graph {seed} at {h}x{w}: {len(net.nodes)} nodes, {mode}")
    up = [i for i, n in enumerate(net.nodes) if n.op == wl.OP_UPSAMPLE2X][0]
    g = ev.EvConvNet(net)
    assert g.kernel_name(up) == ("fused_into_conv_gather" if mode == "bf16" else "fused_into_conv_weights")
    g.destroy()
    x = rng.standard_normal((net.in_c, h, w)).astype(np.float32)
    frames = [x]
    for t in range(5):
        m = rng.random((1, h, w)) < (0.03 if t != 2 else 0.5)
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    if mode == "bf16":
        run_stream(net, frames[0], frames[1:], "frame", tol=2e-2, label=f"fold{seed}", max_flips=40, frobenius=True)
        return
    run_stream(net, frames[0], frames[1:], "frame", label=f"fold{seed}", max_flips=40)
    folded, recomputed = ev.EvConvNet(net), ev.EvConvNet(net)
    plain = ev.EvConvNet(net, flags=ev.FLAG_NO_FOLD)
    assert plain.kernel_name(up) == "fused_into_conv_gather"
    conv = [i for i, n in enumerate(net.nodes) if n.op == wl.OP_CONV2D and n.in0 == up][0]
    for t, f in enumerate(frames):
        for net_ in (folded, plain, recomputed):
            (net_.reset if t == 0 else net_.step_frame)(_dev(f))
        if t == 0:
            recomputed.set_mode(ev.MODE_DENSE_RECOMPUTE)
        np.testing.assert_array_equal(folded.state(conv, ev.STATE_OCC_TOUCHED), plain.state(conv, ev.STATE_OCC_TOUCHED))
        za, zb = folded.state(conv, ev.STATE_Z), plain.state(conv, ev.STATE_Z)
        assert np.abs(za - zb).max() <= 2e-5 * np.abs(zb).max(), (t, np.abs(za - zb).max(), np.abs(zb).max())
    # a regular forward pass through the folded kernels, as a reset and as a dense-recompute step: same bits
    folded.reset(_dev(frames[-1]))
    np.testing.assert_array_equal(folded.state(conv, ev.STATE_Z), recomputed.state(conv, ev.STATE_Z))
    for net_ in (folded, plain, recomputed):
        net_.destroy()


def test_folded_upsampling_ragged_channels_and_output_node():
    """Folded up-sampling conv with an input channel count that is not a multiple of the chunk
    (36: the last chunk is zero-padded in the patch and in the folded weight sets), three blocks
    of output channels, a bias, and the conv being a network output itself."""
    _say("folded up-sampling conv, 36 -> 96 channels on 40x56 -> 80x112, network output")
    b = wl._NetBuilder("fold_ragged", 4, 40, 56, 4242, bias=True)
    x = b.conv(-1, 36, 3)
    u = b.simple(wl.OP_UPSAMPLE2X, x)
    b.conv(u, 96, 5, act=wl.ACT_RELU, out=1)
    net = b.finish()
    g = ev.EvConvNet(net)
    assert [g.kernel_name(i) for i in range(3)] == ["conv_narrow_mfma_f32", "fused_into_conv_weights", "conv_mfma_f32"]
    g.destroy()
    rng = np.random.default_rng(4242)
    x = rng.standard_normal((4, 40, 56)).astype(np.float32)
    frames = [x]
    for t in range(5):
        m = rng.random((1, 40, 56)) < (0.02 if t != 3 else 0.7)
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    run_stream(net, frames[0], frames[1:], "frame", label="fold-ragged", max_flips=10)


@pytest.mark.parametrize("h,w,ci,co", [(18, 18, 32, 32), (17, 33, 32, 32), (26, 19, 96, 32), (48, 21, 32, 64)])
def test_folded_upsampling_smallest_interiors(h, w, ci, co):
    """Stored tensors that have just one tile away from the border (18 rows: sites 8-15 lie 2 or
    more from both edges), none (17 rows), or a single row / column of them."""
    _say(f"folded up-sampling conv, stored tensor {h}x{w}, {ci} -> {co} channels")
    b = wl._NetBuilder("fold_small", 4, h, w, 7 * h + w, bias=True)
    x = b.conv(-1, ci, 3)
    u = b.simple(wl.OP_UPSAMPLE2X, x)
    d = b.conv(u, co, 5)
    b.conv(d, 2, 1, 1, 0, wl.ACT_NONE, out=1)
    net = b.finish()
    g = ev.EvConvNet(net)
    assert g.kernel_name(u) == ("fused_into_conv_weights" if min(h, w) >= 18 else "fused_into_conv_gather")
    g.destroy()
    rng = np.random.default_rng(h * 100 + w)
    x = rng.standard_normal((4, h, w)).astype(np.float32)
    frames = [x]
    for t in range(4):
        m = rng.random((1, h, w)) < (0.03 if t != 2 else 0.6)
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    run_stream(net, frames[0], frames[1:], "frame", label=f"fold{h}x{w}", max_flips=10)


# --------------------------------------------------------------------------- recurrent state

def _running_sum_net(c, h, w):
    nodes = [
        wl.Node(wl.OP_DELAY, wl.ACT_NONE, 1, -1, c, c, 1, 1, 0, -1, -1, 0),
        wl.Node(wl.OP_ADD, wl.ACT_NONE, -1, 0, c, c, 1, 1, 0, -1, -1, 1),
    ]
    return wl.Net("running_sum", c, h, w, nodes, np.zeros(0, np.float32))


def test_delay_running_sum_bit_exact_against_fp32_oracle():
    """s(n) = x(n) + s(n-1) through a DELAY node: every operation is a single fp32 add or
    subtraction, so the GPU must agree bit for bit with the oracle run in binary32, through
    incremental steps, refreshes (regular passes that keep the state) and the steps after them."""
    _say("recurrent running sum, bit-exact, with refreshes")
    c, h, w = 3, 9, 19
    net = _running_sum_net(c, h, w)
    rng = np.random.default_rng(11)
    x = rng.standard_normal((c, h, w)).astype(np.float32)
    gpu, ora = ev.EvConvNet(net), Oracle(net, fp32_state=True)
    gpu.set_refresh_period(4)
    gpu.reset(_dev(x))
    ora.reset(x)
    for t in range(1, 11):
        m = rng.random((1, h, w)) < 0.1
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        gpu.step_frame(_dev(x))
        (ora.refresh if t % 4 == 0 else ora.step_frame)(x)
        import torch
        torch.cuda.synchronize()
        for i in (0, 1):
            np.testing.assert_array_equal(gpu.state(i, ev.STATE_Z).view(np.uint32) if i == 0 else 0,
                                          ora.z(i).astype(np.float32).view(np.uint32) if i == 0 else 0,
                                          err_msg=f"step {t} node {i} accumulated value")
        y = gpu.outputs()[0]["y"].cpu().numpy()
        np.testing.assert_array_equal(y.view(np.uint32), np.transpose(ora.y(1), (2, 0, 1)).astype(np.float32).view(np.uint32),
                                      err_msg=f"step {t} output")
        if t % 4:
            for i in (0, 1):
                np.testing.assert_array_equal(cmp.words_to_mask(gpu.state(i, ev.STATE_OCC), h, w), ora.mask(i),
                                              err_msg=f"step {t} node {i} active set")
                on = ora.mask(i).astype(bool)
                np.testing.assert_array_equal(gpu.state(i, ev.STATE_DY)[on].view(np.uint32),
                                              ora.dy(i).astype(np.float32)[on].view(np.uint32), err_msg=f"step {t} node {i} increment")
    gpu.destroy()


@pytest.mark.parametrize("mode,in_c", [("f32", 4), ("split", 4), ("f32", 5), ("split", 5)])
def test_convlstm_cell_against_oracle(mode, in_c):
    """A ConvLSTM cell (gates on the matrix cores, products, tanh, two recurrent states) and a
    1 x 1 head: all nodes at every step.  With 5 input channels the gate convs read 37 channels
    (not a multiple of four)."""
    net = wl.net_convlstm(41, in_c=in_c, h=24, w=40, hidden=32, out_c=2)
    if mode == "split":
        net = wl.with_weight_dtype(net, wl.WD_F32_SPLIT)
    _say(f"ConvLSTM cell, {mode}, {in_c}x24x40, hidden 32")
    g = ev.EvConvNet(net)
    names = [g.kernel_name(i) for i in range(len(net.nodes))]
    g.destroy()
    assert names[0] == names[1] == "delay", names
    assert names.count("conv_mfma_f32" if mode == "f32" else "conv_mfma_f32_split_bf16x3") == 4, names
    rng = np.random.default_rng(12)
    x = rng.standard_normal((in_c, 24, 40)).astype(np.float32)
    frames = [x]
    for t in range(8):
        m = rng.random((1, 24, 40)) < 0.05
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    run_stream(net, frames[0], frames[1:], "frame", label=f"convlstm-{mode}", max_flips=40)


def test_convlstm_refresh_and_dense_recompute_keep_the_state():
    """Regular forward passes in mid-stream (refresh period; dense-recompute mode) keep the
    recurrent state: outputs follow the oracle's refresh()."""
    _say("ConvLSTM cell with refresh period 3, and in dense-recompute mode")
    net = wl.net_convlstm(42, in_c=4, h=16, w=24, hidden=32, out_c=2)
    rng = np.random.default_rng(13)
    x = rng.standard_normal((4, 16, 24)).astype(np.float32)
    frames = [x]
    for t in range(7):
        m = rng.random((1, 16, 24)) < 0.1
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    import torch
    for which in ("refresh", "dense"):
        gpu, ora = ev.EvConvNet(net), Oracle(net)
        if which == "refresh":
            gpu.set_refresh_period(3)
        else:
            gpu.set_mode(ev.MODE_DENSE_RECOMPUTE)
        gpu.reset(_dev(frames[0]))
        ora.reset(frames[0])
        out = ora.outputs[0]
        for t in range(1, 8):
            gpu.step_frame(_dev(frames[t]))
            regular = which == "dense" or t % 3 == 0
            (ora.refresh if regular else ora.step_frame)(frames[t])
            torch.cuda.synchronize()
            y = gpu.outputs()[0]["y"].cpu().numpy()
            ref = np.transpose(ora.y(out), (2, 0, 1))
            assert np.abs(y - ref).max() <= TOL * np.abs(ref).max(), f"{which} step {t}: {np.abs(y - ref).max():.3e}"
            for d in (0, 1):
                z, zr = gpu.state(d, ev.STATE_Z).astype(np.float64), ora.z(d)
                assert np.abs(z - zr).max() <= TOL * max(np.abs(zr).max(), 1e-30), f"{which} step {t} state {d}"
        gpu.destroy()


def test_convgru_cell_against_oracle():
    """A ConvGRU cell: two sigmoid gates, r * h', a tanh candidate on [x, r * h'], 1 - z, two
    products and an add, one recurrent state; all nodes at every step."""
    net = wl.net_convgru(43, in_c=4, h=24, w=40, hidden=32, out_c=2)
    _say("ConvGRU cell, 4x24x40, hidden 32")
    rng = np.random.default_rng(14)
    x = rng.standard_normal((4, 24, 40)).astype(np.float32)
    frames = [x]
    for t in range(8):
        m = rng.random((1, 24, 40)) < 0.05
        x = (x + rng.standard_normal(x.shape).astype(np.float32) * m).astype(np.float32)
        frames.append(x)
    run_stream(net, frames[0], frames[1:], "frame", label="convgru", max_flips=40)


def test_large_frame_720p():
    """A 720p sensor (5 x 720 x 1280, 14400 tiles; widths 16..128): launch shapes and offsets far
    from the benchmark's size, two steps against the oracle."""
    _say("UNet depth net on a 5x720x1280 frame, width 16, reset + 2 steps")
    net = wl.net_unet_depth(1003, h=720, w=1280, width=16)
    frames = list(wl.stream_voxel(1010, 720, 1280, 2, 0.01, n_prim=12))
    rep = run_stream(net, frames[0], frames[1:], "frame", check_nodes_at={2}, label="720p", max_flips=400)
    _say(f"720p: max rel z err {rep.max_rel_z:.2e}, y err {rep.max_rel_y:.2e}, flips {rep.flips}")
