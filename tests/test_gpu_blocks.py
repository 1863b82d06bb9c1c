"""GPU parity of the composite entry points (inception_fwd, net_fwd) against the oracle on the
seeded workloads: original and slim forms, every execution mode of the module."""
import numpy as np
import pytest

import oracle
import workloads
from paper_1708_04728_amd import binding as B, graph as G
from util import TOL_BF16, TOL_F32, host, close, oracle_in_chunks, rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

MODES = [0, B.DR_FUSE_RELU, B.DR_FUSE_CONCAT, B.DR_FUSE_RELU | B.DR_FUSE_CONCAT,
         B.DR_FUSE_RELU | B.DR_FUSE_CONCAT | B.DR_FUSE_STACK]


def run_inception(layer, params, x, mode, dtype="f32", pack=False):
    xg = G.to_device(x, dtype)
    d = G.inception_desc(layer[1], x.shape[1], mode, pack)
    ws = torch.empty(max(B.inception_workspace_bytes(xg, d), 256), dtype=torch.uint8, device="cuda")
    c_out = G._out_channels([layer], x.shape[1])
    y = torch.full((x.shape[0], c_out, x.shape[2], x.shape[3]), float("nan"), dtype=G.torch_dtype(dtype), device="cuda")
    flat = G.flat_params(params, dtype, pack=pack)
    B.inception_fwd(xg, d, flat[0::2], flat[1::2], y, ws)
    torch.cuda.synchronize()
    return host(y)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("form", ["original", "slim"])
@pytest.mark.parametrize("pack", [False, True])
def test_inception_3a(form, mode, pack):
    layer = workloads.CONFIGS[2][form][0]
    params = workloads.make_params(2, form)
    x = workloads.make_input(2, 3)
    ref = oracle.forward([layer], params, x)
    got = run_inception(layer, params, x, mode, pack=pack)
    assert close(got, ref, TOL_F32)


def _run_stacked(layer, params, x, mode, pack):
    xg = G.to_device(x, "f32")
    c_out = G._out_channels([layer], x.shape[1])
    flat = G.stack_first_steps([layer], G.flat_params(params, "f32", pack=pack))
    d = G.inception_desc(layer[1], x.shape[1], mode, pack)
    ws = torch.empty(max(B.inception_workspace_bytes(xg, d), 256), dtype=torch.uint8, device="cuda")
    y = torch.full((x.shape[0], c_out, x.shape[2], x.shape[3]), float("nan"), dtype=torch.float32, device="cuda")
    B.inception_fwd(xg, d, flat[0::2], flat[1::2], y, ws)
    torch.cuda.synchronize()
    return host(y)


@pytest.mark.parametrize("form", ["original", "slim"])
@pytest.mark.parametrize("pack", [False, True])
def test_inception_3a_stacked_first_steps_fp32(form, pack):
    """DR_FUSE_STACK (Eq. (12)) on fp32 NCHW tensors: with the first-step 1x1 filters laid back to back they run as
    one convolution whose filter ranges go to their own tensors.  Against the oracle on three images; and at
    the full batch, where no contraction is cut over workgroups, bit for bit the result of one convolution per
    branch (same products, same order), with and without the fused concat."""
    layer = workloads.CONFIGS[2][form][0]
    params = workloads.make_params(2, form)
    base = B.DR_FUSE_RELU | B.DR_FUSE_CONCAT
    x3 = workloads.make_input(2, 3)
    ref = oracle.forward([layer], params, x3)
    for mode in (base | B.DR_FUSE_STACK, B.DR_FUSE_RELU | B.DR_FUSE_STACK):
        assert close(_run_stacked(layer, params, x3, mode, pack), ref, TOL_F32), (form, pack, mode)
    x = workloads.make_input(2)
    plain = run_inception(layer, params, x, base, pack=pack)
    for mode in (base | B.DR_FUSE_STACK, B.DR_FUSE_RELU | B.DR_FUSE_STACK):
        assert np.array_equal(_run_stacked(layer, params, x, mode, pack), plain), (form, pack, mode)


@pytest.mark.parametrize("form", ["original", "slim"])
def test_inception_branches_side_by_side_equal_branches_in_turn(form):
    """The branches of a module run on the library's own streams between a fork and a join on the caller's
    stream (DR_CONCURRENT_BRANCHES).  The result must be bit-identical to running them in turn and match the
    oracle, call after call on the same workspace, with work of the caller queued before and after it."""
    layer = workloads.CONFIGS[2][form][0]
    params = workloads.make_params(2, form)
    x = workloads.make_input(2, 8)
    ref = oracle.forward([layer], params, x)
    for mode in (0, B.DR_FUSE_RELU | B.DR_FUSE_CONCAT):
        serial = run_inception(layer, params, x, mode)
        assert close(serial, ref, TOL_F32)
        xg = G.to_device(x, "f32")
        d = G.inception_desc(layer[1], x.shape[1], mode | B.DR_CONCURRENT_BRANCHES, False)
        ws = torch.empty(max(B.inception_workspace_bytes(xg, d), 256), dtype=torch.uint8, device="cuda")
        flat = G.flat_params(params, "f32", pack=False)
        side = torch.cuda.Stream()
        for rep in range(6):
            stream = side if rep % 2 else torch.cuda.current_stream()
            with torch.cuda.stream(stream):
                xin = xg.clone()                       # the module must wait for work queued before it
                y = torch.full(serial.shape, float("nan"), dtype=torch.float32, device="cuda")
                B.inception_fwd(xin, d, flat[0::2], flat[1::2], y, ws, stream=stream)
                ycopy = y.clone()                      # and work queued after it must wait for every branch
                ws.zero_()
            stream.synchronize()
            assert np.array_equal(host(ycopy), serial), (form, mode, rep)


def test_inception_3a_paper_variant_and_ragged_spatial():
    layer = workloads.inception_3a_paper_variant()
    params = workloads.make_params(2, "slim", layers=[layer])
    x = workloads.make_input(2, 2)[:, :, :13, :11]
    ref = oracle.forward([layer], params, x)
    assert ref.shape == (2, 256, 13, 11)
    for mode in (0, B.DR_FUSE_RELU | B.DR_FUSE_CONCAT):
        assert close(run_inception(layer, params, x, mode), ref, TOL_F32)


def run_net(layers, params, x, dtype="f32", fuse_relu=False, inception_mode=0, folded=False, timing=False, pack=True):
    xg = G.to_device(x, dtype)
    net = B.Net(G.net_descs(layers, x.shape[1], inception_mode=inception_mode, fuse_relu=fuse_relu, folded=folded,
                            pack=pack))
    yd = net.output_desc(B.desc(xg))
    y = torch.full((yd.n, yd.c, yd.h, yd.w), float("nan"), dtype=torch.float32 if yd.dtype == B.DR_F32 else torch.bfloat16,
                   device="cuda")
    ws = torch.empty(max(net.workspace_bytes(B.desc(xg)), 256), dtype=torch.uint8, device="cuda")
    if timing:
        net.set_timing(True)
    net.fwd(xg, G.flat_params(params, dtype, pack=pack), y, ws)
    torch.cuda.synchronize()
    out = host(y)
    return (out, net.layer_times()) if timing else out


def test_two_forwards_recorded_as_one_graph():
    """dr_capture_begin / dr_capture_end: the original and the slim form of config 1's block, and a single layer
    call, recorded together; the replay gives the bits of the calls made one by one, three times over with
    other work in between."""
    x = workloads.make_input(1)
    xg = G.to_device(x, "f32")
    nets, outs, wss, flats = [], [], [], []
    for form in ("original", "slim"):
        layers = workloads.CONFIGS[1][form]
        net = B.Net(G.net_descs(layers, x.shape[1], fuse_relu=(form == "slim"), pack="f32"))
        y = G.empty_like_desc(net.output_desc(B.desc(xg)))
        ws = torch.empty(max(net.workspace_bytes(B.desc(xg)), 256), dtype=torch.uint8, device="cuda")
        flat = G.flat_params(workloads.make_params(1, form), "f32", pack=True)
        nets.append(net); outs.append(y); wss.append(ws); flats.append(flat)
    r = torch.empty_like(outs[0])
    for net, y, ws, flat in zip(nets, outs, wss, flats):
        net.fwd(xg, flat, y, ws)
    B.relu(outs[0], r)
    torch.cuda.synchronize()
    want = [outs[0].clone(), outs[1].clone(), r.clone()]
    assert close(host(outs[0]), oracle.forward(workloads.CONFIGS[1]["original"], workloads.make_params(1, "original"), x), TOL_F32)
    side = torch.cuda.Stream()
    with B.capture(side, [xg, r] + outs + wss + flats) as c:
        for net, y, ws, flat in zip(nets, outs, wss, flats):
            net.fwd(xg, flat, y, ws, side)
        B.relu(outs[0], r, side)
    for rep in range(3):
        for t in outs + [r]:
            t.zero_()
        torch.cuda.synchronize()
        c.graph.launch()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(outs + [r], want)), rep
    # a recording the caller gives up: the stream is usable again
    with pytest.raises(ValueError):
        with B.capture(side):
            nets[0].fwd(xg, flats[0], outs[0], wss[0], side)
            raise ValueError("changed my mind")
    with B.capture(side) as c2:
        nets[1].fwd(xg, flats[1], outs[1], wss[1], side)
    outs[1].zero_()
    c2.graph.launch()
    torch.cuda.synchronize()
    assert torch.equal(outs[1], want[1])


@pytest.mark.parametrize("form,fuse", [("original", False), ("original", True), ("slim", True)])
def test_config1_streamline_block(form, fuse):
    layers = workloads.CONFIGS[1][form]
    params = workloads.make_params(1, form)
    x = workloads.make_input(1)
    ref = oracle.forward(layers, params, x)
    assert ref.shape == (1, 192, 28, 28)
    assert close(run_net(layers, params, x, fuse_relu=fuse), ref, TOL_F32)


@pytest.mark.parametrize("form,fuse", [("original", False), ("slim", True)])
def test_config3_alexnet_front(form, fuse):
    layers = workloads.CONFIGS[3][form]
    params = workloads.make_params(3, form)
    x = workloads.make_input(3, 2)
    ref = oracle.forward(layers, params, x)
    assert ref.shape == ((2, 256, 13, 13) if form == "original" else (2, 256, 14, 14))
    got, times = run_net(layers, params, x, fuse_relu=fuse, timing=True)
    assert close(got, ref, TOL_F32)
    assert len(times) == len(G.net_descs(layers, 3, fuse_relu=fuse)) and all(t >= 0 for t in times)


@pytest.mark.parametrize("form,mode", [("original", 0), ("slim", B.DR_FUSE_RELU | B.DR_FUSE_CONCAT)])
def test_config2_through_net_fwd_full_batch(form, mode):
    """Config 2 at its full batch in the launch configuration the benchmark times, every image against the oracle."""
    x = workloads.make_input(2)
    assert x.shape == (32, 192, 28, 28)
    layers = workloads.CONFIGS[2][form]
    params = workloads.make_params(2, form)
    got = run_net(layers, params, x, inception_mode=mode)
    assert got.shape == (32, 256, 28, 28)
    ref = oracle_in_chunks(lambda c: oracle.forward(layers, params, c), x)
    assert close(got, ref, TOL_F32, "32 images")
    assert np.isfinite(got).all() and (got >= 0).all()


@pytest.mark.parametrize("form,fuse", [("original", False), ("slim", True)])
def test_config3_alexnet_front_full_batch(form, fuse):
    """Config 3 at its full batch of 128 as the benchmark launches it, every image against the oracle."""
    x = workloads.make_input(3)
    assert x.shape == (128, 3, 227, 227)
    layers = workloads.CONFIGS[3][form]
    params = workloads.make_params(3, form)
    got = run_net(layers, params, x, fuse_relu=fuse)
    assert got.shape[0] == 128 and np.isfinite(got).all() and (got >= 0).all()
    ref = oracle_in_chunks(lambda c: oracle.forward(layers, params, c), x)
    assert close(got, ref, TOL_F32, "128 images")


def test_module_that_fails_half_way_leaves_no_loose_ends():
    """Branches side by side (DR_CONCURRENT_BRANCHES): a module that fails after some branches have been started (a
    missing filter pointer in the last branch) reports the error with every started branch joined to the caller's
    stream again: the same stream then runs the module correctly, and a recording that met the error can be given
    up and started anew."""
    layer = workloads.CONFIGS[2]["original"][0]
    params = workloads.make_params(2, "original")
    x = workloads.make_input(2, 3)
    ref = oracle.forward([layer], params, x)
    mode = B.DR_FUSE_RELU | B.DR_FUSE_CONCAT | B.DR_CONCURRENT_BRANCHES
    xg = G.to_device(x, "f32")
    d = G.inception_desc(layer[1], x.shape[1], mode, False)
    ws = torch.empty(max(B.inception_workspace_bytes(xg, d), 256), dtype=torch.uint8, device="cuda")
    y = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    flat = G.flat_params(params, "f32", pack=False)
    weights, biases = list(flat[0::2]), list(flat[1::2])
    broken = weights[:-1] + [None]
    side = torch.cuda.Stream()
    with pytest.raises(B.DeepRebirthError) as e:
        B.inception_fwd(xg, d, broken, biases, y, ws, side)
    assert e.value.code == B.DR_ERR_NULL
    B.inception_fwd(xg, d, weights, biases, y, ws, side)
    side.synchronize()
    assert close(host(y), ref, TOL_F32)
    with pytest.raises(B.DeepRebirthError):
        with B.capture(side):
            B.inception_fwd(xg, d, broken, biases, y, ws, side)
    with B.capture(side, [xg, y, ws] + flat) as c:
        B.inception_fwd(xg, d, weights, biases, y, ws, side)
    for rep in range(2):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        c.graph.launch()
        torch.cuda.synchronize()
        assert close(host(y), ref, TOL_F32)
