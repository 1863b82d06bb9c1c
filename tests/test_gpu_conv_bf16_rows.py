"""GPU parity of the row-stack patch convolution kernel (bf16 NHWC, several taps at stride 1 on maps with 16, 32, 48 or 64
channels: a tile is a run of output rows of the whole batch's row stack -- image borders inside it allowed -- whose input
patch is loaded into LDS once) against the fp64 oracle.  The library picks the kernel by rule, restated in `takes` below;
every case satisfies it (and not the rule of the 64-channel patch kernel, which the library asks first), so what is
compared is this kernel.  The cases put image borders at every position inside a tile, several images in one tile,
tiles that end behind the last image, ragged filter blocks, filter rows whose last 64-deep slice is partly empty, and
rectangular filters."""
import numpy as np
import pytest

import oracle
import workloads
from paper_1708_04728_amd import binding as B
from test_gpu_conv_bf16_patch import rows_per_tile as patch_kernel_rows
from util import TOL_BF16, case_seed, close, empty_nhwc, gpu, gpu_nhwc, host_nhwc

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

CUS = 256


def takes(N, C, H, W, K, R, S, stride, pad):
    """The rule of the library's launcher, restated: stacked output rows per tile, 0 = the layer goes elsewhere."""
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(W, S, stride, pad)
    if C % 16 or C > 64 or K % 8 or stride != 1 or R * S < 2 or R > 7 or S > 7 or P < 2 or Q < 2 or Q > 256:
        return 0
    tm = 3 if (K + 95) // 96 * 96 <= (K + 63) // 64 * 64 else 2
    budget = 80 * 1024 - (2 * tm * 32 * 128 + 512 + 1024)
    th = min(256 // Q, N * P)
    while th >= 1:
        segs = min(N, (th + P - 2) // P + 1)
        patch = ((th + (R - 1) * segs) * (W + 2 * pad) * (C // 8 + 1) * 16 + 4095) // 4096 * 4096
        if patch <= budget:
            break
        th -= 1
    if th < 1 or th * Q * 4 < 256 * 3:
        return 0
    tiles, blocks = (N * P + th - 1) // th, (K + tm * 32 - 1) // (tm * 32)
    return th if tiles * blocks * 4 >= CUS else 0


# N, C, H, W, K, R, S, stride, pad
CASES = [
    (12, 16, 28, 28, 128, 5, 5, 1, 2),     # GoogLeNet 3a's slim 5x5: 9 rows per tile, image borders at every offset; 25 k-steps = 6 slices + 1 step
    (8, 32, 28, 28, 288, 5, 5, 1, 2),      # 3b's: three blocks of 96 filters
    (40, 16, 14, 14, 304, 5, 5, 1, 2),     # 4a's: 18 rows per tile, up to three images in a tile; 304 = 3 x 96 + 16 filters
    (84, 32, 14, 14, 72, 5, 5, 1, 2),      # ragged single block of 96
    (70, 32, 7, 7, 320, 5, 5, 1, 2),       # 7 x 7 maps: 36 rows per tile, six images in a tile, the last tile ends behind the batch
    (64, 48, 7, 7, 320, 3, 3, 1, 1),       # 48 channels (three k-steps per tap)
    (80, 64, 10, 10, 136, 3, 3, 1, 1),     # 64 channels on maps too small for the 64-channel patch kernel: 22 rows per tile, four images
    (70, 16, 9, 30, 40, 3, 5, 1, 1),       # 3x5 filter, padding 1: output 7 x 28
    (25, 32, 12, 17, 200, 2, 2, 1, 0),     # 2x2 filter without padding: output 11 x 16, 16 rows per tile
    (24, 16, 10, 100, 24, 3, 3, 1, 1),     # wide map: two rows of 100 per tile
    (20, 32, 31, 23, 96, 7, 1, 1, 3),      # 7x1 filter, padded by 3 both ways
]


def _check(case, relu, bias, images=None):
    N, C, H, W, K, R, S, stride, pad = case
    assert takes(*case) > 0, "the case must be one the row-stack kernel takes"
    assert patch_kernel_rows(C, H, W, K, R, S, stride, pad) == 0, "... and the 64-channel patch kernel does not"
    rng = np.random.default_rng(case_seed(case))
    x = workloads.round_to_bf16(rng.standard_normal((N, C, H, W)).astype(np.float32))
    w = workloads.round_to_bf16(rng.standard_normal((K, C, R, S)).astype(np.float32) * np.float32(np.sqrt(2.0 / (C * R * S))))
    b = (rng.standard_normal(K) * 0.1).astype(np.float32) if bias else None
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(W, S, stride, pad)
    # written at a channel offset of a wider tensor (a branch of a module writing its part of the concatenated output)
    ctot, coff = K + 24, 16
    y = B.NHWC(torch.full((N, P, Q, ctot), -5.0, dtype=torch.bfloat16, device="cuda"))
    B.conv2d_fwd(gpu_nhwc(x, "bf16"), B.conv_desc(K, C, R, S, stride, pad, relu, B.DR_KRSC), B.pack_filters(gpu(w, "bf16")),
                 gpu(b) if bias else None, y, y_c_offset=coff)
    torch.cuda.synchronize()
    got = host_nhwc(y)
    assert not np.isnan(got).any()
    assert (got[:, :coff] == -5.0).all() and (got[:, coff + K:] == -5.0).all()
    pick = list(range(N)) if images is None else images
    ref = oracle.conv2d(x[pick], w, b, stride, pad, relu)
    assert close(got[pick, coff:coff + K], ref, TOL_BF16)
    assert close(got[pick, coff:coff + K], oracle.round_bf16(ref), 2.0 ** -7, "within one bf16 unit of the oracle")


@pytest.mark.parametrize("case", CASES)
def test_conv_rows(case):
    _check(case, relu=case_seed(case) % 2 == 0, bias=case_seed(case) % 3 != 0)


def test_conv_rows_many_tiles_per_workgroup():
    # 128 images of 28 x 28 with one block of filters: 399 tiles on 256 x 2 workgroup slots; with three blocks 1197 on
    # 510, so workgroups walk two or three tiles and the next tile's patch is requested before the last one's store
    _check((128, 32, 28, 28, 96, 5, 5, 1, 2), relu=True, bias=True, images=[0, 1, 63, 126, 127])
    _check((128, 16, 28, 28, 264, 5, 5, 1, 2), relu=False, bias=True, images=[0, 77, 127])


def test_layers_the_rule_leaves_out_still_match():
    # few tiles (the streaming kernel's smaller tiles fill the device better) and 24 channels (not a multiple of 16)
    for case in [(1, 16, 28, 28, 32, 5, 5, 1, 2), (4, 24, 14, 14, 64, 5, 5, 1, 2)]:
        assert takes(*case) == 0
        N, C, H, W, K, R, S, stride, pad = case
        rng = np.random.default_rng(case_seed(case))
        x = workloads.round_to_bf16(rng.standard_normal((N, C, H, W)).astype(np.float32))
        w = workloads.round_to_bf16(rng.standard_normal((K, C, R, S)).astype(np.float32) * np.float32(np.sqrt(2.0 / (C * R * S))))
        y = empty_nhwc((N, K, oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(W, S, stride, pad)), "bf16")
        B.conv2d_fwd(gpu_nhwc(x, "bf16"), B.conv_desc(K, C, R, S, stride, pad, False, B.DR_KRSC), B.pack_filters(gpu(w, "bf16")), None, y)
        torch.cuda.synchronize()
        assert close(host_nhwc(y), oracle.conv2d(x, w, None, stride, pad, False), TOL_BF16)


def stem_takes(N, C, H, W, K, R, stride, pad):
    """The launcher's rule for the packed 4-channel input of a first layer, restated: stacked output rows per tile or 0."""
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(W, R, stride, pad)
    if C > 4 or R > 8 or stride % 2 or stride > 8 or K % 8 or P < 2 or Q < 2 or Q > 256:
        return 0
    hp = max(H + 2 * pad, (P - 1) * stride + 8)
    wp = (max(W + 2 * pad, (Q - 1) * stride + 8) + 7) // 8 * 8
    tm = 3 if (K + 95) // 96 * 96 <= (K + 63) // 64 * 64 else 2
    budget = 80 * 1024 - (2 * tm * 32 * 128 + 512 + 1024)
    th = min(256 // Q, N * P)
    while th >= 1:
        segs = 1 if P % th == 0 else min(N, (th + P - 2) // P + 1)
        rows = stride * (th - 1) + (segs - 1) * (hp - stride * P) + 8
        if (rows * (wp // 2) * 16 + 4095) // 4096 * 4096 <= budget:
            break
        th -= 1
    if th < 1 or th * Q * 4 < 256 * 3:
        return 0
    return th if ((N * P + th - 1) // th) * ((K + tm * 32 - 1) // (tm * 32)) * 4 >= CUS else 0


@pytest.mark.parametrize("case", [
    # N, C, H, W, K, R, stride, pad
    (16, 3, 64, 60, 64, 7, 2, 3),     # the GoogLeNet / ResNet first layer's shape class: 8 rows of 30 per tile, tiles inside images
    (40, 3, 81, 77, 24, 7, 4, 3),     # stride 4 (slim form), 21 x 20 outputs: 12 rows per tile across image borders
    (48, 1, 37, 39, 40, 3, 2, 0),     # one channel, 3x3, no padding
    (40, 4, 40, 40, 72, 5, 2, 2),     # four channels, 5x5
    (3, 3, 224, 224, 64, 7, 2, 3),    # the benchmark's size: two rows of 112 per tile
])
def test_first_layer_packed_input(case):
    """A first layer with up to 4 input channels inside dr_net_fwd: the row-stack kernel on the padded 4-channel copy."""
    from test_gpu_bf16_nets import run_net_bf16
    N, C, H, W, K, R, stride, pad = case
    assert stem_takes(*case) > 0
    rng = np.random.default_rng(case_seed(case))
    x = workloads.round_to_bf16(rng.standard_normal((N, C, H, W)).astype(np.float32))
    w = workloads.round_to_bf16(rng.standard_normal((K, C, R, R)).astype(np.float32) * np.float32(np.sqrt(2.0 / (C * R * R))))
    b = (rng.standard_normal(K) * 0.1).astype(np.float32)
    layers = [workloads.conv(K, R, stride, pad), workloads.relu()]
    params = [{"w": w, "b": b}]
    ref = oracle.forward(layers, params, x)
    got = run_net_bf16(layers, params, x, fuse_relu=True)
    assert got.shape == ref.shape
    assert close(got, ref, TOL_BF16)
    assert close(got, oracle.round_bf16(ref), 2.0 ** -7, "within one bf16 unit of the oracle")


def tail_takes(N, C, H, W, K, R, stride, pad, K2):
    """The launcher's rule for a first layer and the 1x1 convolution behind it as one kernel, restated."""
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(W, R, stride, pad)
    if C > 4 or R > 8 or stride % 2 or stride > 8 or K % 8 or K > 64 or K2 % 8 or K2 < 8 or K2 > 64 or P < 2 or Q < 2 or Q > 256:
        return 0
    hp = max(H + 2 * pad, (P - 1) * stride + 8)
    wp = (max(W + 2 * pad, (Q - 1) * stride + 8) + 7) // 8 * 8
    budget = 80 * 1024 - (2 * 64 * 128 + 512 + 1024) - (64 * 128 + 512)
    th = min(256 // Q, N * P)
    while th >= 1:
        segs = 1 if P % th == 0 else min(N, (th + P - 2) // P + 1)
        rows = stride * (th - 1) + (segs - 1) * (hp - stride * P) + 8
        if (rows * (wp // 2) * 16 + 4095) // 4096 * 4096 <= budget:
            break
        th -= 1
    if th < 1 or th * Q * 4 < 256 * 3:
        return 0
    return th if (N * P + th - 1) // th * 4 >= CUS else 0


@pytest.mark.parametrize("case", [
    # N, C, H, W, K, R, stride, pad, K2
    (16, 3, 224, 224, 64, 7, 4, 3, 64),     # the slim GoogLeNet's first two layers (Table 2: conv1 merged, then conv2's 1x1 reduction)
    (40, 3, 81, 77, 24, 7, 4, 3, 40),       # ragged filter counts on both sides, tiles across image borders
    (48, 1, 37, 39, 40, 3, 2, 0, 8),        # one input channel, the smallest 1x1
    (72, 4, 40, 40, 56, 5, 2, 2, 64),
])
@pytest.mark.parametrize("relus", [(True, True), (False, True), (True, False)])
def test_first_layer_and_1x1_in_one_kernel(case, relus):
    """dr_net_fwd runs a first layer on up to 4 channels and a 1x1 convolution right behind it as ONE kernel that never
    writes the tensor between them.  Against the oracle's composition, and against the library's own two layers run as two
    networks (the tensor between them stored in bf16): the fused kernel rounds it to bf16 as well."""
    from test_gpu_bf16_nets import run_net_bf16
    N, C, H, W, K, R, stride, pad, K2 = case
    assert tail_takes(*case) > 0
    rng = np.random.default_rng(case_seed(case))
    x = workloads.round_to_bf16(rng.standard_normal((N, C, H, W)).astype(np.float32))
    w1 = workloads.round_to_bf16(rng.standard_normal((K, C, R, R)).astype(np.float32) * np.float32(np.sqrt(2.0 / (C * R * R))))
    w2 = workloads.round_to_bf16(rng.standard_normal((K2, K, 1, 1)).astype(np.float32) * np.float32(np.sqrt(2.0 / K)))
    b1 = (rng.standard_normal(K) * 0.1).astype(np.float32)
    b2 = (rng.standard_normal(K2) * 0.1).astype(np.float32)
    first = [workloads.conv(K, R, stride, pad)] + ([workloads.relu()] if relus[0] else [])
    second = [workloads.conv(K2, 1, 1, 0)] + ([workloads.relu()] if relus[1] else [])
    params = [{"w": w1, "b": b1}, {"w": w2, "b": b2}]
    got = run_net_bf16(first + second, params, x, fuse_relu=True)
    # the oracle with the tensor between the layers rounded to bf16, as both forms of the library hold it
    mid = oracle.round_bf16(oracle.forward(first, params[:1], x)).astype(np.float32)
    ref = oracle.forward(second, params[1:], mid)
    assert got.shape == ref.shape
    assert close(got, ref, TOL_BF16)
    assert close(got, oracle.round_bf16(ref), 2.0 ** -7, "within one bf16 unit of the oracle")
    # ... and the two layers as two networks
    mid_gpu = run_net_bf16(first, params[:1], x, fuse_relu=True)
    two = run_net_bf16(second, params[1:], mid_gpu, fuse_relu=True)
    # (the same matrix instruction on the same operands in the same order of k-steps: the values are the same bits)
    assert np.array_equal(got, two), "%d of %d values differ from the two layers run one after the other" % (int((got != two).sum()), got.size)


def test_first_layer_pair_under_layer_timing_and_as_a_graph():
    """The one-kernel pair with per-layer timing on (the kernel's time is booked under the first layer, the 1x1 gets the gap
    between two event records)
    and recorded into a HIP graph: the same bits as the plain call."""
    from paper_1708_04728_amd import graph as G
    case = (40, 3, 81, 77, 24, 7, 4, 3, 40)
    N, C, H, W, K, R, stride, pad, K2 = case
    assert tail_takes(*case) > 0
    rng = np.random.default_rng(case_seed(case, 1))
    x = workloads.round_to_bf16(rng.standard_normal((N, C, H, W)).astype(np.float32))
    params = [{"w": workloads.round_to_bf16(rng.standard_normal((K, C, R, R)).astype(np.float32) * np.float32(0.1)),
               "b": (rng.standard_normal(K) * 0.1).astype(np.float32)},
              {"w": workloads.round_to_bf16(rng.standard_normal((K2, K, 1, 1)).astype(np.float32) * np.float32(0.2)),
               "b": (rng.standard_normal(K2) * 0.1).astype(np.float32)}]
    layers = [workloads.conv(K, R, stride, pad), workloads.relu(), workloads.conv(K2, 1, 1, 0), workloads.relu()]
    xg = G.to_device(x, "bf16", nhwc=True)
    net = B.Net(G.net_descs(layers, C, fuse_relu=True, pack="bf16"))
    assert net.n_layers == 2
    flat = G.flat_params(params, "bf16", pack=True)
    ws = torch.empty(max(net.workspace_bytes(B.desc(xg)), 256), dtype=torch.uint8, device="cuda")
    outs = []
    for mode in ("plain", "timed", "graph"):
        y = G.empty_like_desc(net.output_desc(B.desc(xg)))
        if mode == "timed":
            net.set_timing(True)
            net.fwd(xg, flat, y, ws)
            times = net.layer_times()
            net.set_timing(False)
            assert len(times) == 2 and times[0] > 0.0 and 0.0 <= times[1] < 0.01, times
        elif mode == "graph":
            side = torch.cuda.Stream()
            g = net.capture(xg, flat, y, ws, side)
            for _ in range(3):
                g.launch(torch.cuda.current_stream())
                torch.cuda.synchronize()
        else:
            net.fwd(xg, flat, y, ws)
        torch.cuda.synchronize()
        outs.append(G.to_host(y))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    mid = oracle.round_bf16(oracle.forward(layers[:2], params[:1], x)).astype(np.float32)
    assert close(outs[0], oracle.forward(layers[2:], params[1:], mid), TOL_BF16)
