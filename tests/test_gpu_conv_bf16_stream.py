"""GPU parity of the streaming bf16 convolution kernel (NHWC, KRSC filters, operands loaded straight
into LDS, persistent workgroups) against the fp64 oracle, on shapes chosen to reach every code path:
both slice modes (C a multiple of 64 or not), every tile configuration the launcher picks, several tiles per
workgroup, ragged filter counts / pixel counts / channel runs, strides and paddings on every
border, and the scalar store path (channel offsets that are not multiples of 8)."""
import numpy as np
import pytest

import oracle
import workloads
from paper_1708_04728_amd import binding as B
from util import TOL_BF16, empty_nhwc, gpu, gpu_nhwc, host_nhwc, case_seed, close, rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _vals(rng, shape):
    return workloads.round_to_bf16(rng.standard_normal(shape).astype(np.float32))


def _run(case, relu=False, bias=True, seed=0):
    N, C, H, W, K, R, S, stride, pad = case
    rng = np.random.default_rng(seed + 1000 * (case_seed(case) % 1000))
    x = _vals(rng, (N, C, H, W))
    w = workloads.round_to_bf16(rng.standard_normal((K, C, R, S)).astype(np.float32) * np.float32(np.sqrt(2.0 / (C * R * S))))
    b = (rng.standard_normal(K) * 0.1).astype(np.float32) if bias else None
    ref = oracle.conv2d(x, w, b, stride, pad, relu)
    y = empty_nhwc(ref.shape, "bf16")
    B.conv2d_fwd(gpu_nhwc(x, "bf16"), B.conv_desc(K, C, R, S, stride, pad, relu, B.DR_KRSC), B.pack_filters(gpu(w, "bf16")),
                 gpu(b) if bias else None, y)
    torch.cuda.synchronize()
    got = host_nhwc(y)
    assert not np.isnan(got).any()
    assert close(got, ref, TOL_BF16)
    # against the oracle's result rounded to bf16: at most one unit in the last place apart
    assert close(got, oracle.round_bf16(ref), 2.0 ** -7)


# N, C, H, W, K, R, S, stride, pad
CASES = [
    # --- slices inside one tap (C % 64 == 0)
    (1, 64, 12, 12, 24, 1, 1, 1, 0),        # few tiles: 64 x 64 tiles (as for most small cases below), one slice per tile
    (2, 64, 30, 30, 64, 3, 3, 1, 1),        # one round of 64 x 128 tiles, 9 slices
    (1, 128, 40, 40, 72, 3, 3, 1, 1),       # ragged filter block
    (1, 64, 190, 190, 136, 1, 1, 1, 0),     # many pixels: several channel blocks, ragged last pixel tile, grid not a multiple of 8
    (3, 128, 17, 19, 40, 3, 3, 2, 1),       # stride 2, odd sizes
    (1, 192, 9, 9, 200, 5, 5, 1, 2),        # 5x5 at 192 channels, 75 slices
    (2, 64, 8, 8, 16, 3, 3, 1, 0),          # no padding
    # --- slices running over a filter row (C % 64 != 0)
    (1, 8, 20, 20, 16, 7, 7, 2, 3),         # 8 channels: one chunk per tap, 7x7 stride 2
    (2, 16, 28, 28, 32, 5, 5, 1, 2),
    (2, 24, 14, 14, 64, 5, 5, 1, 2),
    (1, 48, 7, 7, 128, 5, 5, 1, 2),
    (1, 96, 28, 28, 128, 3, 3, 1, 1),
    (1, 112, 14, 14, 224, 3, 3, 1, 1),
    (2, 144, 14, 14, 288, 3, 3, 1, 1),
    (1, 160, 7, 7, 320, 3, 3, 1, 1),
    (2, 480, 14, 14, 96, 1, 1, 1, 0),       # 1x1 at 480 = 7.5 slices
    (1, 528, 14, 14, 32, 1, 1, 1, 0),
    (1, 832, 7, 7, 48, 1, 1, 1, 0),
    (1, 16, 150, 150, 8, 3, 3, 1, 1),       # many pixel tiles per workgroup at K = 8
    (1, 32, 11, 13, 20, 3, 5, 1, 2),        # 3x5 filter, pad 2: whole filter rows in the padding
    (1, 40, 6, 6, 12, 5, 5, 3, 2),          # stride 3
    (1, 8, 3, 3, 8, 3, 3, 1, 1),            # tiny
    (2, 96, 70, 70, 72, 3, 3, 1, 1),        # many pixels (64 x 128 tiles) with slices running over filter rows
    (1, 24, 200, 200, 40, 5, 5, 2, 2),      # the same at stride 2, 5x5
    (1, 64, 100, 100, 192, 3, 3, 1, 1),     # 192 filters, three channel blocks
    (8, 64, 56, 56, 256, 1, 1, 1, 0),       # 256 filters, 25 088 pixels: one round of 128 x 128 tiles (64 x 64 per wave)
    (8, 16, 56, 56, 256, 3, 3, 1, 1),       # the same with slices running over filter rows
    (2, 16, 160, 160, 96, 3, 3, 1, 1),      # 96 filters, 51 200 pixels: one round of 96 x 128 tiles instead of two of 64 x 128
    (2, 64, 160, 160, 96, 1, 1, 1, 0),      # the same with slices inside one tap
    (1, 32, 96, 96, 288, 5, 5, 1, 2),       # 288 filters, slices running over filter rows
    (1, 64, 200, 200, 24, 1, 1, 1, 0),      # K <= 32 and 40 000 pixels: 32 x 128 tiles
    (1, 16, 200, 200, 24, 3, 3, 1, 1),      # the same with slices running over filter rows
    (8, 24, 100, 100, 104, 3, 3, 1, 1),     # 104 filters on 80 000 pixels: one round of 128 x 256 tiles (128 x 64 per wave, half-depth slices)
    (8, 64, 200, 200, 128, 3, 3, 2, 1),     # the same tile with slices inside one tap, stride 2, 128 filters
]


@pytest.mark.parametrize("case", CASES)
def test_conv_stream(case):
    _run(case, relu=(case_seed(case) % 2 == 0))


def _random_cases(count, seed):
    """Seeded random layer shapes inside what the streaming kernel takes (C a multiple of 8, S <= 9, R <= 16):
    small ones of every kind, and every fourth one with enough pixels to leave the 64 x 64 tiles."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        big = len(out) % 4 == 3
        C = 8 * int(rng.integers(1, 18))
        R, S = int(rng.integers(1, 8)), int(rng.integers(1, 8))
        stride = int(rng.integers(1, 4))
        pad = int(rng.integers(0, min(R, S) // 2 + 2))
        N = int(rng.integers(1, 4))
        H, W = (int(rng.integers(60, 130)), int(rng.integers(60, 130))) if big else (int(rng.integers(3, 40)), int(rng.integers(3, 40)))
        K = int(rng.integers(1, 40)) if big else int(rng.integers(1, 200))
        if H + 2 * pad < R or W + 2 * pad < S or pad >= R or pad >= S:
            continue
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        if N * P * Q * K * C * R * S > 3e8:
            continue
        out.append((N, C, H, W, K, R, S, stride, pad))
    return out


@pytest.mark.parametrize("case", _random_cases(48, 20260101))
def test_conv_stream_random_shapes(case):
    _run(case, relu=(case_seed(case) % 2 == 0), bias=(case_seed(case) % 3 != 0))


def test_conv_stream_many_tiles_per_workgroup():
    """More pixel tiles than the device holds workgroups: every workgroup walks several tiles, and the
    loads of one tile are in flight while the previous one is stored."""
    _run((3, 16, 208, 208, 16, 3, 3, 1, 1), relu=True)       # 129 792 pixels = 507 tiles of 256
    _run((2, 64, 200, 200, 16, 1, 1, 1, 0), bias=False)      # one slice per tile, 313 tiles


def test_conv_stream_channel_offsets():
    """Channel ranges of a wider tensor: offset 8 (16-byte stores) and offset 3 (element stores).  (The
    residual sum of the store is reached through the folded bottleneck, see test_gpu_bf16_nets.)"""
    rng = np.random.default_rng(77)
    N, C, H, W, K = 2, 64, 12, 12, 88
    x = _vals(rng, (N, C, H, W))
    w = workloads.round_to_bf16(rng.standard_normal((K, C, 1, 1)).astype(np.float32) * np.float32(0.2))
    b = (rng.standard_normal(K) * 0.1).astype(np.float32)
    ref = oracle.conv2d(x, w, b, 1, 0)
    for off, ctot in ((8, 104), (3, 99)):
        y = B.NHWC(torch.full((N, H, W, ctot), -7.0, dtype=torch.bfloat16, device="cuda"))
        B.conv2d_fwd(gpu_nhwc(x, "bf16"), B.conv_desc(K, C, 1, 1, 1, 0, False, B.DR_KRSC), B.pack_filters(gpu(w, "bf16")), gpu(b), y,
                     y_c_offset=off)
        torch.cuda.synchronize()
        got = host_nhwc(y)
        assert close(got[:, off:off + K], ref, TOL_BF16)
        assert (got[:, :off] == -7.0).all() and (got[:, off + K:] == -7.0).all()
