"""GPU parity of the patch convolution kernel (bf16 NHWC, several taps at stride 1 on 64-channel maps: the input rows of a
tile are loaded into LDS once and every tap multiplies from there) against the fp64 oracle.  The library picks that
kernel by rule: 64 | C, stride 1, more than one tap, a map wide enough that whole output rows fill at least 192 of a
tile's 256 pixel rows while (rows + R - 1) (W + 2 pad) patch pixels per 64 channels fit 352 LDS rows.  Every case
below satisfies the rule (the last test checks one that does not against the same oracle, for contrast).  Where tiles of
HALF rows take fewer tiles per image than tiles of whole rows the kernel uses those (`tiling` restates the choice): the
cases cover both, half-row tiles that start in mid-row, and last tiles of a few segments."""
import numpy as np
import pytest

import oracle
import workloads
from paper_1708_04728_amd import binding as B
from util import TOL_BF16, case_seed, close, empty_nhwc, gpu, gpu_nhwc, host_nhwc

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def rows_per_tile(C, H, W, K, R, S, stride, pad):
    """The rule of the library's launcher, restated: output rows per tile, 0 = the layer goes to the streaming kernel."""
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(W, S, stride, pad)
    if C % 64 or K % 8 or stride != 1 or R * S < 2 or R > 7 or S > 7 or Q < 2 or Q > 256:
        return 0
    th = min(256 // Q, P)
    while th >= 1 and (C // 64) * (((th + R - 1) * (W + 2 * pad) + 31) // 32 * 32) > 352:
        th -= 1
    return th if th >= 1 and th * Q * 4 >= 256 * 3 else 0


def tiling(C, H, W, K, R, S, stride, pad):
    """(segments per row, segments per tile, tiles per image) the launcher chooses, restated."""
    P, Q = oracle.conv_out_size(H, R, stride, pad), oracle.conv_out_size(W, S, stride, pad)
    th = rows_per_tile(C, H, W, K, R, S, stride, pad)
    whole = (1, th, (P + th - 1) // th)
    if Q % 2 or Q < 4:
        return whole
    th2 = min(256 // (Q // 2), 2 * P)
    while th2 >= 1 and (C // 64) * (((th2 // 2 + R) * (W + 2 * pad) + 31) // 32 * 32) > 416:
        th2 -= 1
    return (2, th2, (2 * P + th2 - 1) // th2) if th2 >= 1 and (2 * P + th2 - 1) // th2 < whole[2] else whole


# N, C, H, W, K, R, S, stride, pad
CASES = [
    (2, 64, 56, 56, 192, 3, 3, 1, 1),      # the benchmark's dominant layer: 9 half rows per tile (13 tiles per image, the last of 4 half rows), two blocks of 96 filters
    (3, 64, 56, 56, 64, 3, 3, 1, 1),       # ResNet conv2_x: one block of 64 filters
    (1, 64, 57, 56, 72, 3, 3, 1, 1),       # 114 half rows: a last tile of 6; ragged filter block
    (2, 64, 28, 28, 200, 3, 3, 1, 1),      # 9 rows per tile (252 of 256 pixel rows), 28 = 3 tiles + 1 row; 200 filters
    (1, 64, 30, 68, 40, 3, 3, 1, 1),       # wide map: three rows per tile, 204 of 256 pixel rows
    (2, 64, 20, 66, 24, 3, 3, 1, 0),       # no padding: 64 outputs per row, three rows per tile
    (1, 64, 33, 28, 96, 5, 5, 1, 2),       # 5x5: 17 half rows of 14 per tile (patch of 13 x 32 pixels: all 416 LDS rows) instead of seven rows
    (2, 64, 40, 64, 128, 1, 3, 1, 1),      # 1x3 filter, padded both ways (the row padding adds output rows)
    (1, 64, 31, 63, 136, 3, 2, 1, 1),      # 3x2 filter; 7 half rows of 32 per tile
    (5, 64, 12, 64, 64, 3, 3, 1, 1),       # three rows per tile, four tiles per image, five images
]


# (segments per row, segments per tile, tiles per image) of each case
EXPECTED_TILING = dict(zip(CASES, [(2, 9, 13), (2, 9, 13), (2, 9, 13), (1, 9, 4), (1, 3, 10), (1, 3, 6), (2, 17, 4), (1, 4, 11), (2, 7, 9), (1, 3, 4)]))


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("relu", [False, True])
def test_conv_patch(case, relu):
    N, C, H, W, K, R, S, stride, pad = case
    assert rows_per_tile(C, H, W, K, R, S, stride, pad) > 0, "the case must be one the patch kernel takes"
    assert tiling(C, H, W, K, R, S, stride, pad) == EXPECTED_TILING[case], "the cases are chosen for these tilings"
    rng = np.random.default_rng(case_seed(case))
    x = workloads.round_to_bf16(rng.standard_normal((N, C, H, W)).astype(np.float32))
    w = workloads.round_to_bf16(rng.standard_normal((K, C, R, S)).astype(np.float32) * np.float32(np.sqrt(2.0 / (C * R * S))))
    bias = case_seed(case) % 3 != 0
    b = (rng.standard_normal(K) * 0.1).astype(np.float32) if bias else None
    ref = oracle.conv2d(x, w, b, stride, pad, relu)
    # written at a channel offset of a wider tensor (a branch of a module writing its part of the concatenated output)
    ctot, coff = K + 24, 16
    y = B.NHWC(torch.full((N, ref.shape[2], ref.shape[3], ctot), -5.0, dtype=torch.bfloat16, device="cuda"))
    B.conv2d_fwd(gpu_nhwc(x, "bf16"), B.conv_desc(K, C, R, S, stride, pad, relu, B.DR_KRSC), B.pack_filters(gpu(w, "bf16")),
                 gpu(b) if bias else None, y, y_c_offset=coff)
    torch.cuda.synchronize()
    got = host_nhwc(y)
    assert not np.isnan(got).any()
    assert (got[:, :coff] == -5.0).all() and (got[:, coff + K:] == -5.0).all()
    assert close(got[:, coff:coff + K], ref, TOL_BF16)
    assert close(got[:, coff:coff + K], oracle.round_bf16(ref), 2.0 ** -7, "within one bf16 unit of the oracle")


def test_conv_patch_many_tiles_per_workgroup_and_a_layer_the_rule_leaves_out():
    # 64 images of 56 x 56: 896 tiles on at most 512 workgroups per filter block, so workgroups walk several tiles
    case = (64, 64, 56, 56, 96, 3, 3, 1, 1)
    N, C, H, W, K, R, S, stride, pad = case
    assert rows_per_tile(C, H, W, K, R, S, stride, pad) == 4
    rng = np.random.default_rng(7)
    x = workloads.round_to_bf16(rng.standard_normal((N, C, H, W)).astype(np.float32))
    w = workloads.round_to_bf16(rng.standard_normal((K, C, R, S)).astype(np.float32) * np.float32(np.sqrt(2.0 / (C * R * S))))
    b = (rng.standard_normal(K) * 0.1).astype(np.float32)
    y = empty_nhwc((N, K, 56, 56), "bf16")
    B.conv2d_fwd(gpu_nhwc(x, "bf16"), B.conv_desc(K, C, R, S, stride, pad, True, B.DR_KRSC), B.pack_filters(gpu(w, "bf16")), gpu(b), y)
    torch.cuda.synchronize()
    got = host_nhwc(y)
    pick = [0, 17, 63]
    assert close(got[pick], oracle.conv2d(x[pick], w, b, stride, pad, True), TOL_BF16)
    assert np.isfinite(got).all() and (got >= 0).all()
    # stride 2 is not for the patch kernel; the streaming kernel gives the same layer's strided form
    assert rows_per_tile(C, H, W, K, R, S, 2, pad) == 0
