"""GPU parity: every single-layer entry point of the C ABI against the fp64 CPU oracle on the same
seeded inputs.  Integer-like work (ReLU, max-pool, concat) must be bit-exact; floating-point
layers must stay within the tolerance of the data type."""
import numpy as np
import pytest

import oracle
import workloads
from paper_1708_04728_amd import binding as B
from util import TOL_BF16, TOL_F32, gpu, host, case_seed, close, rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _rng(seed):
    return np.random.default_rng(seed)


def _vals(rng, shape, dtype):
    a = rng.standard_normal(shape).astype(np.float32)
    return workloads.round_to_bf16(a) if dtype == "bf16" else a


def _tdt(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def _tol(dtype):
    return TOL_BF16 if dtype == "bf16" else TOL_F32


# N, C, H, W, K, R, S, stride, pad   -- spans several tiles, ragged tails in M, N and K of the GEMM
CONV_CASES = [
    (1, 64, 56, 56, 192, 3, 3, 1, 1),      # config 1 original
    (1, 64, 56, 56, 192, 3, 3, 2, 1),      # config 1 slim
    (2, 192, 28, 28, 64, 1, 1, 1, 0),      # inception 1x1
    (2, 192, 28, 28, 16, 1, 1, 1, 0),      # M smaller than a tile
    (2, 96, 28, 28, 128, 3, 3, 1, 1),
    (2, 16, 28, 28, 32, 5, 5, 1, 2),
    (2, 16, 28, 28, 128, 5, 5, 1, 2),      # slim 5x5
    (2, 3, 227, 227, 96, 11, 11, 4, 0),    # AlexNet conv1: Kg = 363 (not a multiple of 4 or 16)
    (2, 3, 227, 227, 96, 11, 11, 8, 0),
    (1, 96, 27, 27, 256, 5, 5, 1, 2),
    (1, 96, 27, 27, 256, 5, 5, 2, 2),
    (1, 3, 64, 48, 64, 7, 7, 2, 3),        # GoogLeNet stem filter, Kg = 147
    (3, 5, 9, 7, 7, 3, 3, 1, 1),           # everything ragged and tiny
    (1, 7, 13, 17, 33, 2, 4, 3, 1),        # run-time filter size path, M = 33
    (1, 4, 6, 6, 150, 1, 1, 1, 0),         # M = 150: two tiles with a ragged second one
    (2, 48, 14, 14, 40, 3, 3, 1, 1),       # C = 48: KRSC with 16-deep slices only
    (1, 32, 9, 11, 70, 5, 5, 2, 2),        # KRSC, strided, ragged everything
    (1, 3, 40, 37, 24, 7, 7, 2, 0),        # KCRS without padding: groups of 4 taps, 7 -> 8 wide
    (2, 5, 12, 12, 10, 4, 4, 1, 0),        # the same with a width that is a multiple of 4 (no added taps)
    (1, 2, 9, 30, 6, 3, 10, 1, 0),         # 10 -> 12 wide, windows that end on the tensor's last element
    (3, 1, 14, 14, 20, 12, 12, 1, 0),      # one channel, 12 x 12
]


# every shape in both filter orders where the channel count allows KRSC (a multiple of 16); the ReLU epilogue on three shapes
CONV_GRID = [(case, relu, layout) for case in CONV_CASES for relu in (False, True) for layout in ("kcrs", "krsc")
             if (not relu or case in (CONV_CASES[0], CONV_CASES[4], CONV_CASES[12])) and (layout == "kcrs" or B.can_pack(case[1]))]


@pytest.mark.parametrize("case,relu,layout", CONV_GRID)
def test_conv2d_f32(case, relu, layout):
    N, C, H, W, K, R, S, stride, pad = case
    rng = _rng(case_seed(case))
    x, w = _vals(rng, (N, C, H, W), "f32"), _vals(rng, (K, C, R, S), "f32") * np.float32(np.sqrt(2.0 / (C * R * S)))
    b = (_vals(rng, (K,), "f32") * np.float32(0.1))
    ref = oracle.conv2d(x, w, b, stride, pad, relu)
    y = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    wg = gpu(w)
    if layout == "krsc":
        wg = B.pack_filters(wg)
        assert np.array_equal(host(wg), np.transpose(w, (0, 2, 3, 1)))       # the repack is a pure permutation
    B.conv2d_fwd(gpu(x), B.conv_desc(K, C, R, S, stride, pad, relu, B.DR_KRSC if layout == "krsc" else B.DR_KCRS), wg,
                 gpu(b), y)
    torch.cuda.synchronize()
    assert close(host(y), ref, TOL_F32)


def _random_f32_cases(count, seed):
    """Seeded random fp32 layer shapes: any channel count (KCRS; KRSC as well when it is a multiple of 16), filters
    up to 12 wide, half of them without padding (the groups-of-4-taps order takes those whose width allows it)."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        C = int(rng.integers(1, 9)) if len(out) % 2 else 16 * int(rng.integers(1, 5))
        R, S = int(rng.integers(1, 13)), int(rng.integers(1, 13))
        stride = int(rng.integers(1, 5))
        pad = 0 if len(out) % 4 < 2 else int(rng.integers(0, min(R, S) // 2 + 1))
        N = int(rng.integers(1, 4))
        H, W = int(rng.integers(R, 48)), int(rng.integers(S, 48))
        K = int(rng.integers(1, 150))
        P, Q = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1
        if N * P * Q * K * C * R * S > 2e8:
            continue
        out.append((N, C, H, W, K, R, S, stride, pad))
    return out


@pytest.mark.parametrize("case", _random_f32_cases(40, 20260102))
def test_conv2d_f32_random_shapes(case):
    N, C, H, W, K, R, S, stride, pad = case
    rng = _rng(case_seed(case, 2))
    x, w = _vals(rng, (N, C, H, W), "f32"), _vals(rng, (K, C, R, S), "f32") * np.float32(np.sqrt(2.0 / (C * R * S)))
    b = (_vals(rng, (K,), "f32") * np.float32(0.1))
    relu = case_seed(case) % 2 == 0
    ref = oracle.conv2d(x, w, b, stride, pad, relu)
    xg, bg = gpu(x), gpu(b)
    for layout in ("kcrs", "krsc") if B.can_pack(C) else ("kcrs",):
        cd = B.conv_desc(K, C, R, S, stride, pad, relu, B.DR_KRSC if layout == "krsc" else B.DR_KCRS)
        wg = B.pack_filters(gpu(w)) if layout == "krsc" else gpu(w)
        y = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
        B.conv2d_fwd(xg, cd, wg, bg, y)
        torch.cuda.synchronize()
        assert close(host(y), ref, TOL_F32), layout
        need = B.conv2d_workspace_bytes(xg, cd)
        if need:
            ws = torch.empty((need // 4,), dtype=torch.float32, device="cuda")
            y2 = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
            B.conv2d_fwd_ws(xg, cd, wg, bg, y2, ws)
            torch.cuda.synchronize()
            assert close(host(y2), ref, TOL_F32), (layout, "with workspace")


# layers with few output tiles: the contraction is cut over several workgroups when scratch is given
SPLIT_CASES = [
    (1, 64, 56, 56, 192, 3, 3, 2, 1),      # config 1 slim: 39 tiles
    (1, 64, 64, 64, 128, 3, 3, 1, 1),      # 128 tiles, ranges of 5 slices: with KRSC they start inside a filter tap
    (1, 48, 14, 14, 40, 3, 3, 1, 1),       # ragged filter block, 16-deep slices with KRSC
    (1, 7, 13, 17, 33, 2, 4, 3, 1),        # tiny and ragged, four slices in two ranges
    (2, 32, 9, 11, 70, 5, 5, 2, 2),        # two images
    (1, 96, 27, 27, 256, 5, 5, 2, 2),      # 150 slices of 16 (KCRS) or 75 of 32 (KRSC), 16 tiles
    (3, 16, 6, 6, 20, 3, 3, 1, 0),         # 32-filter tiles
]


@pytest.mark.parametrize("case,layout", [(case, layout) for case in SPLIT_CASES for layout in ("kcrs", "krsc")
                                         if layout == "kcrs" or B.can_pack(case[1])])
def test_conv2d_f32_with_workspace(case, layout):
    N, C, H, W, K, R, S, stride, pad = case
    rng = _rng(case_seed(case, 1))
    x, w = _vals(rng, (N, C, H, W), "f32"), _vals(rng, (K, C, R, S), "f32") * np.float32(np.sqrt(2.0 / (C * R * S)))
    b = (_vals(rng, (K,), "f32") * np.float32(0.1))
    ref = oracle.conv2d(x, w, b, stride, pad, True)
    cd = B.conv_desc(K, C, R, S, stride, pad, True, B.DR_KRSC if layout == "krsc" else B.DR_KCRS)
    xg, wg = gpu(x), gpu(w)
    if layout == "krsc":
        wg = B.pack_filters(wg)
    need = B.conv2d_workspace_bytes(xg, cd)
    assert need > 0 and need % (K * ref.shape[0] * ref.shape[2] * ref.shape[3] * 4) == 0      # whole [K][n] planes
    ws = torch.full((need // 4 + 7,), float("nan"), dtype=torch.float32, device="cuda")
    # written at a channel offset of a wider tensor; the other channels stay as they are
    y = torch.full((ref.shape[0], K + 5, ref.shape[2], ref.shape[3]), -3.0, dtype=torch.float32, device="cuda")
    B.conv2d_fwd_ws(xg, cd, wg, gpu(b), y, ws, y_c_offset=2)
    torch.cuda.synchronize()
    got = host(y)
    assert close(got[:, 2:2 + K], ref, TOL_F32)
    assert (got[:, :2] == -3.0).all() and (got[:, 2 + K:] == -3.0).all()
    # the same call again gives the same bits (fixed order of the sum over the ranges)
    y2 = torch.full_like(y, -3.0)
    B.conv2d_fwd_ws(xg, cd, wg, gpu(b), y2, ws, y_c_offset=2)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


def test_conv2d_with_workspace_refusals_and_layers_that_are_not_cut():
    x = torch.zeros((1, 64, 56, 56), dtype=torch.float32, device="cuda")
    w = torch.zeros((192, 64, 3, 3), dtype=torch.float32, device="cuda")
    y = torch.zeros((1, 192, 28, 28), dtype=torch.float32, device="cuda")
    cd = B.conv_desc(192, 64, 3, stride=2, pad=1)
    need = B.conv2d_workspace_bytes(x, cd)
    assert need > 0
    small = torch.zeros((need // 4 - 1,), dtype=torch.float32, device="cuda")
    with pytest.raises(RuntimeError, match="workspace"):
        B.conv2d_fwd_ws(x, cd, w, None, y, small)
    with pytest.raises(RuntimeError, match="workspace"):
        B.conv2d_fwd_ws(x, cd, w, None, y, None)
    # a layer whose tiles reach half of the compute units needs no scratch and runs without any
    rng = _rng(11)
    xb, wb = _vals(rng, (16, 32, 40, 40), "f32"), _vals(rng, (64, 32, 3, 3), "f32") * np.float32(0.1)
    cdb = B.conv_desc(64, 32, 3, pad=1)
    assert B.conv2d_workspace_bytes(gpu(xb), cdb) == 0
    yb = torch.empty((16, 64, 40, 40), dtype=torch.float32, device="cuda")
    B.conv2d_fwd_ws(gpu(xb), cdb, gpu(wb), None, yb, None)
    torch.cuda.synchronize()
    assert close(host(yb), oracle.conv2d(xb, wb, None, 1, 1), TOL_F32)


def test_conv2d_channel_offset_and_no_bias():
    rng = _rng(7)
    x, w = _vals(rng, (2, 8, 10, 10), "f32"), _vals(rng, (5, 8, 3, 3), "f32")
    ref = oracle.conv2d(x, w, None, 1, 1)
    y = torch.full((2, 12, 10, 10), -7.0, dtype=torch.float32, device="cuda")
    B.conv2d_fwd(gpu(x), B.conv_desc(5, 8, 3, pad=1), gpu(w), None, y, y_c_offset=4)
    torch.cuda.synchronize()
    got = host(y)
    assert close(got[:, 4:9], ref, TOL_F32)
    assert (got[:, :4] == -7.0).all() and (got[:, 9:] == -7.0).all()       # other channels untouched


def test_slim_conv_is_stride_product_with_relu():
    rng = _rng(8)
    x, w, b = _vals(rng, (2, 16, 23, 23), "f32"), _vals(rng, (24, 16, 3, 3), "f32") * np.float32(0.1), _vals(rng, (24,), "f32")
    ref = oracle.conv2d(x, w, b, 2 * 2, 1, relu=True)      # conv stride 2, absorbed pool stride 2
    y = torch.empty(ref.shape, dtype=torch.float32, device="cuda")
    B.slim_conv_fwd(gpu(x), B.conv_desc(24, 16, 3, stride=2, pad=1, relu=False), 2, gpu(w), gpu(b), y)
    torch.cuda.synchronize()
    assert close(host(y), ref, TOL_F32)
    assert (host(y) >= 0).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 3, 5, 7), (1, 192, 56, 56), (1, 1, 1, 1), (3, 1, 1, 13)])
def test_relu_bit_exact(dtype, shape):
    x = _vals(_rng(1), shape, dtype)
    xg = gpu(x, dtype)
    y = torch.empty_like(xg)
    B.relu(xg, y)
    assert np.array_equal(host(y), oracle.relu(x))
    B.relu(xg, xg)                                          # in place
    torch.cuda.synchronize()
    assert np.array_equal(host(xg), oracle.relu(x))
    # unaligned views take the scalar path
    flat = gpu(_vals(_rng(2), (1, 1, 1, 1001), dtype), dtype)
    v = flat[..., 1:]
    out = torch.empty_like(flat)[..., 1:]
    B.lib().dr_relu(B.dr_tensor(1, 1, 1, 1000, B._dtype_code(v)), B._ptr(v), B._ptr(out), B._stream())
    torch.cuda.synchronize()
    assert np.array_equal(host(out), np.maximum(host(v), 0))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(1, 192, 56, 56), (2, 96, 55, 55), (2, 7, 3, 5), (1, 3, 4, 4), (2, 64, 1, 1)])
def test_lrn(dtype, shape):
    x = _vals(_rng(3), shape, dtype) * np.float32(30.0)     # large values so the normaliser matters
    if dtype == "bf16":
        x = workloads.round_to_bf16(x)
    ref = oracle.lrn(x, 5, 1e-4, 0.75, 1.0)
    xg = gpu(x, dtype)
    y = torch.empty_like(xg)
    B.lrn_fwd(xg, y, 5, 1e-4, 0.75, 1.0)
    torch.cuda.synchronize()
    assert close(host(y), ref, _tol(dtype))


@pytest.mark.parametrize("n,alpha,beta,k", [(3, 0.5, 0.5, 2.0), (5, 2.0, 0.6, 1.0), (1, 0.3, 0.75, 1.0), (4, 1.0, 0.75, 1.5)])
def test_lrn_other_parameters(n, alpha, beta, k):
    x = _vals(_rng(4), (2, 9, 6, 5), "f32") * np.float32(3.0)
    ref = oracle.lrn(x, n, alpha, beta, k)
    y = torch.empty(x.shape, dtype=torch.float32, device="cuda")
    B.lrn_fwd(gpu(x), y, n, alpha, beta, k)
    torch.cuda.synchronize()
    assert close(host(y), ref, TOL_F32)


POOL_CASES = [  # N, C, H, W, k, stride, pad
    (1, 192, 56, 56, 3, 2, 0), (2, 192, 28, 28, 3, 1, 1), (2, 96, 55, 55, 3, 2, 0), (1, 256, 27, 27, 3, 2, 0),
    (1, 64, 112, 112, 3, 2, 0), (2, 5, 7, 9, 3, 2, 0), (1, 3, 5, 5, 2, 2, 1), (1, 2, 9, 9, 3, 3, 1), (2, 3, 6, 7, 1, 1, 0),
    (1, 8, 14, 14, 3, 2, 0),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", POOL_CASES)
def test_maxpool_bit_exact(dtype, case):
    N, C, H, W, k, s, pad = case
    x = -np.abs(_vals(_rng(5), (N, C, H, W), dtype)) - np.float32(0.5)       # negative: padding must not win
    if dtype == "bf16":
        x = workloads.round_to_bf16(x)
    ref = oracle.maxpool(x, k, s, pad)
    y = torch.empty(ref.shape, dtype=_tdt(dtype), device="cuda")
    B.maxpool_fwd(gpu(x, dtype), B.pool_desc(k, s, pad), y)
    torch.cuda.synchronize()
    assert np.array_equal(host(y), ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_concat_bit_exact(dtype):
    rng = _rng(6)
    for shapes in ([(2, 64, 28, 28), (2, 128, 28, 28), (2, 32, 28, 28), (2, 32, 28, 28)], [(3, 1, 5, 3), (3, 2, 5, 3), (3, 5, 5, 3)],
                   [(1, 7, 1, 1)]):
        xs = [_vals(rng, s, dtype) for s in shapes]
        ref = oracle.concat(xs)
        y = torch.empty(ref.shape, dtype=_tdt(dtype), device="cuda")
        B.concat([gpu(x, dtype) for x in xs], y)
        torch.cuda.synchronize()
        assert np.array_equal(host(y), ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 64, 56, 56), (3, 5, 7, 3)])
def test_bn_and_add_relu(dtype, shape):
    rng = _rng(9)
    x = _vals(rng, shape, dtype)
    C = shape[1]
    g, be = rng.uniform(0.5, 1.5, C).astype(np.float32), (rng.standard_normal(C) * 0.1).astype(np.float32)
    mu, var = (rng.standard_normal(C) * 0.1).astype(np.float32), rng.uniform(0.5, 1.5, C).astype(np.float32)
    eps = float(np.float32(1e-5))
    ref = oracle.bn(x, g, be, mu, var, eps)
    xg = gpu(x, dtype)
    y = torch.empty_like(xg)
    B.bn_fwd(xg, gpu(g), gpu(be), gpu(mu), gpu(var), eps, False, y)
    torch.cuda.synchronize()
    assert close(host(y), ref, _tol(dtype))
    B.bn_fwd(xg, gpu(g), gpu(be), gpu(mu), gpu(var), eps, True, xg)          # in place, fused ReLU
    torch.cuda.synchronize()
    assert close(host(xg), np.maximum(ref, 0), _tol(dtype))

    a, b = _vals(rng, shape, dtype), _vals(rng, shape, dtype)
    ref = oracle.add_relu(a, b)
    ag = gpu(a, dtype)
    B.add_relu(ag, gpu(b, dtype), ag)
    torch.cuda.synchronize()
    if dtype == "f32":
        assert np.array_equal(host(ag), ref.astype(np.float32).astype(np.float64))   # one rounding of an exact sum
    else:
        assert close(host(ag), ref, TOL_BF16)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_avgpool_fc_softmax(dtype):
    rng = _rng(10)
    x = _vals(rng, (4, 1024, 7, 7), dtype)
    ref = oracle.avgpool(x, 7)
    y = torch.empty(ref.shape, dtype=_tdt(dtype), device="cuda")
    B.avgpool_fwd(gpu(x, dtype), B.pool_desc(7, 1), y)
    torch.cuda.synchronize()
    assert close(host(y), ref, _tol(dtype))

    xf = _vals(rng, (4, 1024, 1, 1), dtype)
    w = _vals(rng, (1000, 1024), dtype) * np.float32(np.sqrt(2.0 / 1024))
    if dtype == "bf16":
        w = workloads.round_to_bf16(w)
    b = _vals(rng, (1000,), "f32") * np.float32(0.01)
    ref = oracle.fc(xf, w, b)
    z = torch.empty((4, 1000, 1, 1), dtype=_tdt(dtype), device="cuda")
    B.fc_fwd(gpu(xf, dtype), gpu(w, dtype), gpu(b), z)
    torch.cuda.synchronize()
    assert close(host(z).reshape(4, 1000), ref, _tol(dtype))

    logits = host(z).reshape(4, 1000)
    p = torch.empty((4, 1000, 1, 1), dtype=torch.float32, device="cuda")
    B.softmax_fwd(z, p)
    torch.cuda.synchronize()
    got = host(p).reshape(4, 1000)
    assert close(got, oracle.softmax(logits), 1e-5)
    np.testing.assert_allclose(got.sum(axis=1), 1.0, rtol=1e-5)


def test_empty_tensors_are_accepted():
    x = torch.empty((0, 4, 5, 5), dtype=torch.float32, device="cuda")
    B.relu(x, torch.empty_like(x))
    B.lrn_fwd(x, torch.empty_like(x))
    y = torch.empty((0, 4, 2, 2), dtype=torch.float32, device="cuda")
    B.maxpool_fwd(x, B.pool_desc(3, 2), y)
    w = torch.empty((3, 4, 3, 3), dtype=torch.float32, device="cuda")
    B.conv2d_fwd(x, B.conv_desc(3, 4, 3, pad=1), w, None, torch.empty((0, 3, 5, 5), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
