"""GPU parity of the pieces that learn a slim layer (Sec. 3.1, Lemma 1) against the fp64 oracle: the loss and its
gradient, the gradient of a convolution's parameters, the descent step, and a short run of the whole loop."""
import numpy as np
import pytest

import oracle
import workloads
from paper_1708_04728_amd import binding as B
from util import TOL_F32, gpu, host, close, rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _ws(nbytes):
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")


def test_regression_loss_and_gradient():
    rng = np.random.default_rng(1)
    for shape in ((2, 5, 7, 9), (1, 3, 1, 1), (3, 192, 28, 28), (1, 1, 1, 300001)):
        f = np.maximum(rng.standard_normal(shape), 0).astype(np.float32)          # about half the entries are zero
        y = np.abs(rng.standard_normal(shape)).astype(np.float32)
        loss_ref, dz_ref = oracle.regression_loss_grad(f, y)
        fg, yg = gpu(f), gpu(y)
        dz = torch.empty_like(fg)
        loss = torch.zeros(1, device="cuda")
        B.regression_loss_grad(fg, yg, dz, loss, _ws(B.regression_loss_workspace_bytes()))
        torch.cuda.synchronize()
        assert float(loss.item()) == pytest.approx(loss_ref, rel=1e-5)
        # each entry is one subtraction and one doubling: exact in fp32 up to the subtraction's rounding
        np.testing.assert_allclose(host(dz), dz_ref, rtol=1e-6, atol=1e-6)
        assert ((host(dz) == 0) == (dz_ref == 0)).all()


# N, C, H, W, K, R, S, stride, pad
WGRAD_CASES = [
    (2, 3, 9, 8, 5, 3, 3, 1, 1),          # one tile, ragged everywhere
    (3, 64, 28, 28, 192, 3, 3, 2, 1),     # the slim layer of the conv2 block: 3 x 9 tiles, stride 2
    (2, 16, 14, 14, 70, 5, 5, 1, 2),      # 5x5, ragged filter block, 400 (c, r, s) columns
    (5, 8, 10, 6, 64, 1, 1, 1, 0),        # 1x1
    (1, 4, 31, 29, 9, 7, 7, 4, 3),        # one image (no partial sums), 7x7 stride 4
    (40, 2, 6, 6, 3, 3, 2, (2, 1), (1, 0)),  # many images: several per workgroup, non-square filter and stride
]


@pytest.mark.parametrize("case", WGRAD_CASES)
def test_conv_parameter_gradients(case):
    N, C, H, W, K, R, S, stride, pad = case
    rng = np.random.default_rng(7 + N * C)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    ph, pw = (pad, pad) if np.isscalar(pad) else pad
    P, Q = oracle.conv_out_size(H, R, sh, ph), oracle.conv_out_size(W, S, sw, pw)
    dz = (rng.standard_normal((N, K, P, Q)) * (rng.random((N, K, P, Q)) < 0.6)).astype(np.float32)   # ReLU zeros
    dw_ref, db_ref = oracle.conv2d_bwd_params(x, dz, R, S, stride, pad)
    xg, dzg = gpu(x), gpu(dz)
    cd = B.conv_desc(K, C, R, S, stride, pad, True, B.DR_KCRS)
    dw = torch.full((K, C, R, S), float("nan"), device="cuda")
    db = torch.full((K,), float("nan"), device="cuda")
    for rep in range(2):       # the same workspace twice: nothing may depend on what it held
        ws = _ws(B.conv2d_bwd_params_workspace_bytes(xg, cd))
        ws.fill_(255)
        B.conv2d_bwd_params(xg, cd, dzg, dw, db, ws)
        torch.cuda.synchronize()
        assert close(host(dw), dw_ref, TOL_F32)
        assert close(host(db), db_ref, TOL_F32)
    first = host(dw).copy()
    B.conv2d_bwd_params(xg, cd, dzg, dw, db, ws)
    torch.cuda.synchronize()
    assert np.array_equal(host(dw), first)      # fixed summation order: bit-identical from run to run


def test_sgd_step_bit_exact():
    rng = np.random.default_rng(3)
    w = rng.standard_normal(100003).astype(np.float32)
    dw = rng.standard_normal(100003).astype(np.float32)
    lr = np.float32(0.0137)
    wg = gpu(w)
    B.sgd_step(wg, gpu(dw), float(lr))
    torch.cuda.synchronize()
    assert np.array_equal(host(wg).astype(np.float32), w - lr * dw)


def test_slim_layer_regression_follows_the_oracle():
    """Config 1's slim layer (3x3, stride 2, ReLU) learned from the output of the original block on a few seeded
    images: twelve descent steps on the GPU and in the oracle from the same start; the losses agree step by
    step and fall."""
    layers = workloads.CONFIGS[1]["original"]
    params = workloads.make_params(1, "original")
    x = workloads.make_input(1, 1)
    x = np.concatenate([x, x[:, ::-1].copy(), x[:, :, ::-1].copy()], axis=0)[:, :16, :20, :20].copy()    # 3 small images
    p16 = [{"w": params[0]["w"][:24, :16].copy(), "b": params[0]["b"][:24].copy()}]
    y = oracle.forward(layers, p16, x)                      # conv - ReLU - LRN - pool
    slim_w = workloads.make_params(1, "slim")[0]
    w0, b0 = slim_w["w"][:24, :16].astype(np.float32).copy(), slim_w["b"][:24].astype(np.float32).copy()
    lr = 5e-5
    w_ref, b_ref, ref_losses = w0.astype(np.float64), b0.astype(np.float64), []
    for _ in range(12):
        loss, w_ref, b_ref = oracle.regression_step(x, w_ref, b_ref, y, 2, 1, lr)
        ref_losses.append(loss)
    xg, yg, wg, bg = gpu(x), gpu(y), gpu(w0), gpu(b0)
    cd = B.conv_desc(24, 16, 3, 3, 1, 1, False, B.DR_KCRS)
    f = torch.empty(y.shape, device="cuda")
    dw, db, loss = torch.empty_like(wg), torch.empty_like(bg), torch.zeros(1, device="cuda")
    ws = _ws(max(B.conv2d_bwd_params_workspace_bytes(xg, B.conv_desc(24, 16, 3, 3, 2, 1, True, B.DR_KCRS)), B.regression_loss_workspace_bytes()))
    cd2 = B.conv_desc(24, 16, 3, 3, 2, 1, True, B.DR_KCRS)
    got = []
    for _ in range(12):
        B.slim_conv_fwd(xg, cd, 2, wg, bg, f)              # stride 1 x pool stride 2, ReLU forced on
        B.regression_loss_grad(f, yg, f, loss, ws)         # dz overwrites f
        got.append(float(loss.item()))
        B.conv2d_bwd_params(xg, cd2, f, dw, db, ws)
        B.sgd_step(wg, dw, lr)
        B.sgd_step(bg, db, lr)
    torch.cuda.synchronize()
    assert y.shape == (3, 24, 10, 10)
    np.testing.assert_allclose(got, ref_losses, rtol=2e-4)
    assert all(b_ < a_ for a_, b_ in zip(got, got[1:]))
    assert close(host(wg), w_ref, 10 * TOL_F32)


def test_degenerate_inputs():
    """No images / no pixels: the gradients are zero (and the kernels dereference nothing); an empty tensor has zero
    loss; unsupported layouts are refused before anything is launched."""
    cd = B.conv_desc(5, 3, 3, 3, 1, 1, True, B.DR_KCRS)
    x = torch.empty((0, 3, 8, 8), device="cuda")
    dz = torch.empty((0, 5, 8, 8), device="cuda")
    dw = torch.full((5, 3, 3, 3), float("nan"), device="cuda")
    db = torch.full((5,), float("nan"), device="cuda")
    B.conv2d_bwd_params(x, cd, dz, dw, db, _ws(B.conv2d_bwd_params_workspace_bytes(x, cd)))
    torch.cuda.synchronize()
    assert not host(dw).any() and not host(db).any()
    f = torch.empty((0, 4, 2, 2), device="cuda")
    loss = torch.full((1,), 7.0, device="cuda")
    B.regression_loss_grad(f, f, f, loss, _ws(B.regression_loss_workspace_bytes()))
    torch.cuda.synchronize()
    assert float(loss.item()) == 0.0
    xb = torch.zeros((1, 8, 4, 4), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(B.DeepRebirthError):
        B.conv2d_bwd_params_workspace_bytes(xb, B.conv_desc(4, 8, 1, 1, 1, 0, True, B.DR_KCRS))
    x1 = torch.zeros((1, 16, 4, 4), device="cuda")
    with pytest.raises(B.DeepRebirthError):                      # KRSC filters
        B.conv2d_bwd_params_workspace_bytes(x1, B.conv_desc(4, 16, 1, 1, 1, 0, True, B.DR_KRSC))
    with pytest.raises(B.DeepRebirthError):                      # dz of the wrong shape
        B.conv2d_bwd_params(x1, B.conv_desc(4, 16, 1, 1, 1, 0, True, B.DR_KCRS), torch.zeros((1, 4, 3, 3), device="cuda"),
                            torch.zeros((4, 16, 1, 1), device="cuda"), None, _ws(256))
