"""dr_conv2d_fwd_static: the convolution whose contraction is cut over workgroups, on scratch memory the library
holds itself (for callers that cannot allocate).  Called through the C ABI; its output must be, bit for bit, that
of dr_conv2d_fwd_ws on caller-supplied scratch, and within the fp32 tolerance of the oracle -- on two calls in a
row, the second on a smaller input (the shared array still holds the first call's partial sums)."""
import ctypes as C

import numpy as np
import pytest

import oracle
from paper_1708_04728_amd import binding as B
from util import TOL_F32, close, gpu, host

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _case(seed, N, Cc, H, W, K, R, S, stride, pad):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, Cc, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, Cc, R, S)) * np.sqrt(2.0 / (Cc * R * S))).astype(np.float32)
    b = (rng.standard_normal(K) * 0.1).astype(np.float32)
    return x, w, b, B.conv_desc(K, Cc, R, S, stride, pad, True, B.DR_KCRS)


def _both_ways(x, w, b, cd, stride, pad):
    L = B.lib()
    xg, wg, bg = gpu(x), gpu(w), gpu(b)
    ref = oracle.conv2d(x, w, b, stride, pad, True)
    need = B.conv2d_workspace_bytes(xg, cd)
    assert 0 < need <= B.STATIC_SCRATCH_BYTES           # a layer that is cut, and whose partial sums fit
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")
    y_ws = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    y_st = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    B.conv2d_fwd_ws(xg, cd, wg, bg, y_ws, ws)
    torch.cuda.synchronize()
    # the entry point itself, straight through ctypes: descriptors, device pointers, the current stream
    xd, yd = B.desc(xg), B.desc(y_st)
    rc = L.dr_conv2d_fwd_static(xd, C.c_void_p(xg.data_ptr()), cd, C.c_void_p(wg.data_ptr()), C.c_void_p(bg.data_ptr()), yd,
                                C.c_void_p(y_st.data_ptr()), 0, C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == B.DR_OK, B.last_error()
    torch.cuda.synchronize()
    assert torch.equal(y_st, y_ws)                      # same kernels, same order of the sums: same bits
    assert close(host(y_st), ref, TOL_F32)
    return need


def test_static_scratch_matches_caller_scratch_twice_in_a_row():
    # the one-image streamline block of the paper's Fig. 3 setting at stride 2 (7.2 MB of partial sums), then a smaller layer
    first = _case(1, 1, 64, 56, 56, 192, 3, 3, 2, 1)
    n1 = _both_ways(*first, 2, 1)
    second = _case(2, 1, 48, 14, 14, 40, 3, 3, 1, 1)
    n2 = _both_ways(*second, 1, 1)
    assert n2 < n1
    # and the first again: nothing of the smaller call is left in the way
    _both_ways(*first, 2, 1)


def test_static_scratch_refuses_what_does_not_fit_and_passes_on_what_needs_none():
    L = B.lib()
    fake = C.c_void_p(4096)   # never dereferenced: refused in validation
    xd = B.dr_tensor(1, 128, 40, 40, B.DR_F32)
    cd = B.conv_desc(64, 128, 7, 7, 1, 3, True, B.DR_KCRS)
    need = C.c_size_t(0)
    assert L.dr_conv2d_workspace_bytes(xd, cd, C.byref(need)) == B.DR_OK and need.value > B.STATIC_SCRATCH_BYTES
    assert L.dr_conv2d_fwd_static(xd, fake, cd, fake, None, B.dr_tensor(1, 64, 40, 40, B.DR_F32), fake, 0, None) == B.DR_ERR_WORKSPACE
    assert "dr_conv2d_fwd_ws" in B.last_error()
    # a layer that is not cut (enough tiles for the device) uses no scratch: same result as dr_conv2d_fwd
    x, w, b, cd = _case(3, 6, 16, 40, 40, 64, 3, 3, 1, 1)
    xg, wg, bg = gpu(x), gpu(w), gpu(b)
    assert B.conv2d_workspace_bytes(xg, cd) == 0
    ref = oracle.conv2d(x, w, b, 1, 1, True)
    y0 = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    y1 = torch.full(ref.shape, float("nan"), dtype=torch.float32, device="cuda")
    B.conv2d_fwd(xg, cd, wg, bg, y0)
    B.conv2d_fwd_static(xg, cd, wg, bg, y1)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and close(host(y1), ref, TOL_F32)
