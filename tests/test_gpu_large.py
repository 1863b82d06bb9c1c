"""GPU parity of the bf16 channels-last convolution at the sizes where the streaming kernel hands over to the
other kernels: more than 2^24 output pixels in one call, and an input of 2 GiB or more (64-bit indexing).
The input is a seeded block repeated down the image (row h holds block row h % rows), so that the host never
holds the whole tensor; the oracle computes sampled output pixels one by one from their input windows."""
import numpy as np
import pytest

import oracle
import workloads
from paper_1708_04728_amd import binding as B
from util import TOL_BF16, gpu, close, rel_err

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _window(block, H, W, p, q, R, S, pad):
    """Input window of output pixel (p, q) at stride 1 as a (1, C, R, S) array, zeros outside the image."""
    C, rows, _ = block.shape
    out = np.zeros((1, C, R, S), dtype=np.float32)
    for r in range(R):
        for s in range(S):
            ih, iw = p + r - pad, q + s - pad
            if 0 <= ih < H and 0 <= iw < W:
                out[0, :, r, s] = block[:, ih % rows, iw]
    return out


def _run(C, H, W, K, R, pad, rows, seed, marks):
    rng = np.random.default_rng(seed)
    block = workloads.round_to_bf16(rng.standard_normal((C, rows, W)).astype(np.float32))
    w = workloads.round_to_bf16(rng.standard_normal((K, C, R, R)).astype(np.float32) * np.float32(np.sqrt(2.0 / (C * R * R))))
    b = (rng.standard_normal((K,)) * 0.1).astype(np.float32)
    assert H % rows == 0
    xb = torch.from_numpy(np.ascontiguousarray(np.transpose(block, (1, 2, 0)))).to(torch.bfloat16).cuda()      # (rows, W, C)
    x = B.NHWC(xb.repeat(H // rows, 1, 1).reshape(1, H, W, C))
    del xb
    y = B.NHWC(torch.empty((1, H, W, K), dtype=torch.bfloat16, device="cuda"))
    wg = B.pack_filters(gpu(w, "bf16")) if B.can_pack(C, "bf16") else gpu(w, "bf16")
    cd = B.conv_desc(K, C, R, R, 1, pad, True, B.DR_KRSC if B.can_pack(C, "bf16") else B.DR_KCRS)
    B.conv2d_fwd(x, cd, wg, gpu(b), y)
    torch.cuda.synchronize()
    pix = {0, W - 1, (H - 1) * W, H * W - 1, H * W // 2}
    for m in marks:
        pix.update(n for n in (m - 1, m, m + 1) if 0 <= n < H * W)
    pix.update(int(v) for v in rng.integers(0, H * W, 300))
    pix = sorted(pix)
    idx = torch.tensor(pix, dtype=torch.long, device="cuda")
    got = y.t.reshape(H * W, K)[idx].float().cpu().numpy().astype(np.float64)
    ref = np.stack([oracle.conv2d(_window(block, H, W, n // W, n % W, R, R, pad), w, b, 1, 0, True)[0, :, 0, 0] for n in pix])
    assert close(got, ref, TOL_BF16)


def test_conv_bf16_more_than_2_to_24_output_pixels():
    # 4200 x 4200 = 17.6 M output pixels in one call (the streaming kernel indexes at most 2^24)
    _run(C=8, H=4200, W=4200, K=16, R=3, pad=1, rows=600, seed=21, marks=[1 << 24])


def test_conv_bf16_input_of_more_than_2_gib():
    # 11600 x 11600 x 8 bf16 = 2.15 GB: byte offsets beyond 32 bits, in the input and in the output
    H = W = 11600
    _run(C=8, H=H, W=W, K=8, R=3, pad=1, rows=400, seed=22, marks=[(1 << 31) // 16, (1 << 32) // 16 if (1 << 32) // 16 < H * W else H * W - 2])
