"""Host-side checks of the C ABI: the library loads, exports every symbol the header declares,
rejects bad arguments before touching a GPU, and its host-only routines (shape rules, Lemma 2
fold) agree with the oracle.  No GPU needed."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import workloads
from paper_1708_04728_amd import binding as B, graph as G, slim

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(dr_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = C.CDLL(B.LIB_PATH)
    syms = declared_symbols()
    assert len(syms) >= 25
    for name in syms:
        assert hasattr(lib, name), name
    assert set(B._SIGNATURES) == set(syms)
    assert B.lib().dr_version().decode().startswith("deeprebirth")


def test_shape_rules_match_oracle():
    for n in range(1, 40):
        for k in (1, 2, 3, 5, 7, 11):
            for s in (1, 2, 3, 4, 8):
                for pad in (0, 1, 2, 3):
                    assert B.conv_out_size(n, k, s, pad) == oracle.conv_out_size(n, k, s, pad), (n, k, s, pad)
                    if pad < k:
                        assert B.pool_out_size(n, k, s, pad) == oracle.pool_out_size(n, k, s, pad), (n, k, s, pad)


def _t(n, c, h, w, dt=B.DR_F32):
    return B.dr_tensor(n, c, h, w, dt)


def test_argument_validation_runs_before_any_launch():
    L = B.lib()
    xd, yd = _t(1, 4, 8, 8), _t(1, 6, 8, 8)
    cd = B.conv_desc(6, 4, 3, pad=1)
    fake = C.c_void_p(4096)   # never dereferenced: every call below must fail in validation
    assert L.dr_conv2d_fwd(xd, None, cd, fake, None, yd, fake, 0, None) == B.DR_ERR_NULL
    assert "NULL" in B.last_error()
    assert L.dr_conv2d_fwd(xd, fake, cd, fake, None, _t(1, 6, 7, 8), fake, 0, None) == B.DR_ERR_SHAPE
    assert L.dr_conv2d_fwd(xd, fake, cd, fake, None, yd, fake, 1, None) == B.DR_ERR_SHAPE        # channels overflow
    assert L.dr_conv2d_fwd(_t(1, 5, 8, 8), fake, cd, fake, None, yd, fake, 0, None) == B.DR_ERR_SHAPE
    assert L.dr_conv2d_fwd(xd, fake, B.conv_desc(6, 4, 3, stride=0), fake, None, yd, fake, 0, None) == B.DR_ERR_SHAPE
    assert L.dr_conv2d_fwd(_t(1, 4, 8, 8, 7), fake, cd, fake, None, yd, fake, 0, None) == B.DR_ERR_UNSUPPORTED
    assert L.dr_slim_conv_fwd(xd, fake, cd, 2, 2, fake, None, yd, fake, 0, None) == B.DR_ERR_SHAPE   # needs 4x4 output
    assert L.dr_maxpool_fwd(xd, fake, B.pool_desc(3, 2), _t(1, 4, 3, 3), fake, None) == B.DR_ERR_SHAPE  # ceil rule: 4x4
    assert L.dr_maxpool_fwd(xd, fake, B.pool_desc(3, 2, 3), _t(1, 4, 4, 4), fake, None) == B.DR_ERR_SHAPE  # pad >= window
    assert L.dr_lrn_fwd(xd, fake, B.dr_lrn(0, 1e-4, 0.75, 1.0), fake, None) in (B.DR_ERR_SHAPE, B.DR_ERR_UNSUPPORTED)
    assert L.dr_relu(None, fake, fake, None) == B.DR_ERR_NULL
    xds = (B.dr_tensor * 2)(_t(1, 2, 4, 4), _t(1, 3, 4, 4))
    ptrs = (C.c_void_p * 2)(4096, 8192)
    assert L.dr_concat(2, xds, ptrs, _t(1, 6, 4, 4), fake, None) == B.DR_ERR_SHAPE
    assert L.dr_concat(9, xds, ptrs, _t(1, 5, 4, 4), fake, None) == B.DR_ERR_SHAPE
    assert L.dr_softmax_fwd(_t(2, 10, 2, 1), fake, fake, None) == B.DR_ERR_SHAPE
    # inner product: i runs over (c, h, w), which a channels-last map larger than 1x1 does not store in that order
    nhwc = B.dr_tensor(2, 8, 3, 3, B.DR_F32, B.DR_NHWC)
    assert L.dr_fc_fwd(nhwc, fake, fake, None, _t(2, 5, 1, 1), fake, None) == B.DR_ERR_UNSUPPORTED
    assert "channels-last" in B.last_error()


def test_sizes_beyond_the_kernels_index_range_are_refused_on_the_host():
    L = B.lib()
    fake = C.c_void_p(4096)   # never dereferenced
    huge = _t(1 << 11, 1 << 10, 1 << 5, 1 << 5)          # 2^31 elements
    assert L.dr_relu(huge, fake, fake, None) == B.DR_ERR_UNSUPPORTED and "2^31" in B.last_error()
    # fp32 convolution: the kernel addresses its operands with 32-bit byte offsets
    xd, yd = _t(1, 16, 8192, 8192), _t(1, 1, 8192, 8192)  # input of 4 GiB
    assert L.dr_conv2d_fwd(xd, fake, B.conv_desc(1, 16, 1), fake, None, yd, fake, 0, None) == B.DR_ERR_UNSUPPORTED
    assert "GiB" in B.last_error()


def test_inception_and_net_planning_on_host():
    layers = workloads.CONFIGS[2]["original"]
    d = G.inception_desc(layers[0][1], 192, 0)
    assert d.n_branches == 4 and [d.branches[i].n_steps for i in range(4)] == [1, 2, 2, 2]
    n = C.c_size_t(0)
    xd = _t(32, 192, 28, 28)
    assert B.lib().dr_inception_workspace_bytes(xd, d, C.byref(n)) == B.DR_OK
    # layer-by-layer form keeps every branch tensor: 64+96+128+16+32+192+32 channels of 32x28x28 fp32; on top of
    # that, the scratch of those convolutions that would leave compute units idle (each rounded up to 256 bytes)
    def scratch(c_in, k, r):
        m = C.c_size_t(0)
        assert B.lib().dr_conv2d_workspace_bytes(_t(32, c_in, 28, 28), B.conv_desc(k, c_in, r, pad=r // 2), C.byref(m)) == B.DR_OK
        return (m.value + 255) // 256 * 256
    convs = [(192, 64, 1), (192, 96, 1), (96, 128, 3), (192, 16, 1), (16, 32, 5), (192, 32, 1)]
    assert scratch(96, 128, 3) == 0
    assert n.value == (64 + 96 + 128 + 16 + 32 + 192 + 32) * 32 * 784 * 4 + sum(scratch(*c) for c in convs)
    d2 = G.inception_desc(layers[0][1], 192, B.DR_FUSE_RELU | B.DR_FUSE_CONCAT)
    assert B.lib().dr_inception_workspace_bytes(xd, d2, C.byref(n)) == B.DR_OK
    assert n.value == (96 + 16 + 192) * 32 * 784 * 4 + sum(scratch(*c) for c in convs)
    # the query itself: whole [K][pixels] planes of partial sums for a one-image layer, nothing for bf16 or big layers
    m = C.c_size_t(0)
    assert B.lib().dr_conv2d_workspace_bytes(_t(1, 64, 56, 56), B.conv_desc(192, 64, 3, stride=2, pad=1), C.byref(m)) == B.DR_OK
    assert m.value > 0 and m.value % (192 * 784 * 4) == 0
    assert B.lib().dr_conv2d_workspace_bytes(_t(128, 64, 56, 56), B.conv_desc(192, 64, 3, pad=1), C.byref(m)) == B.DR_OK and m.value == 0
    assert B.lib().dr_conv2d_workspace_bytes(_t(1, 64, 56, 56, B.DR_BF16), B.conv_desc(192, 64, 3, pad=1), C.byref(m)) == B.DR_OK and m.value == 0
    assert B.lib().dr_conv2d_workspace_bytes(_t(1, 32, 56, 56), B.conv_desc(192, 64, 3, pad=1), C.byref(m)) == B.DR_ERR_SHAPE
    assert B.lib().dr_conv2d_fwd_ws(_t(1, 64, 56, 56), C.c_void_p(4096), B.conv_desc(192, 64, 3, stride=2, pad=1), C.c_void_p(4096), None,
                                    _t(1, 192, 28, 28), C.c_void_p(4096), 0, None, 0, None) == B.DR_ERR_WORKSPACE
    bad = G.inception_desc(layers[0][1], 100, 0)
    assert B.lib().dr_inception_workspace_bytes(xd, bad, C.byref(n)) == B.DR_ERR_SHAPE

    for form in ("original", "slim"):
        net = B.Net(G.net_descs(workloads.CONFIGS[5][form], 3, fuse_relu=(form == "slim")))
        assert net.num_params() == 2 * len(workloads.make_params(5, form))
        yd = net.output_desc(_t(4, 3, 224, 224, B.DR_BF16))
        assert (yd.n, yd.c, yd.h, yd.w, yd.dtype) == (4, 1000, 1, 1, B.DR_F32)
        assert net.workspace_bytes(_t(4, 3, 224, 224, B.DR_BF16)) > 0
    net = B.Net(G.net_descs(workloads.CONFIGS[4]["original"], 64))
    assert net.num_params() == 6 * 4 + 6 * 3 + 6 * 3
    yd = net.output_desc(_t(2, 64, 56, 56, B.DR_BF16))
    assert (yd.n, yd.c, yd.h, yd.w) == (2, 256, 56, 56)
    net = B.Net(G.net_descs(workloads.CONFIGS[1]["original"], 64))
    with pytest.raises(B.DeepRebirthError):
        net.output_desc(_t(2, 32, 56, 56))


def test_fold_bn_host_matches_lemma2():
    rng = np.random.default_rng(5)
    w = rng.standard_normal((7, 3, 3, 3)).astype(np.float32)
    b = rng.standard_normal(7).astype(np.float32)
    g, be = rng.uniform(0.5, 1.5, 7).astype(np.float32), rng.standard_normal(7).astype(np.float32)
    mu, var = rng.standard_normal(7).astype(np.float32), rng.uniform(0.5, 1.5, 7).astype(np.float32)
    wf, bf = B.fold_bn(w, b, g, be, mu, var, 1e-5)
    # fp32 eps is not exactly 1e-5: hand the oracle the value the library saw
    wo, bo = oracle.fold_bn(w, b, g, be, mu, var, float(np.float32(1e-5)))
    np.testing.assert_allclose(wf, wo, rtol=1e-7)
    np.testing.assert_allclose(bf, bo, rtol=2e-7, atol=1e-7)
    assert np.array_equal(wf, wo.astype(np.float32)) and np.array_equal(bf, bo.astype(np.float32))


def test_slim_transforms_reproduce_the_configurations():
    for cid in (1, 2, 3, 5):
        assert slim.slim_network(workloads.CONFIGS[cid]["original"]) == workloads.CONFIGS[cid]["slim"], cid
    # stride rule: new stride = conv stride x pool stride; LRN dropped; ReLU kept
    s = slim.streamline_slim(workloads.CONFIGS[3]["original"])
    assert [k for k, _ in s] == ["conv", "relu", "conv", "relu"]
    assert s[0][1]["stride"] == 8 and s[2][1]["stride"] == 2
    # branch slimming keeps the concatenated width
    for name, wd in workloads.INCEPTION_WIDTHS.items():
        br = slim.branch_slim(workloads.inception_original(name))[1]["branches"]
        assert len(br) == 2
        assert br[0][2][1]["k"] + br[1][2][1]["k"] == wd[1] + wd[3] + wd[5] + wd[6]
        assert br[1][2][1]["r"] == 5


def test_stack_first_steps_lays_reducers_back_to_back():
    """graph.stack_first_steps (the parameter layout DR_FUSE_STACK looks for, Eq. (12)): the first-step 1x1
    convolutions of every module end up adjacent in memory in branch order, values unchanged, everything
    else untouched."""
    layers = workloads.CONFIGS[5]["original"][10:12] + [workloads.CONFIGS[5]["slim"][6]]     # 3a, 3b, slim 3a
    assert all(kind == "inception" for kind, _ in layers)
    per = [sum(1 for br in p["branches"] for k, _ in br if k == "conv") for _, p in layers]
    # any parameter dicts of the right shapes will do: build them from the layer lists
    rng = np.random.default_rng(0)
    dicts, c = [], 192
    for kind, p in layers:
        outc = 0
        for br in p["branches"]:
            ci = c
            for k, q in br:
                if k == "conv":
                    dicts.append({"w": rng.standard_normal((q["k"], ci, q["r"], q["s"])).astype(np.float32), "b": rng.standard_normal(q["k"]).astype(np.float32)})
                    ci = q["k"]
            outc += ci
        c = outc if kind == "inception" else c
        c = 192 if layers.index((kind, p)) == 1 else c          # the third module is another 3a: 192 channels in again
    flat = G.flat_params(dicts, "f32", device="cpu", pack=False)
    stacked = G.stack_first_steps(layers, flat)
    assert len(stacked) == len(flat) == 2 * sum(per)
    for a, b in zip(flat, stacked):
        assert a.shape == b.shape and bool((a == b).all())
    pos = 0
    for (kind, p), n in zip(layers, per):
        first, j = [], pos
        for br in p["branches"]:
            if br[0][0] == "conv" and br[0][1]["r"] == 1:
                first.append(j)
            j += 2 * sum(1 for k, _ in br if k == "conv")
        assert len(first) >= 2
        for f0, f1 in zip(first, first[1:]):
            w0, w1, b0, b1 = stacked[f0], stacked[f1], stacked[f0 + 1], stacked[f1 + 1]
            assert w1.data_ptr() == w0.data_ptr() + w0.numel() * w0.element_size()
            assert b1.data_ptr() == b0.data_ptr() + b0.numel() * b0.element_size()
        pos = j
