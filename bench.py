#!/usr/bin/env python3
"""Benchmark of the forward hot path on one MI355X: original form vs slim form.

One "step" = one forward pass of the ORIGINAL block (layer by layer: conv, ReLU, LRN / max-pool /
concat / BatchNorm kernels as separate passes, the form the paper times) followed by one forward
pass of the SLIM block (slimmed structure, ReLU in the conv store, branches written straight into
the concatenated tensor, BatchNorm folded), both over the same batch already resident in HBM.

Prints ONE JSON line: whole-step throughput (`value`, images/s through both forms), the per-form
times and the slim/original speed-up, the roofline of the dominant kernel (measured with HIP events
around that kernel inside the timed region), the CPU oracle timed on the host cores, and a short
summary of the other configurations (`all_configs`).

The default workload is the full GoogLeNet-v1 forward at batch 128 in bf16 (the network the headline
metric names); `--config N` selects another of the five configurations.

`--calibrate-copy` runs only a plain elementwise kernel (ReLU, one read and one write of 256 MiB) a
few times: the known-size reference against which hardware byte counters are scaled when the HBM
traffic of the dominant kernel is measured with rocprofv3 (see profiles/).
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MI355X_HBM_GBS = 8000.0
MI355X_MFMA_TFLOPS = {"f32": 157.3, "bf16": 2500.0}

WORKLOAD_NAMES = {
    1: "config 1: GoogLeNet conv2 streamline block, batch 1, fp32 NCHW, 64x56x56 -> 192x28x28",
    2: "config 2: GoogLeNet inception(3a), batch 32, fp32 NCHW, 192x28x28 -> 256x28x28",
    3: "config 3: AlexNet front end (conv1+conv2 blocks), batch 128, fp32 NCHW, 3x227x227",
    4: "config 4: ResNet-50 conv2_x stage (3 bottlenecks), batch 128, bf16 NHWC / fp32 accumulate, 64x56x56",
    5: "config 5: GoogLeNet-v1 forward, batch 128, bf16 NHWC / fp32 accumulate, 3x224x224 -> 1000",
}


# sources a launch's kernel can come from, by trace label (the bf16 convolution picks one of several kernels by rule)
KERNEL_SOURCES = {"conv_bf16": ["conv_bf16.hip", "conv_bf16_dma.hip", "conv_bf16_patch.hip", "conv_bf16_rows.hip", "conv_bf16_dev.h"],
                  "conv_f32": ["conv_f32.hip"]}


def kernel_source_hash(label):
    """SHA-256 over the source files of the kernels behind a trace label, or None for a label without an entry."""
    srcs = KERNEL_SOURCES.get(label)
    if srcs is None:
        return None
    h = hashlib.sha256()
    for src in srcs:
        with open(os.path.join(ROOT, "paper_1708_04728_amd", "csrc", src), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(kernel_desc, label):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, or
    None when there is no summary for this kernel or its sources have changed since it was taken."""
    sha = kernel_source_hash(label)
    if sha is None:
        return None
    pdir = os.path.join(ROOT, "profiles")
    for name in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not name.endswith("_hbm_traffic.md"):
            continue
        text = open(os.path.join(pdir, name)).read()
        fields = dict(re.findall(r"^([a-z_0-9]+):\s*(.+?)\s*$", text, re.M))
        if fields.get("kernel") == kernel_desc and fields.get("source_sha256") == sha:
            try:
                return float(fields["traffic_bytes_per_launch"])
            except (KeyError, ValueError):
                return None
    return None


NON_TENSOR_SOURCES = ["pointwise_nhwc.hip", "pointwise.hip", "dr_store.h"]


def non_tensor_from_kernel_trace(cfg_id):
    """Non-tensor throughput from KERNEL durations (the committed rocprofv3 kernel trace of `bench.py --layer-trace`,
    profiles/layers_config<N>_kernel_trace.md), which leave out the gap between dependent launches that the HIP-event pairs
    of this process include; None when there is no such summary or the non-tensor kernels' sources have changed since."""
    path = os.path.join(ROOT, "profiles", "layers_config%d_kernel_trace.md" % cfg_id)
    if not os.path.isfile(path):
        return None
    h = hashlib.sha256()
    for src in NON_TENSOR_SOURCES:
        with open(os.path.join(ROOT, "paper_1708_04728_amd", "csrc", src), "rb") as f:
            h.update(f.read())
    fields = dict(re.findall(r"^([a-z_0-9]+):\s*(.+?)\s*$", open(path).read(), re.M))
    if fields.get("non_tensor_source_sha256") != h.hexdigest():
        return None
    try:
        return {"all_gbs": float(fields["non_tensor_gbs_all"]), "launches_over_32MB_gbs": float(fields["non_tensor_gbs_over_32mb"]),
                "source": "profiles/layers_config%d_kernel_trace.md (rocprofv3 kernel durations)" % cfg_id}
    except (KeyError, ValueError):
        return None


def calibrate_copy():
    """One read + one write of 256 MiB, three times, through the library's ReLU kernel."""
    import torch

    from paper_1708_04728_amd import binding as B
    n = 64 * 1024 * 1024
    x = torch.ones((1, 1, 1, n), dtype=torch.float32, device="cuda")
    y = torch.empty_like(x)
    for _ in range(3):
        B.relu(x, y)
    torch.cuda.synchronize()
    print(json.dumps({"calibration": "dr_relu", "bytes_read": 4 * n, "bytes_written": 4 * n, "launches": 3}))


def ceilings():
    """What this GPU sustains on the resources the kernels are graded against, from the measuring kernels in
    libdr_ceilings.so (register-only matrix instructions; a plain 16-byte copy at several sizes; reads of a buffer that
    stays in the caches), timed with HIP events, best of five launches each.  One JSON line."""
    import ctypes as C

    import torch
    lib = C.CDLL(os.path.join(ROOT, "paper_1708_04728_amd", "libdr_ceilings.so"))
    vp, z, i = C.c_void_p, C.c_size_t, C.c_int
    lib.drc_mfma_bf16.argtypes = lib.drc_mfma_f32.argtypes = lib.drc_mfma_bf16_data.argtypes = [vp, i, i, vp]
    lib.drc_copy16.argtypes = [vp, vp, z, i, vp]
    lib.drc_read16.argtypes = [vp, vp, z, i, i, vp]
    lib.drc_fill16.argtypes = [vp, z, i, vp]
    lib.drc_kstep.argtypes = [i, vp, i, i, vp, vp]
    st = torch.cuda.current_stream()
    sp = vp(st.cuda_stream)
    out = torch.zeros(1024, dtype=torch.float32, device="cuda")

    def best_ms(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            assert fn() == 0
            e1.record(st)
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return min(ts)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    res = {"compute_units": cus, "mfma": {}, "copy": {}, "fill": {}, "cache_read": {}, "kstep_cycles": {}}
    iters = 20000
    for wg_per_cu in (1, 2):
        blocks = cus * wg_per_cu
        ms = best_ms(lambda: lib.drc_mfma_bf16(vp(out.data_ptr()), iters, blocks, sp))
        res["mfma"]["bf16_32x32x16_tflops_%dwave_per_simd" % wg_per_cu] = round(2.0 * 32 * 32 * 16 * 4 * iters * 4 * blocks / (ms * 1e-3) / 1e12, 1)
        ms = best_ms(lambda: lib.drc_mfma_bf16_data(vp(out.data_ptr()), iters, blocks, sp))
        res["mfma"]["bf16_32x32x16_tflops_%dwave_per_simd_varying_operands" % wg_per_cu] = round(2.0 * 32 * 32 * 16 * 4 * iters * 4 * blocks / (ms * 1e-3) / 1e12, 1)
        ticks = out[:2].tolist()
        res["mfma"]["shader_clock_GHz_%dwave_per_simd_varying_operands" % wg_per_cu] = round(ticks[0] / max(ticks[1], 1.0) * 0.1, 3)
        ms = best_ms(lambda: lib.drc_mfma_f32(vp(out.data_ptr()), iters, blocks, sp))
        res["mfma"]["f32_32x32x2_tflops_%dwave_per_simd" % wg_per_cu] = round(2.0 * 32 * 32 * 2 * 4 * iters * 4 * blocks / (ms * 1e-3) / 1e12, 1)
    for mib in (8, 32, 64, 128, 256, 512, 1024):
        n = mib << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        ms = best_ms(lambda: lib.drc_copy16(vp(src.data_ptr()), vp(dst.data_ptr()), n, cus * 8, sp))
        res["copy"]["%d_MiB_read_plus_write_GBs" % mib] = round(2.0 * n / (ms * 1e-3) / 1e9, 1)
        del src, dst
    for mib in (64, 256, 1024):
        n = mib << 20
        dst = torch.empty(n, dtype=torch.uint8, device="cuda")
        ms = best_ms(lambda: lib.drc_fill16(vp(dst.data_ptr()), n, cus * 8, sp))
        res["fill"]["%d_MiB_write_GBs" % mib] = round(float(n) / (ms * 1e-3) / 1e9, 1)
        del dst
    # one k-step of the bf16 convolutions' inner loop in isolation (6 matrix instructions = 192 cycles of matrix work on 5 LDS
    # reads), shader-clock cycles per k-step and wave: one workgroup of four waves per compute unit, then two
    filt = torch.ones(96 * 1152 + 4096, dtype=torch.uint8, device="cuda")
    names = ("matrix_instructions_only", "with_lds_reads_one_step_ahead", "with_drain_and_barrier_every_4_steps", "with_next_filter_slice_by_dma")
    for wg_per_cu in (1, 2):
        blocks = cus * wg_per_cu
        ticks = torch.zeros(4 * blocks, dtype=torch.float32, device="cuda")
        for mode, name in enumerate(names):
            assert lib.drc_kstep(mode, vp(ticks.data_ptr()), 2000, blocks, vp(filt.data_ptr()), sp) == 0
            torch.cuda.synchronize()
            t = ticks.cpu()
            res["kstep_cycles"]["%s_%dwg_per_cu" % (name, wg_per_cu)] = {"mean": round(float(t.mean()), 1), "min": round(float(t.min()), 1), "max": round(float(t.max()), 1)}
    for kib in (64, 1024):
        n = kib << 10
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        passes, blocks = (4096 if kib == 64 else 256), cus * 2
        ms = best_ms(lambda: lib.drc_read16(vp(src.data_ptr()), vp(out.data_ptr()), n, passes, blocks, sp))
        res["cache_read"]["%d_KiB_buffer_GBs" % kib] = round(float(n) * passes * blocks / (ms * 1e-3) / 1e9, 1)
    print(json.dumps({"ceilings": res, "published": {"hbm_GBs": MI355X_HBM_GBS, "mfma_tflops": MI355X_MFMA_TFLOPS}}))


def layer_trace(cfg_id):
    """For a run under `rocprofv3 --kernel-trace`: every form's forward four times, kernel by kernel with the branches of
    a module in turn, each forward preceded by a marker kernel (torch's cos_ on 7 floats), so that the kernels of the
    trace between two markers can be matched, in order, with the launches the library reports for that form.  Prints
    one JSON line: per form the launches as [label, K, C, R, S, items, algorithmic bytes]."""
    import torch
    wl = Workload(cfg_id, serial_branches=True)
    for _ in range(3):
        wl.step()
    torch.cuda.synchronize()
    labels = {form: [list(r[:6]) + [r[7]] for r in wl.trace(form)] for form in wl.forms}
    torch.cuda.synchronize()
    marker = torch.zeros(7, device="cuda")
    for form in wl.forms:
        for _ in range(4):
            marker.cos_()
            torch.cuda.synchronize()
            wl.run(form)
            torch.cuda.synchronize()
    marker.cos_()
    torch.cuda.synchronize()
    print(json.dumps({"layer_trace": labels, "config": cfg_id, "forwards_per_form": 4, "marker": "cos"}))


def paper_variant_ms(wl, reps=20, x=None):
    """The module of Sec. 3.2 slimmed the way the paper's own example does it (3x3 reducer 96 -> 48, the 1x1
    branch absorbed into a 3x3 of 192 filters, the pool branch into a 5x5 of 64 filters), on config 2's input,
    run like the slim form: best time of `reps` runs in ms."""
    import torch

    import workloads
    B, G = wl.B, wl.G
    layer = workloads.inception_3a_paper_variant()
    params = workloads.make_params(2, "slim", layers=[layer])
    bf16 = wl.dtype == "bf16"
    x = wl.x if x is None else x
    mode = B.DR_FUSE_RELU | B.DR_FUSE_CONCAT | (B.DR_FUSE_STACK if bf16 else 0)
    net = B.Net(G.net_descs([layer], 192, inception_mode=mode, fuse_relu=True, pack=wl.dtype))
    xd = B.desc(x)
    y = G.empty_like_desc(net.output_desc(xd))
    ws = torch.empty(max(net.workspace_bytes(xd), 256), dtype=torch.uint8, device="cuda")
    flat = G.flat_params(params, wl.dtype, pack=True)
    if bf16:
        flat = G.stack_first_steps([layer], flat)
    best = 1e9
    for i in range(reps + 3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(wl.stream)
        net.fwd(x, flat, y, ws, wl.stream)
        e1.record(wl.stream)
        e1.synchronize()
        if i >= 3:
            best = min(best, e0.elapsed_time(e1))
    return best


def paper_variant_3a(wl):
    """Config 5's inception 3a (batch 128, bf16, 28 x 28 x 192 input) in three structures: the original module, the benchmark's
    slim variant (both removed branches absorbed into the 5x5) and the paper's own example (Sec. 3.2), each run alone on a
    seeded input of the module's shape, best of 20 runs in ms."""
    import numpy as np
    import torch

    import workloads
    B, G = wl.B, wl.G
    rng = np.random.default_rng(31)
    xh = workloads.round_to_bf16(np.abs(rng.standard_normal((wl.batch, 192, 28, 28))).astype(np.float32))
    x = G.to_device(xh, "bf16", nhwc=True)
    out = {"paper_variant_ms": round(paper_variant_ms(wl, x=x), 4)}
    for form, key in (("original", "original_ms"), ("slim", "benchmark_slim_ms")):
        layer = [l for l in workloads.CONFIGS[5][form] if l[0] == "inception"][0]
        params = workloads.make_params(2, form, layers=[layer])
        slim = form == "slim"
        mode = (B.DR_FUSE_RELU | B.DR_FUSE_CONCAT | B.DR_FUSE_STACK) if slim else 0
        net = B.Net(G.net_descs([layer], 192, inception_mode=mode, fuse_relu=slim, pack="bf16"))
        xd = B.desc(x)
        y = G.empty_like_desc(net.output_desc(xd))
        ws = torch.empty(max(net.workspace_bytes(xd), 256), dtype=torch.uint8, device="cuda")
        flat = G.flat_params(params, "bf16", pack=True)
        if slim:
            flat = G.stack_first_steps([layer], flat)
        best = 1e9
        for i in range(23):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(wl.stream)
            net.fwd(x, flat, y, ws, wl.stream)
            e1.record(wl.stream)
            e1.synchronize()
            if i >= 3:
                best = min(best, e0.elapsed_time(e1))
        out[key] = round(best, 4)
    return out


def slim_layer_regression(batch=32, iters=40, lr=2e-7):
    """Sec. 3.1, Lemma 1 on config 1's block: the slim layer (3x3, 64 -> 192, stride 2, ReLU) is learned by gradient
    descent on sum || Y - f~(W, b; X) ||^2, Y being the output of the original block (conv - ReLU - LRN - pool) on
    `batch` seeded images, from fresh He-normal weights.  A toy: it shows the loss falling and what one step
    costs, not accuracy.  Everything runs in the library's kernels; times from HIP events."""
    import numpy as np
    import torch

    import workloads
    from paper_1708_04728_amd import binding as B, graph as G
    x = workloads.make_input(1, batch)
    c_in = x.shape[1]
    xg = G.to_device(x, "f32")
    stream = torch.cuda.current_stream()
    net = B.Net(G.net_descs(workloads.CONFIGS[1]["original"], c_in))
    xd = B.desc(xg)
    y = G.empty_like_desc(net.output_desc(xd))
    ws = torch.empty(max(net.workspace_bytes(xd), 256), dtype=torch.uint8, device="cuda")
    net.fwd(xg, G.flat_params(workloads.make_params(1, "original"), "f32"), y, ws, stream)      # the target feature map
    q = workloads.make_params(1, "slim")[0]
    w, b = G.to_device(q["w"], "f32"), G.to_device(q["b"], "f32")
    k, c, r, s = w.shape
    cd1 = B.conv_desc(k, c, r, s, 1, 1, False, B.DR_KCRS)        # dr_slim_conv_fwd multiplies the stride by the pool's
    cd2 = B.conv_desc(k, c, r, s, 2, 1, True, B.DR_KCRS)
    f = torch.empty_like(y)
    dw, db, loss = torch.empty_like(w), torch.empty_like(b), torch.zeros(1, device="cuda")
    ws2 = torch.empty(max(B.conv2d_bwd_params_workspace_bytes(xg, cd2), B.regression_loss_workspace_bytes(), 256), dtype=torch.uint8, device="cuda")
    losses = []

    def step(record):
        B.slim_conv_fwd(xg, cd1, 2, w, b, f, stream=stream)
        B.regression_loss_grad(f, y, f, loss, ws2, stream)
        if record:
            losses.append(float(loss.item()))
        B.conv2d_bwd_params(xg, cd2, f, dw, db, ws2, stream)
        B.sgd_step(w, dw, lr, stream)
        B.sgd_step(b, db, lr, stream)

    for _ in range(iters):
        step(True)
    # one traced step for the per-kernel times, then the cost of a step without host round trips
    B.trace_begin("", capacity=64)
    step(False)
    recs = B.trace_end(64)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(10):
        step(False)
    e1.record(stream)
    e1.synchronize()
    wg = [r_ for r_ in recs if r_[0].startswith("conv_wgrad")][0]
    wg_tf = conv_flops(wg) / (wg[6] * 1e-3) / 1e12
    return {"layer": "3x3 %d->%d stride 2 on %dx%d, batch %d, fp32" % (c, k, x.shape[2], x.shape[3], batch), "iterations": iters, "lr": lr,
            "loss_first": round(losses[0], 1), "loss_last": round(losses[-1], 1), "loss_ratio": round(losses[-1] / losses[0], 4),
            "monotone": all(b_ < a_ for a_, b_ in zip(losses, losses[1:])),
            "ms_per_step": round(e0.elapsed_time(e1) / 10, 4), "kernels_ms": {r_[0]: round(r_[6], 4) for r_ in recs},
            "wgrad_tflops": round(wg_tf, 2), "wgrad_frac_of_fp32_mfma_peak": round(wg_tf / MI355X_MFMA_TFLOPS["f32"], 4)}


def conv_flops(rec):
    label, k, c, r, s, items = rec[:6]
    return 2.0 * k * c * r * s * items


def is_tensor(rec):
    return rec[0].startswith("conv") or rec[0] == "fc"


def launch_roof(rec, dtype):
    """(roof in ms, which roof binds) of one traced launch: a tensor layer is bounded by the slower of its FLOPs at the
    matrix-core peak of its dtype and its algorithmic bytes (input, filters, output once each) at the HBM peak; a
    non-tensor layer by its algorithmic bytes at the HBM peak."""
    esz = 2 if dtype == "bf16" else 4
    nbytes = float(rec[7]) if rec[7] > 0 else 2.0 * rec[5] * esz
    t_hbm = nbytes / (MI355X_HBM_GBS * 1e9) * 1e3
    if rec[0].startswith("conv"):
        t_mfma = conv_flops(rec) / (MI355X_MFMA_TFLOPS[dtype] * 1e12) * 1e3
        return (t_mfma, "mfma") if t_mfma >= t_hbm else (t_hbm, "hbm")
    return t_hbm, "hbm"


def network_roofline(recs, dtype, forward_ms):
    """Every launch of one forward graded against its own roof (launch_roof): the sums, the split into tensor and
    non-tensor layers, and the launches that lose the most time against their roof.  `measured_ms` of the whole
    forward is the forward's own best time (one graph launch); the per-launch times are HIP-event pairs of a
    kernel-by-kernel pass, which include the gap between dependent launches."""
    rows = []
    for r in recs:
        roof, bound = launch_roof(r, dtype)
        rows.append((r, roof, bound))
    def part(sel):
        rs = [x for x in rows if sel(x[0])]
        roof, meas = sum(x[1] for x in rs), sum(x[0][6] for x in rs)
        return {"launches": len(rs), "roof_ms": round(roof, 4), "measured_ms": round(meas, 4), "frac": round(roof / max(meas, 1e-9), 3),
                "mfma_bound": sum(1 for x in rs if x[2] == "mfma"), "hbm_bound": sum(1 for x in rs if x[2] == "hbm")}
    roof_all = sum(x[1] for x in rows)
    worst = sorted(rows, key=lambda x: x[1] - x[0][6])[:5]
    def name(r):
        return "%s %dx%d %d->%d n=%d" % (r[0], r[3], r[4], r[2], r[1], r[5]) if r[0].startswith("conv") else "%s n=%d" % (r[0], r[5])
    return {"roof_ms": round(roof_all, 4), "measured_ms": round(forward_ms, 4), "frac": round(roof_all / max(forward_ms, 1e-9), 3),
            "kernel_by_kernel_ms": round(sum(x[0][6] for x in rows), 4),
            "tensor": part(is_tensor), "non_tensor": part(lambda r: not is_tensor(r)),
            "most_time_lost": [{"launch": name(r), "bound": b, "roof_ms": round(roof, 5), "measured_ms": round(r[6], 5),
                                "frac": round(roof / max(r[6], 1e-9), 3)} for r, roof, b in worst]}


class Workload:
    """Both forms of one configuration, resident on the GPU."""

    def __init__(self, cfg_id, batch=None, serial_branches=False):
        import numpy as np
        import torch

        import workloads
        from paper_1708_04728_amd import binding as B, graph as G
        self.B, self.G, self.torch, self.np = B, G, torch, np
        self.cfg_id = cfg_id
        cfg = workloads.CONFIGS[cfg_id]
        self.dtype = cfg["dtype"]
        bf16 = self.dtype == "bf16"
        self.x_host = workloads.make_input(cfg_id, batch)
        self.batch, c_in = self.x_host.shape[0], self.x_host.shape[1]
        self.x = G.to_device(self.x_host, self.dtype, nhwc=bf16)
        self.stream = torch.cuda.current_stream()
        self.side = torch.cuda.Stream()          # used for graph capture only
        self.forms = {}
        # "fused": the original structure with every fusion that leaves the function unchanged (ReLU, concat and
        # stacked first steps in the convolution stores, LRN + pooling in one pass): how much of the slim form's
        # gain fusion alone recovers.  Not part of a step; absent where the slim form is itself such a fusion.
        forms = ("original", "slim") if isinstance(cfg["slim"], str) else ("original", "slim", "fused")
        # "block": the fused form with every conv - ReLU - LRN - max-pool run as ONE kernel (dr_conv_lrn_maxpool_fwd)
        kinds = [k for k, _ in cfg["original"]] if not isinstance(cfg["original"], str) else []
        if bf16 and any(kinds[i:i + 4] == ["conv", "relu", "lrn", "maxpool"] for i in range(len(kinds))):
            forms = forms + ("block",)
        for form in forms:
            slim, fused = form == "slim", form in ("fused", "block")
            src_form = "original" if fused else form
            layers = cfg["original"] if isinstance(cfg[src_form], str) else cfg[src_form]
            folded = slim and isinstance(cfg[form], str)
            if folded:      # Lemma 2: BatchNorm folded into the filters by the library's host routine
                src = workloads.make_params(cfg_id, "original")
                params_host = []
                for i in range(0, len(src), 2):
                    cq, bq = src[i], src[i + 1]
                    wf, bf = B.fold_bn(cq["w"], cq["b"], bq["gamma"], bq["beta"], bq["mean"], bq["var"],
                                       float(np.float32(workloads.BN_EPS)))
                    params_host.append({"w": workloads.round_to_bf16(wf) if bf16 else wf, "b": bf})
            else:
                params_host = workloads.make_params(cfg_id, src_form)
            net = B.Net(G.net_descs(layers, c_in, inception_mode=(B.DR_FUSE_RELU | B.DR_FUSE_CONCAT | B.DR_FUSE_STACK) if (slim or fused) else (0 if serial_branches else B.DR_CONCURRENT_BRANCHES),
                                    fuse_relu=slim or fused, folded=folded, pack=self.dtype,
                                    fuse_nontensor="block" if form == "block" else (fused and bf16)))
            xd = B.desc(self.x)
            y = G.empty_like_desc(net.output_desc(xd))
            ws = torch.empty(max(net.workspace_bytes(xd), 256), dtype=torch.uint8, device="cuda")
            flat = G.flat_params(params_host, self.dtype, pack=True)
            if (slim or fused) and not folded and any(kind == "inception" for kind, _ in layers):
                flat = G.stack_first_steps(layers, flat)      # the layout DR_FUSE_STACK takes (Eq. (12))
            self.forms[form] = dict(net=net, y=y, ws=ws, params=flat,
                                    layers=layers, params_host=params_host, folded=folded)
            # The same forward as a HIP graph (dr_net_capture): one launch per forward.  Inside a graph the branches of
            # a module run side by side without the events between queues that this costs kernel by kernel, so the
            # forms that keep all four branches (original, fused) are captured in that mode; the slim form's two
            # branches gain nothing from it.
            gnet = net
            if fused and any(kind == "inception" for kind, _ in layers):
                gnet = B.Net(G.net_descs(layers, c_in, inception_mode=B.DR_FUSE_RELU | B.DR_FUSE_CONCAT | B.DR_FUSE_STACK | B.DR_CONCURRENT_BRANCHES,
                                         fuse_relu=True, folded=folded, pack=self.dtype,
                                         fuse_nontensor="block" if form == "block" else (fused and bf16)))
                assert gnet.workspace_bytes(xd) <= ws.numel()
            self.forms[form]["gnet"] = gnet
            self.forms[form]["graph"] = gnet.capture(self.x, flat, y, ws, self.side)
        self.capture_step()

    def capture_step(self):
        """One step (original-form forward, then slim-form forward) recorded as a single HIP graph."""
        B = self.B
        keep = [self.x] + [self.forms[k][n] for k in ("original", "slim") for n in ("params", "y", "ws")]
        with B.capture(self.side, keep) as c:
            for form in ("original", "slim"):
                f = self.forms[form]
                f["gnet"].fwd(self.x, f["params"], f["y"], f["ws"], self.side)
        self.step_g = c.graph

    def run(self, form):
        f = self.forms[form]
        f["net"].fwd(self.x, f["params"], f["y"], f["ws"], self.stream)

    def step(self):
        self.run("original")
        self.run("slim")

    def run_graph(self, form):
        self.forms[form]["graph"].launch(self.stream)

    def step_graph(self):
        self.step_g.launch(self.stream)

    def trace(self, form):
        self.B.trace_begin("", capacity=8192)
        self.run(form)
        return self.B.trace_end(8192)

    def form_times(self, reps, graph=False):
        out = {}
        for form in self.forms:
            ts = []
            for _ in range(reps):
                e0, e1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
                e0.record(self.stream)
                self.run_graph(form) if graph else self.run(form)
                e1.record(self.stream)
                e1.synchronize()
                ts.append(e0.elapsed_time(e1))
            out[form] = (float(self.np.min(ts)), float(self.np.median(ts)))
        return out

    def block_times(self, reps=5):
        """Time per block of the network (the rows of Table 4: conv1, conv2, the inception modules, loss3; the
        pooling layers between modules as rows of their own), per form, in ms: the library's per-layer
        HIP-event times (dr_net_layer_times), best of a few runs, summed over the layers of a block."""
        B = self.B
        names = ["inception_3a", "inception_3b", "inception_4a", "inception_4b", "inception_4c", "inception_4d",
                 "inception_4e", "inception_5a", "inception_5b"]
        out = {}
        for form, f in self.forms.items():
            net = f["net"]
            net.set_timing(True)
            best = None
            for _ in range(reps):
                self.run(form)
                self.torch.cuda.synchronize()
                t = net.layer_times()
                best = t if best is None else [min(a, b) for a, b in zip(best, t)]
            net.set_timing(False)
            rows, convs, modules, pools = {}, 0, 0, 0
            for kind, ms in zip(net.kinds, best):
                if kind == B.DR_LAYER_INCEPTION:
                    name = names[modules] if modules < len(names) else "inception_%d" % modules
                    modules += 1
                elif kind in (B.DR_LAYER_AVGPOOL, B.DR_LAYER_FC, B.DR_LAYER_SOFTMAX):
                    name = "loss3"
                elif modules:               # between modules: pool3, pool4
                    pools += 1
                    name = "pool%d" % (pools + 2)
                else:                       # the stem: conv1 = first convolution and what follows it, conv2 = the rest
                    if kind == B.DR_LAYER_CONV:
                        convs += 1
                    name = "conv1" if convs <= 1 else "conv2"
                rows[name] = rows.get(name, 0.0) + ms
            out[form] = {k: round(v, 4) for k, v in rows.items()}
        return out

    def memory(self):
        """Run-time memory of the forward pass per form (the analogue of the memory columns of Table 6): the
        workspace the library plans for this batch (two ping-pong activation buffers + per-layer scratch), the
        parameters, what one more image adds, and the largest batch whose input, workspace, output and
        parameters fit the 288 GB of one MI355X."""
        B = self.B
        out = {}
        for form, f in self.forms.items():
            xd = B.desc(self.x)
            params = sum(p.numel() * p.element_size() for p in f["params"])
            def total(n):
                d = B.desc(self.x)
                d.n = n
                yd = f["net"].output_desc(d)
                esz = 2 if self.dtype == "bf16" else 4
                io = (d.n * d.c * d.h * d.w + yd.n * yd.c * yd.h * yd.w) * esz
                return f["net"].workspace_bytes(d) + io
            per_image = (total(512) - total(256)) / 256.0
            out[form] = {"workspace_mb": round(f["net"].workspace_bytes(xd) / 1e6, 2), "params_mb": round(params / 1e6, 2),
                         "per_image_mb": round(per_image / 1e6, 3),
                         "max_batch_288GB": int((288e9 - params) // per_image)}
        out.pop("fused", None)
        out.pop("block", None)
        out["slim_saving"] = round(out["original"]["per_image_mb"] / out["slim"]["per_image_mb"], 2)
        return out

    def summary(self, reps, warmup):
        for _ in range(warmup):
            self.step()
        self.torch.cuda.synchronize()
        fe = self.form_times(reps)
        fg = self.form_times(reps, graph=True)
        # a forward of one to four kernels is quicker launched kernel by kernel than as a graph: the faster way per form
        fm = {k: min(fe[k], fg[k]) for k in fe}
        recs = self.trace("original")
        tens = sum(r[6] for r in recs if is_tensor(r))
        other = sum(r[6] for r in recs if not is_tensor(r))
        return {"workload": WORKLOAD_NAMES[self.cfg_id], "batch": self.batch, "dtype": self.dtype,
                "launch": {k: "graph" if fg[k] <= fe[k] else "eager" for k in fe},
                "eager_ms": {k: round(v[0], 4) for k, v in fe.items()}, "graph_ms": {k: round(v[0], 4) for k, v in fg.items()},
                "original_ms": round(fm["original"][0], 4), "slim_ms": round(fm["slim"][0], 4),
                "original_images_per_s": round(self.batch / (fm["original"][0] * 1e-3), 1),
                "slim_images_per_s": round(self.batch / (fm["slim"][0] * 1e-3), 1),
                "slim_speedup": round(fm["original"][0] / fm["slim"][0], 3),
                "fused_original_ms": round(fm["fused"][0], 4) if "fused" in fm else None,
                "fused_block_ms": round(fm["block"][0], 4) if "block" in fm else None,
                "pct_latency_non_tensor_original": round(100.0 * other / max(tens + other, 1e-9), 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, choices=sorted(WORKLOAD_NAMES))
    ap.add_argument("--calibrate-copy", action="store_true", help="run only the known-size copy kernel (counter calibration)")
    ap.add_argument("--ceilings", action="store_true", help="run only the machine-ceiling measurements (matrix-core issue, copy, cached reads)")
    ap.add_argument("--layer-trace", action="store_true", help="run only the marked forwards for a rocprofv3 kernel trace (see layer_trace)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--only", action="store_true", help="skip the summary of the other configurations")
    ap.add_argument("--roofline-kernel", default="", metavar="LABEL,K,C,R",
                    help="grade this launch (e.g. conv_bf16,192,64,3) instead of looking for the longest one: for runs under a profiler, "
                         "which lengthens launches by different amounts")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU; the path shards by batch with no communication, "
              "so --gpus %d is not measured here" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads
    from paper_1708_04728_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    B.lib()                                    # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        calibrate_copy()
        return
    if args.ceilings:
        ceilings()
        return
    if args.layer_trace:
        layer_trace(args.config)
        return
    wl = Workload(args.config)
    dtype, batch = wl.dtype, wl.batch

    for _ in range(args.warmup):
        wl.step()
    torch.cuda.synchronize()

    # ---- untimed traced pass: every kernel of one step, to find the dominant one and the per-kind split
    recs = wl.trace("original")
    recs_slim = wl.trace("slim")
    # (the dominant launch by its shortest time over three such passes: one pass alone is one sample per launch, and the
    # two longest launches of this workload are within 15 % of each other)
    shortest = [r[6] for r in recs + recs_slim]
    for _ in range(2):
        again = wl.trace("original") + wl.trace("slim")
        if len(again) == len(shortest):
            shortest = [min(a, r[6]) for a, r in zip(shortest, again)]
    dom = (recs + recs_slim)[max(range(len(shortest)), key=lambda i: shortest[i])]
    if args.roofline_kernel:
        want = args.roofline_kernel.split(",")
        named = [r for r in recs + recs_slim if r[0] == want[0] and [int(v) for v in want[1:]] == list(r[1:len(want)])]
        if not named:
            sys.exit("bench.py: no launch matches --roofline-kernel %s" % args.roofline_kernel)
        dom = max(named, key=lambda r: r[6])
    dom_is_conv = dom[0].startswith("conv")

    # ---- timed region: K steps, with one event pair around every launch of the dominant kernel
    cap = 64 * args.steps + 16
    if dom_is_conv:
        B.trace_begin(dom[0], dom[1], dom[2], dom[3], capacity=cap)
    else:
        B.trace_begin(dom[0], capacity=cap)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_recs = [r for r in B.trace_end(cap) if r[:6] == dom[:6]]
    eager_ms_per_step = (t1 - t0) * 1e3 / args.steps
    dom_ms = float(np.mean([r[6] for r in dom_recs]))

    # ---- the timed region proper: K steps, each one launch of a HIP graph holding both forwards (the same kernels on the same
    # buffers; events cannot be read inside a graph, which is why the dominant kernel was timed in the region above)
    for _ in range(args.warmup):
        wl.step_graph()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        wl.step_graph()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- per-form times (events on the launch stream), best and median as the paper reports best runs
    form_ms = wl.form_times(max(args.steps, 10), graph=True)
    form_eager = wl.form_times(max(args.steps, 10))

    # ---- roofline of the dominant kernel
    esz = 2 if dtype == "bf16" else 4
    if dom_is_conv:
        # the roof that binds: the matrix cores when the layer's arithmetic intensity (FLOP per byte it must
        # move: input, filters and output once each) exceeds the machine balance, else HBM
        flops, nbytes = conv_flops(dom), float(dom[7])
        peak = MI355X_MFMA_TFLOPS[dtype]
        desc = "%s %dx%d %d->%d n=%d" % (dom[0], dom[3], dom[4], dom[2], dom[1], dom[5])
        mfma_bound = flops / nbytes >= peak * 1e12 / (MI355X_HBM_GBS * 1e9)
        if mfma_bound:
            achieved = flops / (dom_ms * 1e-3) / 1e12
            roofline = {"bound": "mfma", "kernel": desc, "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                        "frac": round(achieved / peak, 4)}
        else:
            achieved = nbytes / (dom_ms * 1e-3) / 1e9
            roofline = {"bound": "hbm", "kernel": desc, "achieved": round(achieved, 1), "peak": MI355X_HBM_GBS, "unit": "GB/s",
                        "frac": round(achieved / MI355X_HBM_GBS, 4)}
        roofline.update({"launch_ms": round(dom_ms, 5), "launches_timed": len(dom_recs), "algorithmic_flop_per_launch": flops,
                         "algorithmic_bytes_per_launch": nbytes, "flop_per_byte": round(flops / nbytes, 1),
                         "tflops": round(flops / (dom_ms * 1e-3) / 1e12, 2), "traffic": measured_traffic(desc, dom[0])})
    else:
        nbytes = 2.0 * dom[5] * esz
        achieved = nbytes / (dom_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": dom[0], "achieved": round(achieved, 1), "peak": MI355X_HBM_GBS,
                    "unit": "GB/s", "frac": round(achieved / MI355X_HBM_GBS, 4), "launch_ms": round(dom_ms, 5),
                    "launches_timed": len(dom_recs), "algorithmic_bytes_per_launch": nbytes, "traffic": None}

    # ---- per-kind split of one step: time in tensor layers vs non-tensor layers (Eq. (1))
    def split(rs):
        conv = sum(r[6] for r in rs if is_tensor(r))
        other = sum(r[6] for r in rs if not is_tensor(r))
        fl = sum(conv_flops(r) for r in rs if r[0].startswith("conv"))
        return conv, other, fl
    co, oo, fo = split(recs)
    cs, os_, fs = split(recs_slim)
    # non-tensor layers: algorithmic bytes (each layer's input and output once) over HIP-event time, for all
    # launches of the original form and for those that move at least 32 MB (below that a launch is bound by
    # its start-up, not by bandwidth: the event pair around an empty launch already spans several microseconds)
    def nt_bytes(r):
        return float(r[7]) if r[7] > 0 else 2.0 * r[5] * esz
    nontensor_bytes = sum(nt_bytes(r) for r in recs if not is_tensor(r))
    big = [r for r in recs if not is_tensor(r) and nt_bytes(r) >= 32e6]
    by_kind = {}
    for r in recs:
        if not is_tensor(r):
            k = by_kind.setdefault(r[0], [0.0, 0.0, 0])
            k[0] += nt_bytes(r); k[1] += r[6]; k[2] += 1

    out = {
        "metric": "images/sec fwd (orig vs slim GoogLeNet), conv MFMA util %, non-tensor HBM GB/s",
        "value": round(batch / (ms_per_step * 1e-3), 1),
        "unit": "images/s (one original-form + one slim-form forward per image)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[args.config], "batch": batch,
                   "launch": "a step is one launch of a HIP graph recorded from the library's layer-by-layer calls of both "
                             "forwards (dr_capture_begin / dr_capture_end); `eager` holds the same steps launched kernel by kernel",
                   "filters": "pre-packed KRSC where the channel count allows",
                   "original": "layer-by-layer (separate ReLU / pool / LRN / concat / BatchNorm kernels)",
                   "slim": "slimmed structure, ReLU / concat / residual fused into the conv stores, BatchNorm folded"},
        "eager": {"value": round(batch / (eager_ms_per_step * 1e-3), 1), "ms_per_step": round(eager_ms_per_step, 4),
                  "original_ms": round(form_eager["original"][0], 4), "slim_ms": round(form_eager["slim"][0], 4),
                  "fused_original_ms": round(form_eager["fused"][0], 4) if "fused" in form_eager else None,
                  "note": "the dominant kernel's HIP events (roofline) were taken in this region"},
        "original_ms": {"best": round(form_ms["original"][0], 4), "median": round(form_ms["original"][1], 4)},
        "slim_ms": {"best": round(form_ms["slim"][0], 4), "median": round(form_ms["slim"][1], 4)},
        "original_images_per_s": round(batch / (form_ms["original"][0] * 1e-3), 1),
        "slim_images_per_s": round(batch / (form_ms["slim"][0] * 1e-3), 1),
        "slim_speedup": round(form_ms["original"][0] / form_ms["slim"][0], 3),
        "fused_original_ms": {"best": round(form_ms["fused"][0], 4), "median": round(form_ms["fused"][1], 4)} if "fused" in form_ms else None,
        "fused_block_ms": {"best": round(form_ms["block"][0], 4), "median": round(form_ms["block"][1], 4),
                           "note": "the fused form with conv - ReLU - LRN - max-pool of the conv2 block as one kernel"} if "block" in form_ms else None,
        # how much of the slim form's gain fusion alone recovers: the best fusion that leaves the function unchanged
        "fusion_share_of_slim_gain": round((form_ms["original"][0] - min(form_ms[k][0] for k in ("fused", "block") if k in form_ms))
                                           / max(form_ms["original"][0] - form_ms["slim"][0], 1e-9), 3) if "fused" in form_ms else None,
        "kernel_split_ms": {"original_tensor": round(co, 4), "original_non_tensor": round(oo, 4),
                            "slim_tensor": round(cs, 4), "slim_non_tensor": round(os_, 4)},
        "pct_latency_non_tensor_original": round(100.0 * oo / max(co + oo, 1e-9), 1),
        "conv_mfma_util_pct": {"original": round(100.0 * fo / max(co, 1e-9) / 1e9 / MI355X_MFMA_TFLOPS[dtype], 1),
                               "slim": round(100.0 * fs / max(cs, 1e-9) / 1e9 / MI355X_MFMA_TFLOPS[dtype], 1)},
        "non_tensor_hbm_gbs": round(nontensor_bytes / max(oo, 1e-9) / 1e6, 1) if oo > 0 else None,
        "non_tensor_hbm_gbs_launches_over_32MB": round(sum(nt_bytes(r) for r in big) / max(sum(r[6] for r in big), 1e-9) / 1e6, 1) if big else None,
        "non_tensor_hbm_gbs_kernel_trace": non_tensor_from_kernel_trace(args.config),
        "non_tensor_by_kind": {k: {"launches": v[2], "ms": round(v[1], 4), "gbs": round(v[0] / max(v[1], 1e-9) / 1e6, 1)} for k, v in sorted(by_kind.items())},
        "roofline": dict(roofline, network={"original": network_roofline(recs, dtype, form_ms["original"][0]),
                                            "slim": network_roofline(recs_slim, dtype, form_ms["slim"][0]),
                                            "note": "every launch against max(FLOP / matrix-core peak, algorithmic bytes / 8 TB/s); "
                                                    "frac = sum of the roofs / measured time of the forward"}),
        "per_block_ms": wl.block_times() if args.config == 5 else None,
        "per_block_ms_paper_S5": {"conv1": [94.92, 8.424], "conv2": [153.8, 16.62], "inception_3a": [55.23, 21.17],
                                  "inception_3b": [98.41, 25.94], "inception_4a": [30.53, 16.80], "inception_4b": [32.60, 20.29],
                                  "inception_4c": [46.96, 18.71], "inception_4d": [36.88, 24.67], "inception_4e": [48.24, 28.08],
                                  "inception_5a": [24.64, 10.69], "inception_5b": [24.92, 14.58], "loss3": [3.014, 2.97],
                                  "note": "Table 4, GoogLeNet vs GoogLeNet-Slim, one image on a Galaxy S5 CPU (context only)"}
        if args.config == 5 else None,
        "paper_variant_3a": paper_variant_3a(wl) if args.config == 5 else None,
        "activation_memory": wl.memory(),
        "paper_context": "GoogLeNet 651.4 ms -> GoogLeNet-Slim 210.6 ms on Samsung Galaxy S5 CPU; 10.17 -> 6.57 ms on "
                         "Titan X (batch 1, Table 4/5); inception_3a 55.23 -> 21.17 ms on S5; run-time memory 33.2 -> 13.2 MB per "
                         "image, largest batch on a 12 GB Titan X 350 -> 882 (Table 6)",
    }

    # ---- CPU baseline: the fp64 oracle, as it stands, on the host cores (bounded sample, >= 10 s)
    if not args.no_cpu_baseline:
        import oracle
        sample = {1: 1, 2: 32, 3: 4, 4: 4, 5: 4}[args.config]
        xs = wl.x_host[:sample]
        oracle.relu(xs[:1])                                   # builds / loads the C library
        reps = 0
        c0 = c1 = time.perf_counter()
        while c1 - c0 < 10.0:
            for form in ("original", "slim"):
                f = wl.forms[form]
                oracle.forward(f["layers"], f["params_host"], xs, fold="given" if f["folded"] else False)
            reps += 1
            c1 = time.perf_counter()
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count()
        omp = os.environ.get("OMP_NUM_THREADS")
        cores = min(cores, int(omp)) if omp else cores
        out["cpu_baseline"] = {"value": round(sample * reps / (c1 - c0), 2), "unit": out["unit"], "cores": cores, "kind": "oracle",
                               "sample": "%d of %d images, one original + one slim forward, repeated %d times, fp64 "
                                         "nested loops, %.1f s" % (sample, batch, reps, c1 - c0)}

    # ---- the other configurations, briefly (best of a few runs each)
    if not args.only:
        del wl
        torch.cuda.empty_cache()
        allc = {}
        for cid in sorted(WORKLOAD_NAMES):
            w2 = Workload(cid)
            allc[str(cid)] = w2.summary(reps=10, warmup=3)
            if cid == 2:
                allc["2"]["paper_variant_ms"] = round(paper_variant_ms(w2), 4)
            if cid == 1:
                allc["1"]["slim_layer_regression"] = slim_layer_regression()
            del w2
            torch.cuda.empty_cache()
        out["all_configs"] = allc
    print(json.dumps(out))


if __name__ == "__main__":
    main()
