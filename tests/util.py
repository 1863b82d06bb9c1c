"""Helpers shared by the tests (no arithmetic of the method)."""
import numpy as np

TOL_F32 = 1e-4    # max relative error, fp32 path
TOL_BF16 = 2e-2   # max relative error, bf16 storage with fp32 accumulation


def rel_err(got, ref):
    """max_i |g_i - r_i| / max(|r_i|, rms(r)): relative error with an RMS floor, so that exact
    zeros after a ReLU and softmax tails do not divide by ~0."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref * ref))
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den))


def rms_err(got, ref):
    """rms(got - ref) / rms(ref): the typical (not the worst) relative deviation over a tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    return float(np.sqrt(np.mean((got - ref) ** 2)) / max(np.sqrt(np.mean(ref * ref)), 1e-300))


def note(what, value, bound):
    """Records a measured figure that is not a rel_err of two tensors (a ratio, an rms error); True when value < bound."""
    import os
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0]
    MEASURED.append((test, what, float(value), float(bound)))
    if not value < bound:
        print("note(): %s %s: measured %.3e, bound %.3e" % (test, what, value, bound))
    return value < bound


def oracle_in_chunks(fn, x, chunk=16):
    """fn applied to x in chunks of images (images are independent): bounds the oracle's fp64 working set."""
    return np.concatenate([fn(x[i:i + chunk]) for i in range(0, x.shape[0], chunk)], axis=0)


# every comparison a test makes through close(): (test id, what, measured error, tolerance); the terminal summary
# of the run prints the worst case of each test function (tests/conftest.py)
MEASURED = []


def close(got, ref, tol, what=""):
    """True when rel_err(got, ref) < tol; records the measured error for the run's summary."""
    import os
    err = rel_err(got, ref)
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0]
    MEASURED.append((test, what, err, float(tol)))
    if not err < tol:
        print("close(): %s %s: measured %.3e, tolerance %.3e" % (test, what, err, tol))
    return err < tol


def case_seed(case, salt=0):
    """A seed that depends only on the printed form of a test case (not on the interpreter's hash)."""
    import zlib
    return (zlib.crc32(repr(case).encode()) + salt) % (2 ** 31)


def gpu(a, dtype="f32"):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda()


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


def gpu_nhwc(a, dtype="f32"):
    """(n, c, h, w) numpy array -> channels-last device tensor wrapped for the binding."""
    from paper_1708_04728_amd import graph as G
    return G.to_device(a, dtype, nhwc=True)


def host_nhwc(t):
    from paper_1708_04728_amd import graph as G
    return G.to_host(t)


def empty_nhwc(shape_nchw, dtype="f32"):
    import torch
    from paper_1708_04728_amd import binding as B
    n, c, h, w = shape_nchw
    return B.NHWC(torch.full((n, h, w, c), float("nan"), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32,
                             device="cuda"))
