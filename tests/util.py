"""Helpers shared by the GPU parity tests (no method arithmetic here)."""
import numpy as np

TOL = 1e-4   # max |gpu - oracle| / max |oracle| per output tensor (fp32 path vs fp64 oracle)


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    denom = np.max(np.abs(ref))
    if denom == 0.0:
        return float(np.max(np.abs(got)))
    value = float(np.max(np.abs(got - ref)) / denom)
    _report("rel_err", value)
    return value


def per_step_err(got, ref, floor=1e-30):
    """max over steps t of ||got_t - ref_t||_inf / ||ref_t||_inf, for steps above `floor`."""
    got = np.asarray(got, dtype=np.float64).reshape(got.shape[0], -1)
    ref = np.asarray(ref, dtype=np.float64).reshape(ref.shape[0], -1)
    n = np.max(np.abs(ref), axis=1)
    keep = n >= floor
    if not np.any(keep):
        return 0.0
    value = float(np.max(np.max(np.abs(got - ref), axis=1)[keep] / n[keep]))
    _report("per_step_err", value)
    return value


def _report(what, value):
    """With BPPSA_TEST_REPORT=<file> in the environment, every measured figure is appended to that
    file with the name of the running test (the bounds in the tests are limits, not measurements)."""
    import os
    path = os.environ.get("BPPSA_TEST_REPORT")
    if path:
        with open(path, "a") as f:
            f.write("%s %s %.3e\n" % (os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0], what, value))


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_np(t):
    return t.detach().cpu().numpy()
