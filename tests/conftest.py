import os
import sys
from pathlib import Path

import numpy as np
import pytest

ROOT = Path(__file__).resolve().parents[1]
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))
# test_oracle_mutants.py runs the pins in a child process against a copy of the oracle with a planted mistake:
# that copy's parent directory then goes in front of the repository
if os.environ.get("ASTRAEA_TEST_ORACLE_ROOT"):
    sys.path.insert(0, os.environ["ASTRAEA_TEST_ORACLE_ROOT"])


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped (not failed) when no GPU is visible and they were not asked for."""
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def to_np(t):
    """torch tensor -> numpy as the oracle wants it (fp32 stays, bf16 becomes uint16 bit patterns)."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def bf16_bits_to_f64(a):
    """uint16 bf16 bit patterns -> float64 values."""
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def assert_rel_l2(got, ref, tol=1e-2, tag=""):
    """The bf16 parity bar, applied twice: relative L2 error over the whole comparison and over every group
    taken by itself, a group being the last axis (one head of one row of an attention result, one row of a
    per-token layer), so that one bad group among thousands cannot hide under the global figure.  Returns
    (global, worst group)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{tag}: non-finite values"
    diff = got - ref
    glob = float(np.linalg.norm(diff.ravel()) / max(np.linalg.norm(ref.ravel()), 1e-300))
    num = np.linalg.norm(diff.reshape(-1, ref.shape[-1]), axis=1)
    den = np.linalg.norm(ref.reshape(-1, ref.shape[-1]), axis=1)
    # a group whose reference is zero has no relative error: compare it absolutely against the typical size
    typical = float(np.sqrt(np.mean(den ** 2))) if den.size else 0.0
    worst_each = num / np.where(den > 0.0, den, max(typical, 1e-300))
    worst = float(worst_each.max()) if worst_each.size else 0.0
    assert glob <= tol, f"{tag}: relative L2 error {glob:.3g} > {tol}"
    assert worst <= tol, (f"{tag}: group {int(worst_each.argmax())} of {worst_each.size} has relative L2 error "
                          f"{worst:.3g} > {tol} (global {glob:.3g})")
    return glob, worst
