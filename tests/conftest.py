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
