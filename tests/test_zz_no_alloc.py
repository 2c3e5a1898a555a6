"""astraea_select_topk_static, the selection for callers that cannot allocate: the same kernels as
astraea_select_topk with the selection state, histogram and per-workgroup counts in a device array built
into the library instead of a caller's workspace.  Its output must equal the workspace entry point's bit for
bit (indices, complement, mask, counters), on calls that follow each other on one GPU, the later ones with
smaller inputs (the array keeps the earlier call's contents), and the size limit must be an error."""
import numpy as np
import pytest
import torch

from paper_2506_05096_amd import binding as ab
from paper_2506_05096_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _both(score, k):
    """(workspace entry point, static entry point) results for one score array."""
    n = score.numel()
    dscore = score.to(DEV)
    skip0 = (torch.arange(n, dtype=torch.int32) % 7).to(DEV)
    out = []
    for static in (False, True):
        idx = torch.full((max(k, 1),), -7, dtype=torch.int32, device=DEV)
        rem = torch.full((max(n - k, 1),), -7, dtype=torch.int32, device=DEV)
        mask = torch.full((n,), 9, dtype=torch.uint8, device=DEV)
        skip = skip0.clone()
        if static:
            ab.astraea_select_topk_static(dscore, k, idx, idx_remain=rem, sel_mask=mask, skip_count=skip)
        else:
            ws = torch.empty(ab.workspace_bytes(ab.OP_SELECT_TOPK, n), dtype=torch.uint8, device=DEV)
            ws.random_(0, 255)
            ab.astraea_select_topk(dscore, k, idx, ws, idx_remain=rem, sel_mask=mask, skip_count=skip)
        torch.cuda.synchronize()
        out.append((idx[:k].cpu().numpy(), rem[:n - k].cpu().numpy(), mask.cpu().numpy(), skip.cpu().numpy()))
    return out


def test_static_scratch_selection_equals_the_workspace_one_on_calls_in_a_row():
    # sizes above 32768 take the multi-launch path, the one that uses the scratch array; the sequence shrinks,
    # grows again and ends on a single-workgroup size (which leaves the array alone)
    cases = [(1000000, 300000, "narrow"), (118800, 35640, "narrow"), (50000, 20000, "tied"), (40000, 0, "normal"),
             (524288, 524288, "lognormal"), (33000, 1, "narrow"), (5000, 1234, "tied")]
    for n, k, kind in cases:
        a, b = _both(synth.random_scores(n, 17 + n, kind), k)
        for x, y, what in zip(a, b, ("idx_sel", "idx_remain", "sel_mask", "skip_count")):
            assert np.array_equal(x, y), (n, k, kind, what)
        assert len(b[0]) == k and (k == 0 or np.all(np.diff(b[0]) > 0))


def test_static_scratch_selection_rejects_what_its_array_cannot_hold():
    lim = 1 << 22
    dummy = torch.zeros(8, device=DEV)
    idx = torch.zeros(8, dtype=torch.int32, device=DEV)
    L = ab.lib()
    rc = L.astraea_select_topk_static(dummy.data_ptr(), lim + 1, 4, idx.data_ptr(), None, None, None, None)
    assert rc == ab.ERR_UNSUPPORTED and b"4194304" in L.astraea_last_error()
    assert L.astraea_select_topk_static(dummy.data_ptr(), 8, 9, idx.data_ptr(), None, None, None, None) == ab.ERR_INVALID
    assert L.astraea_select_topk_static(None, 0, 0, None, None, None, None, None) == ab.OK
    # the largest size it takes runs, and agrees with the workspace entry point
    a, b = _both(synth.random_scores(lim, 5, "normal"), lim // 3)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
