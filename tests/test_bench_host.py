"""Host-side checks of the benchmark's bookkeeping (no GPU): the HBM traffic it quotes comes from the tracked
counter summary and is withheld when that summary was made for other kernel sources."""
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parents[1]
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

import bench  # noqa: E402


def test_traffic_is_read_from_the_profile_and_tied_to_the_kernel_sources(tmp_path, monkeypatch):
    h = bench.kernel_source_hash("attn_bf16_kernel")
    assert len(h) == 16 and int(h, 16) >= 0
    prof = tmp_path / "counters.txt"
    line = ("roofline_traffic kernel=attn_bf16_kernel workload=cfg3 budget_pct=30 fetched_bytes=8.0e9 "
            "written_bytes=2.5e8 source_sha256_16={}\n")
    monkeypatch.setattr(bench, "TRAFFIC_PROFILE", prof)
    # no summary at all, a summary for the present sources, one for other sources, one for another workload
    got, note = bench.measured_traffic("attn_bf16_kernel", "cfg3", 30)
    assert got is None and note
    prof.write_text("# header\n" + line.format(h))
    got, note = bench.measured_traffic("attn_bf16_kernel", "cfg3", 30)
    assert got == 8.0e9 + 2.5e8 and h in note
    assert bench.measured_traffic("attn_bf16_kernel", "cfg3", 40)[0] is None
    assert bench.measured_traffic("attn_bf16_kernel", "cfg2", 30)[0] is None
    assert bench.measured_traffic("attn_f32_kernel", "cfg0", 50)[0] is None
    prof.write_text(line.format("0123456789abcdef"))
    got, note = bench.measured_traffic("attn_bf16_kernel", "cfg3", 30)
    assert got is None and "another version" in note


def test_the_tracked_summary_matches_the_tracked_sources():
    """The committed counter summary must have been made for the committed kernel: otherwise the benchmark prints
    no traffic figure."""
    got, note = bench.measured_traffic("attn_bf16_kernel", "cfg3", 30)
    assert got is not None and got > 1.9e9, note      # at least the algorithmic bytes
