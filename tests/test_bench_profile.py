"""bench.py reads `roofline.traffic` from the committed rocprofv3 summary: the summary must carry a
traffic line, naming its kernels, for every call of the default step, and a summary without them must
be refused rather than silently ignored."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench  # noqa: E402

CALLS = {"mm_fwd_l1": "k_roast_mfma", "mm_fwd_l2": "k_roast_mfma", "mm_bwd_dx_l1": "k_roast_mfma",
         "mm_bwd_dx_l2": "k_roast_mfma", "mm_bwd_dM_l1": "k_roast_mfma", "mm_bwd_dM_l2": "k_roast_mfma",
         "embed_fwd": "k_embed", "embed_bwd": "k_embed_accum"}


def test_committed_summary_has_a_traffic_line_for_every_call():
    rows = bench.load_measured_traffic()
    for call, kernel in CALLS.items():
        b = bench.traffic_of(rows, [call], kernel)
        assert b > 0
    # algorithmic bytes are a lower bound of what the counters can read
    assert bench.traffic_of(rows, ["embed_fwd"], "k_embed") >= 872e6
    assert bench.traffic_of(rows, ["embed_bwd"], "k_embed_accum") >= 872e6


def test_missing_or_malformed_summary_is_an_error(tmp_path):
    p = tmp_path / "empty.txt"
    p.write_text("no counters here\n")
    with pytest.raises(ValueError):
        bench.load_measured_traffic(str(p))
    p.write_text("traffic: mm_fwd_l1 | | 1 | 2\n")
    with pytest.raises(ValueError):
        bench.load_measured_traffic(str(p))
    p.write_text("traffic: mm_fwd_l1 | k_other | 1 | 2\n")
    rows = bench.load_measured_traffic(str(p))
    with pytest.raises(KeyError):
        bench.traffic_of(rows, ["mm_fwd_l1"], "k_roast_mfma")
    with pytest.raises(KeyError):
        bench.traffic_of(rows, ["embed_fwd"], "k_embed")
    with pytest.raises(OSError):
        bench.load_measured_traffic(str(tmp_path / "absent.txt"))


@pytest.mark.gpu
@pytest.mark.parametrize("flags", [["--mm-only"], ["--embed-only"], ["--reduce", "deterministic"]])
def test_profiling_runs_of_the_bench_print_a_line(flags):
    """The flag combinations the committed rocprofv3 summaries were collected with must run to the end
    and print one JSON line with the fields the summaries quote."""
    import json
    import subprocess
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--no-cpu-baseline", "--hot-path-only",
           "--steps", "2", "--warmup", "1"] + flags
    r = subprocess.run(cmd, cwd=ROOT, capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, r.stderr[-2000:]
    line = json.loads(r.stdout.strip().splitlines()[-1])
    assert line["steps"] == 2 and line["ms_per_step"] > 0
    if "--embed-only" not in flags:
        assert line["roofline"]["avg_launch_us"] > 0 and set(line["kernel_ms"]) == set(line["roofline_per_call"])
    if "--mm-only" not in flags:
        assert line["embedding"]["value"] > 0
