"""The benchmark's one JSON line (GPU): every field the measurement contract names is there and sane, on a short run
(20 timed steps, a 60-step sample pass, one oracle sequence), run inside this process (no child process is started)."""
import io
import json
import os
import sys
from contextlib import redirect_stdout

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(argv):
    sys.path.insert(0, ROOT)
    import bench
    old = sys.argv
    sys.argv = ["bench.py"] + argv
    out = io.StringIO()
    try:
        with redirect_stdout(out):
            bench.main()
    finally:
        sys.argv = old
    lines = [l for l in out.getvalue().splitlines() if l.startswith("{")]
    assert len(lines) == 1, out.getvalue()
    return json.loads(lines[0])


def test_default_workload_line():
    d = run_bench(["--steps", "20", "--warmup", "5", "--sample-steps", "60", "--oracle-seqs", "1", "--ramp-seconds", "0.1"])
    assert d["metric"].startswith("committed tokens/sec") and d["unit"] == "tokens/s"
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 5 and d["higher_is_better"] is True
    assert d["dtype"] == "bf16" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["config"]["workload"].startswith("c2") and "model" not in d["config"]
    assert 1e4 < d["value"] < 1e6 and 0.05 < d["ms_per_step"] < 2.0
    assert abs(d["value"] - d["config"]["committed_tokens"] / (d["ms_per_step"] * 1e-3 * 20)) < 0.01 * d["value"]
    r = d["roofline"]
    assert r["bound"] in ("hbm", "mfma") and r["unit"] in ("GB/s", "TFLOP/s") and r["peak"] in (8000.0, 2500.0)
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and 0.3 < r["frac"] < 1.0 and r["traffic"] > 1e9
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and c["unit"] and c["sample"]
    for call in ("dlm_block_attn", "dlm_lmhead_confidence", "dlm_unmask_commit", "dlm_kv_refresh"):
        k = d["kernels"][call]
        assert k is not None and k["calls"] > 0 and k["avg_us"] > 0, call
    assert d["peaks"]["measured"]["copy_gbs"] > 3000


def test_more_than_one_gpu_is_refused(capsys):
    with pytest.raises(SystemExit) as e:
        run_bench(["--gpus", "2"])
    assert e.value.code != 0
    assert "--gpus 1" in capsys.readouterr().err
