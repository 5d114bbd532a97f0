"""bench.py prints one JSON line with the fields its consumers rely on (run on the smallest
workload so that the test stays short)."""
import json
import subprocess
import sys
from pathlib import Path

import pytest

pytestmark = pytest.mark.gpu

ROOT = Path(__file__).resolve().parent.parent


def test_bench_line_has_the_contract_fields():
    proc = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--workload", "c1", "--configs", "c1",
                           "--steps", "20", "--warmup", "2", "--repeats", "3", "--cpu-seconds", "0.5",
                           "--inject-seconds", "0"], capture_output=True, text=True, timeout=300)
    assert proc.returncode == 0, proc.stderr[-2000:]
    lines = [ln for ln in proc.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "configs"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 2 and d["vs_baseline"] is None
    assert d["value"] > 0 and abs(d["value"] * d["ms_per_step"] - 1000.0) < 1e-6 * 1000.0
    assert set(d["roofline"]) >= {"bound", "achieved", "peak", "unit", "frac", "traffic"}
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["cores"] >= 1
    assert d["cpu_baseline"]["label_agreement_first_assign"]["differ_outside_tie_band"] == 0
    c1 = d["configs"]["c1"]
    assert "workload" in d["config"] and set(c1["ft"]) >= {"strict", "correct"}
    # a second GPU is not part of this build
    proc = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                          timeout=60)
    assert proc.returncode != 0 and "one GPU" in proc.stderr
