"""The workload timing drivers run end to end on down-scaled inputs and print one JSON line
with positive stage times (they share the library calls of the parity tests, not their checks)."""
import io
import json
from contextlib import redirect_stdout

import pytest

from paper_1905_03381_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,n", [("sparse", 140_000), ("images", 4096), ("translation", 60_000),
                                    ("sk", 70_000), ("stale", 70_000), ("rho", 70_000)])
def test_workload_driver_runs(name, n):
    buf = io.StringIO()
    with redirect_stdout(buf):
        workloads.main([name, "--n", str(n), "--repeats", "2", "--threads", "4"])
    lines = [l for l in buf.getvalue().splitlines() if l.startswith("{")]
    assert len(lines) == 1
    out = json.loads(lines[0])
    assert out["data"] == "synthetic" and out["stages"]
    for stage in out["stages"]:
        assert stage["us"] > 0 and stage["calls"] >= 1
