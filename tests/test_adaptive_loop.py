"""The adaptive-loop study script (host only): it runs, the static baseline admits what arithmetic says it must,
and on-demand slabs admit several times more under the same budget."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_adaptive_loop_small_run():
    cmd = [sys.executable, os.path.join(ROOT, "adaptive_loop.py"), "--requests", "3000", "--budget-tokens", str(1 << 20),
           "--l-max", "8192", "--safety-slabs", "16", "--window", "1000", "--refresh", "100", "--max-live", "2048"]
    out = subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=300, cwd=ROOT).stdout
    res = json.loads(out.strip().splitlines()[-1])
    by = {r["policy"]: r for r in res["policies"]}
    assert set(by) == {"odma", "odma-fixed", "static"}
    for r in by.values():
        assert r["requests"] == 3000 and r["steps"] > 0
        assert 0.0 < r["utilization_completed"] <= 1.0
    # static: every resident request holds L_max, so at most budget / L_max of them fit
    assert by["static"]["mean_resident_requests"] <= (1 << 20) / 8192
    assert by["static"]["mean_resident_requests"] > 0.9 * (1 << 20) / 8192
    assert by["static"]["migrations"] == 0 and by["static"]["final_boundaries"] == [8192]
    assert by["odma"]["mean_resident_requests"] > 3 * by["static"]["mean_resident_requests"]
    assert by["odma"]["utilization_completed"] > 5 * by["static"]["utilization_completed"]
    assert by["odma"]["recalibrations"] == 3000 // 100
    traj = by["odma"]["boundary_trajectory"]
    assert traj[0] == {"epoch": 0, "boundaries": [512, 1024, 2048, 4096]}
    assert all(b["boundaries"] == sorted(b["boundaries"]) and b["boundaries"][-1] <= 8192 for b in traj)
    assert by["odma-fixed"]["final_boundaries"] == [512, 1024, 2048, 4096] and by["odma-fixed"]["recalibrations"] == 0
