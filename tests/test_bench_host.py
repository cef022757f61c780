"""Host-only checks of the benchmark's bookkeeping: the HBM traffic it reports is read from the
committed rocprofv3 summary, not typed in."""
import os
import re

import bench


def test_traffic_comes_from_the_committed_counter_summary():
    t = bench.traffic_from_profiles()
    assert {"summarize_mfma", "merge_mfma", "attend_mfma"} <= set(t)
    text = open(os.path.join(bench.ROOT, "profiles", "hbm_traffic_pmc.txt")).read()
    m = re.search(r"stage 1 = .*? = ([\d.]+) MB per launch; stage 2 = .*? = ([\d.]+) MB", text)
    assert abs(t["summarize_mfma"] / 1e6 - float(m.group(1))) < 0.06
    assert abs(t["attend_mfma"] / 1e6 - float(m.group(2))) < 0.06
    # traffic close to the algorithmic bytes of the two default workloads (no re-reads)
    assert 0.95 < t["attend_mfma"] / (524288 * 640) < 1.05
    assert bench.traffic_from_profiles("/nonexistent") == {}


def test_more_than_one_gpu_is_refused(monkeypatch, capsys):
    import pytest
    monkeypatch.setattr("sys.argv", ["bench.py", "--gpus", "2"])
    with pytest.raises(SystemExit) as e:
        bench.main()
    assert "one GPU" in str(e.value)


def test_calibration_modes_match_the_header():
    """bench.py's table of loop bodies names every value of the header's enum, and nothing else."""
    text = open(os.path.join(bench.ROOT, "include", "vista_calibrate.h")).read()
    enum = {int(v) for v in re.findall(r"VISTA_CAL_[A-Z0-9_]+ = (\d+)", text)}
    assert enum == set(bench.CAL_MODES.values())
    assert len(bench.CAL_MODES) == len(enum) == max(enum) + 1
