"""profile_run --summarize: the per-kernel figures of the LAST n launches of a rocprofv3
kernel-trace or counter-collection CSV (host logic, no GPU)."""
import csv

from paper_2603_06664_amd import profile_run


def _write(path, header, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)


def test_kernel_trace_uses_last_launches(tmp_path, capsys):
    p = tmp_path / "kt_kernel_trace.csv"
    rows = []
    t = 1000
    for i, d in enumerate([900, 800, 100, 110, 120]):     # two cold launches, then three warm ones
        rows.append(["KERNEL_DISPATCH", i + 1, "attn", t, t + d])
        t += 10000
    rows.append(["KERNEL_DISPATCH", 9, "rope", t, t + 15])
    _write(p, ["Kind", "Dispatch_Id", "Kernel_Name", "Start_Timestamp", "End_Timestamp"], rows)
    profile_run.summarize(str(p), 3)
    out = capsys.readouterr().out
    line = [l for l in out.splitlines() if "attn" in l][0]
    assert "launches    5" in line and "mean        110" in line and "median        110" in line
    assert "min        100" in line and "max        120" in line
    assert [l for l in out.splitlines() if "rope" in l][0].count("15") >= 3


def test_counter_collection_means_and_max(tmp_path, capsys):
    p = tmp_path / "f_counter_collection.csv"
    rows = [[i + 1, "attn", "FETCH_SIZE", v, 0, 0] for i, v in enumerate([500.0, 100.0, 200.0, 300.0])]
    rows += [[10, "copy", "FETCH_SIZE", 524288.0, 0, 0]]
    _write(p, ["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value", "Start_Timestamp", "End_Timestamp"], rows)
    profile_run.summarize(str(p), 3)
    out = capsys.readouterr().out
    line = [l for l in out.splitlines() if "attn" in l][0]
    assert "dispatches    4" in line and "mean            200.0" in line and "max of all            500.0" in line
    assert "524288.0" in [l for l in out.splitlines() if "copy" in l][0]
