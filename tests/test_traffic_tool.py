"""The tool that writes profiles/traffic.json, on synthetic counter files (no GPU): calibration by
the copy dispatch, largest dispatch of the last steps per kernel substring, sum over the worker
call's kernels."""
import csv
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _write(path, rows):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for i, (name, value) in enumerate(rows):
            w.writerow([i + 1, name, "X", value])


def test_traffic_tool_scales_and_sums(tmp_path):
    steps = [("void (anonymous namespace)::k_a<true>(int)", 1000.0), ("k_b", 10.0), ("k_shared", 50.0), ("k_shared", 7.0)]
    fetch = steps * 8 + [("__amd_rocclr_copyBuffer", 524288.0)]                # the counter reads half of what a copy moves
    write = [(n, v * 2) for n, v in steps] * 8 + [("__amd_rocclr_copyBuffer", 1048576.0)]
    fetch[0] = (fetch[0][0], 9999.0)                                            # an early (cold) dispatch must not count
    _write(tmp_path / "f.csv", fetch)
    _write(tmp_path / "w.csv", write)
    # the tool writes next to the package: run a private copy so the tracked file is left alone
    pkg = tmp_path / "pkg"
    os.makedirs(pkg / "paper_1905_05957_amd")
    os.makedirs(pkg / "profiles")
    with open(os.path.join(ROOT, "paper_1905_05957_amd", "traffic.py")) as src, open(pkg / "paper_1905_05957_amd" / "traffic.py", "w") as dst:
        dst.write(src.read())
    r = subprocess.run([sys.executable, str(pkg / "paper_1905_05957_amd" / "traffic.py"), "--workload", "demo", "--fetch", str(tmp_path / "f.csv"),
                        "--write", str(tmp_path / "w.csv"), "--kernel", "k_a<", "--kernel", "k_shared", "--commit", "abc", "--steps-in-run", "8"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    entry = json.load(open(pkg / "profiles" / "traffic.json"))["demo"]
    assert entry["fetch_scale"] == 2.0 and entry["write_scale"] == 1.0 and entry["commit"] == "abc"
    assert entry["kernels"]["k_a<"] == {"read_bytes": 1000 * 2 * 1024, "written_bytes": 2000 * 1024}
    assert entry["kernels"]["k_shared"] == {"read_bytes": 50 * 2 * 1024, "written_bytes": 100 * 1024}
    assert entry["worker_call_bytes"] == (1000 * 2 + 2000 + 50 * 2 + 100) * 1024
