"""Host-only checks of bench.py's command line and of the profile summariser."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_profile_summaries(tmp_path):
    from paper_2411_00662_amd import profiling
    stats_csv = tmp_path / "k_stats.csv"
    stats_csv.write_text('"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
                         '"monta::regather_kernel(unsigned int __vector(4) const*, int)",10,100000,10000.0,50.0,9000,11000,1.0\n'
                         '"void monta::combine_kernel<true, 2>(float const*)",10,100000,10000.0,50.0,9000,11000,1.0\n')
    out = tmp_path / "stats.txt"
    profiling.stats(str(stats_csv), str(out), "rocprofv3 ... -- python3 bench.py")
    text = out.read_text()
    assert "regather_kernel" in text and "combine_kernel<true, 2>" in text and "python3 bench.py" in text

    def pmc(path, counter, vals):
        rows = ['"Kernel_Name","Counter_Name","Counter_Value"']
        for name, v in vals:
            rows.append(f'"{name}","{counter}",{v}')
        path.write_text("\n".join(rows) + "\n")

    f, w = tmp_path / "f.csv", tmp_path / "w.csv"
    pmc(f, "FETCH_SIZE", [("monta::copy_kernel(a)", 512.0), ("monta::regather_kernel(b)", 100.0), ("monta::regather_kernel(b)", 300.0)])
    pmc(w, "WRITE_SIZE", [("monta::copy_kernel(a)", 1024.0), ("monta::regather_kernel(b)", 400.0)])
    tj = tmp_path / "traffic.json"
    profiling.traffic(str(f), str(w), "1", "wl/S4/mode1", str(tmp_path / "t.txt"), str(tj), "cmd f", "cmd w")
    entry = json.loads(tj.read_text())["wl/S4/mode1"]["regather_kernel"]
    # 1 MiB copy read 512 units => 2 KiB per FETCH unit; 1024 units => 1 KiB per WRITE unit
    assert entry["read_bytes"] == 200 * 2 * 1024 and entry["write_bytes"] == 400 * 1024
    assert entry["total_bytes"] == entry["read_bytes"] + entry["write_bytes"]
