"""bench.py's host-side contract (no GPU): it refuses more than one GPU with a message, and its HBM-traffic figure comes from the tracked
profiles/traffic.json, which records the commit it was measured at and the counters' scale factors."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_file_is_consistent():
    sys.path.insert(0, ROOT)
    import bench

    t = json.load(open(bench.TRAFFIC_FILE))
    assert t["kernel"] == bench.HEADLINE_KERNEL and t["commit"] not in ("", "unknown")
    want = sum(t[c]["kib_per_launch"] * t[c]["factor"] for c in ("FETCH_SIZE", "WRITE_SIZE")) * 1024.0
    assert abs(t["bytes_per_launch"] - want) <= 1e-6 * want
    # the scale factors are what the counters read for a copy of known size: reads are reported in half units, writes in full
    assert abs(t["copy_kernel_kib"] / t["FETCH_SIZE"]["copy_kernel_reads_kib"] - t["FETCH_SIZE"]["factor"]) < 0.01
    assert abs(t["copy_kernel_kib"] / t["WRITE_SIZE"]["copy_kernel_reads_kib"] - t["WRITE_SIZE"]["factor"]) < 0.01
    # more than the algorithmic bytes (q, k, v read once, out written once), less than ten times as much
    algorithmic = 4 * 80640 * 40 * 128 * 2
    assert algorithmic < t["bytes_per_launch"] < 10 * algorithmic
    assert bench.read_traffic() == (t["bytes_per_launch"], t["commit"])


def test_traffic_is_rebuilt_from_counter_files(tmp_path, monkeypatch):
    """--traffic-from on two tiny counter_collection files of the shape rocprofv3 writes."""
    sys.path.insert(0, ROOT)
    import bench

    hdr = "Kernel_Name,Counter_Name,Counter_Value\n"
    k = '"void skiparse::attn_fwd_bf16_kernel<128, 1, false>(skiparse::AttnArgs, unsigned int, unsigned int, unsigned int)"'
    c = '"void skiparse::permute_rows_kernel<5, false>(HIP_vector_type<unsigned int, 4u> const*)"'
    (tmp_path / "f").mkdir()
    (tmp_path / "w").mkdir()
    (tmp_path / "f" / "x_counter_collection.csv").write_text(hdr + f"{k},FETCH_SIZE,3000000\n{k},FETCH_SIZE,3200000\n{c},FETCH_SIZE,403200\n")
    (tmp_path / "w" / "x_counter_collection.csv").write_text(hdr + f"{k},WRITE_SIZE,830000\n{c},WRITE_SIZE,806400\n")
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "traffic.json"))
    bench.write_traffic([str(tmp_path / "f"), str(tmp_path / "w")], "abc1234")
    t = json.load(open(tmp_path / "traffic.json"))
    assert t["commit"] == "abc1234" and t["FETCH_SIZE"]["factor"] == 2.0 and t["WRITE_SIZE"]["factor"] == 1.0
    assert t["bytes_per_launch"] == (3100000 * 2.0 + 830000 * 1.0) * 1024.0
