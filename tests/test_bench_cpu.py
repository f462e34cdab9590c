"""bench.py contract checks that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_comes_from_a_measurement_of_the_current_kernels(tmp_path, monkeypatch):
    """roofline.traffic is read from the file the profile step writes, and only while the kernels are the ones
    the counters were taken from."""
    sys.path.insert(0, ROOT)
    import json
    import bench
    assert bench.PEAK_BF16_TFLOPS == 2516.6 and bench.PEAK_HBM_GBS == 8000.0
    f = tmp_path / "traffic.json"
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    assert bench.measured_traffic("c2") is None                       # no file
    f.write_text(json.dumps({"kernel_source_hash": bench.kernel_source_hash(), "workloads": {"c2": {"read_bytes": 3.0, "write_bytes": 4.0}}}))
    assert bench.measured_traffic("c2") == 7.0 and bench.measured_traffic("c3") is None
    f.write_text(json.dumps({"kernel_source_hash": "stale", "workloads": {"c2": {"read_bytes": 3.0, "write_bytes": 4.0}}}))
    assert bench.measured_traffic("c2") is None                       # the kernels have changed since


def test_summarize_traffic_scales_by_the_calibration_copy(tmp_path, monkeypatch):
    sys.path.insert(0, ROOT)
    import json
    import bench
    d = tmp_path / "traffic_c2"
    d.mkdir()
    head = "Kernel_Name,Grid_Size,Counter_Name,Counter_Value\n"
    rows = ""
    for counter, copy_kib, kern_kib in (("FETCH_SIZE", 262144.0, 1000.0), ("WRITE_SIZE", 524288.0, 500.0)):
        rows += '"__amd_rocclr_copyBuffer",131072,%s,%f\n' % (counter, copy_kib)
        rows += '"void fle::gemm_tiled_256<1, false>(fle::GemmArgs)",65536,%s,%f\n' % (counter, kern_kib)
    (d / "x_counter_collection.csv").write_text(head + rows)
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "traffic.json"))
    bench.summarize_traffic([str(d)])
    w = json.load(open(tmp_path / "traffic.json"))["workloads"]["c2"]
    assert abs(w["fetch_scale"] - 2.0) < 1e-9 and abs(w["write_scale"] - 1.0) < 1e-9
    assert abs(w["read_bytes"] - 1000 * 1024 * 2.0) < 1e-3 and abs(w["write_bytes"] - 500 * 1024) < 1e-3


def test_kernel_hash_ignores_comments_and_white_space(tmp_path, monkeypatch):
    """A comment edit does not change what the counters describe; a code edit does."""
    sys.path.insert(0, ROOT)
    import bench
    d = tmp_path / "csrc"
    d.mkdir()
    monkeypatch.setattr(bench, "KERNEL_SOURCES", str(d))
    (d / "k.h").write_text("// one\nint f(int a) { return a + 1; }  /* two */\n")
    h0 = bench.kernel_source_hash()
    (d / "k.h").write_text("// another comment\n\nint f(int a)   {\n    return a + 1;\n}\n")
    assert bench.kernel_source_hash() == h0
    (d / "k.h").write_text("int f(int a) { return a + 2; }\n")
    assert bench.kernel_source_hash() != h0
