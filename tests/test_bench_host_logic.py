"""Host-side logic of bench.py that needs no GPU: the algorithmic byte counts it prices the
kernels with, the refusal of more than one GPU, and the rule that figures taken from a
committed profile are handed out only for the very kernel source they were measured on."""
import hashlib
import importlib.util
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load_bench():
    spec = importlib.util.spec_from_file_location("zpp_bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_algorithmic_bytes_follow_the_layouts():
    """codes n*bits/8 + one fp32 scale per block + the 16-bit or fp32 payload; the reduce stages
    read every peer's codes and scales once (Sec. 3.1, 3.3.2)"""
    B = load_bench().Bytes
    n = 1811939328                                           # one layer of the step, hidden 12288
    assert B.dequantize(n, 2048, 8) == n + 4 * (n // 2048) + 2 * n == 5439356928
    assert B.quantize(n, 512, 4) == 2 * n + n // 2 + 4 * (n // 512) == 4544004096
    assert B.quantize(1 << 20, 256, 8, in_bytes=4) == (4 << 20) + (1 << 20) + 4 * 4096
    m = n // 8
    assert B.intra(m, 512, 4, 8) == 9 * (m // 2 + 4 * (m // 512)) == 1035141120
    L = n // 384
    assert B.inter(L, 512, 4, 48) == 48 * (L // 2 + 4 * (L // 512)) + 4 * L == 133890048


def test_more_than_one_gpu_is_refused_before_anything_runs():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert run.returncode == 2
    assert "one GPU" in run.stderr and run.stdout.strip() == ""


def test_profile_figures_only_for_the_source_they_were_measured_on(tmp_path, monkeypatch):
    bench = load_bench()
    src = tmp_path / "kernel.hip"
    src.write_text("// some kernel source\n")
    digest = hashlib.sha256(src.read_bytes()).hexdigest()
    prof = tmp_path / "profiles"
    prof.mkdir()
    (prof / "t.txt").write_text(
        "TRAFFIC qwz_dequantize bytes_per_launch=1000 elements=300 kernel=k<1> grid_threads=64\n"
        f"SOURCE sha256={digest} file=kernel.hip\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "KERNEL_SOURCE", str(src))
    row, where = bench.profile_figures("t.txt", "qwz_dequantize", 300)
    assert row["bytes_per_launch"] == "1000" and where["kernel"] == "k<1>" and where["grid_threads"] == 64
    row, where = bench.profile_figures("t.txt", "qwz_dequantize", 301)
    assert row is None and "another problem size" in where["refused"]
    row, where = bench.profile_figures("t.txt", "qgz_reorder", 300)
    assert row is None and "no row" in where["refused"]
    row, where = bench.profile_figures("absent.txt", "qwz_dequantize", 300)
    assert row is None and "not present" in where["refused"]
    src.write_text("// the kernel source after an edit\n")
    row, where = bench.profile_figures("t.txt", "qwz_dequantize", 300)
    assert row is None and "another version" in where["refused"]
