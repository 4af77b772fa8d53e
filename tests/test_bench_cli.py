"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "ONE GPU" in r.stderr


def test_kernel_fingerprint_ignores_comments_and_white_space(tmp_path, monkeypatch):
    sys.path.insert(0, ROOT)
    import bench
    a = tmp_path / "a.hip"
    b = tmp_path / "b.hip"
    a.write_text("int f(int x) { return x + 1; }  // plus one\n")
    b.write_text("/* a function */\nint f(int x)\n{\n    return x + 1;\n}\n")
    monkeypatch.setattr(bench, "KERNEL_SRC", str(a))
    h1 = bench.kernel_fingerprint()
    monkeypatch.setattr(bench, "KERNEL_SRC", str(b))
    assert bench.kernel_fingerprint() == h1
    b.write_text("int f(int x) { return x + 2; }\n")
    assert bench.kernel_fingerprint() != h1


def test_recorded_counter_traffic_belongs_to_the_current_kernel_source():
    """profiles/*.json are only reported while the kernel source has the recorded hash; this fails
    when the kernels were changed and the counters not taken again (bench.py would then print
    traffic = null, which is allowed, but the records should not be left stale unnoticed)."""
    sys.path.insert(0, ROOT)
    import bench
    t = bench.counter_traffic("c2_7b_uniform", "fp16")
    alg = 8594128896
    assert t is None or 1.0 <= t / alg < 1.03
