"""CPU checks of bench.py's contract pieces that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert out.returncode != 0 and "ONE GPU" in out.stderr and out.stdout.strip() == ""


def test_algorithmic_bytes_and_traffic_key():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.grad_bytes_per_elem("adamw", "bf16") == 26 and bench.grad_bytes_per_elem("adamw", "f32") == 28
    assert bench.grad_bytes_per_elem("sgdm", "f32") == 20 and bench.grad_bytes_per_elem("sgdm", "bf16") == 18
    # the counter-derived traffic is reported only for the kernel source it was measured with
    same = bench.kernel_source_digest() == bench.TRAFFIC["kernel_source_sha256"]
    got, alg = bench.measured_traffic("gptneo125m_k8")
    assert (got == bench.TRAFFIC["bytes_per_launch"]) if same else (got is None and alg is None)
    assert bench.measured_traffic("resnet50_k8") == (None, None)
    if got is not None:                                 # reported next to the algorithmic bytes of the SAME launches
        assert alg == bench.TRAFFIC["algorithmic_bytes_same_launches"] and abs(got / alg - 1) < 0.01


def test_cpu_model_is_a_string_here():
    sys.path.insert(0, ROOT)
    import bench
    m = bench.cpu_model()
    assert m is None or (isinstance(m, str) and m)
