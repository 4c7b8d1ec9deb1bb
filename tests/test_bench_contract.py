"""Host-side checks of bench.py's command line contract (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       cwd=ROOT, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_roofline_constants_are_consistent():
    sys.path.insert(0, ROOT)
    import bench
    # dense MFMA peaks of the part: 256 compute units x 2.4 GHz x 256 (fp32) / 4096 (bf16) flop per clock
    assert abs(bench.PEAK_TFLOPS["f32"] - 256 * 2.4e9 * 256 / 1e12) < 0.1
    assert abs(bench.PEAK_TFLOPS["bf16"] - 256 * 2.4e9 * 4096 / 1e12) < 0.1
    # the headline's two GEMMs: (m*k + k*n + m*n) * 4 bytes, the second with beta*C_in on top
    m, d, h = 2048, 1024, 4096
    first = (m * d + d * h + m * h) * 4
    second = (m * h + h * d + 2 * m * d) * 4
    assert abs(bench.GEMM_ALGORITHMIC_BYTES - (first + second) / 2) < 2 ** 20
    assert bench.GEMM_TRAFFIC_BYTES >= bench.GEMM_ALGORITHMIC_BYTES
