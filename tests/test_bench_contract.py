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
    assert bench.HBM_PEAK_GBPS == 8000.0
    assert bench.BF16_POWER_LIMITED_TFLOPS < bench.PEAK_TFLOPS["bf16"]
    assert bench.HEADLINE == "deep_chain" and "4096" in bench.HEADLINE_TEXT


def test_algorithmic_bytes_of_a_gemm_stage():
    """One GEMM of the headline chain: (m*k + k*n + m*n) * 4 bytes; with beta != 0 C_in is read too."""
    sys.path.insert(0, ROOT)
    import bench
    from paper_2604_04599_amd import api
    n = 4096
    a_d, b_d = api.desc(api.LPG_PACKED_A, api.LPG_F32, n, n), api.desc(api.LPG_PACKED_B, api.LPG_F32, n, n)
    s = api.stage_gemm(1.0, 256, a_d, 512, b_d, 0.0, None, 768, a_d)
    assert bench.stage_bytes(s) == 3 * n * n * 4
    s = api.stage_gemm(1.0, 256, a_d, 512, b_d, 1.0, 1024, 768, a_d)
    assert bench.stage_bytes(s) == 4 * n * n * 4


def test_traffic_figure_comes_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    traffic, src = bench.profile_traffic("gemm_kernel")
    if traffic is not None:
        assert src.startswith("profiles/") and traffic >= 3 * 4096 * 4096 * 4 * 0.9
