"""bench.py contract pieces that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_measured_traffic_constants_match_the_committed_profile():
    """The roofline `traffic` figures are constants of the profile summary under profiles/: keep the two in step."""
    sys.path.insert(0, ROOT)
    import importlib
    bench = importlib.import_module("bench")
    text = open(os.path.join(ROOT, "profiles", "gemm_nt_bf16_7b.md")).read()
    rows = {}
    for line in text.splitlines():
        if line.startswith("| `gemm_nt_bf16") and line.count("|") == 4:
            name, fetched, written = [c.strip() for c in line.strip("|").split("|")]
            rows.setdefault(name.strip("`"), []).append(float(fetched) + float(written))
    want = {"stash": {"gemm_fwd": rows["gemm_nt_bf16_kernel<EpiFwdStash>"][0], "gemm_bwd": rows["gemm_nt_bf16_pair_kernel<EpiDX, EpiDW>"][0]},
            "recompute": {"gemm_fwd": rows["gemm_nt_bf16_kernel<EpiFwd>"][0], "gemm_ds": rows["gemm_nt_bf16_kernel<EpiDS>"][0],
                          "gemm_dx": rows["gemm_nt_bf16_kernel<EpiDX>"][0], "gemm_dw": rows["gemm_nt_bf16_kernel<EpiDW>"][0]}}
    for mode, d in want.items():
        for k, gb in d.items():
            assert abs(bench.MEASURED_TRAFFIC_7B[mode][k] / 1e9 - gb) < 0.06, (mode, k, gb)
