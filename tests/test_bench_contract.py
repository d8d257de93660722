"""Host-side parts of bench.py that need no GPU: the single-GPU refusal and the oracle baseline leg."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert out.returncode != 0
    assert "single-GPU" in out.stderr and out.stdout.strip() == ""


def test_one_timed_step_cannot_weigh_both_kinds_of_step():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "1"], capture_output=True, text=True)
    assert out.returncode != 0 and "--steps >= 2" in out.stderr and out.stdout.strip() == ""


def test_oracle_baseline_leg_reports_the_contract_fields():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2510_09103_amd import workloads as WL
    wl = WL.CONFIGS["llama_60m"]()
    r = bench.cpu_baseline(wl, 100, wl.lr, nlayers=1, held_steps=1)
    assert r["kind"] == "oracle" and r["unit"] == "params/s" and r["value"] > 0
    assert isinstance(r["cores"], int) and r["cores"] >= 1
    assert "layers" in r["sample"] and "Alg. 2" in r["sample"]
