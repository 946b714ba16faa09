"""Bounds of the workspace layout and of every kernel's LDS plan, checked on the CPU: the index
helpers the kernels share with the host are compiled by hipcc into a small host
program (tests/host_plans.hip) that walks the extreme accepted shapes.  GPU sanitizers are not
available on the target machines; this is the net under the carved regions."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_workspace_and_lds_plans_stay_in_bounds(tmp_path):
    exe = str(tmp_path / "host_plans")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-std=c++17", "-O1", "-Wall", "-Wno-unused-function",
                           "-Wno-unused-value", "-o", exe, os.path.join(ROOT, "tests", "host_plans.hip")])
    run = subprocess.run([exe], capture_output=True, text=True)
    assert run.returncode == 0, run.stdout[-4000:] + run.stderr[-2000:]
    assert "host plans ok" in run.stdout
