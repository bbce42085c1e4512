"""A C99 program drives the library on the GPU through the C ABI alone (no Python in the process):
prefill quantization, draft / verify attention, flush, qs_attn_static and the code export, against a
fixture that tests/c_abi/make_fixture.py writes from the CPU oracle."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_c_program_runs_the_hot_path_on_the_gpu(tmp_path):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2502_10424_amd import binding
    assert os.path.exists(binding.LIB_PATH)
    fixture, exe = str(tmp_path / "fixture.bin"), str(tmp_path / "gpu_run")
    subprocess.run([sys.executable, os.path.join(ROOT, "tests", "c_abi", "make_fixture.py"), fixture], check=True)
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-Werror", "-I" + os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_abi", "gpu_run.c"), "-o", exe, "-ldl", "-lm"], check=True)
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = "/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    print("[case] C program: prefill, draft, verify, flush, static-scratch verify, export", flush=True)
    res = subprocess.run([exe, binding.LIB_PATH, fixture], env=env, capture_output=True, text=True, timeout=120)
    print(res.stdout, res.stderr, flush=True)
    assert res.returncode == 0 and res.stdout.strip().endswith("ok"), res.stderr
