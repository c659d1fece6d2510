"""The C boundary used from plain C (no Python, no PyTorch in the loop): a host program
links libes.so and the C oracle, runs two global steps and compares all outputs."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
EXE = os.path.join(HERE, "c_abi", "est_step")


def build_c_abi_program(force=False) -> str:
    src = os.path.join(HERE, "c_abi", "est_step.c")
    if force or not os.path.exists(EXE) or os.path.getmtime(EXE) < os.path.getmtime(src):
        pkg = os.path.join(ROOT, "paper_2208_14228_amd")
        subprocess.check_call([
            "gcc", "-O1", "-std=c11", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
            "-I", "/opt/rocm/include", src, os.path.join(ROOT, "oracle", "es_oracle.c"),
            "-ffp-contract=off", "-o", EXE,
            "-L", pkg, "-l:libes.so", "-L", "/opt/rocm/lib", "-lamdhip64",
            "-Wl,-rpath,$ORIGIN/../../paper_2208_14228_amd", "-Wl,-rpath,/opt/rocm/lib"])
    return EXE


def test_c_program_matches_oracle():
    exe = build_c_abi_program()
    print(f"[gpu-case] running {exe}", flush=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "bit-exact" in out.stdout
