"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only)."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_is_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", os.path.join(HERE, "c_abi", "oracle_san.c"),
           os.path.join(ROOT, "oracle", "es_oracle.c"), "-o", exe]
    try:
        subprocess.check_call(cmd, stderr=subprocess.STDOUT)
    except (subprocess.CalledProcessError, FileNotFoundError) as e:      # pragma: no cover
        pytest.skip(f"sanitizer build not available: {e}")
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    if "ASan runtime does not come first" in out.stderr:
        pytest.skip("a preloaded library prevents running ASan binaries in this environment")
    assert out.returncode == 0, out.stdout + out.stderr
    assert "geometries clean" in out.stdout


def test_host_runtime_is_clean_under_asan_ubsan(tmp_path):
    """libes' host logic (layout validation, tile planning, argument checks, plan search) with the kernel
    launchers stubbed out: host code only, no device code is built or run."""
    exe = str(tmp_path / "host_san")
    pkg = os.path.join(ROOT, "paper_2208_14228_amd", "csrc")
    cmd = ["g++", "-O1", "-g", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "include"), "-I", pkg, "-I", "/opt/rocm/include",
           os.path.join(HERE, "c_abi", "host_san.cpp"), os.path.join(pkg, "es_api.cpp"),
           os.path.join(pkg, "es_sched.cpp"),
           "-o", exe, "-L", "/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"]
    try:
        subprocess.check_call(cmd, stderr=subprocess.STDOUT)
    except (subprocess.CalledProcessError, FileNotFoundError) as e:      # pragma: no cover
        pytest.skip(f"sanitizer build of the host runtime not available: {e}")
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                         env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
    if "ASan runtime does not come first" in out.stderr:
        pytest.skip("a preloaded library prevents running ASan binaries in this environment")
    assert out.returncode == 0, out.stdout + out.stderr
    assert "plans clean" in out.stdout
