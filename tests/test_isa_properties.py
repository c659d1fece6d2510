"""Properties of the compiled gfx950 code, read off the compiler's assembly listing of the
library's own kernels (cross-compiled, no GPU needed): no atomics anywhere (the summation
order is fixed by program order alone), no packed-fp32 arithmetic, no writes through the
scalar data cache, no register spills, and streaming hints on the gradient loads."""
import os
import re
import subprocess

import pytest

from paper_2208_14228_amd import build as hip_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def listing(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("isa") / "es_kernels.s")
    flags = [f for f in hip_build.FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hip_build.hipcc(), *flags, "-S", "--cuda-device-only", hip_build.SOURCES[0], "-o", out]
    try:
        subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    except (subprocess.CalledProcessError, FileNotFoundError) as e:       # pragma: no cover
        pytest.skip(f"hipcc not available: {e}")
    return open(out).read()


def test_no_atomics_no_packed_fp32_no_scalar_stores(listing):
    code = "\n".join(l for l in listing.splitlines() if l.startswith("\t") and not l.startswith("\t."))
    assert not re.search(r"\b(global|flat|buffer|ds)_atomic|\bds_(add|sub|min|max|and|or|xor|cmpst)_", code)
    assert not re.search(r"\bv_pk_(add|mul|fma)_f32\b", code)
    assert not re.search(r"\bs_(store|buffer_store|atomic|dcache_wb)", code)


def test_no_kernel_spills_registers(listing):
    sizes = [int(x) for x in re.findall(r"\.private_segment_fixed_size:\s+(\d+)", listing)]
    assert len(sizes) > 50 and max(sizes) == 0


def test_gradient_loads_carry_the_streaming_hint(listing):
    body = listing[listing.index("k_ring_reduceILi2ELi8ELi1ELb1EE"):]
    body = body[:body.index("s_endpgm")]
    loads = re.findall(r"global_load_dwordx4 [^\n]*", body)
    assert len(loads) >= 16 and sum(" nt" in l for l in loads) >= 16      # 2 vectors x 8 ranks per batch
