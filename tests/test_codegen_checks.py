"""Code-generation checks that need no GPU: hipcc cross-compiles a few lines against the kernels'
header and the test reads the gfx950 assembly of that translation unit.

The run-time choice between a streaming and an ordinary store is two stores that differ only in a
hint; a compiler that merges them (hoisting or sinking the store out of the branch) keeps one store
without the hint, silently.  The helpers in the header guard against that, and this test checks that
both forms are still in the generated code.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "paper_2404_00438_amd", "csrc", "dlion_kernels.hpp")

SOURCE = r'''
#include "%s"
using namespace dlion;
extern "C" __global__ void probe_counts8(uint16_t *counts, int stream)
{
    u32x4 v;
    v.x = v.y = v.z = v.w = threadIdx.x;
    counts_store8(v, counts + threadIdx.x * 8, stream != 0);
}
extern "C" __global__ void probe_counts4(uint16_t *counts, int stream)
{
    u16x4 v;
    v.x = v.y = v.z = v.w = static_cast<uint16_t>(threadIdx.x);
    counts_store4(v, counts + threadIdx.x * 4, stream != 0);
}
extern "C" __global__ void probe_rows(float *__restrict__ m, const uint16_t *__restrict__ g, float *__restrict__ x)
{
    const int j = threadIdx.x * 4;
    f32x4 a = row_load4(m + j);
    const u32x2 b = row_load4(g + j);
    f32x4 c = x_load4(x + j);
    a.x += __uint_as_float(b.x << 16);
    a.y += __uint_as_float(b.x & 0xFFFF0000u);
    a.z += __uint_as_float(b.y << 16);
    a.w += __uint_as_float(b.y & 0xFFFF0000u);
    c += a;
    row_store4(a, m + j);
    x_store4(c, x + j);
}
'''


def kernel_body(asm: str, name: str) -> str:
    start = asm.index(f"\n{name}:")
    end = asm.index(".Lfunc_end", start)
    return asm[start:end]


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    hipcc = os.environ.get("HIPCC") or shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc) and shutil.which(hipcc) is None:
        pytest.skip("hipcc not available")
    tmp = tmp_path_factory.mktemp("codegen")
    src = os.path.join(tmp, "probe.hip")
    out = os.path.join(tmp, "probe.s")
    with open(src, "w") as f:
        f.write(SOURCE % HEADER)
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-ffp-contract=off", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only", "-o", out, src]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    with open(out) as f:
        return f.read()


def stores(body: str, width: str):
    return [line.strip() for line in body.splitlines() if re.search(rf"global_store_{width}\b", line)]


def test_streaming_and_ordinary_count_stores_both_survive(asm):
    for name, width in (("probe_counts8", "dwordx4"), ("probe_counts4", "dwordx2")):
        found = stores(kernel_body(asm, name), width)
        streaming = [s for s in found if s.endswith(" nt")]
        ordinary = [s for s in found if not s.endswith(" nt")]
        assert streaming and ordinary, f"{name}: expected a streaming and an ordinary store, got {found}"


def test_row_and_weight_accesses_are_full_width_and_streaming(asm):
    """Element-aligned vector types must still give one 128-bit (64-bit for bf16) access, with the hint."""
    body = kernel_body(asm, "probe_rows")
    loads4 = [l for l in body.splitlines() if "global_load_dwordx4" in l]
    loads2 = [l for l in body.splitlines() if "global_load_dwordx2" in l]
    st4 = stores(body, "dwordx4")
    assert len(loads4) == 2 and len(loads2) == 1 and len(st4) == 2, (loads4, loads2, st4)
    assert all(l.strip().endswith(" nt") for l in loads4 + loads2 + st4)
    assert "global_load_dword " not in body and "global_load_ushort" not in body
