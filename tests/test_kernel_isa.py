"""Properties of the fused kernel's machine code that cost microseconds when they are lost and
that no functional test notices (CPU only: hipcc cross-compiles gfx950 without a GPU).

The latency-bound builds of query_aware_decode_kernel (one unit per cluster) must
  - fetch every kernel argument their first loads are addressed with in ONE trip to memory:
    a single wait for scalar loads ahead of the first vector load (scalar registers running
    out at the head of the kernel, or an argument first used behind a branch, brought a second
    and a third trip, 0.1-0.5 us each on every launch);
  - use no scratch memory (a fragment held through a pointer once put 208 bytes per lane
    there: +9 us).
"""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

from paper_2509_12211_amd import build as tsbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# head_dim 64, page size, no loop, append folded in, bf16, clusters: the builds the
# benchmark's 64-, 16- and 8-sequence shapes run
KERNELS = {
    "page 16": "_ZN2ts25query_aware_decode_kernelILi64ELi16ELb0ELb1ELb0ELb0ELb1EEEvNS_11FusedParamsE",
    "page 32": "_ZN2ts25query_aware_decode_kernelILi64ELi32ELb0ELb1ELb0ELb0ELb1EEEvNS_11FusedParamsE",
}


@pytest.fixture(scope="module")
def fused_asm():
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    tmp = tempfile.mkdtemp(prefix="ts_isa_")
    try:
        out = os.path.join(tmp, "fmt_bf16_d64.s")
        flags = [f for f in tsbuild.HIPCC_FLAGS if f not in ("-fPIC",)]
        cmd = [HIPCC] + flags + ["--offload-device-only", "-S",
                                 os.path.join(ROOT, "paper_2509_12211_amd", "csrc", "fmt_bf16_d64.hip"),
                                 "-o", out]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-2000:]
        with open(out) as f:
            yield f.read()
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def kernel_body(asm, symbol):
    m = re.search(r"^" + re.escape(symbol) + r":.*?\n\s*s_endpgm", asm, re.S | re.M)
    assert m, f"{symbol} not in the assembly"
    return [l.strip() for l in m.group(0).split("\n") if l.strip() and not l.strip().startswith(";")]


@pytest.mark.parametrize("which", sorted(KERNELS))
def test_arguments_arrive_in_one_trip(fused_asm, which):
    body = kernel_body(fused_asm, KERNELS[which])
    trips, pending, spills = 0, False, 0
    for line in body:
        if line.startswith(("global_load", "buffer_load", "flat_load")):
            break
        if line.startswith("s_load"):
            pending = True
        elif line.startswith("s_waitcnt") and "lgkmcnt" in line and pending:
            trips, pending = trips + 1, False
        elif line.startswith("v_writelane"):
            spills += 1
    else:
        pytest.fail("no vector load in the kernel")
    assert not pending, "a scalar load ahead of the first vector load is never waited for?"
    assert trips == 1, f"{trips} dependent trips for kernel arguments ahead of the first load"
    assert spills == 0, f"{spills} scalar registers parked in vector lanes ahead of the first load"


@pytest.mark.parametrize("which", sorted(KERNELS))
def test_no_scratch_memory(fused_asm, which):
    sym = KERNELS[which]
    m = re.search(r"\.amdhsa_kernel " + re.escape(sym) + r"\n(.*?)\.end_amdhsa_kernel", fused_asm, re.S)
    assert m, "kernel descriptor not found"
    size = re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", m.group(1))
    assert size and int(size.group(1)) == 0, f"scratch bytes per lane: {size.group(1) if size else '?'}"
    assert not any(l.startswith("scratch_") for l in kernel_body(fused_asm, sym))
