"""Properties of the compiled kernels that no run-time test can see, read off the ISA that hipcc emits for this
repository's own sources (cross-compiled, no GPU needed):

* gemm_w4_midp_kernel issues its vector-memory loads from asm statements and keeps the wait counts by hand, so
  the compiler does not know when a loaded register becomes valid.  Nothing may read or write such a register
  between its load and the wait that covers it (a register copy placed there by the allocator would copy stale
  data): checked by replaying the in-order completion of vector-memory loads over the instruction stream.
* The kernels whose speed depends on it keep everything in registers (no scratch).
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_13915_amd", "csrc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only"]

pytestmark = pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")


def _isa(src, tmp_path, extra=()):
    out = os.path.join(str(tmp_path), src.replace(".hip", ".s"))
    r = subprocess.run(["hipcc", *FLAGS, *extra, os.path.join(CSRC, src), "-o", out], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    with open(out) as fh:
        return fh.read()


def _kernel_body(txt, pattern):
    names = [l.split(":")[0] for l in txt.split("\n") if re.match(r"^_Z\w*" + pattern + r"\w*:", l)]
    assert len(names) == 1, names
    start = txt.index("\n" + names[0] + ":")
    return names[0], txt[start:txt.index(".Lfunc_end", start)]   # every exit of the kernel, not only the first


def _regs(tok):
    m = re.match(r"v\[(\d+):(\d+)\]$", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def _scratch_bytes(txt, name):
    m = re.search(r"\.name:\s+" + re.escape(name) + r"\n(?:.*\n){0,12}?\s+\.private_segment_fixed_size:\s+(\d+)", txt)
    assert m, name
    return int(m.group(1))


@pytest.fixture(scope="module")
def mid_isa(tmp_path_factory):
    return _isa("gemm_w4_mid.hip", tmp_path_factory.mktemp("isa"))


# <depth, row groups, steps per batch, loader waves, operand window, 16-row image, canonical weights>
@pytest.mark.parametrize("inst", ["ILi2ELi1ELi8ELi4ELi5ELb0ELb0E", "ILi2ELi1ELi8ELi4ELi5ELb1ELb0E", "ILi2ELi2ELi8ELi4ELi5ELb0ELb0E",
                                  "ILi2ELi3ELi4ELi4ELi5ELb0ELb0E", "ILi2ELi4ELi4ELi4ELi5ELb0ELb0E",
                                  # the canonical weight layout
                                  "ILi2ELi1ELi8ELi4ELi5ELb0ELb1E", "ILi2ELi1ELi8ELi4ELi5ELb1ELb1E", "ILi2ELi2ELi4ELi4ELi5ELb0ELb1E",
                                  "ILi2ELi3ELi4ELi4ELi5ELb0ELb1E", "ILi1ELi4ELi4ELi0ELi5ELb0ELb1E"])
def test_midp_loads_are_not_touched_before_their_wait(mid_isa, inst):
    txt = mid_isa
    name, body = _kernel_body(txt, "gemm_w4_midp_kernel" + inst)
    assert _scratch_bytes(txt, name) == 0
    in_flight = []   # destination registers of the loads issued and not yet waited for, oldest first
    loads = waits = 0
    for line in body.split("\n"):
        t = line.strip()
        if not t or t[0] in ";.":
            continue
        toks = re.split(r"[ ,]+", t)
        if toks[0] == "global_load_dwordx4":
            in_flight.append(_regs(toks[1]))
            loads += 1
            continue
        if toks[0] == "global_load_lds_dwordx4":   # a fill: counts, writes no register
            in_flight.append(set())
            continue
        if toks[0] == "s_endpgm":                  # an exit (the loader waves leave early): nothing may be pending
            assert not in_flight, "exit with loads in flight"
            continue
        if toks[0] == "s_waitcnt" and "vmcnt" in t:
            n = int(re.search(r"vmcnt\((\d+)\)", t).group(1))
            in_flight = in_flight[len(in_flight) - n:] if n else []
            waits += 1
            continue
        used = set()
        for tok in toks[1:]:
            used |= _regs(tok)
        pending = set().union(*in_flight) if in_flight else set()
        assert not (used & pending), (t, sorted(used & pending))
    assert loads >= 15 and waits >= 2   # the scan saw the kernel it was written for


@pytest.mark.parametrize("src,pattern,extra", [
    ("gemm_w4_prefill.hip", "gemm_w4_dma_kernelILi4ELb0ELb0E", ()),
    ("gemm_w8.hip", "gemm_w8_dma_kernelILi128ELi256ELi4ELi4ELi4ELb0ELb0ELi64ELi1E", ()),
    ("gemm_w4.hip", "gemm_w4_rows_kernelILi2ELb1E", ()),   # three weight batches and two x blocks in registers
    ("gemm_w4.hip", "gemm_w4_rows_kernelILi2ELb0E", ()),   # ... on the canonical layout
    ("attn_mla.hip", "attn_mla_dequant_kernelILb1E", ()),   # 128 output registers per lane
])
def test_register_bound_kernels_use_no_scratch(tmp_path, src, pattern, extra):
    txt = _isa(src, tmp_path, extra)
    name, _ = _kernel_body(txt, pattern)
    assert _scratch_bytes(txt, name) == 0
