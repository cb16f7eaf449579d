"""Host-side check of the generated gfx950 code of the tile kernels (no GPU needed; compiles to assembly).

The tile kernels load X straight into LDS and end every pipeline stage with an explicit wait on the load counter
followed by a plain barrier instruction.  That wait is only right if, in the instruction stream the compiler finally
emits, (1) the direct-to-LDS loads of a stage precede all of the stage's other loads, (2) the wait allows at most as
many outstanding loads as were issued between them and the wait, and (3) the wave's own LDS reads are waited for before
the barrier.  A violation would be a data race that a parity test may or may not catch.
"""
import concurrent.futures
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_15601_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
UNITS = {"tm_w4_tile_small": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "tm_w4_tile_kgroup": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "tm_w4_tile_grouped": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "tm_w4_tile_w8": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
         "tm_w4_tile_large": [],
         "tm_w4_tile32": []}
VMCNT_MAX = 63          # six-bit counter: a wave cannot have more loads outstanding, so a larger bound is no wait at all


def _assembly(unit, extra, outdir):
    out = os.path.join(outdir, unit + ".s")
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
           os.path.join(CSRC, unit + ".hip"), "-o", out]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    return open(out).read()


def _stage_regions(text):
    """(kernel name, instructions of one barrier-terminated region) for every region that loads into LDS."""
    for m in re.finditer(r"^(_ZN4tmw4[^\n]*tile(?:32)?_kernel[^\n]*):\s*;[^\n]*\n(.*?)^\.Lfunc_end", text, re.S | re.M):
        region = []
        for line in m.group(2).splitlines():
            t = line.strip()
            if not t or t[0] in ";.":
                continue
            region.append(t)
            if t.startswith("s_barrier"):
                if any(x.startswith("buffer_load") and x.endswith("lds") for x in region):
                    yield m.group(1), region
                region = []


@pytest.mark.skipif(shutil.which(HIPCC) is None, reason="hipcc not available")
def test_stage_end_wait_covers_the_direct_to_lds_loads(tmp_path):
    with concurrent.futures.ThreadPoolExecutor(max_workers=3) as pool:
        texts = list(pool.map(lambda kv: _assembly(kv[0], kv[1], str(tmp_path)), UNITS.items()))
    checked = 0
    for text in texts:
        for name, reg in _stage_regions(text):
            is_load = [t.startswith("buffer_load") for t in reg]
            is_lds = [ld and t.endswith("lds") for ld, t in zip(is_load, reg)]
            first, last = is_lds.index(True), len(reg) - 1 - is_lds[::-1].index(True)
            assert not any(is_load[i] and not is_lds[i] for i in range(first, last)), (name, "loads interleaved")
            # (a) the direct-to-LDS loads have landed before the barrier: some wait after the last of them leaves at
            #     most as many loads outstanding as were issued between that load and the wait (the counter retires
            #     in order); a wait without a vmcnt field only counts where 63 or more loads separate them
            covered = False
            for i in range(last + 1, len(reg)):
                if not reg[i].startswith("s_waitcnt"):
                    continue
                younger = sum(1 for k in range(last + 1, i) if is_load[k])
                m = re.search(r"vmcnt\((\d+)\)", reg[i])
                if (m and int(m.group(1)) <= younger) or (not m and "lgkmcnt" in reg[i] and younger >= VMCNT_MAX):
                    covered = True
            assert covered, (name, "no wait covers the direct-to-LDS loads before the barrier")
            # (b) this wave's own LDS reads are done before it lets others overwrite the buffer
            ds = [i for i, t in enumerate(reg) if t.startswith("ds_read")]
            if ds:
                assert any(t.startswith("s_waitcnt") and "lgkmcnt(0)" in t for t in reg[ds[-1] + 1:]), (name, "LDS reads")
            checked += 1
    assert checked > 1200        # every instantiation has a prologue and PD*(PD+1) unrolled stages
