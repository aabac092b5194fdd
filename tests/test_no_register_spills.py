"""Host-only: the kernels of the library compile without register spills and without scratch memory.

The tuned main loop fences its global -> LDS pipeline with hand-counted `s_waitcnt vmcnt(N)`; scratch loads and
stores that the compiler inserts for spilled registers use the same counter, so a spill inside that loop would
silently break the count, and spills anywhere turn into memory traffic per tile.  This compiles the library's
source for gfx950 with the compiler's own resource-usage remarks and checks every kernel (no GPU needed).
"""
import re
import subprocess

import pytest

from paper_2511_17599_amd import build as BLD


def kernel_resource_usage(tmp_path):
    out = tmp_path / "remarks.so"
    flags = [f for f in BLD.HIPCC_FLAGS]
    cmd = [BLD.hipcc_path(), *flags, "-Rpass-analysis=kernel-resource-usage", BLD.SRC, "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    usage = {}
    for block in re.split(r"remark: [^\n]*Function Name: ", res.stderr)[1:]:
        name = block.split()[0]
        fields = {}
        for key, pat in (("vgpr_spill", r"VGPRs Spill: (\d+)"), ("sgpr_spill", r"SGPRs Spill: (\d+)"),
                         ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"), ("vgprs", r" VGPRs: (\d+)"),
                         ("agprs", r"AGPRs: (\d+)"), ("occupancy", r"Occupancy \[waves/SIMD\]: (\d+)")):
            m = re.search(pat, block)
            assert m, (name, key)
            fields[key] = int(m.group(1))
        usage[name] = fields
    return usage


def test_no_kernel_spills_or_uses_scratch(tmp_path):
    usage = kernel_resource_usage(tmp_path)
    tuned = [n for n in usage if "FastLoop" in n]
    # the benchmarked instantiations are all there: forward, recompute, both contractions
    for piece in ("fwd_tiles_kernel", "recompute_kernel", "contract_kernel"):
        assert any(piece in n for n in tuned), piece
    assert len(usage) >= 30
    bad = {n: u for n, u in usage.items() if u["vgpr_spill"] or u["sgpr_spill"] or u["scratch"]}
    assert not bad, bad
    # one wavefront per SIMD in the tuned kernels: the whole accumulation register file holds the 256 x 256 tile
    for n in tuned:
        assert usage[n]["agprs"] == 256 and usage[n]["occupancy"] == 1, (n, usage[n])
