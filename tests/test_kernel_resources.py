"""Compile-time guard (no GPU): the register-blocked min-plus kernel keeps its
table values in VGPRs, so a register spill in its loop costs a large factor.
Every instantiation must compile with zero scratch and reach the occupancy its
blocking table asks for."""
import os
import re
import subprocess

from paper_2307_02031_amd import build as b


def test_minplus_instantiations_do_not_spill(tmp_path):
    src = os.path.join(b.CSRC, "gbmw_kernels.hip")
    flags = [f for f in b.FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [b.HIPCC, *flags, "--cuda-device-only", "-c", "-Rpass-analysis=kernel-resource-usage", src,
           "-o", str(tmp_path / "k.o")]
    out = subprocess.run(cmd, check=True, capture_output=True, text=True).stderr
    blocks = re.split(r"remark: Function Name: ", out)[1:]
    seen = 0
    for blk in blocks:
        name = blk.split()[0]
        m = re.match(r"_ZN4gbmw9k_minplusILi(\d+)ELi\d+ELi\d+ELi\d+ELi(\d+)E", name)
        if not m:
            continue
        seen += 1
        scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", blk).group(1))
        occ = int(re.search(r"Occupancy \[waves/SIMD\]: (\d+)", blk).group(1))
        assert scratch == 0, f"{name}: {scratch} bytes of scratch per lane"
        assert occ >= int(m.group(2)), f"{name}: occupancy {occ} below the requested {m.group(2)}"
    assert seen == 288         # S' = 4..64 in steps of 4; first-layer and later-layer; with and without argmin records;
                               # three launch shapes (split, and unsplit with and without the run shortcut), and the
                               # counting twin of the last (measurements only, no occupancy target); S' = 68..128: with and
                               # without records
