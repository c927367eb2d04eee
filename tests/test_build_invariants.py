"""Properties of the compiled gfx950 code that the kernels rely on and the compiler does not promise.

The dK/dV pass of the gradient kernels keeps its accumulators in the accumulation registers a0..a127 by name,
inside inline assembly.  That is only sound while the compiler allocates no accumulation register of its own
in those kernels (it would be free to use one between two of the assembly statements).  The check compiles the
translation unit to assembly (device side only, no GPU needed) and reads the register counts from the kernel
metadata: exactly the 128 named registers, no scratch memory.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="hipcc not available")
def test_dkv_kernels_keep_only_accumulators_and_owner_rows_in_accumulation_registers(tmp_path):
    from paper_2401_09486_amd import build as hip_build
    src = os.path.join(hip_build.CSRC, "loma_bwd_dkv.hip")
    out = str(tmp_path / "dkv.s")
    cmd = [hip_build.HIPCC, *hip_build.FLAGS, "--cuda-device-only", "-S", src, "-o", out]
    subprocess.run(cmd, check=True, capture_output=True)
    text = open(out).read()
    kernels = re.findall(r"\.agpr_count:\s+(\d+).*?\.name:\s+(\S+).*?\.private_segment_fixed_size:\s+(\d+)"
                         r".*?\.sgpr_spill_count:\s+(\d+).*?\.vgpr_count:\s+(\d+).*?\.vgpr_spill_count:\s+(\d+)", text, flags=re.S)
    dkv = [(name, int(agpr), int(scratch), int(sspill), int(vgpr), int(vspill))
           for agpr, name, scratch, sspill, vgpr, vspill in kernels if "bwd_dkv_kernel" in name]
    assert len(dkv) == 6, [k[0] for k in dkv]           # head_dim 64 and 128, 1, 2 and 4 waves
    for name, agpr, scratch, sspill, vgpr, vspill in dkv:
        head_dim = 128 if "ILi128E" in name else 64
        # a0..a127 by name, and past them the owner rows' k and v (operands of the S' and dP' MFMAs, head_dim / 2 registers)
        assert agpr == 128 + head_dim // 2, f"{name}: {agpr} accumulation registers allocated"
        assert scratch == 0, f"{name}: {scratch} bytes of scratch memory"
        # a value the compiler parks in an accumulation register between two assembly statements would be a spill
        # copy: none may exist, and the ordinary registers must not be exhausted (256 is the file's limit per wave)
        assert vspill == 0, f"{name}: {vspill} vector registers spilled"
        # vgpr_count is the sum of both files; 256 ordinary registers is the limit per wave
        assert vgpr - agpr <= 248, f"{name}: {vgpr - agpr} ordinary vector registers leave no headroom"
        # every access to an accumulation register outside the MFMAs is one of the kernel's own 128 clears or of its
        # final reads (one per accumulator: 2 * head_dim / 2); a copy the compiler parked there would add to these
        body = re.search(re.escape(name) + r":.*?\.Lfunc_end", text, flags=re.S).group(0)
        assert body.count("v_accvgpr_write") == 128, f"{name}: {body.count('v_accvgpr_write')} writes to accumulation registers"
        assert body.count("v_accvgpr_read") == head_dim, f"{name}: {body.count('v_accvgpr_read')} reads of accumulation registers"
        assert "v_accvgpr_mov" not in body
