"""The build's device pass really has packed fp32 arithmetic switched off: the gfx950 assembly of
the kernels holds no packed fp32 add / multiply / fma (the kernels add float4 vectors, which is
exactly the shape those instructions would be made from)."""
import re
import shutil
import subprocess

import pytest

from paper_2004_14020_amd import build


@pytest.mark.skipif(shutil.which(build.hipcc()) is None, reason="hipcc not available")
def test_device_assembly_has_no_packed_fp32_arithmetic():
    src = f"{build.HERE}/csrc/kernels.hip"
    cmd = [build.hipcc(), *build.flags(), "--cuda-device-only", "-S", src, "-o", "-"]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-2000:]
    asm = res.stdout
    assert "k_ring_reduce" in asm and "v_add_f32" in asm
    assert not re.search(r"\bv_pk_(add|mul|fma)_f32\b", asm)
    # the same sources without the switch do use them, so the check above is not vacuous
    plain = [a for a in cmd if a not in build.DEVICE_FEATURE]
    res2 = subprocess.run(plain, capture_output=True, text=True, timeout=600)
    assert res2.returncode == 0 and re.search(r"\bv_pk_(add|mul|fma)_f32\b", res2.stdout)
