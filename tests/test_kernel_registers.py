"""Host-side guard on the compiled kernels: the pipelined kernels run at the register limit, and a
spill inside their main loop is reloaded behind a wait for every outstanding global load, which
silently serialises the software pipeline.  The device assembly of the hot kernels must therefore
report no spilled registers.  (Compiles to assembly only: no GPU needed.)"""
import os
import re
import subprocess

import pytest

from paper_2605_07230_amd import build as B

# kernels that are allowed to spill: the widest residual-walk instantiation keeps 64 values per lane
ALLOWED = ("select_residual_kernelILi16E",)
HOT = ["lmhead.hip", "attn.hip", "accept.hip", "select.hip", "commit.hip", "weights.hip"]


def _kernel_stats(src, tmp_path):
    out = os.path.join(str(tmp_path), src.replace(".hip", ".s"))
    cmd = [B._hipcc(), *B.DEVICE_FLAGS, "-S", "--cuda-device-only", os.path.join(B.CSRC, src), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    text = open(out).read()
    stats = re.findall(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.vgpr_spill_count:\s+(\d+)", text)
    return stats


@pytest.mark.parametrize("src", HOT)
def test_hot_kernels_do_not_spill(src, tmp_path):
    stats = _kernel_stats(src, tmp_path)
    assert stats, "no kernels found in the assembly"
    bad = [(name, int(n)) for name, n in stats if int(n) and not any(a in name for a in ALLOWED)]
    assert not bad, bad
