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
    return stats, text


@pytest.mark.parametrize("src", HOT)
def test_hot_kernels_do_not_spill(src, tmp_path):
    stats, _ = _kernel_stats(src, tmp_path)
    assert stats, "no kernels found in the assembly"
    bad = [(name, int(n)) for name, n in stats if int(n) and not any(a in name for a in ALLOWED)]
    assert not bad, bad


def test_tiled_projection_m0_and_waits(tmp_path):
    """The tiled projection sets M0 by hand for its LDS-direct loads (the compiler is not told), and
    its software pipeline relies on partial waits: M0 must have no other user in that kernel, and
    its main loop must not contain a wait for ALL outstanding loads."""
    _, text = _kernel_stats("lmhead.hip", tmp_path)
    bodies = re.findall(r"^(_ZN\S*lmhead_bf16_tiled_kernel\S*):[^\n]*\n(.*?)s_endpgm", text, flags=re.S | re.M)
    assert len(bodies) == 3          # guidance pairs, plain rows, plain rows in 128-row tiles
    for name, body in bodies:
        m0 = [l.strip() for l in body.splitlines() if re.search(r"\bm0\b", l)]
        assert m0 and all(l.startswith("s_mov_b32 m0,") for l in m0), (name, m0[:5])
        assert body.count("global_load_lds_dwordx4") >= 16
        loop = body[body.index("Inner Loop Header"):]
        loop = loop[:loop.index("s_cbranch_scc")]
        assert "vmcnt(0)" not in loop, name
        half = "Lb0ELb1E" in name        # <CFG = false, HALF = true>: 2 x 2 accumulators per wave
        assert loop.count("s_barrier") == 4 and loop.count("v_mfma_f32_32x32x16_bf16") == (32 if half else 64), name


def test_ring_attention_m0_and_waits(tmp_path):
    """The large-tree attention kernel fills its LDS rings with LDS-direct loads (M0 set by hand) three
    tiles ahead and waits with partial counts: inside the tile loop (unrolled once per ring stage, one
    barrier each) there must be no wait for ALL outstanding loads, and nothing in the kernel may go
    through scratch memory; the only full wait is the one that drains the ring before the epilogue."""
    _, text = _kernel_stats("attn.hip", tmp_path)
    bodies = re.findall(r"^(_ZN\S*attn_bf16_ring_kernel\S*):[^\n]*\n(.*?)s_endpgm", text, flags=re.S | re.M)
    assert len(bodies) == 2
    for name, body in bodies:
        m0 = [l.strip() for l in body.splitlines() if re.search(r"\bm0\b", l)]
        assert m0 and all(l.startswith("s_mov_b32 m0,") for l in m0), (name, m0[:5])
        assert "scratch_" not in body, name
        start = body.index("=>This Loop Header: Depth=1")       # the tile loop (it has the masks' climbs inside)
        end = body.rindex("vmcnt(0)")                           # the drain after the loop
        loop = body[start:end]
        assert "vmcnt(0)" not in loop, name
        assert loop.count("s_barrier") == 3, name
        assert loop.count("global_load_lds_dwordx4") >= 6
        # Inline assembly is invisible to the compiler's hazard padding: a vector ALU instruction in it could read
        # an MFMA result before the matrix core has written it.  Only waits, barriers, M0 and the LDS-direct
        # loads may be written that way.
        inline = re.findall(r";;#ASMSTART\n(.*?);;#ASMEND", body, flags=re.S)
        ops = {l.split()[0] for blk in inline for l in blk.strip().splitlines()}
        assert ops <= {"s_waitcnt", "s_barrier", "s_mov_b32", "s_nop", "global_load_lds_dwordx4"}, (name, ops)


def test_row_statistics_prefetch_uses_m0_only_for_its_loads(tmp_path):
    """The long-row statistics kernel prefetches part of the next row with LDS-direct loads (M0 set by hand,
    the compiler is not told): nothing else in that kernel may touch M0."""
    _, text = _kernel_stats("lmhead.hip", tmp_path)
    bodies = re.findall(r"^(_ZN\S*row_stats_kernelILi64ELb1E\S*):[^\n]*\n(.*?)\.amdhsa_kernel", text, flags=re.S | re.M)
    assert len(bodies) == 1
    name, body = bodies[0]
    m0 = [l.strip() for l in body.splitlines() if re.search(r"\bm0\b", l)]
    assert m0 and all(l.startswith("s_mov_b32 m0,") for l in m0), (name, m0[:5])
    assert body.count("global_load_lds_dwordx4") >= 8 and "scratch_" not in body
