"""Static check of the attention kernel's generated code (CPU only: hipcc cross-compiles to assembly).

attn_h_kernel issues its LDS fragment reads and the wait for them as separate asm statements so that the reads
of one group of fragments fly under the MFMAs of the previous group.  That is only correct if the compiler leaves
the destination registers of an issued read alone until the wait: this test reads the listing of the built code
and fails if any instruction between a `ds_read_b128` of the main loop and the next `s_waitcnt lgkmcnt(0)`
touches a register that read is still writing.  It also fails on register spills in the attention kernels."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_16864_amd", "csrc")


@pytest.fixture(scope="module")
def listing(tmp_path_factory):
    if shutil.which("hipcc") is None:
        pytest.skip("no hipcc")
    out = str(tmp_path_factory.mktemp("isa") / "jenga_attn.s")
    cmd = ["hipcc", "-O3", "--offload-arch=gfx950", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-S", "--cuda-device-only",
           "-o", out, os.path.join(CSRC, "jenga_attn.hip")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return open(out).read()


def _regs(text):
    """Set of VGPR numbers named in an operand string."""
    regs = set()
    for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text):
        regs.update(range(int(a), int(b) + 1))
    for a in re.findall(r"\bv(\d+)\b", text):
        regs.add(int(a))
    return regs


def _kernel_bodies(listing, name):
    for m in re.finditer(r"^(_Z\w*%s\w*):.*?^\.Lfunc_end" % name, listing, re.S | re.M):
        yield m.group(1), m.group(0)


def test_fragment_registers_untouched_between_read_and_wait(listing):
    checked = 0
    for sym, body in _kernel_bodies(listing, "attn_h_kernel"):
        pending = set()
        for line in body.split("\n"):
            ins = line.split(";")[0].strip()
            if not ins or ins.endswith(":") or ins.startswith("."):
                continue
            op, _, rest = ins.partition(" ")
            if op == "s_waitcnt" and "lgkmcnt(0)" in rest:
                pending.clear()
                continue
            if op == "ds_read_b128":
                dst, _, addr = rest.partition(",")
                assert not (_regs(dst) & pending), "%s: %s overwrites a fragment still being read" % (sym, ins)
                assert not (_regs(addr) & pending), "%s: %s" % (sym, ins)
                pending |= _regs(dst)
                checked += 1
                continue
            assert not (_regs(rest) & pending), "%s: `%s` touches a fragment register before the wait" % (sym, ins)
    assert checked >= 32 + 16         # fragment reads per step: 32 at head dim 128, 16 at head dim 64


def test_attention_kernels_do_not_spill(listing):
    meta = re.findall(r"\.name:\s+(\S*attn\w*)\n(?:.*\n)*?\s+\.vgpr_spill_count:\s+(\d+)", listing)
    blocks = re.split(r"\n  - \.agpr_count", listing)
    n = 0
    for b in blocks:
        m = re.search(r"\.name:\s+(\S+)", b)
        if not m or "attn" not in m.group(1) or "kernel" not in m.group(1):
            continue
        if m.group(1).endswith(".kd"):
            continue
        sp = re.search(r"\.vgpr_spill_count:\s+(\d+)", b)
        ss = re.search(r"\.sgpr_spill_count:\s+(\d+)", b)
        vg = re.search(r"\.vgpr_count:\s+(\d+)", b)
        assert sp and ss and vg
        assert int(sp.group(1)) == 0, (m.group(1), "vgpr spills", sp.group(1))
        if "attn_h_kernelILi128" in m.group(1):
            assert int(vg.group(1)) <= 168, "three wavefronts per SIMD need at most 168 registers"
            assert int(ss.group(1)) == 0
        n += 1
    assert n >= 6
