"""Static check of the attention kernel's generated code (CPU only: hipcc cross-compiles to assembly).

attn_h_kernel issues its LDS fragment reads and the wait for them as separate asm statements so that the reads
of one group of fragments fly under the MFMAs of the previous group.  That is only correct if the compiler leaves
the destination registers of an issued read alone until the wait: this test reads the listing of the built code
and fails if any instruction between a `ds_read_b128` of the main loop and the next `s_waitcnt lgkmcnt(0)`
touches a register that read is still writing.  It also fails on register spills inside the main loop of an attention kernel."""
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
    assert checked >= 2 * (32 + 16)   # fragment reads per step: 32 at head dim 128, 16 at head dim 64; two walks each


def _main_loop(body):
    """Text of the innermost loop that holds the MFMAs: from its label to the backward branch to that label."""
    best = ""
    for m in re.finditer(r"^(\.LBB\d+_\d+):", body, re.M):
        label = m.group(1)
        back = [b.end() for b in re.finditer(r"s_cbranch_\w+ %s\b|s_branch %s\b" % (re.escape(label), re.escape(label)),
                                             body[m.end():])]
        if back:
            span = body[m.end(): m.end() + back[-1]]
            if "v_mfma" in span and (not best or len(span) < len(best)):
                best = span
    return best


def test_attention_main_loops_do_not_spill(listing):
    n = 0
    for name in ("attn_h_kernel", "attn_kernel"):
        for sym, body in _kernel_bodies(listing, name):
            loop = _main_loop(body)
            assert loop.count("v_mfma") >= 8, sym
            assert "scratch_" not in loop, "%s: register spill inside the main loop" % sym
            n += 1
    assert n >= 8          # two head dims x (in-order, paced) for 128-token blocks, four shapes for the others
    # three wavefronts per SIMD need at most 168 registers in the 128-token kernels
    for b in re.split(r"\n  - \.agpr_count", listing):
        m = re.search(r"\.name:\s+(\S+)", b)
        if m and "attn_h_kernelILi128" in m.group(1) and not m.group(1).endswith(".kd"):
            assert int(re.search(r"\.vgpr_count:\s+(\d+)", b).group(1)) <= 168, m.group(1)
            # a few values that only the epilogue needs may sit in scratch over the loop; none is touched inside it
            assert int(re.search(r"\.vgpr_spill_count:\s+(\d+)", b).group(1)) <= 4, m.group(1)
