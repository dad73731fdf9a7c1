"""Host-side check of the compiled gfx950 code for two hazards around the tile copies (LDS-DMA loads issued as
assembly text, which the compiler's hazard recogniser does not look into):
  * a vector-memory instruction must not read a scalar register within five wait states of a vector-ALU write to it
    (v_readlane restoring a spilled scalar, v_readfirstlane, v_cmp): the copy would fetch from a stale address;
  * an LDS-DMA instruction needs one wait state after a scalar write of M0.
The kernels' sources are compiled to assembly here (no GPU needed) and every copy instruction is checked against the
instructions before it.  The scanner itself is pinned on two hand-written snippets that contain the mistakes."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2605_14877_amd import build as hb

SOURCES_WITH_COPIES = ["attend.hip", "calibrate.hip", "probe.hip"]
VALU_SGPR_WRITERS = ("v_readlane_b32", "v_readfirstlane_b32", "v_cmp", "v_add_co", "v_sub_co", "v_subrev_co",
                     "v_addc_co", "v_subb_co", "v_div_scale")


def _sregs(tok):
    tok = tok.strip(",")
    m = re.fullmatch(r"s\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"s(\d+)", tok)
    if m:
        return {int(m.group(1))}
    if tok == "vcc":
        return {"vcc"}
    return set()


def scan(asm_text):
    """Returns (number of copy instructions seen, list of hazard descriptions)."""
    valu_age = {}   # scalar register -> wait states since a vector-ALU instruction wrote it
    m0_age = None   # wait states since a scalar instruction wrote M0
    copies, hazards = 0, []
    for no, raw in enumerate(asm_text.split("\n"), 1):
        line = raw.split(";")[0].strip()
        if not line or line.startswith(".") or line.endswith(":"):
            continue
        toks = line.split()
        op, args = toks[0], toks[1:]
        if op.startswith("global_load_lds"):
            copies += 1
            base = set()
            for a in args:
                base |= _sregs(a)
            for r in sorted(base, key=str):
                if r in valu_age and valu_age[r] < 5:
                    hazards.append(f"line {no}: {line}: s{r} written by the vector ALU {valu_age[r]} wait states before")
            if m0_age is not None and m0_age < 1:
                hazards.append(f"line {no}: {line}: M0 written by the instruction right before")
        step = int(args[0]) + 1 if op == "s_nop" else 1
        valu_age = {r: a + step for r, a in valu_age.items() if a + step < 16}
        if m0_age is not None:
            m0_age += step
        if args:
            dst = args[0].strip(",")
            if op.startswith("s_") and not op.startswith(("s_cmp", "s_cbranch", "s_branch", "s_waitcnt", "s_nop",
                                                          "s_barrier", "s_endpgm", "s_setprio", "s_sleep")):
                for r in _sregs(dst):
                    valu_age.pop(r, None)  # the scalar ALU wrote it last: no wait states needed
                if dst == "m0":
                    m0_age = 0
            elif op.startswith(VALU_SGPR_WRITERS):
                for r in _sregs(dst):
                    valu_age[r] = 0
    return copies, hazards


def test_scanner_sees_a_planted_stale_address_and_a_planted_m0_hazard():
    stale = """
    v_readlane_b32 s6, v255, 4
    v_readlane_b32 s7, v255, 5
    s_nop 0
    global_load_lds_dwordx4 v213, s[6:7]
    """
    n, hz = scan(stale)
    assert n == 1 and len(hz) == 2 and "s6" in hz[0] and "s7" in hz[1]
    fixed = stale.replace("s_nop 0", "s_mov_b64 s[8:9], s[6:7]").replace("v213, s[6:7]", "v213, s[8:9]")
    assert scan(fixed) == (1, [])
    waited = stale.replace("s_nop 0", "s_nop 4")
    assert scan(waited) == (1, [])
    m0 = """
    s_add_u32 s4, s2, 0x1000
    s_mov_b32 m0, s11
    global_load_lds_dwordx4 v2, s[4:5]
    """
    n, hz = scan(m0)
    assert n == 1 and len(hz) == 1 and "M0" in hz[0]
    assert scan(m0.replace("global_load_lds", "s_mov_b64 s[6:7], s[4:5]\n    global_load_lds")) == (1, [])


def test_no_tile_copy_reads_a_stale_scalar_or_a_fresh_m0():
    with tempfile.TemporaryDirectory() as tmp:
        procs = []
        for src in SOURCES_WITH_COPIES:
            out = os.path.join(tmp, src + ".s")
            cmd = ["hipcc", *hb.HIP_FLAGS, "-S", "--cuda-device-only", os.path.join(hb.CSRC, src), "-o", out]
            procs.append((src, out, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        total = 0
        for src, out, pr in procs:
            log, _ = pr.communicate()
            assert pr.returncode == 0, (src, log[-2000:])
            with open(out) as f:
                copies, hazards = scan(f.read())
            assert copies > 0, src
            assert not hazards, (src, hazards[:8])
            total += copies
        print(f"{total} copy instructions checked")
