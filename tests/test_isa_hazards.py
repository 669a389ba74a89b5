"""Static check of the compiled GEMM kernels (no GPU needed).

The tall tiles (256 and 288 rows) issue every MFMA through inline asm that names the register file of the
accumulator (AGPRs, and VGPRs for two token blocks of the 288-row tile), which the compiler's hazard
recogniser cannot see into.  Two things it would otherwise guarantee are checked here on the compiled code,
instruction by instruction and following branches: nothing but the next accumulating MFMA touches an MFMA's
result until it has been written (7 wait states after a 4-pass MFMA), and nothing writes an operand of an
asm MFMA in the wait states right before it.
"""
import os
import re
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from paper_2605_19945_amd import build as moe_build  # noqa: E402

NEED = 8           # wait states before anything else may touch the result (7 by the ISA tables, one to spare)
MFMA_PASSES = 4    # v_mfma_f32_16x16x32_bf16; the pipe takes the next MFMA when the previous one has gone through


def _regs(tok):
    """Registers named by an operand token, as (file, index) pairs: v7, v[2:5], a3, a[0:3]."""
    m = re.fullmatch(r"([va])\[(\d+):(\d+)\]", tok)
    if m:
        return {(m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1)}
    m = re.fullmatch(r"([va])(\d+)", tok)
    return {(m.group(1), int(m.group(2)))} if m else set()


def _split(line):
    body = line.split(";")[0].strip()
    parts = body.split(None, 1)
    if not parts:
        return "", []
    return parts[0], ([t.strip() for t in re.split(r",\s*", parts[1])] if len(parts) > 1 else [])


def find_hazards(lines, agpr_too=False):
    """Returns (number of MFMAs checked, list of hazard descriptions).  Checked are the MFMAs with a VGPR
    destination and, with agpr_too, those with an AGPR destination as well (kernels that issue every MFMA
    through inline asm)."""
    labels = {}
    for i, l in enumerate(lines):
        m = re.match(r"(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = i
    pinned, bad = 0, []
    for i, l in enumerate(lines):
        op, ops = _split(l)
        if not op.startswith("v_mfma") or not ops:
            continue
        if not (ops[0].startswith("v") or (agpr_too and ops[0].startswith("a"))):
            continue
        pinned += 1
        dst = _regs(ops[0])
        work, seen = [(i + 1, 0, MFMA_PASSES)], set()
        while work:
            j, t, free = work.pop()
            while j < len(lines) and t < NEED:
                s = lines[j].strip()
                j += 1
                if not s or s.startswith(";") or s.startswith("."):
                    continue
                o, oo = _split(s)
                if o == "s_nop":
                    t += int(oo[0]) + 1
                    continue
                if o.startswith("v_mfma"):
                    t = max(t, free)
                    free = t + MFMA_PASSES
                    touched = set().union(*[_regs(x) for x in oo]) & dst
                    if touched and not (oo[0] == oo[3] and _regs(oo[0]) == dst):
                        bad.append(f"line {j}: MFMA touches the result of line {i + 1} after {t} states: {s}")
                    t += 1
                    continue
                touched = set()
                for x in oo:
                    for tok in re.findall(r"[va]\[\d+:\d+\]|\b[va]\d+\b", x):
                        touched |= _regs(tok)
                if touched & dst:
                    bad.append(f"line {j}: touches the result of line {i + 1} after {t} states: {s}")
                    break
                if o == "s_endpgm":
                    break
                if o == "s_branch":
                    if oo[0] in seen:
                        break
                    seen.add(oo[0])
                    j = labels[oo[0]]
                elif o.startswith("s_cbranch") and oo[0] not in seen:
                    seen.add(oo[0])
                    work.append((labels[oo[0]], t + 1, free))
                t += 1
    return pinned, bad


WRITE_TO_MFMA = 4  # wait states between an instruction that writes a register and an asm MFMA that reads it


def find_late_writers(lines):
    """The other direction, for the MFMAs issued through inline asm (between the compiler's ASMSTART / ASMEND
    marks): an instruction other than an MFMA that writes one of their operand registers must lie at least
    WRITE_TO_MFMA wait states before them (the compiler inserts those states for the MFMAs it knows).  Scans
    back inside the basic block; loads are waited for explicitly and are not instructions of this kind."""
    bad, checked, in_asm = [], 0, False
    for i, l in enumerate(lines):
        s = l.strip()
        if s.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if s.startswith(";;#ASMEND"):
            in_asm = False
            continue
        op, ops = _split(s)
        if not in_asm or not op.startswith("v_mfma"):
            continue
        checked += 1
        reads = set().union(*[_regs(x) for x in ops[1:]])
        t, j = 0, i - 1
        while j >= 0 and t < WRITE_TO_MFMA:
            p = lines[j].strip()
            j -= 1
            if not p or p.startswith(";") or p.startswith("."):
                if re.match(r"\.LBB\d+_\d+:", p):
                    break
                continue
            o, oo = _split(p)
            if o == "s_nop":
                t += int(oo[0]) + 1
                continue
            if o.startswith("v_") and not o.startswith("v_mfma") and oo and (_regs(oo[0]) & reads):
                bad.append(f"line {j + 2}: writes an operand of the asm MFMA at line {i + 1} only {t} states before it: {p}")
                break
            t += 1
    return checked, bad


def find_touched_before_arrival(lines, limit=4000):
    """The weight loads are inline asm too (global_load_dwordx4 between ASMSTART / ASMEND), waited for with
    explicit counts: the compiler does not know that their destination registers are not valid yet and could
    copy or reuse them.  From every such load, walk forward along the fall-through path (a taken branch is
    followed, a conditional one is not) until an s_waitcnt whose vmcnt is no larger than the number of
    vector-memory instructions issued since -- or the next barrier, in front of which the kernel waits with a
    count it picks at run time -- and flag anything that names a destination register before that.  Returns
    (loads checked, hazards)."""
    labels = {}
    for i, l in enumerate(lines):
        m = re.match(r"(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = i
    bad, checked, in_asm = [], 0, False
    for i, l in enumerate(lines):
        s = l.strip()
        if s.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if s.startswith(";;#ASMEND"):
            in_asm = False
            continue
        op, ops = _split(s)
        if not in_asm or not op.startswith("global_load_dwordx4"):
            continue
        checked += 1
        dst = _regs(ops[0])
        later, j, steps, seen = 0, i + 1, 0, set()
        while j < len(lines) and steps < limit:
            p = lines[j].strip()
            j += 1
            if not p or p.startswith(";") or p.startswith("."):
                continue
            steps += 1
            o, oo = _split(p)
            if o == "s_waitcnt":
                m = re.search(r"vmcnt\((\d+)\)", p)
                if m and int(m.group(1)) <= later:
                    break
                continue
            if o == "s_barrier":
                break  # every load is waited for (with a count chosen at run time) before the next barrier
            touched = set()
            for x in oo:
                for tok in re.findall(r"[va]\[\d+:\d+\]|\b[va]\d+\b", x):
                    touched |= _regs(tok)
            if touched & dst:
                bad.append(f"line {j}: names a register of the load at line {i + 1} before it has been waited for: {p}")
                break
            if o.startswith(("global_", "buffer_", "scratch_", "flat_")):
                later += 1
            if o == "s_endpgm":
                break
            if o == "s_branch":
                if oo[0] in seen:
                    break
                seen.add(oo[0])
                j = labels[oo[0]]
    return checked, bad


def test_lint_flags_a_register_used_before_its_load_arrived():
    ld = ["\t;;#ASMSTART", "\tglobal_load_dwordx4 v[10:13], v1, s[2:3] offset:0", "\t;;#ASMEND"]
    other = ["\t;;#ASMSTART", "\tglobal_load_dwordx4 v[20:23], v1, s[2:3] offset:1024", "\t;;#ASMEND"]
    ok = ld + other + ["s_waitcnt vmcnt(1)", "v_mov_b32_e32 v5, v10", "s_endpgm"]
    assert find_touched_before_arrival(ok)[1] == []
    early = ld + other + ["v_mov_b32_e32 v5, v10", "s_waitcnt vmcnt(1)", "s_endpgm"]
    assert len(find_touched_before_arrival(early)[1]) == 1
    third = ["\t;;#ASMSTART", "\tglobal_load_dwordx4 v[30:33], v1, s[2:3] offset:2048", "\t;;#ASMEND"]
    not_enough = ld + other + third + ["s_waitcnt vmcnt(3)", "v_mov_b32_e32 v5, v11", "s_waitcnt vmcnt(0)", "s_endpgm"]
    assert len(find_touched_before_arrival(not_enough)[1]) == 1


def test_lint_flags_a_late_writer():
    mf = ["\t;;#ASMSTART", "\tv_mfma_f32_16x16x32_bf16 a[0:3], v[90:93], v[54:57], a[0:3]", "\t;;#ASMEND"]
    assert len(find_late_writers(["v_accvgpr_write_b32 a1, 0"] + mf)[1]) == 1
    assert len(find_late_writers(["v_mov_b32_e32 v91, 0", "s_nop 1"] + mf)[1]) == 1
    assert find_late_writers(["v_accvgpr_write_b32 a1, 0", "s_nop 3"] + mf) == (1, [])
    assert find_late_writers(["v_accvgpr_write_b32 a9, 0"] + mf) == (1, [])
    assert find_late_writers(["v_accvgpr_write_b32 a1, 0", mf[1]]) == (0, [])   # not an asm MFMA: the compiler's job


def test_lint_flags_an_early_reader():
    ok = ["v_mfma_f32_16x16x32_bf16 v[2:5], v[90:93], v[50:53], v[2:5]",
          "v_mfma_f32_16x16x32_bf16 a[0:3], v[90:93], v[54:57], a[0:3]",
          "v_mfma_f32_16x16x32_bf16 a[4:7], v[90:93], v[58:61], a[4:7]",
          "v_mfma_f32_16x16x32_bf16 a[8:11], v[90:93], v[62:65], a[8:11]",
          "v_mov_b32_e32 v100, v2", "s_endpgm"]
    assert find_hazards(ok) == (1, [])
    assert find_hazards(ok, agpr_too=True)[0] == 4
    early = [ok[0], ok[1], "v_mov_b32_e32 v100, v2", "s_endpgm"]
    assert len(find_hazards(early)[1]) == 1
    via_branch = [ok[0], "s_cbranch_scc1 .LBB0_1", ok[1], ok[2], ok[3], "s_endpgm", ".LBB0_1:",
                  "v_add_f32_e32 v3, v3, v4", "s_endpgm"]
    assert len(find_hazards(via_branch)[1]) == 1
    in_place = [ok[0], ok[0], "s_endpgm"]          # accumulating into the same registers again is fine
    assert find_hazards(in_place) == (2, [])
    # an accumulator in the other register file read too early
    early_agpr = [ok[1], "v_accvgpr_read_b32 v7, a1", "s_endpgm"]
    assert find_hazards(early_agpr) == (0, [])
    assert len(find_hazards(early_agpr, agpr_too=True)[1]) == 1
    late_agpr = [ok[1], ok[2], ok[3], "v_accvgpr_read_b32 v7, a1", "s_endpgm"]
    assert find_hazards(late_agpr, agpr_too=True) == (3, [])


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_no_hazard_around_the_mfmas_of_the_compiled_kernels(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    units = [u for u in moe_build.SOURCES if u.startswith("moe_gemm_")]   # every unit that instantiates the kernel
    assert len(units) == 7

    def compile_one(src):
        out = str(tmp_path / src.replace(".hip", ".s"))
        r = subprocess.run([hipcc, *moe_build.FLAGS, "-S", "--cuda-device-only", "-o", out,
                            os.path.join(moe_build.CSRC, src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        return out

    with ThreadPoolExecutor(len(units)) as ex:
        outs = list(ex.map(compile_one, units))
    for out in outs:
        with open(out) as fh:
            pinned, bad = find_hazards(fh.read().splitlines(), agpr_too=True)
        if out.endswith("pairsum.s"):
            assert pinned > 0
        else:
            assert pinned > 0, f"{out}: expected MFMAs"
        assert not bad, f"{out}:\n" + "\n".join(bad[:10])
        with open(out) as fh:
            n_asm, late = find_late_writers(fh.read().splitlines())
        assert not late, f"{out}:\n" + "\n".join(late[:10])
        with open(out) as fh:
            n_loads, early = find_touched_before_arrival(fh.read().splitlines())
        assert n_loads > 0 and not early, f"{out}:\n" + "\n".join(early[:10])
