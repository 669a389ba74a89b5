"""Static check of the compiled GEMM kernels (no GPU needed).

The 288-row tile keeps its ninth row block's accumulators in VGPRs and issues those MFMAs through
inline asm, which the compiler's hazard recogniser cannot see into: nothing but the next accumulating
MFMA may touch such a result until the MFMA has written it (11 wait states after an 8-pass MFMA).  The
kernel places these MFMAs first in every sub-step so that other MFMAs always follow; this test
compiles the kernels to ISA and verifies it instruction by instruction, following branches.
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

NEED = 12          # wait states before anything else may touch the result
MFMA_PASSES = 8    # v_mfma_f32_32x32x16_bf16; the pipe takes the next MFMA when the previous one has gone through


def _regs(tok):
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", tok)
    return {int(m.group(1))} if m else set()


def _split(line):
    body = line.split(";")[0].strip()
    parts = body.split(None, 1)
    if not parts:
        return "", []
    return parts[0], ([t.strip() for t in re.split(r",\s*", parts[1])] if len(parts) > 1 else [])


def find_hazards(lines):
    """Returns (number of VGPR-destination MFMAs, list of hazard descriptions)."""
    labels = {}
    for i, l in enumerate(lines):
        m = re.match(r"(\.LBB\d+_\d+):", l)
        if m:
            labels[m.group(1)] = i
    pinned, bad = 0, []
    for i, l in enumerate(lines):
        op, ops = _split(l)
        if not op.startswith("v_mfma") or not ops or not ops[0].startswith("v"):
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
                    for tok in re.findall(r"v\[\d+:\d+\]|v\d+", x):
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


def test_lint_flags_an_early_reader():
    ok = ["v_mfma_f32_32x32x16_bf16 v[2:17], v[90:93], v[50:53], v[2:17]",
          "v_mfma_f32_32x32x16_bf16 a[0:15], v[90:93], v[54:57], a[0:15]",
          "v_mfma_f32_32x32x16_bf16 a[16:31], v[90:93], v[58:61], a[16:31]",
          "v_mov_b32_e32 v100, v2", "s_endpgm"]
    assert find_hazards(ok) == (1, [])
    early = [ok[0], "s_nop 0", "v_mov_b32_e32 v100, v2", "s_endpgm"]
    assert len(find_hazards(early)[1]) == 1
    via_branch = [ok[0], "s_cbranch_scc1 .LBB0_1", ok[1], ok[2], "s_endpgm", ".LBB0_1:", "v_add_f32_e32 v3, v3, v4",
                  "s_endpgm"]
    assert len(find_hazards(via_branch)[1]) == 1
    in_place = [ok[0], ok[0], "s_endpgm"]          # accumulating into the same registers again is fine
    assert find_hazards(in_place) == (2, [])


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_no_reader_follows_a_vgpr_accumulating_mfma_too_closely(tmp_path):
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
            pinned, bad = find_hazards(fh.read().splitlines())
        if out.endswith("pairsum.s"):
            assert pinned == 0, f"{out}: the router-logit unit is built without the 288-row tile"
        else:
            assert pinned > 0, f"{out}: expected MFMAs with a VGPR destination (the ninth row block of the 288-row tile)"
        assert not bad, f"{out}:\n" + "\n".join(bad[:10])
