"""Host-side check of the attention kernels' machine code (no GPU): the first instruction that
reads an MFMA result must come a number of issue slots after the MFMA: its passes + 3, i.e. 11
for the 8-pass 16x16x32 and 7 for the 4-pass 16x16x16.  The compiler inserts that wait inside a basic block; behind a
branch it was seen to leave it out, which is why the kernels idle explicitly
(mfma_result_wait in csrc/ha_rag_attend_dev.h).  This test compiles the two kernel sources to
assembly with the library's flags and follows every path from every MFMA, taken branches
included, until its destination registers are read or overwritten."""
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2510_20878_amd import build

NEED = {"16x16x32": 11, "16x16x16": 7}  # 8-pass and 4-pass MFMAs: passes + 3


def _need(instr, need):
    if need is not None:
        return need
    for shape, n in NEED.items():
        if shape in instr:
            return n
    return max(NEED.values())


def _regs(text):
    r = set()
    for a, b in re.findall(r"v\[(\d+):(\d+)\]", text):
        r |= set(range(int(a), int(b) + 1))
    for a in re.findall(r"\bv(\d+)\b", text):
        r.add(int(a))
    return r


def _split(instr):
    """(destination operand text, source operands text) of one instruction line."""
    parts = instr.split(None, 1)
    if len(parts) < 2:
        return "", ""
    ops = parts[1].split(",", 1)
    return ops[0], ops[1] if len(ops) > 1 else ""


def early_readers(asm_text, need=None):
    lines = asm_text.split("\n")
    label = {l.split(":")[0]: i for i, l in enumerate(lines) if re.match(r"\.LBB\d+_\d+:", l)}
    found, n_mfma = [], 0
    for i, l in enumerate(lines):
        m = re.match(r"\s+v_mfma_\S+ v\[(\d+):(\d+)\]", l)
        if not m:
            continue
        n_mfma += 1
        limit = _need(l, need)
        dst = set(range(int(m.group(1)), int(m.group(2)) + 1))
        work, seen = [(i + 1, 0)], set()
        while work:
            j, slots = work.pop()
            while j < len(lines) and slots < limit and j not in seen:
                seen.add(j)
                t = lines[j].strip()
                if not t or t[0] in ";.":
                    j += 1
                    continue
                if t.startswith("s_endpgm"):
                    break
                if t.startswith("s_nop"):
                    slots += int(t.split()[1]) + 1
                elif t.startswith(("s_cbranch", "s_branch")):
                    tgt = t.split()[-1]
                    if tgt in label:
                        work.append((label[tgt] + 1, slots + 1))
                    if t.startswith("s_branch"):
                        break
                    slots += 1
                else:
                    d, s = _split(t)
                    is_store = t.startswith(("ds_write", "global_store", "flat_store", "scratch_store", "buffer_store"))
                    if t.startswith("v_mfma"):
                        if _regs(d) & dst:
                            break  # the next MFMA of the chain: the hardware orders those
                    elif _regs(s) & dst or (is_store and _regs(t) & dst):
                        found.append((i + 1, j + 1, slots, t))
                        break
                    elif _regs(d) & dst:
                        break  # overwritten before anything read it
                    slots += 1
                j += 1
    return n_mfma, found


def test_the_scan_sees_a_reader_behind_a_taken_branch_and_accepts_explicit_idling():
    bad = """
	v_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]
	v_or_b32_e32 v20, s0, v1
	s_cbranch_vccz .LBB0_2
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
	v_mov_b32_e32 v21, v20
.LBB0_2:
	v_max_f32_e32 v22, v6, v7
	s_endpgm
"""
    n, found = early_readers(bad)
    assert n == 1 and len(found) == 1 and found[0][2] == 2
    good = bad.replace("	v_or_b32_e32 v20, s0, v1\n", "	s_nop 7\n	s_nop 3\n")
    assert early_readers(good) == (1, [])


@pytest.mark.timeout(600)
def test_no_attention_kernel_reads_an_mfma_result_too_early():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc here")
    sources = ["ha_rag_attend_kernels.hip", "ha_rag_attend_shared.hip"]
    with tempfile.TemporaryDirectory() as tmp:
        def asm(src):
            out = os.path.join(tmp, src + ".s")
            flags = [f for f in build.HIPCC_FLAGS if f != "-fPIC"]
            r = subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only", "-o", out,
                                                  os.path.join(build.CSRC, src)], capture_output=True, text=True)
            assert r.returncode == 0, r.stderr[-2000:]
            return open(out).read()
        with ThreadPoolExecutor(2) as pool:
            texts = list(pool.map(asm, sources))
    for src, text in zip(sources, texts):
        n, found = early_readers(text)
        assert n > 100, (src, n)
        assert not found, (src, found[:5])
