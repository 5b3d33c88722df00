"""The instruction order the compiler chose for the matrix-core kernels, read from the gfx950
assembly that the build leaves beside the objects (no GPU needed).

A matrix instruction delivers its 16 result registers some issue slots after it starts, and nothing
in the hardware holds back a vector, LDS or memory instruction that reads one of them too early:
the compiler inserts wait states (11 for this instruction when it sees the pair in straight-line
code).  One order tried in the long-row scan had the compiler leave five issue slots between a
matrix instruction in the middle of one block and the first read of its results in the next, and
the GPU then lost candidates now and then.  The kernels keep every read at least 11 issue slots
behind the matrix instruction on every fall-through path; this test holds them to it."""
import os
import re

import pytest

from paper_2110_08919_amd import build as lpq_build

NEED = 11


def _regs(tok):
    out = []
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", tok):
        if m.group(1):
            out += list(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.append(int(m.group(3)))
    return out


def _closest_reads(path):
    """(kernel, issue slots, line of the read, line of the matrix instruction, text) for every read of
    a matrix result closer than NEED issue slots on a fall-through path."""
    found = []
    kern, pos, last = None, 0, {}
    for ln, line in enumerate(open(path), 1):
        m = re.match(r"^(_Z\S+):", line)
        if m:
            kern, pos, last = m.group(1), 0, {}
            continue
        if kern is None:
            continue
        if line.startswith(".Lfunc_end"):
            kern = None
            continue
        s = line.strip()
        if not s or s[0] in ";." or s.endswith(":"):
            continue
        op = s.split()[0]
        if op == "s_nop":
            pos += int(s.split()[1]) + 1
            continue
        pos += 1
        if op in ("s_branch", "s_setpc_b64", "s_endpgm"):
            last = {}                      # nothing falls through
            continue
        parts = s[len(op):].split(";")[0].split(",")
        if op.startswith("v_mfma"):
            for r in _regs(parts[0]):
                last[r] = (pos, ln)
            continue
        if not op.startswith(("v_", "ds_", "global_", "scratch_", "buffer_", "flat_")):
            continue
        writes_first = op.startswith("v_") and not (op.startswith("v_cmp") and not op.endswith("_e64"))
        for tok in (parts[1:] if writes_first else parts):
            for r in _regs(tok):
                if r in last:
                    if pos - last[r][0] < NEED:
                        found.append((kern, pos - last[r][0], ln, last[r][1], s[:70]))
                    del last[r]
        if writes_first:
            for r in _regs(parts[0]):
                last.pop(r, None)
    return found


@pytest.mark.parametrize("source", ["search_mfma.hip", "search_mfma_lds.hip"])
def test_no_read_of_a_matrix_result_sooner_than_the_wait_states_it_needs(source):
    lpq_build.build()                      # incremental; writes the assembly if it is not there yet
    path = lpq_build.device_asm(os.path.join(lpq_build.CSRC, source))
    assert os.path.exists(path), f"{path} missing: the build keeps the device assembly of {source}"
    kernels = sum(1 for line in open(path) if re.match(r"^_Z\S+:", line))
    assert kernels >= 4, "no kernels found in the assembly"
    bad = _closest_reads(path)
    assert not bad, f"{len(bad)} reads of matrix results within {NEED} issue slots, e.g. {sorted(bad, key=lambda b: b[1])[:3]}"


def test_the_checker_sees_a_planted_early_read(tmp_path):
    text = """_Zkernel:
\tv_mfma_i32_32x32x32_i8 v[0:15], v[20:23], v[24:27], v[0:15]
\tv_add_u32_e32 v40, v41, v42
\ts_nop 3
\tv_max_i32_e32 v30, v0, v1
\tv_mfma_i32_32x32x32_i8 v[0:15], v[20:23], v[24:27], v[0:15]
\ts_nop 10
\tv_max_i32_e32 v30, v0, v1
.Lfunc_end0:
"""
    p = tmp_path / "k.s"
    p.write_text(text)
    bad = _closest_reads(str(p))
    assert len(bad) == 2 and {b[1] for b in bad} == {6} and {b[2] for b in bad} == {5}   # v0 and v1, six slots after line 2; the second read is fine
