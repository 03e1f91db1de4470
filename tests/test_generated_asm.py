"""Static checks of the gfx950 assembly the compiler generates for the attention kernels (CPU only: hipcc
cross-compiles).  The kernels issue their LDS operand reads through inline assembly and wait for them with
explicit s_waitcnt; the compiler knows nothing about those waits, so two things are checked on its output:

  1. inline assembly contains nothing but LDS reads/writes and s_waitcnt (a vector instruction issued through
     inline assembly gets none of the wait states the hardware needs after a matrix instruction);
  2. no instruction touches the destination registers of a hand-issued LDS read before an s_waitcnt lgkmcnt that
     covers it (LDS operations return in order, so a read is complete once at most N operations issued after
     it are outstanding and the wait asks for <= N).

The walk is linear over the text of each kernel, which is how the kernels' loops are laid out."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2502_04507_amd import build_lib

KERNEL_FILES = ["sta_attention.hip", "sta_backward.hip"]


def _assembly(src):
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [build_lib.HIPCC] + build_lib.FLAGS + ["-save-temps=obj", "-c", os.path.join(build_lib.CSRC, src), "-o",
                                                     os.path.join(tmp, "x.o")]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        name = [f for f in os.listdir(tmp) if f.endswith(".s") and "amdgcn" in f]
        assert len(name) == 1, os.listdir(tmp)
        return open(os.path.join(tmp, name[0])).read()


def _kernels(text):
    for m in re.finditer(r"^(\S+):\s*; @\S+\n", text, re.M):
        end = text.find(".Lfunc_end", m.end())
        if end > 0:
            yield m.group(1), text[m.end():end]


def _vregs(line):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", line):
        out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", line):
        out.add(int(m.group(1)))
    return out


@pytest.fixture(scope="module", params=KERNEL_FILES)
def asm(request):
    return request.param, _assembly(request.param)


def test_inline_assembly_is_only_lds_access_and_waits(asm):
    src, text = asm
    seen = 0
    for name, body in _kernels(text):
        for block in re.findall(r";;#ASMSTART\n(.*?);;#ASMEND", body, re.S):
            for line in block.split("\n"):
                line = line.split(";")[0].strip()
                if not line:
                    continue
                seen += 1
                op = line.split()[0]
                assert op.startswith("ds_read") or op.startswith("ds_write") or op == "s_waitcnt", (src, name, line)
    assert seen > 100, "expected the hand-issued operand reads in %s" % src


def test_hand_issued_lds_reads_are_waited_for_before_use(asm):
    src, text = asm
    checked = 0
    for name, body in _kernels(text):
        lines = [l.split(";")[0].strip() for l in body.split("\n")]
        lines = [l for l in lines if l and not l.startswith(".") and not l.endswith(":")]
        pending = []                                    # [destination registers, LDS/SMEM ops issued after, text]
        for l in lines:
            op = l.split()[0]
            if op == "s_waitcnt":
                m = re.search(r"lgkmcnt\((\d+)\)", l)
                if m:
                    pending = [p for p in pending if p[1] < int(m.group(1))]
                continue
            used = _vregs(l)
            for p in pending:
                assert not (p[0] & used), "%s %s: '%s' touches v%s before the wait that covers '%s'" % (
                    src, name, l, sorted(p[0] & used), p[2])
            if op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load"):
                for p in pending:
                    p[1] += 1
            if op.startswith("ds_read"):
                pending.append([_vregs(l.split(",")[0]), 0, l])
                checked += 1
    assert checked > 100, "expected the hand-issued operand reads in %s" % src


def test_checker_catches_a_planted_early_use():
    """The same walk on a hand-written snippet in which a register is used one wait too early."""
    snippet = ["ds_read_b128 v[4:7], v1 offset:0", "ds_read_b128 v[8:11], v1 offset:32", "s_waitcnt lgkmcnt(1)",
               "v_add_f32 v20, v4, v5", "v_add_f32 v21, v8, v9"]
    pending, hit = [], None
    for l in snippet:
        op = l.split()[0]
        if op == "s_waitcnt":
            n = int(re.search(r"lgkmcnt\((\d+)\)", l).group(1))
            pending = [p for p in pending if p[1] < n]
            continue
        for p in pending:
            if p[0] & _vregs(l):
                hit = l
        if op.startswith("ds_"):
            for p in pending:
                p[1] += 1
        if op.startswith("ds_read"):
            pending.append([_vregs(l.split(",")[0]), 0, l])
    assert hit == "v_add_f32 v21, v8, v9"
