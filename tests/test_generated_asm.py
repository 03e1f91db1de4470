"""Static checks of the gfx950 assembly the compiler generates for the attention kernels (CPU only: hipcc
cross-compiles).  The kernels issue their LDS operand reads through inline assembly and wait for them with
explicit s_waitcnt; the compiler knows nothing about those waits, so two things are checked on its output:

  1. inline assembly contains nothing but LDS reads/writes and s_waitcnt (a vector instruction issued through
     inline assembly gets none of the wait states the hardware needs after a matrix instruction);
  2. no instruction touches the destination registers of a hand-issued LDS read before an s_waitcnt lgkmcnt that
     covers it (LDS operations return in order, so a read is complete once at most N operations issued after
     it are outstanding and the wait asks for <= N).

The second check is a forward data-flow analysis over each kernel's control-flow graph (basic blocks from the
labels and branches of the text), so a read pending on any path into an instruction counts."""
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


def _blocks(body):
    """Basic blocks of one kernel's text: name -> (instructions, successors).  A block starts at a label or after
    a branch; it falls through to the next block unless it ends in s_branch / s_endpgm / s_setpc."""
    blocks, order = {}, []
    name, cur, auto = "entry", [], 0
    for raw in body.split("\n"):
        l = raw.split(";")[0].strip()
        if not l or l.startswith("."):
            m = re.match(r"^(\.LBB\S+):", l)
            if not m:
                continue
            blocks[name] = cur
            order.append(name)
            name, cur = m.group(1), []
            continue
        if l.endswith(":"):
            continue
        cur.append(l)
        op = l.split()[0]
        if op.startswith("s_cbranch") or op in ("s_branch", "s_endpgm") or op.startswith("s_setpc"):
            blocks[name] = cur
            order.append(name)
            auto += 1
            name, cur = "after%d" % auto, []
    blocks[name] = cur
    order.append(name)
    succ = {}
    for i, n in enumerate(order):
        out = []
        last = blocks[n][-1] if blocks[n] else ""
        op = last.split()[0] if last else ""
        if op.startswith("s_cbranch") or op == "s_branch":
            out.append(last.split()[-1])
        if not (op in ("s_branch", "s_endpgm") or op.startswith("s_setpc")) and i + 1 < len(order):
            out.append(order[i + 1])
        succ[n] = out
    return blocks, order, succ


def _walk_block(lines, pending, report):
    """pending: {(destination registers, text): LDS/SMEM operations issued after it}.  Returns the state at the
    end of the block; report(line, registers, read) is called for every early use."""
    pending = dict(pending)
    reads = 0
    for l in lines:
        op = l.split()[0]
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", l)
            if m:
                pending = {k: c for k, c in pending.items() if c < int(m.group(1))}
            continue
        used = _vregs(l)
        for (regs, text) in pending:
            if regs & used:
                report(l, sorted(regs & used), text)
        if op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load"):
            pending = {k: min(c + 1, 64) for k, c in pending.items()}
        if op.startswith("ds_read"):
            pending[(frozenset(_vregs(l.split(",")[0])), l)] = 0
            reads += 1
    return pending, reads


def _check_kernel(body, report):
    """Forward data-flow over the control-flow graph: at a join a read stays pending if it is pending on any
    incoming path, with the fewest operations behind it."""
    blocks, order, succ = _blocks(body)
    state_in = {order[0]: {}}
    work = [order[0]]
    reads = 0
    while work:
        n = work.pop()
        out, _ = _walk_block(blocks[n], state_in[n], lambda *a: None)
        for t in succ[n]:
            if t not in blocks:
                continue
            old = state_in.get(t)
            new = dict(old) if old is not None else {}
            for k, c in out.items():
                new[k] = min(c, new[k]) if k in new else c
            if old is None or new != old:
                state_in[t] = new
                work.append(t)
    for n in order:
        if n in state_in:
            _, r = _walk_block(blocks[n], state_in[n], report)
            reads += r
    return reads


def test_hand_issued_lds_reads_are_waited_for_before_use(asm):
    src, text = asm
    checked = 0
    for name, body in _kernels(text):
        def report(line, regs, read, name=name):
            raise AssertionError("%s %s: '%s' touches v%s before the wait that covers '%s'" % (src, name, line, regs, read))
        checked += _check_kernel(body, report)
    assert checked > 100, "expected the hand-issued operand reads in %s" % src


def test_checker_catches_a_planted_early_use():
    """The same walk on hand-written snippets in which a register is used one wait too early: in straight-line
    code, and on one of two paths that join."""
    hits = []
    snippet = "\n".join(["ds_read_b128 v[4:7], v1 offset:0", "ds_read_b128 v[8:11], v1 offset:32", "s_waitcnt lgkmcnt(1)",
                         "v_add_f32 v20, v4, v5", "v_add_f32 v21, v8, v9"])
    _check_kernel(snippet, lambda line, regs, read: hits.append(line))
    assert hits == ["v_add_f32 v21, v8, v9"]
    hits = []
    joined = "\n".join(["s_cbranch_scc1 .LBB0_2", "ds_read_b128 v[4:7], v1 offset:0", "s_branch .LBB0_3", ".LBB0_2:",
                        "v_mov_b32 v4, 0", ".LBB0_3:", "v_add_f32 v20, v4, v5", "s_endpgm"])
    _check_kernel(joined, lambda line, regs, read: hits.append(line))
    assert hits == ["v_add_f32 v20, v4, v5"]
    hits = []
    unrelated = "\n".join(["s_cbranch_scc1 .LBB0_2", "ds_read_b128 v[4:7], v1 offset:0", "s_waitcnt lgkmcnt(0)", "s_endpgm",
                           ".LBB0_2:", "v_mov_b32 v4, 0", "s_endpgm"])
    _check_kernel(unrelated, lambda line, regs, read: hits.append(line))
    assert hits == []
