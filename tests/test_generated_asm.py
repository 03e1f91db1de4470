"""Static checks of the gfx950 assembly the compiler generates for the attention kernels (CPU only: hipcc
cross-compiles).  The kernels issue their LDS operand reads through inline assembly and wait for them with
explicit s_waitcnt; the compiler knows nothing about those waits, so two things are checked on its output:

  1. inline assembly contains nothing but LDS reads/writes, s_waitcnt, s_nop and the in-place v_mul_f32 of the
     accumulator rescaling (a vector instruction issued through inline assembly gets none of the wait states the
     hardware needs after a matrix instruction);
  2. no instruction touches the destination registers of a hand-issued LDS read before an s_waitcnt lgkmcnt that
     covers it (LDS operations return in order, so a read is complete once at most N operations issued after
     it are outstanding and the wait asks for <= N);
  3. every hand-written v_mul_f32 is at least 20 instructions behind the last matrix instruction that wrote one of
     its registers, on every path (the longest wait the hardware asks for after a matrix instruction is 18 wait
     states), at least 2 instructions ahead of the next matrix instruction that reads one of them, and not directly
     behind a transcendental instruction that produced one of its inputs.

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
                assert op.startswith("ds_read") or op.startswith("ds_write") or op in ("s_waitcnt", "s_nop", "v_mul_f32_e32"), \
                    (src, name, line)
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


ASM_TAG = " hand_written"


def _tag_inline_vector(body):
    """The kernel text with every vector instruction that stands inside an inline-assembly block marked."""
    out, inside = [], False
    for raw in body.split("\n"):
        if ";;#ASMSTART" in raw:
            inside = True
        elif ";;#ASMEND" in raw:
            inside = False
        elif inside and raw.split(";")[0].strip().startswith("v_"):
            raw = raw.split(";")[0].rstrip() + ASM_TAG
        out.append(raw)
    return "\n".join(out)


FAR = 64
MFMA_GAP, READ_GAP = 20, 2


def _walk_vector(lines, state, report):
    """state: ({register: instructions since a matrix instruction wrote it}, {register: instructions since a
    hand-written vector instruction wrote it}, registers written by the previous instruction if it was
    transcendental).  Distances saturate at FAR; s_nop N counts N + 1."""
    since_mfma, since_hand, trans = dict(state[0]), dict(state[1]), set(state[2])
    found = 0
    for l in lines:
        op = l.split()[0]
        step = 1
        if op == "s_nop":
            step = int(l.split()[1]) + 1
        hand = l.endswith(ASM_TAG)
        text = l[:-len(ASM_TAG)] if hand else l
        operands = text.split(None, 1)[1] if " " in text else ""
        dst = _vregs(operands.split(",")[0]) if op.startswith("v_") else set()
        src = _vregs(operands.split(",", 1)[1]) if op.startswith("v_") and "," in operands else set()
        if hand:
            found += 1
            for r in dst | src:
                if since_mfma.get(r, FAR) < MFMA_GAP:
                    report(l, r, "%d instructions behind a matrix instruction that wrote it" % since_mfma[r])
            if trans & src:
                report(l, sorted(trans & src)[0], "directly behind the transcendental instruction that wrote it")
        if op.startswith("v_mfma"):
            for r in src:
                if since_hand.get(r, FAR) < READ_GAP:
                    report(l, r, "read %d instructions behind a hand-written write" % since_hand[r])
        since_mfma = {r: min(c + step, FAR) for r, c in since_mfma.items() if c + step < FAR}
        since_hand = {r: min(c + step, FAR) for r, c in since_hand.items() if c + step < FAR}
        if op.startswith("v_mfma"):
            for r in dst:
                since_mfma[r] = 0
        if hand:
            for r in dst:
                since_hand[r] = 0
        trans = dst if op in ("v_exp_f32_e32", "v_log_f32_e32", "v_rcp_f32_e32", "v_rsq_f32_e32", "v_sqrt_f32_e32") else set()
    return (since_mfma, since_hand, trans), found


def _check_vector(body, report):
    blocks, order, succ = _blocks(_tag_inline_vector(body))
    state_in = {order[0]: ({}, {}, set())}
    work = [order[0]]
    while work:
        n = work.pop()
        out, _ = _walk_vector(blocks[n], state_in[n], lambda *a: None)
        for t in succ[n]:
            if t not in blocks:
                continue
            old = state_in.get(t)
            new = ({}, {}, set()) if old is None else (dict(old[0]), dict(old[1]), set(old[2]))
            for i in (0, 1):
                for r, c in out[i].items():
                    new[i][r] = min(c, new[i][r]) if r in new[i] else c
            new[2].update(out[2])
            if old is None or new != old:
                state_in[t] = new
                work.append(t)
    found = 0
    for n in order:
        if n in state_in:
            _, f = _walk_vector(blocks[n], state_in[n], report)
            found += f
    return found


def test_hand_written_vector_instructions_keep_their_distance_from_matrix_instructions(asm):
    src, text = asm
    found = 0
    for name, body in _kernels(text):
        def report(line, reg, why, name=name):
            raise AssertionError("%s %s: '%s' uses v%d %s" % (src, name, line, reg, why))
        found += _check_vector(body, report)
    if src == "sta_attention.hip":
        assert found >= 64, "expected the in-place accumulator rescaling in %s" % src


def test_vector_checker_catches_planted_hazards():
    tagged = lambda l: l + ASM_TAG
    close = "\n".join(["v_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]", "v_add_f32 v20, v21, v22",
                       tagged("v_mul_f32_e32 v4, v30, v4"), "s_endpgm"])

    def run(snippet):
        found = []
        b, order, succ = _blocks(snippet)
        state = ({}, {}, set())
        for n in order:
            state, _ = _walk_vector(b[n], state, lambda l, r, why: found.append((l.split()[0], r)))
        return found
    assert run(close) == [("v_mul_f32_e32", 4)]
    far = "\n".join(["v_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]"] + ["v_add_f32 v20, v21, v22"] * 20 +
                    [tagged("v_mul_f32_e32 v4, v30, v4"), "v_add_f32 v20, v21, v22", "v_add_f32 v20, v21, v22",
                     "v_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]", "s_endpgm"])
    assert run(far) == []
    early_read = "\n".join([tagged("v_mul_f32_e32 v4, v30, v4"), "v_mfma_f32_16x16x32_bf16 v[4:7], v[8:11], v[12:15], v[4:7]"])
    assert run(early_read) == [("v_mfma_f32_16x16x32_bf16", 4)]
    after_exp = "\n".join(["v_exp_f32_e32 v30, v31", tagged("v_mul_f32_e32 v4, v30, v4")])
    assert run(after_exp) == [("v_mul_f32_e32", 30)]
    nop_between = "\n".join(["v_exp_f32_e32 v30, v31", "s_nop 1", tagged("v_mul_f32_e32 v4, v30, v4")])
    assert run(nop_between) == []
