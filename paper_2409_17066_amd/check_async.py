"""Build-time audit of the kernels that load registers asynchronously from inline assembly.

Such a load (buffer_load / global_load / ds_read inside an asm statement) leaves its destination registers
pending until a later s_waitcnt; the compiler does not know that and is free to copy, spill or reuse them in
between (it has done all three, typically right after the load, at the end of its basic block, or at a loop's
back-edge).  This script reads the device assembly of a source file and follows, per kernel, the queue of
outstanding loads through the control-flow graph: registers written by an inline-assembly load are pending until an
s_waitcnt retires them (vector-memory loads and LDS reads each retire in issue order, so `vmcnt(N)` / `lgkmcnt(N)`
keeps the youngest N; the compiler's own loads take their place in the queue with no registers attached), and any
other instruction that names a pending register is reported.  A block starts from the merge of what its predecessors
leave behind -- queues aligned at their youngest entry, register sets united position by position, which can only
add pending registers -- iterated over the graph to a fixed point (queues are cut at the 64 loads the hardware's
counters can tell apart).  Sound for the mistakes this guards against under two assumptions it cannot check: loads
retire in issue order, and branch targets are the labels of the same function.  It is not complete: it follows every
path through the graph, also those that no run takes because two branches test the same loop-invariant value (a wave
either has vectors in a codebook group or has none, in every copy of an unrolled loop body), and on such a path a
counted wait meets fewer loads than it counts on.  The build therefore fails on any finding in the files whose graphs
come out clean, and for the two files with such paths (build.py names them) on any finding inside a single basic block,
printing the number of cross-block findings for the reader to compare with the number recorded there.
"""
import re
import subprocess
import sys

REG = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
VM_LOAD = re.compile(r"^(buffer_load_\w+|global_load_\w+)\s+(\S+?),")
LDS_LOAD = re.compile(r"^(ds_read\w*)\s+(\S+?),")
LABEL = re.compile(r"^(\.LBB\w+):")
BRANCH = re.compile(r"^(s_cbranch_\w+|s_branch)\s+(\.LBB\w+)")
QUEUE_CAP = 64


def regs_of(text):
    out = set()
    for m in REG.finditer(text):
        if m.group(1) is not None:
            out.add(int(m.group(1)))
        else:
            out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return frozenset(out)


def kernels(asm_text):
    """Yield (name, [(text, in_asm)]) for every function in the file."""
    name, body, in_asm = None, [], False
    for raw in asm_text.splitlines():
        m = re.match(r"^(_Z\w+):", raw)
        if m:
            name, body, in_asm = m.group(1), [], False
            continue
        if name is None:
            continue
        if "#ASMSTART" in raw:
            in_asm = True
            continue
        if "#ASMEND" in raw:
            in_asm = False
            continue
        text = raw.split(";")[0].strip()
        if not text:
            continue
        if text.startswith(".") and not LABEL.match(text):
            continue
        body.append((text, in_asm))
        if text.startswith("s_endpgm"):
            yield name, body
            name = None


def blocks_of(body):
    """Basic blocks: list of dicts with label, instructions, successor indices."""
    blocks, cur = [], {"label": None, "ins": []}
    for text, in_asm in body:
        m = LABEL.match(text)
        if m:
            if cur["ins"] or cur["label"]:
                blocks.append(cur)
            cur = {"label": m.group(1), "ins": []}
            continue
        cur["ins"].append((text, in_asm))
        if BRANCH.match(text) or text.startswith("s_endpgm"):
            blocks.append(cur)
            cur = {"label": None, "ins": []}
    if cur["ins"] or cur["label"]:
        blocks.append(cur)
    index = {b["label"]: i for i, b in enumerate(blocks) if b["label"]}
    for i, b in enumerate(blocks):
        succ = []
        last = b["ins"][-1][0] if b["ins"] else ""
        m = BRANCH.match(last)
        if m:
            if m.group(2) in index:
                succ.append(index[m.group(2)])
            if m.group(1) != "s_branch" and i + 1 < len(blocks):
                succ.append(i + 1)
        elif not last.startswith("s_endpgm") and i + 1 < len(blocks):
            succ.append(i + 1)
        b["succ"] = succ
    return blocks


def step(state, text, in_asm, report):
    vm, lds = state
    m = re.search(r"s_waitcnt\s+(.*)", text)
    if m:
        v = re.search(r"vmcnt\((\d+)\)", m.group(1))
        if v:
            vm = vm[len(vm) - int(v.group(1)):] if int(v.group(1)) else ()
        g = re.search(r"lgkmcnt\((\d+)\)", m.group(1))
        if g:
            lds = lds[len(lds) - int(g.group(1)):] if int(g.group(1)) else ()
        return vm, lds
    pend_vm = frozenset().union(*vm) if vm else frozenset()
    pend_lds = frozenset().union(*lds) if lds else frozenset()
    v, d = VM_LOAD.match(text), LDS_LOAD.match(text)
    named = regs_of(text)
    if v or d:
        # a load may name, as its destination, registers that an older load of the SAME queue still owes: they retire in
        # order, so the younger value lands last; its address registers, and the other queue's registers, may not be pending
        dest = regs_of((v or d).group(2))
        rest = regs_of(text[(v or d).end(2):])
        hit = (rest & (pend_vm | pend_lds)) | (dest & (pend_lds if v else pend_vm))
    else:
        hit = named & (pend_vm | pend_lds)
    if hit:
        report(text, sorted(hit))
    if v and not text.rstrip().endswith(" lds"):
        vm = (vm + ((regs_of(v.group(2)) if in_asm else frozenset()),))[-QUEUE_CAP:]
    elif d:
        lds = (lds + ((regs_of(d.group(2)) if in_asm else frozenset()),))[-QUEUE_CAP:]
    return vm, lds


def merge(a, b):
    """Two queues of pending-register sets, youngest last: aligned at the youngest entry, united position by position."""
    if len(a) < len(b):
        a, b = b, a
    pad = len(a) - len(b)
    return a[:pad] + tuple(x | y for x, y in zip(a[pad:], b))


def audit_blocks(asm_text):
    """Every basic block on its own, starting with nothing pending: what no path can excuse."""
    problems = []
    for name, body in kernels(asm_text):
        for b in blocks_of(body):
            state = ((), ())
            for text, in_asm in b["ins"]:
                state = step(state, text, in_asm,
                             lambda t, regs, _b=b: problems.append((name, _b["label"] or "(entry)", t, regs)))
    return problems


def audit(asm_text):
    """The queues carried through the control-flow graph (see the module's text)."""
    problems = []
    for name, body in kernels(asm_text):
        blocks = blocks_of(body)
        if not blocks:
            continue
        entry = [None] * len(blocks)              # state at the start of each block; None: not reached yet
        entry[0] = ((), ())
        work = [0]
        while work:
            i = work.pop()
            state = entry[i]
            for text, in_asm in blocks[i]["ins"]:
                state = step(state, text, in_asm, lambda t, regs: None)
            for j in blocks[i]["succ"]:
                new = state if entry[j] is None else (merge(entry[j][0], state[0]), merge(entry[j][1], state[1]))
                if new != entry[j]:
                    entry[j] = new
                    work.append(j)
        for i, b in enumerate(blocks):            # the states are final: report
            if entry[i] is None:
                continue
            state = entry[i]
            for text, in_asm in b["ins"]:
                state = step(state, text, in_asm,
                             lambda t, regs, _b=b: problems.append((name, _b["label"] or "(entry)", t, regs)))
    return problems


def device_asm(hipcc, flags, src):
    cmd = [hipcc] + [f for f in flags if not f.startswith("-Rpass")] + ["--cuda-device-only", "-S", src, "-o", "-"]
    return subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True).stdout


if __name__ == "__main__":
    bad = audit(open(sys.argv[1]).read())
    for name, label, text, regs in bad[:40]:
        print("%s %s\n    %s\n    names v%s while a load into it may be pending" % (name, label, text, regs[:6]))
    print("%d finding(s)" % len(bad))
