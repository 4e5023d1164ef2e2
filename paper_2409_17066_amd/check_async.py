"""Build-time audit of the kernels that load registers asynchronously from inline assembly.

Such a load (buffer_load / global_load / ds_read inside an asm statement) leaves its destination registers
pending until a later s_waitcnt; the compiler does not know that and is free to copy, spill or reuse them in
between (it has done all three, typically right after the load or at the end of its basic block).  This script
reads the device assembly of a source file and checks every basic block on its own: registers written by an
inline-assembly load are pending until an s_waitcnt in the same block retires them (vector-memory loads and LDS
reads each retire in issue order, so `vmcnt(N)` / `lgkmcnt(N)` keeps the youngest N), and any other instruction of
the block that names a pending register is reported.  Nothing is carried across block boundaries, so this is a
net for the mistakes seen in practice, not a proof; the build fails on a finding.
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
    pending = frozenset().union(*vm, *lds) if (vm or lds) else frozenset()
    hit = regs_of(text) & pending
    if hit:
        report(text, sorted(hit))
    v = VM_LOAD.match(text)
    if v and not text.rstrip().endswith(" lds"):
        vm = (vm + ((regs_of(v.group(2)) if in_asm else frozenset()),))[-QUEUE_CAP:]
    else:
        d = LDS_LOAD.match(text)
        if d:
            lds = (lds + ((regs_of(d.group(2)) if in_asm else frozenset()),))[-QUEUE_CAP:]
    return vm, lds


def audit(asm_text):
    problems = []
    for name, body in kernels(asm_text):
        for b in blocks_of(body):
            state = ((), ())
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
