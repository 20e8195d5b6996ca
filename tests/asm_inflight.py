"""Reads gfx950 assembly text and reports instructions that touch a vector register while an LDS
read that will write that register is still in flight.

The tile kernels that fill LDS with direct-to-LDS loads issue their LDS fragment reads as inline
assembly and wait for them by counter (s_waitcnt lgkmcnt) themselves, because the compiler would
otherwise make every LDS access wait for all loads in flight.  The compiler therefore believes a
fragment register holds its value as soon as the read has been issued, and is free to copy such a
register (to merge two paths, to make room) before the kernel's wait: the copy then carries what the
register held before.  Nothing in the source can forbid that outright, so the generated code is
checked instead.

Model: LDS operations of a wave complete in order, so after s_waitcnt lgkmcnt(n) only the n most
recent ones are outstanding.  Every basic block is analysed with the outstanding reads that can
reach it along any path of the control-flow graph (merged position by position from the newest
end, to a fixed point).  Any instruction other than the wait that names a register of an
outstanding read is a finding; a later LDS read may write such a register again (in-order return).
Scalar loads share the counter; they are kept in the queue as operations without vector registers.
The analysis is path-insensitive: a path that the program never takes can produce a finding.
"""
import collections
import re

REG = re.compile(r"\b([va])(?:(\d+)|\[(\d+):(\d+)\])")
QUEUE_CAP = 48          # more LDS operations than a wait can count never stay distinguishable


def regs(text):
    out = set()
    for m in REG.finditer(text):
        kind = m.group(1)
        if m.group(2) is not None:
            out.add((kind, int(m.group(2))))
        else:
            out.update((kind, i) for i in range(int(m.group(3)), int(m.group(4)) + 1))
    return frozenset(out)


def functions(lines):
    """(name, [(line number, instruction or label)]) for every function of an assembly listing."""
    name, body = None, []
    for n, line in enumerate(lines, 1):
        code = line.split(";")[0].strip()
        if not code:
            continue
        if code.endswith(":") and code.startswith("_Z"):
            if name:
                yield name, body
            name, body = code[:-1], []
            continue
        if name is None or (code.startswith(".") and not code.endswith(":")):
            continue
        body.append((n, code))
    if name:
        yield name, body


def _is_terminator(op):
    return op.startswith("s_cbranch") or op in ("s_branch", "s_endpgm", "s_setpc_b64")


def basic_blocks(body):
    blocks, cur = [], {"label": None, "ins": []}
    for n, code in body:
        if code.endswith(":"):
            if cur["ins"] or cur["label"]:
                blocks.append(cur)
            cur = {"label": code[:-1], "ins": []}
            continue
        cur["ins"].append((n, code))
        if _is_terminator(code.split()[0]):
            blocks.append(cur)
            cur = {"label": None, "ins": []}
    if cur["ins"] or cur["label"]:
        blocks.append(cur)
    index = {b["label"]: i for i, b in enumerate(blocks) if b["label"]}
    for i, b in enumerate(blocks):
        last = b["ins"][-1][1] if b["ins"] else ""
        op = last.split()[0] if last else ""
        succ = []
        if op.startswith("s_cbranch") or op == "s_branch":
            target = last.split()[-1]
            if target in index:
                succ.append(index[target])
        if not (op == "s_branch" or op in ("s_endpgm", "s_setpc_b64")) and i + 1 < len(blocks):
            succ.append(i + 1)
        b["succ"] = succ
    return blocks


def _merge(a, b):
    if a is None:
        return b
    n = max(len(a), len(b))
    pa = (frozenset(),) * (n - len(a)) + a
    pb = (frozenset(),) * (n - len(b)) + b
    return tuple(x | y for x, y in zip(pa, pb))


def _transfer(state, ins, report=None):
    queue = list(state)
    for n, code in ins:
        op = code.split()[0]
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", code)
            if m:
                keep = int(m.group(1))
                queue = queue[len(queue) - keep:] if keep else []
            elif re.fullmatch(r"s_waitcnt\s+(0|0x0)", code):
                queue = []
            continue
        pending = frozenset().union(*queue) if queue else frozenset()
        if op.startswith(("ds_", "s_load", "s_buffer_load")):
            if op.startswith(("ds_read", "ds_load")):
                operands = code[len(op):].split(",")
                hit = regs(",".join(operands[1:])) & pending
                queue.append(regs(operands[0]))
            else:
                hit = regs(code) & pending
                queue.append(frozenset())
            queue = queue[-QUEUE_CAP:]
        else:
            hit = regs(code) & pending
        if hit and report is not None:
            report.append((n, sorted(hit), code))
    return tuple(queue)


def check_function(body):
    blocks = basic_blocks(body)
    if not blocks:
        return []
    reach = [None] * len(blocks)
    reach[0] = ()
    work = collections.deque([0])
    while work:
        i = work.popleft()
        out = _transfer(reach[i], blocks[i]["ins"])
        for s in blocks[i]["succ"]:
            merged = _merge(reach[s], out)
            if merged != reach[s]:
                reach[s] = merged
                if s not in work:
                    work.append(s)
    report = []
    for i, b in enumerate(blocks):
        if reach[i] is not None:
            _transfer(reach[i], b["ins"], report)
    return report


def check_listing(lines, only=None):
    """[(function, line number, registers, instruction)] over every function whose name contains `only`."""
    findings, seen = [], 0
    for name, body in functions(lines):
        if only and only not in name:
            continue
        seen += 1
        findings += [(name,) + r for r in check_function(body)]
    return seen, findings


WIDE_STORE = re.compile(r"^(global|flat|buffer|scratch)_store_dwordx[34]\b")


def check_wide_store_data(lines, only=None, wait_states=2):
    """A vector instruction that writes a data register of a store of more than 8 bytes must stay
    `wait_states` instructions behind that store (gfx940 family: 2; s_nop n counts as n + 1).  The compiler
    sees to it after its own stores; a store written as inline assembly must bring the distance along.
    [(function, line number, registers, instruction)]"""
    findings = []
    for name, body in functions(lines):
        if only and only not in name:
            continue
        data, left = None, 0
        for n, code in body:
            if code.endswith(":"):
                continue
            op = code.split()[0]
            if left > 0 and op.startswith("v_"):
                hit = regs(code[len(op):].split(",")[0]) & data
                if hit:
                    findings.append((name, n, sorted(hit), code))
            left -= (int(code.split()[1], 0) + 1) if op == "s_nop" else 1
            if WIDE_STORE.match(op):
                operands = code[len(op):].split(",")
                # global/flat/scratch: address, data; buffer: data first
                data, left = regs(operands[0] if op.startswith("buffer") else operands[1]), wait_states
    return findings
