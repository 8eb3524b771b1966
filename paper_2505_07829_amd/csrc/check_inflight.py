#!/usr/bin/env python3
"""Hazard check for the streaming kernels, which request their weights with inline-asm loads and
wait with explicit s_waitcnt (the compiler does not know that those destination registers are in
flight, so a spill or a copy it inserts between a load and its wait would read garbage, and a
register it reuses too early is overwritten when the load returns).

    check_inflight.py <device assembly (.s)> <kernel symbol> [...]

Forward data-flow analysis over the kernel's control-flow graph.  State: for every vector
register (vector or accumulation) that an asm load has been issued to, the least number of vector-memory instructions
issued after that load on any path ("younger").  Loads of a wavefront return in order, so
"s_waitcnt vmcnt(N)" completes every load with at least N younger ones; states of joining paths
are merged register by register with the minimum.  Any instruction outside the asm blocks that
mentions a register whose load may be outstanding is reported.  Exit status 1 if anything was
reported."""
import re
import sys

BIG = 1 << 20


AGPR = 1000     # accumulation register aN is tracked as register number AGPR + N


def regs(text):
    out = set()
    for m in re.finditer(r'\b([va])\[(\d+):(\d+)\]', text):
        base = AGPR if m.group(1) == 'a' else 0
        out.update(range(base + int(m.group(2)), base + int(m.group(3)) + 1))
    for m in re.finditer(r'\b([va])(\d+)\b', text):
        out.add((AGPR if m.group(1) == 'a' else 0) + int(m.group(2)))
    return out


def parse(lines):
    """-> blocks: list of dicts {label, ins: [(lineno, text, in_asm)], succ: [labels or indices]}"""
    blocks, cur, in_asm = [], {"label": None, "ins": [], "succ": [], "fall": True}, False
    for i, raw in enumerate(lines):
        s = raw.strip()
        if 'ASMSTART' in s:
            in_asm = True
            continue
        if 'ASMEND' in s:
            in_asm = False
            continue
        m = re.match(r'^(\.LBB\d+_\d+):', raw)
        if m:
            blocks.append(cur)
            cur = {"label": m.group(1), "ins": [], "succ": [], "fall": True}
            continue
        if not s or s.startswith(';') or s.startswith('.'):
            continue
        cur["ins"].append((i, s, in_asm))
        m = re.match(r'(s_branch|s_cbranch_\w+)\s+(\.LBB\d+_\d+)', s)
        if m:
            cur["succ"].append(m.group(2))
            if m.group(1) == 's_branch':
                cur["fall"] = False
            blocks.append(cur)
            cur = {"label": None, "ins": [], "succ": [], "fall": True}
        elif s.startswith('s_endpgm'):
            cur["fall"] = False
            blocks.append(cur)
            cur = {"label": None, "ins": [], "succ": [], "fall": True}
    blocks.append(cur)
    index = {b["label"]: k for k, b in enumerate(blocks) if b["label"]}
    for k, b in enumerate(blocks):
        succ = [index[l] for l in b["succ"] if l in index]
        if b["fall"] and k + 1 < len(blocks):
            succ.append(k + 1)
        b["succ"] = succ
    return blocks


def transfer(state, block, report=None):
    st = dict(state)
    for lineno, s, in_asm in block["ins"]:
        m = re.match(r's_waitcnt\b(.*)', s)
        if m:
            mm = re.search(r'vmcnt\((\d+)\)', s)
            n = int(mm.group(1)) if mm else (0 if re.match(r's_waitcnt\s+(0x0+|0)\s*$', s) else None)
            if n is not None:
                st = {r: y for r, y in st.items() if y < n}
            continue
        is_vmem = re.match(r'(global_load|global_store|global_atomic|buffer_|flat_|scratch_)', s) is not None
        if in_asm:
            m = re.match(r'global_load_dword(?:x[234])?\s+([va])(?:\[(\d+):(\d+)\]|(\d+))', s)
            if m:
                st = {r: y + 1 for r, y in st.items()}
                base = AGPR if m.group(1) == 'a' else 0
                lo, hi = (int(m.group(2)), int(m.group(3))) if m.group(2) else (int(m.group(4)), int(m.group(4)))
                for r in range(base + lo, base + hi + 1):
                    st[r] = 0
            continue
        hit = regs(s) & set(st)
        if hit and report is not None:
            report.append((lineno, s, sorted(hit)))
        if is_vmem:
            st = {r: y + 1 for r, y in st.items()}
    return st


def check(path, kernel):
    txt = open(path).read().split('\n')
    start = [i for i, l in enumerate(txt) if l.startswith(kernel + ':')][0]
    end = next(i for i in range(start, len(txt)) if 's_endpgm' in txt[i])
    blocks = parse(txt[start:end + 1])
    n = len(blocks)
    inst = [None] * n
    inst[0] = {}
    work = [0]
    while work:
        k = work.pop()
        out = transfer(inst[k], blocks[k])
        for j in blocks[k]["succ"]:
            if inst[j] is None:
                new = dict(out)
            else:
                new = dict(inst[j])
                for r, y in out.items():
                    new[r] = min(new.get(r, BIG), y)
            if new != inst[j]:
                inst[j] = new
                work.append(j)
    report = []
    for k in range(n):
        if inst[k] is not None:
            transfer(inst[k], blocks[k], report)
    seen = set()
    for lineno, s, hit in report:
        if lineno in seen:
            continue
        seen.add(lineno)
        if len(seen) <= 12:
            names = ["a%d" % (r - AGPR) if r >= AGPR else "v%d" % r for r in hit[:4]]
            print("  line %d: %s   <- registers %s may be in flight" % (lineno, s[:72], names))
    print("%s: %d suspicious instruction(s)" % (kernel, len(seen)))
    return len(seen)


if __name__ == '__main__':
    sys.exit(1 if sum(check(sys.argv[1], k) for k in sys.argv[2:]) else 0)
