#!/usr/bin/env python3
"""Hazard check for the streaming kernels, which request their weights with inline-asm loads and
wait with explicit s_waitcnt (the compiler does not know that those destination registers are in
flight, so a spill or a copy it inserts between a load and its wait would read garbage).

    check_inflight.py <device assembly (.s)> <kernel symbol> [...]

Linear simulation of the wavefront's vector-memory queue over the kernel's text (loads return in
order; "s_waitcnt vmcnt(N)" retires all but the N youngest): flags any instruction outside the
asm blocks that mentions a register whose asm load may still be outstanding.  Not aware of the
control flow: a block placed before its loop header in the text can give a false alarm, which
has to be read; a clean run means no spill or copy stands between a load and its wait in text
order.  Exit status 1 if anything was flagged."""
import re, sys
def regs(l):
    out=set()
    for m in re.finditer(r'\bv\[(\d+):(\d+)\]',l): out.update(range(int(m.group(1)),int(m.group(2))+1))
    for m in re.finditer(r'\bv(\d+)\b',l): out.add(int(m.group(1)))
    return out
def check(path, kernel):
    txt=open(path).read().split('\n')
    L=[i for i,l in enumerate(txt) if l.startswith(kernel+':')][0]
    E=next(i for i in range(L,len(txt)) if 's_endpgm' in txt[i])
    lines=txt[L:E]
    queue=[]      # (is_asm, regs) in issue order
    inflight={}   # reg -> issue line
    inapp=False; bad=0
    def wait(n):
        nonlocal queue
        done=queue[:max(0,len(queue)-n)]; queue=queue[max(0,len(queue)-n):]
        for isasm,rs,_ in done:
            for r in rs:
                # only clear if no younger load to the same register remains
                if not any(r in q[1] for q in queue): inflight.pop(r,None)
    for i,l in enumerate(lines):
        s=l.strip()
        if 'ASMSTART' in s: inapp=True; continue
        if 'ASMEND' in s: inapp=False; continue
        if not s or s.startswith(';') or s.startswith('.'): continue
        m=re.match(r's_waitcnt\b(.*)',s)
        if m:
            mm=re.search(r'vmcnt\((\d+)\)',s)
            if mm: wait(int(mm.group(1)))
            elif re.match(r's_waitcnt\s+(0x0+|0)\s*$',s): wait(0)
            continue
        if inapp:
            m=re.match(r'global_load_dwordx4 v\[(\d+):(\d+)\]',s)
            if m:
                rs=set(range(int(m.group(1)),int(m.group(2))+1))
                queue.append((True,rs,i))
                for r in rs: inflight[r]=i
            continue
        if re.match(r'(global_load|global_store|global_atomic|buffer_|flat_)',s):
            queue.append((False,set(),i))          # compiler's own vector memory op: only counts
        hit=regs(s)&set(inflight)
        if hit:
            bad+=1
            if bad<=12: print("  line %d: %s   <- registers %s in flight since line %s"%(i,s[:70],sorted(hit)[:4],sorted(set(inflight[r] for r in hit))[:2]))
    print("%s: %d suspicious instruction(s)"%(kernel,bad))
    return bad
if __name__=='__main__':
    sys.exit(1 if sum(check(sys.argv[1],k) for k in sys.argv[2:]) else 0)
