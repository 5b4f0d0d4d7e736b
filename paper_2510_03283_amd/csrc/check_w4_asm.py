#!/usr/bin/env python3
"""Build step: check the generated code of the gemm_bf16_w4_kernel instantiations (the gfx950 .s file that
hipcc -save-temps leaves beside gemm.o).

The kernel issues its operand loads as asm and counts them itself, so the compiler does not know which
registers have a load in flight.  This walks the prologue once and the main loop twice in program order,
keeps the queue of loads in flight (s_waitcnt vmcnt(N) retires the oldest down to N; the conditional
vmcnt(0) at the end of a phase is ignored) and reports any instruction that names a register whose load has
not been waited for, and any scratch access in that region."""
import re, sys

def regs(tok):
    out = set()
    for m in re.finditer(r'\bv\[(\d+):(\d+)\]', tok):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r'\bv(\d+)\b', tok):
        out.add(int(m.group(1)))
    return out

def check(name, lines):
    code = [l.split(';')[0].rstrip() for l in lines]
    loads = [i for i, l in enumerate(code) if 'buffer_load_dwordx4' in l]
    if not loads:
        return False, f"{name}: no buffer loads found"
    labels = {m.group(1): i for i, l in enumerate(code) for m in [re.match(r'^(\.LBB\d+_\d+):', l)] if m}
    first_store = next((i for i, l in enumerate(code) if 'global_store' in l), len(code))
    barriers = [i for i, l in enumerate(code) if 's_barrier' in l]
    if len(barriers) != 5:
        return False, f"{name}: expected 5 barriers (prologue, two loop phases, two tail phases), found {len(barriers)}"
    # the main loop: the backward branch behind the third barrier, up to the block it reaches
    back = [(i, labels[m.group(1)]) for i, l in enumerate(code) for m in [re.search(r's_c?branch\S*\s+(\.LBB\d+_\d+)', l)]
            if m and m.group(1) in labels and labels[m.group(1)] <= i and barriers[2] < i < barriers[3]]
    if not back:
        return False, f"{name}: no loop found"
    back = [(i, t) for i, t in back if barriers[0] < t < barriers[1]]
    if not back:
        return False, f"{name}: no loop found"
    hi, head = max(i for i, _ in back), min(t for _, t in back)
    if not (barriers[0] < head < barriers[1]):
        return False, f"{name}: loop head {head} not between the first two barriers"
    bad = []
    def walk(order, inflight, what):
        maxq = nwait = 0
        last0 = max([i for i in order if re.search(r's_waitcnt vmcnt\(0\)\s*$', code[i])], default=None)
        for i in order:
            l = code[i].strip()
            if not l or l.startswith('.') or l.endswith(':'):
                continue
            if what == 'tail' and last0 is not None and i >= last0:
                break
            if l.startswith('s_waitcnt'):
                m = re.search(r'vmcnt\((\d+)\)', l)
                if m and int(m.group(1)) > 0:
                    nwait += 1
                    while len(inflight) > int(m.group(1)):
                        inflight.pop(0)
                continue
            pending = set().union(*inflight) if inflight else set()
            # (behind the loop nothing is in flight any more and spills are harmless)
            if ('scratch_' in l and (what != 'tail' or inflight)) or (regs(l) & pending):
                bad.append((i, what + ': ' + l))
            if 'buffer_load_dwordx4' in l:
                inflight.append(regs(l.split(',')[0]))
                maxq = max(maxq, len(inflight))
        return maxq, nwait, last0
    q = []
    m1, w1, _ = walk(list(range(loads[0], head)), q, 'prologue')
    m2, w2, d2 = walk(2 * list(range(head, hi + 1)), q, 'loop')
    if d2 is None:
        bad.append((0, "no vmcnt(0) drain in the loop body"))
    m3, w3, d3 = walk(list(range(hi + 1, first_store)), [], 'tail')
    if m3:
        bad.append((0, "loads issued behind the loop"))
    msg = f"{name}: prologue {loads[0]}..{head - 1}, loop {head}..{hi}, tail ..{d3}, at most {max(m1, m2, m3)} loads in flight, {w1 + w2 + w3} counted waits"
    if max(m1, m2, m3) > 48:
        bad.append((0, "more than 48 loads in flight"))
    if bad:
        return False, msg + "\n  VIOLATIONS:\n" + "\n".join(f"    line {i}: {l}" for i, l in bad[:20])
    return True, msg + "  OK"

def main(path):
    txt = open(path).read().split('\n')
    starts = [(i, m.group(1)) for i, l in enumerate(txt) for m in [re.match(r'^(_ZN\S*gemm_bf16_w4_kernel\S*):', l)] if m]
    rc = 0 if starts else 1
    for i, nm in starts:
        j = next(k for k in range(i, len(txt)) if txt[k].startswith('.Lfunc_end'))
        ok, r = check(nm[-40:], txt[i:j])
        print(r)
        rc |= 0 if ok else 1
    if not starts:
        print("no w4 kernels in", path)
    return rc

if __name__ == '__main__':
    sys.exit(main(sys.argv[1]))
