#!/usr/bin/env python3
"""Static check of the library's own kernels, on the assembly hipcc emits for them (`hipcc -S`).

An MFMA's result may be read by another kind of instruction only after a number of wait states (8 for the
16x16 forms used here: what the compiler itself puts between the two when they sit in one basic block).  Across a
branch the compiler has been seen to leave them out: a wave-uniform choice among the four accumulator elements
right after a chain of MFMAs compiled to `v_mfma; s_cbranch; <target:> v_accvgpr_read`, and the read returned a
half-finished accumulator.  This script follows every control-flow path from every MFMA and reports reads of
its destination registers that come earlier than `need` wait states.

    python -m paper_2502_06766_amd.isa_check file.s [need]      (file.s from hipcc -S --offload-device-only)
"""
import re
import sys
from collections import deque


def check(path: str, need: int = 8):
    """Returns a list of (kernel, mfma line, wait states, reader line, reader) for every early read."""
    lines = open(path).read().split('\n')
    return _check_lines(lines, need)


def _check_lines(lines, need):
    found = []
    def regs(tok):
        out = set()
        for m in re.finditer(r'\b([av])\[(\d+):(\d+)\]|\b([av])(\d+)\b', tok):
            if m.group(1):
                out |= {(m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1)}
            else:
                out.add((m.group(4), int(m.group(5))))
        return out
    # split into functions
    funcs, cur, name = [], None, None
    for i, l in enumerate(lines):
        m = re.match(r'^(_Z\S+):', l)
        if m:
            name, cur = m.group(1), []
            funcs.append((name, cur))
        elif cur is not None:
            if l.startswith('.Lfunc_end'):
                cur = None
            else:
                cur.append((i + 1, l))
    for name, body in funcs:
        ins, labels = [], {}
        for ln, l in body:
            t = l.strip()
            m = re.match(r'^(\.LBB\S+):', t)
            if m:
                labels[m.group(1)] = len(ins); continue
            if not t or t.startswith(';') or t.startswith('.') or t.endswith(':'):
                continue
            t = t.split(';')[0].strip()
            if t: ins.append((ln, t))
        for idx, (ln, t) in enumerate(ins):
            if not t.startswith('v_mfma'): continue
            dst = regs(t.split(None, 1)[1].split(',')[0])
            # only the last MFMA of a chain matters; a following MFMA reading dst as SrcC is handled by the hardware
            best = None
            q = deque([(idx + 1, 0)]); seen = {}
            while q:
                j, ws = q.popleft()
                while j < len(ins) and ws < need:
                    if seen.get(j, 99) <= ws: break
                    seen[j] = ws
                    ln2, u = ins[j]
                    op = u.split(None, 1)
                    args = op[1] if len(op) > 1 else ''
                    if u.startswith('v_mfma'):
                        break
                    parts = args.split(',')
                    srcs = ','.join(parts[1:]) if not u.startswith(('global_store', 'buffer_store', 'ds_write', 'ds_store', 'scratch_store')) else args
                    if regs(srcs) & dst:
                        if best is None or ws < best[0]: best = (ws, ln2, u)
                        break
                    if regs(parts[0]) & dst and not u.startswith(('global_store', 'buffer_store', 'ds_write')):
                        break                       # overwritten by something else: stop this path (a write hazard is another matter)
                    mm = re.match(r's_nop (\d+)', u)
                    ws += int(mm.group(1)) + 1 if mm else 1
                    if u.startswith('s_endpgm'): break
                    if u.startswith('s_branch'):
                        j = labels.get(args.strip(), len(ins)); continue
                    if u.startswith('s_cbranch'):
                        q.append((labels.get(args.strip(), len(ins)), ws))
                    j += 1
            if best is not None:
                found.append((name, ln, best[0], best[1], best[2]))
    return found


if __name__ == "__main__":
    hits = check(sys.argv[1], int(sys.argv[2]) if len(sys.argv) > 2 else 8)
    for name, ln, ws, ln2, u in hits:
        print(f"{name[:70]}: MFMA at line {ln} -> read after {ws} wait states at line {ln2}: {u}")
    print("hazards found:", len(hits))
    sys.exit(1 if hits else 0)
