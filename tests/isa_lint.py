"""Lint of a gfx950 ISA listing (hipcc -S) of the library's own kernels.

The weight stream and the activation fragments are loaded by hand-issued (inline asm) loads whose
completion the compiler does not track.  Between such a load and the s_waitcnt that releases it no
compiler-generated instruction may touch the destination registers: a copy or a spill there moves
data that has not arrived yet.  Forward dataflow over basic blocks; the state is the ordered tuple
of in-flight hand-issued load destinations (oldest first); at joins the longest state wins (states
from different paths are almost always equal, or one is empty).  A wave can have at most 64
loads outstanding, which also bounds the state around loops that issue loads.
"""
import re, sys
def regs(tok):
    tok = tok.strip()
    m = re.match(r'v\[(\d+):(\d+)\]', tok)
    if m: return frozenset(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r'v(\d+)$', tok)
    if m: return frozenset({int(m.group(1))})
    return frozenset()
def parse_function(lines):
    # returns blocks: list of dict(label, instrs=[(lineno, in_asm, op, rest)], succ=[labels or '+1'])
    blocks = []; cur = {'label': None, 'ins': [], 'succ': []}
    in_asm = False
    for no, ln in lines:
        if 'ASMSTART' in ln: in_asm = True; continue
        if 'ASMEND' in ln: in_asm = False; continue
        s = ln.strip()
        if not s or s.startswith(';'): continue
        m = re.match(r'(\.LBB\d+_\d+):', s)
        if m:
            if cur['ins'] or cur['label']:
                if not cur['succ_final']: cur['succ'].append('+1')
                blocks.append(cur)
            cur = {'label': m.group(1), 'ins': [], 'succ': []}
            cur['succ_final'] = False
            continue
        if s.startswith('.'): continue
        cur.setdefault('succ_final', False)
        t = s.split(None, 1); op = t[0]; rest = t[1].split(';')[0] if len(t) > 1 else ''
        cur['ins'].append((no, in_asm, op, rest))
        if op == 's_branch':
            cur['succ'].append(rest.strip()); cur['succ_final'] = True
            blocks.append(cur); cur = {'label': None, 'ins': [], 'succ': [], 'succ_final': False}
        elif op.startswith('s_cbranch'):
            cur['succ'].append(rest.strip()); cur['succ'].append('+1'); cur['succ_final'] = True
            blocks.append(cur); cur = {'label': None, 'ins': [], 'succ': [], 'succ_final': False}
        elif op in ('s_endpgm', 's_setpc_b64'):
            cur['succ_final'] = True
            blocks.append(cur); cur = {'label': None, 'ins': [], 'succ': [], 'succ_final': False}
    if cur['ins'] or cur['label']:
        blocks.append(cur)
    return blocks
def transfer(state, blk, report):
    st = list(state)
    for no, in_asm, op, rest in blk['ins']:
        if op.startswith('s_waitcnt'):
            mm = re.search(r'vmcnt\((\d+)\)', rest)
            if mm:
                n = int(mm.group(1))
                if n < len(st): st = st[len(st) - n:] if n > 0 else []
            continue
        if in_asm and re.match(r'global_load_dword', op):
            st.append((regs(rest.split(',')[0]), no))
            st = st[-64:]  # the 6-bit counter: a wave cannot have more loads on their way
            continue
        if in_asm: continue
        touched = frozenset()
        for o in rest.split(','): touched |= regs(o)
        for d, l in st:
            if touched & d:
                report.add((no, op + ' ' + rest.strip(), l)); break
        # compiler-issued vector memory loads also occupy vmcnt slots: counting them would only make the
        # hand-issued waits look weaker than they are, so they are ignored here
    return tuple(st)
def check(path):
    raw = open(path).read().split('\n')
    # split into functions at non-local labels
    funcs = []; cur = []; name = None
    for i, ln in enumerate(raw):
        m = re.match(r'^([A-Za-z_][\w$.]*):', ln)
        if m and not ln.startswith('.L'):
            if cur: funcs.append((name, cur))
            name = m.group(1); cur = []
        cur.append((i + 1, ln))
    if cur: funcs.append((name, cur))
    total = 0
    for name, lines in funcs:
        if name is None: continue
        blocks = parse_function(lines)
        if not blocks: continue
        idx = {b['label']: k for k, b in enumerate(blocks) if b['label']}
        instate = {0: ()}
        work = [0]; report = set(); iters = 0
        while work and iters < 20000:
            iters += 1
            k = work.pop()
            out = transfer(instate[k], blocks[k], report)
            for sname in blocks[k]['succ']:
                j = k + 1 if sname == '+1' else idx.get(sname)
                if j is None or j >= len(blocks): continue
                old = instate.get(j)
                if old is None or len(out) > len(old):
                    instate[j] = out; work.append(j)
        for no, txt, l in sorted(report):
            print(f"{path}:{no}: '{txt}' touches registers in flight since line {l}  [{name}]")
        total += len(report)
    print(path, "suspicious:", total)
    return total
# ---------------------------------------------------------------------------------------------
# Second check: results of the matrix cores read too early across a basic-block boundary.
# A v_mfma delivers its destination registers many cycles after issue and only software (wait
# states: independent instructions or s_nop) keeps a later reader away.  The compiler pads for that
# inside a basic block; behind a block boundary it was seen to pad too little (an LDS store of an
# accumulator right after a branch target stored what the registers held before).  Flagged: a
# non-MFMA instruction in ANOTHER block than the v_mfma that touches its destination after fewer than
# MFMA_WAIT_STATES wait states on some path (every instruction counts one, s_nop N counts N + 1).
MFMA_WAIT_STATES = 18  # the slowest shape (16 passes) needs 18; the 16x16x32 products here need fewer
def _states(op, rest):
    if op == 's_nop':
        try: return int(rest.strip(), 0) + 1
        except ValueError: return 1
    return 1
def _touched(rest):
    t = frozenset()
    for o in rest.split(','): t |= regs(o)
    return t
def check_mfma(path):
    raw = open(path).read().split('\n')
    funcs = []; cur = []; name = None
    for i, ln in enumerate(raw):
        m = re.match(r'^([A-Za-z_][\w$.]*):', ln)
        if m and not ln.startswith('.L'):
            if cur: funcs.append((name, cur))
            name = m.group(1); cur = []
        cur.append((i + 1, ln))
    if cur: funcs.append((name, cur))
    total = 0
    for name, lines in funcs:
        if name is None: continue
        blocks = parse_function(lines)
        if not blocks: continue
        idx = {b['label']: k for k, b in enumerate(blocks) if b['label']}
        def succs(k):
            out = []
            for sname in blocks[k]['succ']:
                j = k + 1 if sname == '+1' else idx.get(sname)
                if j is not None and j < len(blocks): out.append(j)
            return out
        report = set()
        for k, blk in enumerate(blocks):
            ins = blk['ins']
            for i, (no, in_asm, op, rest) in enumerate(ins):
                if not op.startswith('v_mfma'): continue
                dst = regs(rest.split(',')[0])
                # rest of the own block: the compiler's own padding is trusted there
                count = 0; alive = True
                for (no2, _, op2, rest2) in ins[i + 1:]:
                    if _touched(rest2) & dst: alive = False; break
                    count += _states(op2, rest2)
                if not alive or count >= MFMA_WAIT_STATES: continue
                work = [(j, count) for j in succs(k)]; seen = {}
                while work:
                    j, c = work.pop()
                    if seen.get(j, 1 << 30) <= c: continue
                    seen[j] = c
                    stop = False
                    for (no2, _, op2, rest2) in blocks[j]['ins']:
                        if c >= MFMA_WAIT_STATES: stop = True; break
                        if _touched(rest2) & dst:
                            if not op2.startswith('v_mfma'):
                                report.add((no2, op2 + ' ' + rest2.strip(), no, c))
                            stop = True; break
                        c += _states(op2, rest2)
                    if not stop and c < MFMA_WAIT_STATES:
                        work.extend((jj, c) for jj in succs(j))
        for no2, txt, no, c in sorted(report):
            print(f"{path}:{no2}: '{txt}' touches the result of the v_mfma of line {no} after {c} wait states  [{name}]")
        total += len(report)
    print(path, "early reads of matrix-core results:", total)
    return total
if __name__ == "__main__":
    rc = 0
    for p in sys.argv[1:]:
        rc |= 1 if check(p) else 0
        rc |= 1 if check_mfma(p) else 0
    sys.exit(rc)
