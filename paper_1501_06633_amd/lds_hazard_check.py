"""Static check on gfx950 assembly (test infrastructure for test_kernel_isa.py).

The kernels issue their LDS reads through inline asm and wait for them later with a hand-counted
`s_waitcnt lgkmcnt(N)`.  The compiler believes the destination registers are valid right after the
read instruction, so nothing stops it from copying one (or reusing it) before the wait -- which
happened once, on a path with a branch between read and wait, and gave a wrong tile now and then.
This check makes that a build-time failure: walking every path of a kernel's control-flow graph it
tracks the LDS operations in flight (they complete in order, so after lgkmcnt(N) only the last N
issued may be outstanding) and reports every instruction that reads or writes a VGPR an
outstanding LDS read is going to fill."""
import re, sys

REG = re.compile(r'\bv(\d+)\b|\bv\[(\d+):(\d+)\]')

def regs_of(text):
    out = set()
    for m in REG.finditer(text):
        if m.group(1) is not None: out.add(int(m.group(1)))
        else: out.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return out

def parse_functions(asm):
    funcs = {}; cur = None
    for raw in asm.splitlines():
        line = raw.split(';')[0].rstrip()
        if not line.strip(): continue
        m = re.match(r'^([A-Za-z_.$][\w.$]*):', line)
        if m:
            name = m.group(1)
            if not name.startswith('.L'):
                cur = name; funcs[cur] = []
            if cur is not None: funcs[cur].append(('label', name, ''))
            continue
        if cur is None: continue
        t = line.strip()
        if t.startswith('.'):
            if t.startswith('.end_amdhsa_kernel') or t.startswith('.section') or t.startswith('.Lfunc_end'): pass
            continue
        parts = t.split(None, 1)
        funcs[cur].append(('inst', parts[0], parts[1] if len(parts) > 1 else ''))
    return funcs

def check_function(items, name, max_states=200000):
    # split into blocks
    blocks = []; labels = {}; cur = []
    for kind, a, b in items:
        if kind == 'label':
            if cur: blocks.append(cur); cur = []
            labels[a] = len(blocks)
            continue
        cur.append((a, b))
        if a.startswith('s_branch') or a.startswith('s_cbranch') or a == 's_endpgm':
            blocks.append(cur); cur = []
    if cur: blocks.append(cur)
    # labels may point at len(blocks) if trailing; fix mapping: label index = index of the block that starts after it
    violations = []
    seen = set(); work = [(0, ())]
    while work:
        bi, state = work.pop()
        if bi >= len(blocks) or (bi, state) in seen: continue
        seen.add((bi, state))
        if len(seen) > max_states: raise RuntimeError('state explosion in ' + name)
        st = list(state)
        succ = [bi + 1]
        for mn, ops in blocks[bi]:
            if mn == 's_waitcnt':
                m = re.search(r'lgkmcnt\((\d+)\)', ops)
                if m:
                    n = int(m.group(1)); st = st[len(st) - n:] if n < len(st) else st
                elif re.fullmatch(r'\s*(0x[0-9a-fA-F]+|\d+)\s*', ops):
                    st = []          # raw immediate: assume a full wait
                continue
            is_ds = mn.startswith('ds_')
            is_smem = mn.startswith('s_load') or mn.startswith('s_buffer_load')
            touched = regs_of(ops)
            if is_ds and (mn.startswith('ds_read') or mn.startswith('ds_bpermute') or mn.startswith('ds_permute') or mn.startswith('ds_swizzle')):
                first, _, rest = ops.partition(',')
                dest = regs_of(first); touched = regs_of(rest)
            else:
                dest = set()
            for ent in st:
                if ent & touched:
                    violations.append((name, bi, mn + ' ' + ops, sorted(ent & touched)))
            if is_ds or is_smem:
                st.append(frozenset(dest))
            if mn.startswith('s_branch'):
                succ = [labels[ops.strip()]]
            elif mn.startswith('s_cbranch'):
                succ = [labels[ops.strip()], bi + 1]
            elif mn == 's_endpgm':
                succ = []
        while st and not st[0]: st.pop(0)          # oldest entries without registers cannot matter
        st = st[-24:]
        for s in succ: work.append((s, tuple(st)))
    return violations

def check(asm):
    """-> (number of kernels analysed, list of violations (kernel, block, instruction, registers))"""
    v = []
    n = 0
    for name, items in parse_functions(asm).items():
        if any(k == 'inst' and a.startswith('ds_read') for k, a, b in items):
            n += 1
            v += check_function(items, name)
    return n, v

