"""Static check of hand-pipelined kernels: no instruction may read (or overwrite) a register whose
global load is still outstanding according to the s_waitcnt vmcnt counts.  Walks the control-flow
graph of every kernel in a hipcc -S listing (both ways of every conditional branch), carrying the
ordered queue of outstanding vector-memory operations.  The weight FIFOs of the tiled GEMM issue their
loads from inline asm and count the waits by hand, which the compiler knows nothing about: it must
never copy, spill or reuse such a register while its load is in flight.  Used by test_asm_pipelines.py."""
import re, sys

def regs(tok):
    out = []
    for m in re.finditer(r'\b([va])\[(\d+):(\d+)\]|\b([va])(\d+)\b', tok):
        if m.group(1):
            out += [(m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1)]
        else:
            out.append((m.group(4), int(m.group(5))))
    return out

def parse(path):
    """-> {kernel: (blocks, order)}; blocks[label] = list of (lineno, ins)."""
    kernels = {}
    cur = None
    label = None
    for ln, line in enumerate(open(path), 1):
        s = line.strip()
        if not s or s.startswith(';'):
            continue
        m = re.match(r'^([A-Za-z_.$][\w.$]*):', s)
        if m:
            name = m.group(1)
            if not name.startswith('.'):
                cur = {'blocks': {}, 'order': []}
                kernels[name] = cur
                label = '<entry>'
                cur['blocks'][label] = []
                cur['order'].append(label)
            elif cur is not None and name.startswith('.LBB'):
                label = name
                cur['blocks'][label] = []
                cur['order'].append(label)
            continue
        if s.startswith('.'):
            if s.startswith('.end_amdhsa_kernel') or s.startswith('.section') or s.startswith('.Lfunc_end'):
                pass
            continue
        if cur is None:
            continue
        ins = s.split(';')[0].strip()
        if ins:
            cur['blocks'][label].append((ln, ins))
    return kernels

def step(ins, queue):
    """-> (new_queue, hit_registers)."""
    op = ins.split()[0]
    if op == 's_waitcnt':
        v = re.search(r'vmcnt\((\d+)\)', ins)
        if v:
            n = int(v.group(1))
            if len(queue) > n:
                queue = queue[len(queue) - n:] if n else ()
        return queue, []
    if op.startswith('s_'):
        return queue, []
    args = ins[len(op):]
    parts = [a.strip() for a in args.split(',')]
    is_load = op.startswith(('global_load', 'scratch_load', 'buffer_load', 'flat_load'))
    is_store = op.startswith(('global_store', 'scratch_store', 'buffer_store', 'global_atomic', 'flat_store', 'flat_atomic'))
    is_dma = op.startswith('global_load_lds') or (op.startswith('buffer_load') and ' lds' in ins)
    touched = []
    for i, a in enumerate(parts):
        # reads and writes alike: a write into a pending register is a hazard too -- except the destination of
        # another load: vector-memory loads of a wave return in order, so the later load lands later
        if is_load and i == 0:
            continue
        touched += regs(a)
    pend = set()
    for d in queue:
        pend |= d
    hit = [r for r in touched if r in pend]
    if is_load or is_store:
        dst = frozenset(regs(parts[0])) if (is_load and not is_dma) else frozenset()
        queue = queue + (dst,)
        if not any(queue):
            queue = ()          # nothing pending can be touched any more
    return queue, hit

def check_kernel(path, name, k, limit=3000000):
    blocks, order = k['blocks'], k['order']
    nxt = {order[i]: (order[i + 1] if i + 1 < len(order) else None) for i in range(len(order))}
    seen = set()
    work = [('<entry>', ())]
    bad = {}
    visits = 0
    while work:
        label, queue = work.pop()
        if label is None or (label, queue) in seen:
            continue
        seen.add((label, queue))
        visits += 1
        if visits > limit:
            print(f"{name}: state limit reached")
            return 1
        ended = False
        for ln, ins in blocks[label]:
            op = ins.split()[0]
            if op == 's_endpgm':
                ended = True
                break
            if op == 's_branch':
                work.append((ins.split()[1], queue))
                ended = True
                break
            if op.startswith('s_cbranch'):
                work.append((ins.split()[1], queue))
                continue
            queue, hit = step(ins, queue)
            if hit and ln not in bad:
                bad[ln] = (hit, ins)
        if not ended:
            work.append((nxt[label], queue))
    for ln in sorted(bad)[:10]:
        print(f"{path}:{ln}: [{name[:60]}] touches pending {bad[ln][0][:4]}: {bad[ln][1]}")
    return len(bad)

def check(path):
    total = 0
    for name, k in parse(path).items():
        n = check_kernel(path, name, k)
        total += n
    print(path, "violations:", total)
    return total

if __name__ == "__main__":
    sys.exit(1 if sum(check(p) for p in sys.argv[1:]) else 0)
