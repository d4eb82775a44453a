"""Static check of compiled gfx950 ISA for kernels that issue loads by hand (inline assembly) and count their
own waits: no instruction may read or write a vector register that is the destination of a load still in
flight.

The projection kernel's wide form requests weights (global_load) and activation fragments (ds_read) in inline
assembly and waits with literal s_waitcnt counts; the compiler does not know that such a register is written
later than the statement that names it, so a register it considers dead, or a copy it inserts, would be
corrupted when the data lands (found the hard way: a weight load nobody consumed landed in a register that by
then held an address).  This walker replays every path through a kernel's basic blocks with the ordered list of
outstanding loads per counter (vmcnt, lgkmcnt), retires entries at each s_waitcnt exactly as the hardware does
(loads complete in issue order), and reports any instruction that names a register of an outstanding load.
It also validates the compiler's own waits for the loads it tracks itself.

Usage: python tests/isa_check.py file.s [substring of the mangled kernel names to check]
"""
import re, sys
from collections import deque

REG = re.compile(r'\bv\[(\d+):(\d+)\]|\bv(\d+)\b')

def regs_of(text):
    out = []
    for m in REG.finditer(text):
        if m.group(1) is not None:
            out.append((int(m.group(1)), int(m.group(2))))
        else:
            out.append((int(m.group(3)), int(m.group(3))))
    return out

def overlap(a, b):
    return a[0] <= b[1] and b[0] <= a[1]

def parse(fn_text):
    blocks, cur, order = {}, None, []
    for raw in fn_text.splitlines():
        line = raw.split(';')[0].strip()
        if not line:
            continue
        m = re.match(r'^(\.LBB\d+_\d+):', line)
        if m:
            cur = m.group(1); blocks[cur] = []; order.append(cur); continue
        if cur is None:
            cur = 'entry'; blocks[cur] = []; order.append(cur)
        if line.endswith(':') or line.startswith('.'):
            continue
        blocks[cur].append(line)
    return blocks, order

def walk(blocks, order, kernel):
    # state: (vm tuple of (dest or None), lgkm tuple of dest)
    start = (order[0], 0, (), ())
    seen = set()
    work = deque([start])
    errors = set()
    steps = 0
    while work:
        name, pc, vm, lg = work.popleft()
        # entries without a destination at the OLD end of a queue retire first and retire nothing else with
        # them: dropping them changes no later verdict, and lets paths that differ only there (a store under a
        # branch) fall together
        while vm and vm[0] is None:
            vm = vm[1:]
        while lg and lg[0] == (-1, -1):
            lg = lg[1:]
        key = (name, pc, vm, lg)
        if key in seen:
            continue
        seen.add(key)
        ins = blocks[name]
        vm, lg = list(vm), list(lg)
        i = pc
        while True:
            steps += 1
            if steps > 600_000:
                errors.add("step bound reached: kernel not fully explored"); return errors
            if i >= len(ins):
                idx = order.index(name)
                if idx + 1 < len(order):
                    work.append((order[idx + 1], 0, tuple(vm), tuple(lg)))
                break
            line = ins[i]
            op = line.split()[0]
            rest = line[len(op):]
            if op == 's_waitcnt':
                m = re.search(r'vmcnt\((\d+)\)', rest)
                if m:
                    n = int(m.group(1)); vm = vm[len(vm) - n:] if n < len(vm) else vm
                    if n == 0: vm = []
                m = re.search(r'lgkmcnt\((\d+)\)', rest)
                if m:
                    n = int(m.group(1)); lg = lg[len(lg) - n:] if n < len(lg) else lg
                    if n == 0: lg = []
                i += 1; continue
            if op == 's_endpgm':
                break
            if op.startswith('s_cbranch') or op == 's_branch':
                tgt = rest.strip()
                if tgt in blocks:
                    work.append((tgt, 0, tuple(vm), tuple(lg)))
                if op == 's_branch':
                    break
                i += 1; continue
            rs = regs_of(rest)
            for d in [x for x in vm if x] + list(lg):
                for r in rs:
                    if overlap(d, r):
                        errors.add(f"{name}+{i}: `{line}` touches v[{d[0]}:{d[1]}] while its load is in flight")
            if op.startswith('global_load_lds') or op.startswith('buffer_load') and 'lds' in rest:
                vm.append(None)
            elif op.startswith('global_load') or op.startswith('buffer_load') or op.startswith('scratch_load') or op.startswith('flat_load'):
                vm.append(rs[0] if rs else None)
            elif op.startswith('global_store') or op.startswith('buffer_store') or op.startswith('scratch_store') or op.startswith('global_atomic') or op.startswith('flat_store') or op.startswith('flat_atomic'):
                vm.append(None)
            elif op.startswith('ds_read') or op.startswith('ds_load'):
                lg.append(rs[0])
            elif op.startswith('ds_write') or op.startswith('ds_store') or op.startswith('s_load') or op.startswith('s_buffer_load'):
                lg.append((-1, -1))
            # keep the state bounded (older entries beyond what any wait distinguishes are complete in practice? no: keep)
            if len(vm) > 64: vm = vm[-64:]           # (the hardware counter holds 63: older ones have completed)
            i += 1
    return errors

def check_text(s, pat):
    """{mangled kernel name: sorted list of violations} for every function whose name contains `pat`."""
    out = {}
    for m in re.finditer(r'^(_Z\w+):', s, re.M):
        name = m.group(1)
        if pat not in name:
            continue
        j = s.find('.Lfunc_end', m.end())
        blocks, order = parse(s[m.end():j if j >= 0 else len(s)])
        out[name] = sorted(walk(blocks, order, name))
    return out


def scratch_bytes(s, pat):
    """{kernel name: bytes of scratch per lane} from the code object metadata in the assembly text."""
    out = {}
    for m in re.finditer(r'\.name:\s+(_Z\w+)\n(?:.*\n)*?\s+\.private_segment_fixed_size:\s+(\d+)', s):
        if pat in m.group(1):
            out[m.group(1)] = int(m.group(2))
    return out


def main():
    s = open(sys.argv[1]).read()
    pat = sys.argv[2] if len(sys.argv) > 2 else 'gemm_wide_kernel'
    total = 0
    for name, errs in check_text(s, pat).items():
        total += len(errs)
        print(name, 'violations:', len(errs))
        for e in errs[:6]:
            print('   ', e)
    print('TOTAL', total)
    return 1 if total else 0

if __name__ == '__main__':
    sys.exit(main())
