"""Build-time check of the tuned attention kernel's generated ISA.

The kernel issues its LDS operand reads as inline assembly (ds_read_b128 / ds_read_b64_tr_b16) and
waits for them with an explicit ``s_waitcnt lgkmcnt(0)``.  The compiler does not know that those
registers are still being written between the two; this script verifies, on the assembly hipcc
produced, that no instruction touches the destination registers of such a read before the next
explicit wait (a register copy or a spill in that window would read stale data).
"""
import re
import sys


def check(path: str, verbose: bool = True) -> int:
    lines = open(path).read().split('\n')
    return _check_lines(lines, verbose)


def _check_lines(lines, verbose):
    def regs(tok):
        m = re.match(r'v\[(\d+):(\d+)\]', tok)
        if m: return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.match(r'v(\d+)$', tok)
        if m: return {int(m.group(1))}
        return set()
    pending = {}   # reg -> line of read
    in_asm = False
    bad = 0
    for i, l in enumerate(lines):
        t = l.strip()
        if t.startswith(';;#ASMSTART'): in_asm = True; continue
        if t.startswith(';;#ASMEND'): in_asm = False; continue
        if not t or t.startswith((';', '.', '//')): continue
        if re.match(r'^\.?LBB', t): continue
        ops = re.findall(r'v\[\d+:\d+\]|v\d+', t)
        used = set().union(*[regs(o) for o in ops]) if ops else set()
        if in_asm and t.startswith('ds_read'):
            dst = regs(t.split()[1].rstrip(','))
            for r in dst: pending[r] = i + 1
            continue
        if in_asm and t.startswith('s_waitcnt'):
            pending.clear(); continue
        hit = used & set(pending)
        if hit:
            bad += 1
            if bad <= 10 and verbose: print(f"line {i+1}: '{t[:70]}' touches regs {sorted(hit)[:6]} of an in-flight asm LDS read (issued line {pending[min(hit)]})")
    if verbose:
        print("asm-read discipline violations:", bad)
    return bad


if __name__ == "__main__":
    sys.exit(1 if check(sys.argv[1]) else 0)
