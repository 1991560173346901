"""Build-time check of the tuned attention kernel's generated ISA.

The kernel issues its LDS operand reads as inline assembly (ds_read_b128 / ds_read_b64_tr_b16) and
waits for them with an explicit ``s_waitcnt lgkmcnt(N)``.  The compiler does not know that those
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
    def regs(tok):   # vector registers (v) and accumulation registers (a), as (file, index)
        m = re.match(r'([va])\[(\d+):(\d+)\]', tok)
        if m: return {(m.group(1), r) for r in range(int(m.group(2)), int(m.group(3)) + 1)}
        m = re.match(r'([va])(\d+)$', tok)
        if m: return {(m.group(1), int(m.group(2)))}
        return set()
    pending = {}   # reg -> (line of read, sequence number of that read)
    nread = 0      # inline-asm LDS reads seen so far
    in_asm = False
    bad = 0
    for i, l in enumerate(lines):
        t = l.strip()
        if t.startswith(';;#ASMSTART'): in_asm = True; continue
        if t.startswith(';;#ASMEND'): in_asm = False; continue
        if not t or t.startswith((';', '.', '//')): continue
        if re.match(r'^\.?LBB', t): continue
        if t.startswith(('s_branch', 's_endpgm', 's_setpc')):
            # straight-line approximation of the control flow: nothing falls through an unconditional jump, so
            # what follows in the text is not reached with these reads in flight
            pending = {}
            continue
        ops = re.findall(r'\b[va]\[\d+:\d+\]|\b[va]\d+\b', t)
        used = set().union(*[regs(o) for o in ops]) if ops else set()
        if in_asm and t.startswith('ds_read'):
            dst = regs(t.split()[1].rstrip(','))
            nread += 1
            for r in dst: pending[r] = (i + 1, nread)
            continue
        if in_asm and t.startswith('s_waitcnt'):
            # lgkmcnt(N) leaves at most N LDS operations outstanding and they complete in order, so all but the
            # N most recent asm reads have landed (other LDS traffic in between only makes the wait stricter)
            m = re.search(r'lgkmcnt\((\d+)\)', t)
            if m:
                keep = int(m.group(1))
                pending = {r: v for r, v in pending.items() if v[1] > nread - keep}
            continue
        hit = used & set(pending)
        if hit:
            bad += 1
            if bad <= 10 and verbose: print(f"line {i+1}: '{t[:70]}' touches regs {sorted(hit)[:6]} of an in-flight asm LDS read (issued line {pending[min(hit)][0]})")
    if verbose:
        print("asm-read discipline violations:", bad)
    return bad


if __name__ == "__main__":
    sys.exit(1 if check(sys.argv[1]) else 0)
