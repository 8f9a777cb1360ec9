"""Build-time check of a kernel's ISA listing (no GPU needed).

The bulk layer kernels wait by hand (s_waitcnt vmcnt) for loads that inline asm issues and the compiler does
not track.  As they stand those loads are direct copies into LDS, which have no destination registers; an
earlier form loaded into registers the same way, and the compiler, unaware of the loads, copied, reused and
overwrote their destination registers while they were in flight (once a GPU memory fault, once rare wrong
sums).  This check keeps that form from coming back unnoticed: it walks the listing in file order and reports
any instruction outside inline asm that reads or writes the destination registers of an asm load before an
s_waitcnt vmcnt has covered that load.  Loads pending at a branch are carried to its target, and the walk is
repeated until nothing new arrives at any label, so loads that stay in flight across a loop's back edge are
still pending at the loop's head.  build.py runs it on every build.

Usage: python -m paper_2209_12769_amd.isa_check [listing.s [kernel-symbol-regex ...]]
With no arguments it compiles the two layer-kernel sources to listings and checks every layer256 kernel."""
import re, sys

def regs(tok):
    out = set()
    for m in re.finditer(r'\bv\[(\d+):(\d+)\]', tok):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r'\bv(\d+)\b', tok):
        out.add(int(m.group(1)))
    return out

def vmcnt(line):
    m = re.search(r'vmcnt\((\d+)\)', line)
    if m: return int(m.group(1))
    m = re.search(r's_waitcnt\s+(0x[0-9a-f]+|\d+)$', line)
    if m:
        v = int(m.group(1), 0)
        return (v & 15) | (((v >> 14) & 3) << 4)
    return None

def _merge(a, b):
    """Union of two pending lists, oldest first (by the line of the load)."""
    seen = {}
    for d, ln in list(a) + list(b):
        seen[ln] = d
    return [(seen[ln], ln) for ln in sorted(seen)]


def check(path, kernel_pat):
    """Hazards of one kernel: (line, instruction, line of the load) for every instruction outside inline asm
    that reads or writes the destination of an asm load not yet covered by an s_waitcnt vmcnt.  The loads
    pending at a label are those pending where control falls into it plus those pending at every branch
    to it; the listing is walked until these sets stop growing, so that loads kept in flight across a
    loop's back edge are still pending at the loop's head."""
    L = open(path).read().splitlines()
    start = [i for i, l in enumerate(L) if re.match(kernel_pat, l)][0]
    end = [i for i in range(start, len(L)) if L[i].strip().startswith('.Lfunc_end')][0]
    at_label = {}                     # label -> pending loads carried in by branches (grows over the passes)
    hazards = []
    for _ in range(6):
        before = {k: len(v) for k, v in at_label.items()}
        hazards = _walk(L, start, end, at_label)
        if {k: len(v) for k, v in at_label.items()} == before:
            break
    return sorted(set(hazards))


def _walk(L, start, end, at_label):
    pending = []      # list of (dest regs, line no)
    in_asm = False
    fell_off = False  # the previous instruction was an unconditional branch: nothing falls into the next label
    hazards = []
    for n in range(start, end):
        t = L[n].strip()
        if t.startswith(';;#ASMSTART'): in_asm = True; continue
        if t.startswith(';;#ASMEND'): in_asm = False; continue
        if not t or t.startswith(';'): continue
        m = re.match(r'^(\.?[A-Za-z_0-9$]+):', t)
        if m:                                        # label: what falls in, plus what the branches to it carry
            pending = _merge([] if fell_off else pending, at_label.get(m.group(1), []))
            fell_off = False
            continue
        if t.startswith('.'): continue
        op = t.split()[0]
        if op.startswith('s_waitcnt'):
            k = vmcnt(t)
            if k is not None:
                pending = pending[len(pending) - k:] if k < len(pending) else pending
                if k == 0: pending = []
            continue
        if op.startswith('s_cbranch') or op.startswith('s_branch'):
            target = t.split()[-1]
            at_label[target] = _merge(at_label.get(target, []), pending)
            fell_off = op.startswith('s_branch')
            if fell_off: pending = []
            continue
        if op.startswith('s_endpgm'):
            fell_off = True
            pending = []
            continue
        fell_off = False
        if op.startswith('s_barrier'):
            continue
        args = t[len(op):]
        parts = [p.strip() for p in args.split(',')]
        if in_asm and op.startswith('global_load_dwordx4') and 'lds' not in op:
            dest = regs(parts[0])
            src = set()
            for p in parts[1:]: src |= regs(p)
            for d, ln in pending:
                if d & src: hazards.append((n + 1, t, ln))
            pending = [(d, ln) for d, ln in pending if ln != n + 1] + [(dest, n + 1)]
            continue
        if in_asm:
            continue          # the pin statements name registers without touching them
        # ordinary instruction: first operand is usually the destination
        src = set()
        for p in (parts[1:] if len(parts) > 1 else parts): src |= regs(p)
        dst = regs(parts[0]) if parts else set()
        if op.startswith(('ds_write', 'global_store', 'scratch_store', 'v_cmp', 'buffer_store')):
            src |= dst
        for d, ln in pending:
            if d & src:
                hazards.append((n + 1, t, ln))
            if d & dst and not op.startswith(('ds_write', 'global_store', 'v_cmp')):
                hazards.append((n + 1, 'WRITE ' + t, ln))
    return hazards

def listing_of(source, out):
    """Compiles one HIP source to a gfx950 ISA listing with the library's flags."""
    import subprocess
    from . import build
    subprocess.check_call(["hipcc", *build.COMPILE_FLAGS, "--cuda-device-only", "-S", source, "-o", out],
                          stderr=subprocess.DEVNULL)
    return out


def kernels_in(path, name):
    return [l.split(':')[0] for l in open(path).read().splitlines() if re.match(r'^_Z\w*' + name + r'\w*:', l)]


def check_layer256(listing=None):
    """{kernel symbol: hazards} for every layer256 kernel of csrc/gnn_layer256.hip and csrc/gnn_layer256w.hip
    (or of the given listing)."""
    import os, tempfile
    here = os.path.dirname(os.path.abspath(__file__))
    listings = [listing] if listing else [
        listing_of(os.path.join(here, "csrc", f + ".hip"), os.path.join(tempfile.mkdtemp(), f + ".s"))
        for f in ("gnn_layer256", "gnn_layer256w")]
    return {k: check(l, '^' + re.escape(k) + ':') for l in listings for k in kernels_in(l, "layer256")}


if __name__ == '__main__':
    if len(sys.argv) > 2:
        res = {pat: check(sys.argv[1], pat) for pat in sys.argv[2:]}
    else:
        res = check_layer256(sys.argv[1] if len(sys.argv) > 1 else None)
    for k, hz in res.items():
        print(k[:90], 'hazards:', len(hz))
        for h in hz[:12]:
            print('   line', h[0], h[1], '<- load at line', h[2])
    sys.exit(1 if any(res.values()) else 0)
