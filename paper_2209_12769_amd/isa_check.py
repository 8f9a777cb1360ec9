"""Build-time check of a kernel's ISA listing (no GPU needed).

The data-moving waves of the bulk layer kernel issue their loads through inline asm that the compiler does
not track, and wait for them by hand.  The compiler is then free to copy, reuse or overwrite a load's
destination registers while the load is still in flight: it did so when a loop was restructured (copies of
descriptor registers on the way into the loop) and when loads were issued whose results nothing used (their
registers were reused at once, and the data that arrived later overwrote addresses: a GPU memory fault).
This walks every basic block in file order, with no load pending at its entry, and reports any instruction
outside inline asm that reads or writes the destination registers of an asm load before an s_waitcnt vmcnt
has covered that load.  It only sees hazards inside a block, which is where such copies land.

Usage: python -m paper_2209_12769_amd.isa_check [listing.s [kernel-symbol-regex ...]]
With no arguments it compiles csrc/gnn_layer256.hip to a listing and checks every layer256_*kernel in it."""
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

def check(path, kernel_pat):
    L = open(path).read().splitlines()
    start = [i for i, l in enumerate(L) if re.match(kernel_pat, l)][0]
    end = [i for i in range(start, len(L)) if L[i].strip().startswith('.Lfunc_end')][0]
    pending = []      # list of (dest regs, line no)
    in_asm = False
    hazards = []
    for n in range(start, end):
        t = L[n].strip()
        if t.startswith(';;#ASMSTART'): in_asm = True; continue
        if t.startswith(';;#ASMEND'): in_asm = False; continue
        if not t or t.startswith(';'): continue
        if re.match(r'^\.?[A-Za-z_0-9]+:', t):       # label: new block, forget (unknown) pending state
            pending = []
            continue
        if t.startswith('.'): continue
        op = t.split()[0]
        if op.startswith('s_waitcnt'):
            k = vmcnt(t)
            if k is not None:
                pending = pending[len(pending) - k:] if k < len(pending) else pending
                if k == 0: pending = []
            continue
        if op.startswith('s_barrier') or op.startswith('s_cbranch') or op.startswith('s_branch'):
            continue
        args = t[len(op):]
        parts = [p.strip() for p in args.split(',')]
        if in_asm and op.startswith('global_load_dwordx4') and 'lds' not in op:
            dest = regs(parts[0])
            src = set()
            for p in parts[1:]: src |= regs(p)
            for d, ln in pending:
                if d & src: hazards.append((n + 1, t, ln))
            pending.append((dest, n + 1))
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
    import os, subprocess
    here = os.path.dirname(os.path.abspath(__file__))
    subprocess.check_call(["hipcc", "-O3", "--offload-arch=gfx950", "--cuda-device-only", "-S", "-std=c++17",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-I", os.path.join(here, "..", "include"), "-I", os.path.join(here, "csrc"),
                           source, "-o", out], stderr=subprocess.DEVNULL)
    return out


def kernels_in(path, name):
    return [l.split(':')[0] for l in open(path).read().splitlines() if re.match(r'^_Z\w*' + name + r'\w*:', l)]


def check_layer256(listing=None):
    """{kernel symbol: hazards} for every instantiation of layer256_kernel and layer256_dma1_kernel."""
    import os, tempfile
    here = os.path.dirname(os.path.abspath(__file__))
    if listing is None:
        listing = listing_of(os.path.join(here, "csrc", "gnn_layer256.hip"),
                             os.path.join(tempfile.mkdtemp(), "gnn_layer256.s"))
    return {k: check(listing, '^' + re.escape(k) + ':') for k in kernels_in(listing, "layer256_")}


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
