"""Static checks of the compiled gfx950 code.

scan(): a guard for scalar loads written as inline asm.  The compiler does not know that the
destination SGPRs of such a load are in flight until the next s_waitcnt lgkmcnt(0); the scan
walks every kernel linearly and reports any instruction that reads or writes an SGPR of an
inline-asm scalar load between its issue and that wait.  (Unconditional branches and s_endpgm
end a straight-line run.)  The kernels here fetch their wave-uniform operands with ordinary
constant-address-space loads, which the compiler tracks itself, so the scan finds no such load
at all; it stays in the build as a guard against one coming back.

kernel_stats(): spill counts and instruction histograms per kernel, for the code-generation
checks of the build.
"""
import re, sys

def regs(tok):
    tok = tok.strip()
    m = re.match(r'^s\[(\d+):(\d+)\]$', tok)
    if m: return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r'^s(\d+)$', tok)
    if m: return {int(m.group(1))}
    return set()

NO_SDST = ('s_cmp', 's_cbranch', 's_branch', 's_waitcnt', 's_barrier', 's_nop', 's_endpgm', 's_bitcmp',
           's_setprio', 's_sleep', 's_setreg', 's_sendmsg', 's_icache', 's_dcache', 's_store', 's_buffer_store')

def scan(path):
    """Returns a list of (kernel, line, text, 'reads'|'writes', registers, issue line)."""
    lines = open(path).read().split('\n')
    label_in = {}  # (kernel, label) -> loads in flight at some branch to that label
    for _ in range(4):  # a few sweeps so that states carried by backward branches settle
        out = set()
        kern, inflight, in_asm = None, [], False
        for i, l in enumerate(lines):
            t = l.strip()
            if t.startswith(';;#ASMSTART'): in_asm = True; continue
            if t.startswith(';;#ASMEND'): in_asm = False; continue
            m = re.match(r'^(_Z\w+):', t)
            if m: kern, inflight = m.group(1), []; continue
            m = re.match(r'^(\.LBB\w+):', t)
            if m:
                for e in label_in.get((kern, m.group(1)), []):
                    if e not in inflight: inflight.append(e)
                continue
            if not t or t[0] in ';.':
                continue
            t = t.split(';')[0].strip()
            op = t.split()[0]
            args = [a.strip() for a in t[len(op):].split(',')] if len(t) > len(op) else []
            if op == 's_waitcnt':
                if 'lgkmcnt(0)' in t: inflight = []
                continue
            if op.startswith(('s_cbranch', 's_branch')):
                tgt = label_in.setdefault((kern, args[0]), [])
                for e in inflight:
                    if e not in tgt: tgt.append(e)
                if op == 's_branch': inflight = []
                continue
            if op in ('s_endpgm', 's_setpc_b64'):
                inflight = []; continue
            dst = regs(args[0]) if args else set()
            writes = set()
            if op.startswith('s_') and not op.startswith(NO_SDST): writes = dst
            elif op.startswith(('v_readlane', 'v_readfirstlane')): writes = dst
            elif op.startswith('v_cmp') and op.endswith('_e64'): writes = dst
            srcs = set()
            for a in (args if not writes else args[1:]): srcs |= regs(a)
            for r, ln in inflight:
                if writes & set(r): out.add((kern, i + 1, t, 'writes', tuple(sorted(writes & set(r))), ln + 1))
                if srcs & set(r): out.add((kern, i + 1, t, 'reads', tuple(sorted(srcs & set(r))), ln + 1))
            if in_asm and op.startswith('s_load_dword'):
                inflight.append((tuple(sorted(dst)), i))
    return sorted(out, key=lambda e: e[1])

def report(bad, limit=40):
    lines = ["%s: line %d: '%s' %s SGPR %s of the scalar load issued at line %d" % e for e in bad[:limit]]
    return "\n".join(lines)


if __name__ == "__main__":
    bad = scan(sys.argv[1])
    for k, ln, t, what, rr, l0 in bad[:40]:
        print(f"{k}: line {ln}: '{t}' {what} SGPR {rr} of the load issued at line {l0}")
    print("violations:", len(bad))


def kernel_stats(path):
    """Per kernel of a device listing: VGPR spill count from the metadata and how often each
    instruction mnemonic occurs in its body.  Returns {mangled name: (spills, {mnemonic: n})}."""
    import collections
    import re
    body = {}
    name = None
    spills = {}
    cur_meta = None
    for ln in open(path):
        m = re.match(r"^(_Z\w+):", ln)
        if m:
            name = m.group(1)
            body[name] = collections.Counter()
            continue
        t = ln.strip()
        if name and t and not t.startswith((";", ".", "_Z")) and ":" not in t.split()[0]:
            body[name][t.split()[0]] += 1
        if t.startswith("s_endpgm"):
            name = None
        m = re.match(r"^\s+\.name:\s+(\S+)", ln)
        if m:
            cur_meta = m.group(1)
        m = re.match(r"^\s+\.vgpr_spill_count:\s+(\d+)", ln)
        if m and cur_meta:
            spills[cur_meta] = int(m.group(1))
    return {k: (spills.get(k, 0), v) for k, v in body.items() if k in spills}


def scratch_bytes(path):
    """Per kernel of a device listing: bytes of private (scratch) memory per lane, from the
    metadata.  Returns {mangled name: bytes}."""
    out = {}
    text = open(path).read()
    for block in text.split("  - .agpr_count:")[1:]:
        n = re.search(r"\.name:\s+(\S+)", block)
        v = re.search(r"\.private_segment_fixed_size:\s+(\d+)", block)
        if n and v:
            out[n.group(1)] = int(v.group(1))
    return out
