"""Static check of compiled GPU assembly for one hazard class of hand-scheduled LDS reads.

The streamed GEMM kernels issue their LDS reads from inline assembly and wait for them with explicit counters, so
the compiler believes a read is complete when its statement ends.  If nothing consumes a read's destination (a
prefetch past the last stage), the register allocator may hand those registers to something else, for instance the
address of the next LDS-direct load, while the data is still on its way: it then lands on top of the new value and
the load goes to a wild address.  This walks a kernel's instructions in program order, tracks the LDS reads still in
flight (the LGKM counter completes in order; `s_waitcnt lgkmcnt(n)` leaves the n newest) and reports every
instruction that writes or reads a vector register an in-flight read will still write.
"""
import re


def _regs(tok):
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", tok)
    return {int(m.group(1))} if m else set()


_NO_VGPR_DEST = ("v_mfma", "v_cmp", "v_accvgpr_write", "v_readfirstlane", "v_readlane")
_LOADS_WITH_DEST = ("global_load_dword", "global_load_ushort", "global_load_ubyte", "global_load_short", "buffer_load", "scratch_load", "flat_load")


def _merge(states):
    """In-flight lists of several predecessors -> one list that is at least as pending as each: position by position
    from the newest end, the union of the destinations."""
    out = []
    for k in range(1, max((len(s) for s in states), default=0) + 1):
        dest = set()
        for s in states:
            if len(s) >= k:
                dest |= s[-k][0]
        out.append((dest, -1))
    return out[::-1]


def check_kernel(lines):
    """Returns a list of (line index, message) for the instruction lines of one kernel.

    Program order is file order, except at a label that cannot be fallen into (the instruction before it is an
    unconditional branch or the end of the program) and whose every branch to it lies earlier in the file: there the
    state is the merge of the states at those branches (the compiler moves cold blocks, such as the tail of the
    epilogue, behind the main loop, where file order would pair them with the loop's last reads)."""
    targets = {}
    for ln in lines:
        t = ln.split(";")[0].strip()
        if t.startswith(("s_branch", "s_cbranch")):
            lab = t.split()[-1]
            targets[lab] = targets.get(lab, 0) + 1
    inflight, found = [], []
    at_branch = {}                    # label -> states at the branches to it seen so far
    falls_through = True
    for n, ln in enumerate(lines):
        t = ln.split(";")[0].strip()
        if t.endswith(":") and not t.startswith(".amdhsa") and " " not in t:
            lab = t[:-1]
            seen = at_branch.get(lab, [])
            if not falls_through and seen and len(seen) == targets.get(lab, 0):
                inflight = _merge(seen)
            elif falls_through and seen:
                inflight = _merge(seen + [inflight])
            falls_through = True
            continue
        if not t or t.endswith(":") or t.startswith("."):
            continue
        parts = t.replace(",", " ").split()
        op, args = parts[0], parts[1:]
        if op.startswith(("s_branch", "s_cbranch")):
            at_branch.setdefault(args[-1], []).append(list(inflight))
            falls_through = op != "s_branch"
            continue
        falls_through = op != "s_endpgm"
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", t)
            if m:
                keep = int(m.group(1))
                inflight = inflight[len(inflight) - keep:] if 0 < keep < len(inflight) else ([] if keep == 0 else inflight)
            continue
        is_lds_read = op.startswith("ds_read") or op.startswith("ds_load")
        dest = set()
        if is_lds_read:
            dest = _regs(args[0])
        elif op.startswith(_NO_VGPR_DEST) or op.startswith("global_load_lds"):
            dest = set()
        elif op.startswith("v_") or op.startswith(_LOADS_WITH_DEST):
            dest = _regs(args[0]) if args else set()
        srcs = set()
        for a in (args[1:] if dest else args):
            srcs |= _regs(a)
        pending = set().union(*[d for d, _ in inflight]) if inflight else set()
        if dest & pending:
            found.append((n, "writes v%s while an LDS read into it is in flight: %s" % (sorted(dest & pending), t)))
        if srcs & pending:
            found.append((n, "reads v%s before the LDS read into it has been waited for: %s" % (sorted(srcs & pending), t)))
        if is_lds_read:
            inflight.append((dest, n))
        elif op.startswith(("ds_write", "ds_store", "s_load", "s_buffer_load")):
            inflight.append((set(), n))          # these count on the same counter
    return found


def _aregs(tok):
    m = re.fullmatch(r"a\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"a(\d+)", tok)
    return {int(m.group(1))} if m else set()


def check_accumulator_reads(lines, min_idle=32):
    """The MFMAs of these kernels are issued from inline assembly, so the compiler inserts no wait states behind them.
    Reports every instruction other than an MFMA that reads (or overwrites) an accumulation register within `min_idle`
    idle cycles of the MFMA that writes it.  Cycles are counted from what follows that MFMA: `s_nop n` is n + 1, a
    later MFMA 16 (they run one after another), anything else 1 - an underestimate, which errs on the safe side."""
    found, recent = [], []                     # recent: [set(agprs), cycles since issue]
    for n, ln in enumerate(lines):
        t = ln.split(";")[0].strip()
        if not t or t.startswith("."):
            continue
        if t.endswith(":"):
            continue
        parts = t.replace(",", " ").split()
        op, args = parts[0], parts[1:]
        if op.startswith("v_mfma"):
            for r in recent:
                r[1] += 16
            recent.append([_aregs(args[0]), 0])
        else:
            touched = set()
            for a in args:
                touched |= _aregs(a)
            for regs_, cyc in recent:
                if cyc < min_idle and touched & regs_:
                    found.append((n, "touches a%s %d cycles behind the MFMA that writes it: %s" % (sorted(touched & regs_), cyc, t)))
            m = re.fullmatch(r"s_nop", op)
            step = int(args[0]) + 1 if m and args else 1
            for r in recent:
                r[1] += step
        recent = [r for r in recent if r[1] < min_idle]
    return found


def kernels(asm_text, name_pattern):
    """Yields (mangled name, instruction lines) for the kernels whose mangled name matches name_pattern."""
    src = asm_text.split("\n")
    for i, l in enumerate(src):
        m = re.match(r"^(_Z\w+):", l)
        if m and re.search(name_pattern, m.group(1)):
            j = i
            while j < len(src) and "s_endpgm" not in src[j]:
                j += 1
            yield m.group(1), src[i:j]
