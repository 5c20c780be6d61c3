"""Build-time check of the compiler's output for the kernels whose global loads are assembly statements.

Those loads (buffer_load ... in an asm statement) are invisible to the compiler: it inserts no wait for
them and does not know that their destination registers are still to be written.  The kernels place the
waits by hand (s_waitcnt vmcnt), which is sound only while, on every path through the code, nothing reads
or writes a load's destination registers between the load and the wait that covers it: a register the
compiler reused in between would be overwritten when the load lands, and if it then held an address the
kernel would access memory it does not own.  This module walks the generated assembly (control-flow graph
of each kernel, the queue of outstanding loads as the state) and reports every such use.
"""
import re


def _vregs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(3) is not None:
            out.add(int(m.group(3)))
        else:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return frozenset(out)


def parse_functions(text, pattern):
    """{kernel symbol: [("label", name, line) | ("inst", text, line)]} for symbols matching `pattern`"""
    fns, cur = {}, None
    for ln, line in enumerate(text.splitlines(), 1):
        t = line.split(";")[0].strip()
        if not t:
            continue
        m = re.match(r"^(_Z\w+):", t)
        if m:
            cur = [] if re.search(pattern, m.group(1)) else None
            if cur is not None:
                fns[m.group(1)] = cur
            continue
        if cur is None:
            continue
        if t.startswith(".Lfunc_end"):
            cur = None
            continue
        m = re.match(r"^(\.LBB\w+):", t)
        if m:
            cur.append(("label", m.group(1), ln))
        elif not t.startswith("."):
            cur.append(("inst", t, ln))
    return fns


def _blocks(items):
    blocks, cur = [], {"labels": [], "insts": [], "succ": None}

    def close():
        nonlocal cur
        if cur["insts"] or cur["labels"]:
            blocks.append(cur)
        cur = {"labels": [], "insts": [], "succ": None}

    for kind, t, ln in items:
        if kind == "label":
            if cur["insts"]:
                close()
            cur["labels"].append(t)
            continue
        cur["insts"].append((t, ln))
        op = t.split()[0]
        if op == "s_branch":
            cur["succ"] = ("jump", t.split()[1])
            close()
        elif op.startswith("s_cbranch"):
            cur["succ"] = ("cond", t.split()[1])
            close()
        elif op in ("s_endpgm", "s_setpc_b64"):
            cur["succ"] = ("end", None)
            close()
    close()
    return blocks


_LOADS = ("buffer_load", "global_load", "flat_load", "scratch_load")
_STORES = ("buffer_store", "global_store", "flat_store", "scratch_store", "global_atomic", "buffer_atomic", "flat_atomic")


def _step(state, t, ln, bad):
    """state: the outstanding vector-memory operations, oldest first, each the set of registers an
    assembly-statement load will still write (empty for everything the compiler tracks itself)"""
    op = t.split()[0]
    if op == "s_waitcnt":
        m = re.search(r"vmcnt\((\d+)\)", t)
        n = None
        if m:
            n = int(m.group(1))
        elif re.match(r"s_waitcnt\s+(0x[0-9a-fA-F]+|\d+)$", t):
            v = int(t.split()[1], 0)
            n = (v & 0xf) | (((v >> 14) & 3) << 4)
        if n is not None and len(state) > n:
            state = state[len(state) - n:] if n else ()
    elif op.startswith(_LOADS):
        dst = _vregs(t.split(",")[0]) if op.startswith("buffer_load") else frozenset()
        src = _vregs(",".join(t.split(",")[1:]))
        if any(p & (src | dst) for p in state):
            bad.add((ln, t))
        state = state + (dst,)
    else:
        r = _vregs(t)
        if any(p & r for p in state):
            bad.add((ln, t))
        if op.startswith(_STORES):
            state = state + (frozenset(),)
    if len(state) > 64:
        state = state[-64:]
    while state and not state[0]:   # operations older than every watched load cannot matter
        state = state[1:]
    return state


def check_function(items, max_states=512):
    """(number of buffer loads, [(line, instruction)] violations, True if the state space was cut short)"""
    blocks = _blocks(items)
    by_label = {l: i for i, b in enumerate(blocks) for l in b["labels"]}
    seen = [set() for _ in blocks]
    bad, work, overflow = set(), [(0, ())], False
    while work:
        i, st = work.pop()
        if st in seen[i]:
            continue
        if len(seen[i]) >= max_states:
            overflow = True
            continue
        seen[i].add(st)
        b = blocks[i]
        for t, ln in b["insts"]:
            st = _step(st, t, ln, bad)
        kind, tgt = b["succ"] if b["succ"] else ("fall", None)
        if kind in ("jump", "cond"):
            work.append((by_label[tgt], st))
        if kind in ("cond", "fall") and i + 1 < len(blocks):
            work.append((i + 1, st))
    n_loads = sum(1 for b in blocks for t, _ in b["insts"] if t.startswith("buffer_load"))
    return n_loads, sorted(bad), overflow


def check_assembly(text, pattern=r"gemm_kernel|conv_dw_halo_kernel|conv_rows_halo_kernel"):
    """Checks every kernel whose symbol matches `pattern`; returns the number of kernels checked and raises
    RuntimeError on the first kernel with a violation (or whose walk could not be completed)."""
    n = 0
    for name, items in parse_functions(text, pattern).items():
        loads, bad, overflow = check_function(items)
        if overflow:
            raise RuntimeError(f"{name}: the walk over outstanding loads did not finish")
        if bad:
            lines = "\n".join(f"    line {ln}: {t}" for ln, t in bad[:8])
            raise RuntimeError(f"{name}: {len(bad)} instruction(s) touch the destination of an assembly-statement load "
                               f"before the wait that covers it:\n{lines}")
        n += 1
    return n
