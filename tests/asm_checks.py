"""Checks on the compiler's assembly output of the kernels (used by tests/test_host_abi.py; not collected by pytest)."""

import re


def readlanes_of_loads_under_narrowed_exec(asm_path, kernel_re=r"^(_ZN5dadam[A-Za-z0-9_]*k_direct[A-Za-z0-9_]*):"):
    """Follows the exec-mask nesting of every matching kernel along its control flow (basic blocks, branch
    targets and fall-through; s_and_saveexec pushes the register pair the mask is saved in, restoring exec
    from a pair pops back to where it was pushed; where paths meet, the deeper nesting is kept).  Returns
    (checked, bad): the number of v_readlane sites whose source register holds (directly or through register
    copies) what a global_load_dword loaded, and the kernels in which such a load ran under a narrowed mask."""
    lines = open(asm_path).read().split("\n")
    checked, bad = 0, []
    i = 0
    while i < len(lines):
        m = re.match(kernel_re, lines[i])
        if not m:
            i += 1
            continue
        name = m.group(1)
        j = i + 1
        body = []
        while j < len(lines) and not lines[j].startswith(".Lfunc_end"):      # not s_endpgm: there may be several exits
            body.append(lines[j]); j += 1
        # split into blocks
        blocks, order, cur = {}, [], "__entry"
        blocks[cur] = []; order.append(cur)
        for l in body:
            ml = re.match(r"^(\.LBB\d+_\d+):", l)
            if ml:
                cur = ml.group(1); blocks[cur] = []; order.append(cur)
                continue
            t = l.strip()
            if t and not t.startswith(";") and not t.startswith("."):
                blocks[cur].append(t)
        nxt = {b: (order[k + 1] if k + 1 < len(order) else None) for k, b in enumerate(order)}
        state_in = {"__entry": ((), ())}     # (stack of saved pairs, tuple of (reg, depth) of loads) - loads tracked separately
        load_depth = {}                      # per block processing we recompute
        work = ["__entry"]
        seen_state = {}
        results = []
        while work:
            b = work.pop()
            stack, loads = state_in[b]
            stack = list(stack); loads = dict(loads)
            succ = []
            fall = True
            snapshot = lambda: (tuple(stack), tuple(sorted(loads.items())))
            for t in blocks[b]:
                m1 = re.match(r"s_and_saveexec_b64 (s\[\d+:\d+\])", t)
                m0 = re.match(r"s_(or|andn2)_saveexec_b64 (s\[\d+:\d+\]), (s\[\d+:\d+\])", t)
                m2 = re.match(r"s_or_b64 exec, exec, (s\[\d+:\d+\])", t)
                m3 = re.match(r"s_cbranch_\w+ (\.LBB\d+_\d+)", t)
                m4 = re.match(r"s_branch (\.LBB\d+_\d+)", t)
                m5 = re.match(r"global_load_dword (v\d+),", t)
                m6 = re.match(r"v_readlane_b32 s\d+, (v\d+),", t)
                m7 = re.match(r"v_mov_b32_e32 (v\d+), (v\d+)$", t)
                m8 = re.match(r"\w+ (v\d+|v\[(\d+):(\d+)\])[, ]", t)       # any other write to vector registers
                if m1: stack.append(m1.group(1))
                elif m0:
                    # the switch from the then-side to the else-side of a divergent branch: the lanes saved in the
                    # second pair come back (or take over), the mask at this point is saved in the first pair
                    if m0.group(3) in stack: del stack[stack.index(m0.group(3)):]
                    stack.append(m0.group(2))
                elif m2:
                    if m2.group(1) in stack: del stack[stack.index(m2.group(1)):]
                elif m3: succ.append((m3.group(1), snapshot()))        # the state at the branch, not at the block's end
                elif m4: succ.append((m4.group(1), snapshot())); fall = False
                elif m5: loads[m5.group(1)] = len(stack)
                elif m6:
                    if m6.group(1) in loads:
                        results.append((b, m6.group(1), loads[m6.group(1)]))
                elif m7:                                     # a copy carries the source's history along
                    if m7.group(2) in loads: loads[m7.group(1)] = loads[m7.group(2)]
                    else: loads.pop(m7.group(1), None)
                elif m8 and not t.startswith(("global_store", "buffer_store", "ds_write", "v_cmp", "v_readfirstlane")):
                    regs = [m8.group(1)] if m8.group(2) is None else [f"v{k}" for k in range(int(m8.group(2)), int(m8.group(3)) + 1)]
                    for r in regs: loads.pop(r, None)
            if fall and nxt[b]: succ.append((nxt[b], snapshot()))
            for s_, out in succ:
                if s_ not in blocks: continue
                if s_ not in state_in:
                    state_in[s_] = out; work.append(s_)
                else:
                    # merge: keep the deeper nesting per load (pessimistic), shorter stack
                    old_stack, old_loads = state_in[s_]
                    ol = dict(old_loads); changed = False
                    for r, d in out[1]:
                        if ol.get(r, -1) < d: ol[r] = d; changed = True
                    new_stack = old_stack if len(old_stack) <= len(out[0]) else out[0]
                    if new_stack != old_stack: changed = True
                    if changed:
                        state_in[s_] = (new_stack, tuple(sorted(ol.items()))); work.append(s_)
        seen = set()
        for b, r, d in results:
            key = (b, r)
            if key in seen: continue
            seen.add(key); checked += 1
            if d > 0: bad.append(name)
        i = j
    return checked, bad


def streaming_hints(asm_path):
    """Per kernel of the library: (wide stores with the non-temporal hint, wide stores without, wide loads
    with, wide loads without), wide = 8 or 16 bytes per lane, keyed by mangled kernel name."""
    out, name = {}, None
    for l in open(asm_path):
        m = re.match(r"^(_ZN5dadam\w+):", l)
        if m:
            name = m.group(1)
            out[name] = [0, 0, 0, 0]
            continue
        if name is None:
            continue
        t = l.split(";")[0].strip()
        if re.match(r"global_store_dwordx[24]\b", t):
            out[name][0 if " nt" in t else 1] += 1
        elif re.match(r"global_load_dwordx[24]\b", t):
            out[name][2 if " nt" in t else 3] += 1
        elif l.startswith(".Lfunc_end"):          # not s_endpgm: a kernel may have several exits
            name = None
    return out
