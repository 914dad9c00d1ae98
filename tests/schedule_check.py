"""Independent validator for a step's command list (the oracle's or the HIP library's).

It knows nothing about how the schedule was built.  It checks that
  * every access stays inside the arena,
  * any two accesses to overlapping bytes, one of them a write, are ordered by the
    stream/event structure (happens-before via vector clocks), whatever the timings,
  * replayed in emission order, every read finds the tensor it expects at that offset.
"""
KF, KR, KB, KO, KI, KREC, KWAIT = range(7)
M_NONE, M_WRITE, M_ACC, M_TRANSFER = range(4)
OFF_INPUT, OFF_NONE = -2, -1


def _accesses(G, c):
    """[(offset, size, is_write, label)] of one command; label = ('v'|'g', tensor)"""
    k = c[0]
    acc = []
    relabel = []
    if k in (KF, KR):
        i = c[1]
        ins = G.finputs[i]
        offs = [c[3], c[4]]
        for j, t in enumerate(ins):
            if offs[j] >= 0:
                acc.append((offs[j], G.bytes[t], False, ("v", t)))
        if c[2] >= 0 and G.bytes[i] > 0:
            acc.append((c[2], G.bytes[i], True, ("v", i)))
    elif k == KO:
        acc.append((c[2], G.bytes[c[1]], False, ("v", c[1])))
    elif k == KI:
        acc.append((c[2], G.bytes[c[1]], True, ("v", c[1])))
    elif k == KB:
        i, dy, need = c[1], c[2], c[3]
        op = G.ops[i]
        if op != "softmax_ce":
            acc.append((dy, G.gbytes[i], False, ("g", i)))
        if G.needs[i] and need >= 0:
            acc.append((need, G.bytes[G.needs[i][0]], False, ("v", G.needs[i][0])))
        outs = [(c[4], c[5]), (c[6], c[7])]
        for j, t in enumerate(G.inputs[i]):
            off, mode = outs[j]
            if mode == M_NONE:
                continue
            # only element-wise backward passes may produce their result in the buffer they read dy from
            assert off != dy or op in ("relu", "bn", "bnrelu", "add", "addrelu"), ("backward writes into its own dy", c)
            if mode == M_WRITE:
                acc.append((off, G.gbytes[t], True, ("g", t)))
            elif mode == M_ACC:
                acc.append((off, G.gbytes[t], False, ("g", t)))
                acc.append((off, G.gbytes[t], True, ("g", t)))
            elif mode == M_TRANSFER:
                assert off == dy
                if op == "add":
                    relabel.append((off, ("g", t)))
                elif op == "addrelu":
                    # masked in place: a read-modify-write of the dy buffer, which changes owner
                    acc.append((off, G.gbytes[t], True, ("g", t)))
                else:
                    acc.append((off, G.gbytes[t], True, ("g", t)))
    return acc, relabel


def check(G, cmds, cap):
    nstream = 3
    pos = [0, 0, 0]
    clock = [[0, 0, 0] for _ in range(nstream)]   # vector clock of each stream
    ev_clock = {}
    recs = []   # (stream, position, clock-at-start, accesses)
    for c in cmds:
        k = c[0]
        if k == KREC:
            ev_clock[c[2]] = list(clock[c[1]])
            continue
        if k == KWAIT:
            assert c[2] in ev_clock, "wait on an event that was never recorded before it"
            clock[c[1]] = [max(a, b) for a, b in zip(clock[c[1]], ev_clock[c[2]])]
            continue
        s = {KF: 0, KR: 0, KB: 0, KO: 1, KI: 2}[k]
        pos[s] += 1
        clock[s][s] = pos[s]
        acc, relabel = _accesses(G, c)
        for off, size, _, _ in acc:
            assert 0 <= off and off + size <= cap, ("access outside the arena", c)
            assert off % 256 == 0
        recs.append((s, pos[s], list(clock[s]), acc, relabel, c))

    # happens-before between conflicting accesses: sweep by address
    items = []
    for r, (s, p, vc, acc, _, c) in enumerate(recs):
        for off, size, w, _ in acc:
            if size > 0:
                items.append((off, off + size, w, r))
    items.sort()
    active = []
    for a0, a1, aw, ar in items:
        active = [x for x in active if x[1] > a0]
        for b0, b1, bw, br in active:
            if br == ar or not (aw or bw):
                continue
            sa, pa, vca = recs[ar][0], recs[ar][1], recs[ar][2]
            sb, pb, vcb = recs[br][0], recs[br][1], recs[br][2]
            a_before_b = vcb[sa] >= pa
            b_before_a = vca[sb] >= pb
            assert a_before_b or b_before_a, ("unordered conflicting accesses", recs[ar][5], recs[br][5])
        active.append((a0, a1, aw, ar))

    # contents, replayed in emission order.  A range may hold several tensors at once: the backward of
    # an add can hand its dy buffer to both inputs (one of them only ever reads it).
    live = {}   # offset -> (size, set of labels)
    for s, p, vc, acc, relabel, c in recs:
        for off, size, w, label in acc:
            if size == 0:
                continue
            if not w:
                assert off in live and live[off][0] == size and label in live[off][1], ("read finds wrong contents", c, off, live.get(off))
        written = {}
        for off, size, w, label in acc:
            if w and size > 0:
                written.setdefault((off, size), set()).add(label)
        for (off, size), labels in written.items():
            for o in [o for o, (sz, _) in live.items() if o < off + size and off < o + sz]:
                del live[o]
            live[off] = (size, labels)
        renamed = {}
        for off, label in relabel:
            renamed.setdefault(off, set()).add(label)
        for off, labels in renamed.items():
            live[off] = (live[off][0], labels)
    return len(recs)
