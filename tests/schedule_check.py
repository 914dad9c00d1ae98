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


# --------------------------------------------------------------------------------------------------------------
# Timeline of a command list, written independently of the oracle's and the library's simulators.
#
# Every executed command becomes an interval [start, end).  A command starts when the command before it on its
# stream has ended and every event its stream waited for since then has fired; an event fires when the stream that
# recorded it had finished everything issued before the record (its last command's end, and the events it had
# itself waited for by then).  From the intervals, by their definitions (paper section 4.4.2):
#   step time  = the latest end;
#   L_I        = maps whose arrival the compute stream really waited for: at the wait, the arrival event fires
#                later than everything else the compute stream was waiting for up to that point;
#   L_O        = maps whose swap-out is not hidden by computation: it ends after the last forward command has
#                ended, or some stream, ready to go on, had to sit out a device-to-host completion event while
#                that swap-out (issued no later than the awaited one) was still running.

class Interval:
    __slots__ = ("cmd", "stream", "start", "end")

    def __init__(self, cmd, stream, start, end):
        self.cmd, self.stream, self.start, self.end = cmd, stream, start, end


def timeline(G, cmds, t_fwd, t_bwd, t_refwd, t_out, t_in):
    """returns (intervals of the executed commands in list order, step time, L_O, L_I); L_O / L_I as sets of tensor ids"""
    stream_of = {KF: 0, KR: 0, KB: 0, KO: 1, KI: 2}
    ready = [0.0, 0.0, 0.0]          # per stream: when it could start its next command
    fires = {}                       # event -> time
    d2h_done_event = {}              # event recorded right after a swap-out -> position of that swap-out in issue order
    arrive_event = {}                # event recorded right after a swap-in -> tensor
    outs = []                        # swap-out intervals in issue order
    ivs = []
    LO, LI = set(), set()
    prev_kind = [None, None, None]   # last executed command per stream: (kind, tensor / node)
    for c in cmds:
        k = c[0]
        if k == KREC:
            s, e = c[1], c[2]
            fires[e] = ready[s]
            if prev_kind[s] is not None and prev_kind[s][0] == KO and s == 1:
                d2h_done_event.setdefault(e, prev_kind[s][2])
            if prev_kind[s] is not None and prev_kind[s][0] == KI and s == 2:
                arrive_event.setdefault(e, prev_kind[s][1])
            prev_kind[s] = None          # a later record on this stream marks no copy
            continue
        if k == KWAIT:
            s, e = c[1], c[2]
            assert e in fires, "wait on an event that has not been recorded"
            if fires[e] > ready[s]:
                if e in d2h_done_event:
                    for iv in outs[:d2h_done_event[e] + 1]:
                        if iv.end > ready[s]:
                            LO.add(iv.cmd[1])
                elif e in arrive_event and s == 0:
                    LI.add(arrive_event[e])
                ready[s] = fires[e]
            continue
        s = stream_of[k]
        dur = {KF: t_fwd, KR: t_refwd, KB: t_bwd}[k][c[1]] if k in (KF, KR, KB) else (t_out if k == KO else t_in)[G.fidx[c[1]]]
        iv = Interval(c, s, ready[s], ready[s] + dur)
        ready[s] = iv.end
        ivs.append(iv)
        if k == KO:
            outs.append(iv)
            prev_kind[s] = (KO, c[1], len(outs) - 1)
        else:
            prev_kind[s] = (k, c[1], None)
    fwd_end = max([iv.end for iv in ivs if iv.cmd[0] == KF], default=0.0)
    for iv in outs:
        if iv.end > fwd_end:
            LO.add(iv.cmd[1])
    T = max([iv.end for iv in ivs], default=0.0)
    return ivs, T, LO, LI
