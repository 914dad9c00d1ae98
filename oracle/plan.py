"""Plan oracle: the paper's classification method written out step by step in plain Python.

TEST INFRASTRUCTURE ONLY (slow, obvious, no sharing with the HIP library).  It covers

  * the feature-map set and its sizes (section 2.2: feature maps must be preserved until
    backward consumes them; section 4.1.1: only feature maps are classified),
  * the static schedule of one step under a classification: swap-out after the last forward
    use, swap-in before the first backward use (section 3.1), discard and recursive
    recomputation (section 3.2), swap-ins moved up as far as memory has room (section 4.3)
    or started together with the preceding backward computation (section 5.1, the variant
    without scheduling), all inside a fixed-size arena with a first-fit allocator,
  * the timeline simulation over three serial resources -- compute, device-to-host,
    host-to-device -- from profiled durations (section 4.1.2),
  * the two-step heuristic search (section 4.4): L_O / L_I extraction on the all-swap
    timeline, binary tree over L_I with a greedy scan of L_O \\ L_I from the output layer,
    then r(X) = recompute_overhead / swap_overhead (equation 1) for the maps left in swap,
  * mode "superneurons": the static policy of section 5.2 (keep from the output end, then
    convolution outputs swap, the rest is recomputed; swap-ins not moved up),
  * mode "refine" (not in the paper): the two steps followed by an iterated local search over
    single class changes, judged by the same simulation.

Where the paper is silent, the reading taken is stated at the function that needs it.
"""
from collections import deque

KEEP, SWAP, RECOMPUTE = 0, 1, 2
ALIGN = 256

# command kinds
KF, KR, KB, KO, KI, KREC, KWAIT = 0, 1, 2, 3, 4, 5, 6
S_COMPUTE, S_D2H, S_H2D = 0, 1, 2
# gradient-output modes of a backward command
M_NONE, M_WRITE, M_ACC, M_TRANSFER = 0, 1, 2, 3
OFF_INPUT = -2  # the network input lives in the resident region
OFF_NONE = -1


class Budget(Exception):
    """the classification does not fit the arena (or the pinned buffer)"""


def _round(n):
    return (n + ALIGN - 1) // ALIGN * ALIGN


# ------------------------------------------------------------------ graph analysis

class Graph:
    """static facts about a layer list (see workloads.py for the format).

    fuse=True applies the executor's layer fusion: a BN or add whose only consumer is a ReLU
    is executed inside that ReLU ("bnrelu", "addrelu"); the BN / add output is then never
    materialised (op "dead", zero bytes, no commands).  The feature-map set does not change:
    backward of a bnrelu reads the BN's input (the ReLU decision is re-derived from it),
    backward of an addrelu reads the ReLU's output.
    One more step: a BN whose only consumer is the add of such an addrelu is applied inside the
    addrelu's forward kernel (apply_into[bn] = addrelu; either input or both).  The BN node stays:
    its forward is the statistics alone and writes no tensor (zero bytes), its backward is unchanged
    and still receives the gradient along the edge from the addrelu.  Hence two edge sets:
    `inputs` / `consumers` carry gradients, `finputs` / `fconsumers` say what a forward kernel reads
    (the addrelu reads the BN's input in place of the BN's output) and decide how long tensors live."""

    def __init__(self, net, fuse=False, masks=False):
        self.net = net
        n = len(net)
        self.n = n
        self.ops = [L["op"] for L in net]
        self.inputs = []
        for L in net:
            if L["op"] == "input":
                self.inputs.append([])
            elif L["op"] == "add":
                if L["a"] == L["b"]:
                    raise ValueError("add takes two different tensors")
                self.inputs.append([L["a"], L["b"]])
            else:
                self.inputs.append([L["x"]])
        self.shape = self._shapes()
        self.fused_into = [-1] * n
        if fuse:
            raw = [[] for _ in range(n)]
            for i in range(n):
                for t in self.inputs[i]:
                    if i not in raw[t]:
                        raw[t].append(i)
            for i in range(n):
                if self.ops[i] in ("bn", "add") and len(raw[i]) == 1 and self.ops[raw[i][0]] == "relu":
                    j = raw[i][0]
                    self.ops[j] = "bnrelu" if self.ops[i] == "bn" else "addrelu"
                    self.inputs[j] = list(self.inputs[i])
                    self.ops[i] = "dead"
                    self.inputs[i] = []
                    self.fused_into[i] = j
        self.apply_into = [-1] * n
        if fuse:
            for a in range(n):
                if self.ops[a] != "addrelu":
                    continue
                for b in self.inputs[a]:
                    if self.ops[b] == "bn" and len(raw[b]) == 1 and self.fused_into[raw[b][0]] == a:
                        self.apply_into[b] = a
        self.finputs = []
        for i in range(n):
            self.finputs.append([self.inputs[t][0] if self.apply_into[t] == i else t for t in self.inputs[i]])
        self.bytes = []
        self.gbytes = []
        for i in range(n):
            numel = 1
            for v in self.shape[i]:
                numel *= v
            self.bytes.append(0 if self.ops[i] in ("softmax_ce", "dead") or self.apply_into[i] >= 0 else _round(4 * numel))
            # its gradient: a full tensor also where the output itself is never written (apply_into)
            self.gbytes.append(0 if self.ops[i] in ("softmax_ce", "dead") else _round(4 * numel))
        self.consumers = [[] for _ in range(n)]
        self.fconsumers = [[] for _ in range(n)]
        for i in range(n):
            for t in self.inputs[i]:
                if i not in self.consumers[t]:
                    self.consumers[t].append(i)
            for t in self.finputs[i]:
                if i not in self.fconsumers[t]:
                    self.fconsumers[t].append(i)
        self.last_consumer = [max(c) if c else -1 for c in self.fconsumers]
        # tensors the backward of node i reads
        self.needs = []
        for i, op in enumerate(self.ops):
            if op in ("conv", "bn", "bnrelu", "maxpool", "fc", "softmax_ce"):
                self.needs.append([self.inputs[i][0]])
            elif op in ("relu", "addrelu"):
                self.needs.append([i])
            else:
                self.needs.append([])
        # masks=True: a relu / addrelu whose output no other layer's backward reads keeps one bit per element for its own
        # backward instead of the output, which then is no feature map
        self.mask_only = [False] * n
        if masks:
            read_by_other = set(t for i in range(n) for t in self.needs[i] if t != i)
            for i, op in enumerate(self.ops):
                if op in ("relu", "addrelu") and i not in read_by_other:
                    self.mask_only[i] = True
                    self.needs[i] = []
        needed = set()
        for i in range(n):
            needed.update(self.needs[i])
        needed.discard(0)
        self.fmaps = sorted(needed)                      # tensor id of every feature map
        self.fidx = {t: k for k, t in enumerate(self.fmaps)}

    def _shapes(self):
        out = []
        for L in self.net:
            op = L["op"]
            if op == "input":
                s = tuple(L["shape"])
            elif op in ("conv", "maxpool"):
                i = out[L["x"]]
                sp = tuple((i[2 + d] + 2 * L["pad"][d] - L["k"][d]) // L["stride"][d] + 1 for d in range(len(L["k"])))
                s = (i[0], L["cout"] if op == "conv" else i[1]) + sp
            elif op in ("bn", "relu"):
                s = out[L["x"]]
            elif op == "add":
                s = out[L["a"]]
            elif op == "gavgpool":
                s = out[L["x"]][:2]
            elif op == "fc":
                s = (out[L["x"]][0], L["nout"])
            else:
                s = ()
            out.append(s)
        return out

    def fmap_bytes(self):
        return [self.bytes[t] for t in self.fmaps]


# ------------------------------------------------------------------ arena allocator

class Arena:
    """Free list over [0, cap).  A free block carries a tag: the index of the swap-out
    (device-to-host copy) that must have completed before the block may be overwritten,
    or -1.  Copies complete in issue order, so a stream that has waited for swap-out k
    may use every block with tag <= k."""

    def __init__(self, cap):
        self.cap = cap
        self.blocks = [[0, cap, -1]] if cap > 0 else []
        self.used = 0
        self.peak = 0
        self.lo = None
        self.hi = None

    def _normalize(self, seen):
        for b in self.blocks:
            if b[2] <= seen:
                b[2] = -1
        out = []
        for b in self.blocks:
            if out and out[-1][0] + out[-1][1] == b[0] and out[-1][2] == b[2]:
                out[-1][1] += b[1]
            else:
                out.append(b)
        self.blocks = out

    def alloc(self, size, top, seen):
        """returns (offset, tag) or None.  Among all runs of adjacent free blocks that hold
        `size` bytes, take the one whose largest tag is smallest; ties go to the lowest
        address (bottom) or the highest address (top)."""
        if size == 0:
            return (0, -1)
        self._normalize(seen)
        B = self.blocks
        best = None
        if not top:
            for i in range(len(B)):
                total, tag, j = 0, -1, i
                while True:
                    total += B[j][1]
                    tag = max(tag, B[j][2])
                    if total >= size:
                        break
                    if j + 1 < len(B) and B[j][0] + B[j][1] == B[j + 1][0]:
                        j += 1
                    else:
                        j = -1
                        break
                if j < 0:
                    continue
                if best is None or tag < best[0]:
                    best = (tag, i, j)
            if best is None:
                return None
            tag, i, j = best
            off = B[i][0]
            end = off + size
            rest = B[j][0] + B[j][1] - end
            repl = [[end, rest, B[j][2]]] if rest > 0 else []
            self.blocks = B[:i] + repl + B[j + 1:]
        else:
            for i in range(len(B) - 1, -1, -1):
                total, tag, j = 0, -1, i
                while True:
                    total += B[j][1]
                    tag = max(tag, B[j][2])
                    if total >= size:
                        break
                    if j - 1 >= 0 and B[j - 1][0] + B[j - 1][1] == B[j][0]:
                        j -= 1
                    else:
                        j = -1
                        break
                if j < 0:
                    continue
                if best is None or tag < best[0]:
                    best = (tag, i, j)
            if best is None:
                return None
            tag, i, j = best
            end = B[i][0] + B[i][1]
            off = end - size
            rest = off - B[j][0]
            repl = [[B[j][0], rest, B[j][2]]] if rest > 0 else []
            self.blocks = B[:j] + repl + B[i + 1:]
        self.used += size
        self.peak = max(self.peak, self.used)
        self.lo = off if self.lo is None else min(self.lo, off)
        self.hi = off + size if self.hi is None else max(self.hi, off + size)
        return (off, tag)

    def free(self, off, size, tag):
        if size == 0:
            return
        self.used -= size
        B = self.blocks
        k = 0
        while k < len(B) and B[k][0] < off:
            k += 1
        B.insert(k, [off, size, tag])
        if k + 1 < len(B) and B[k][0] + B[k][1] == B[k + 1][0] and B[k][2] == B[k + 1][2]:
            B[k][1] += B[k + 1][1]
            del B[k + 1]
        if k > 0 and B[k - 1][0] + B[k - 1][1] == B[k][0] and B[k - 1][2] == B[k][2]:
            B[k - 1][1] += B[k][1]
            del B[k]


# ------------------------------------------------------------------ static schedule

class Schedule:
    def __init__(self):
        self.cmds = []          # tuples, first element is the kind
        self.peak = 0
        self.extent = 0
        self.swap_bytes = 0
        self.n_events = 0
        self.d2h_event = []     # completion event of swap-out k
        self.d2h_map = []       # tensor id of swap-out k
        self.arrive_event = {}  # tensor id -> event recorded after its swap-in
        self.n_refwd = 0


def _uniq(seq):
    out = []
    for v in seq:
        if v not in out:
            out.append(v)
    return out


def build_schedule(G, cls, cap, ahead=True, pinned_cap=None):
    """cls: class per feature map (index into G.fmaps).  Returns a Schedule or raises Budget."""
    info = _walk(G, cls, None, ahead, None)              # dry pass: who touches what, when
    total_swap = sum(G.bytes[t] for t in G.fmaps if cls[G.fidx[t]] == SWAP)
    if pinned_cap is not None and total_swap > pinned_cap:
        raise Budget("pinned buffer too small")
    return _walk(G, cls, cap, ahead, info)


def _walk(G, cls, cap, ahead, info):
    dry = info is None
    n = G.n
    arena = None if dry else Arena(cap)
    S = Schedule()
    cmds = S.cmds
    klass = {t: cls[G.fidx[t]] for t in G.fmaps}
    loc = [None] * n
    gloc = [None] * n
    loc[0] = OFF_INPUT
    state = {}            # swap maps: "out" (on host), "flight" (swap-in issued), "in"
    seen = [-1]           # highest swap-out index the compute stream has waited for
    pinned_off = {}
    alloc_tag = {}        # tensor -> tag returned when its current buffer was carved (for cancel)
    pending = deque()     # swap maps awaiting swap-in, in order of first backward touch
    outstanding = []      # prefetched, not yet consumed: (tensor, first cmd index, last cmd index)
    in_backward = [False]
    blocked = [False]
    first_touch, last_touch, touch_seq, bwd_steps = {}, {}, [], []

    def new_event():
        S.n_events += 1
        return S.n_events - 1

    def emit(*c):
        cmds.append(c)

    def cancel_last_prefetch():
        t, a, b = outstanding.pop()
        for k in range(a, b):
            cmds[k] = None
        arena.free(loc[t], G.bytes[t], alloc_tag[t])
        loc[t] = None
        state[t] = "out"
        pending.appendleft(t)
        blocked[0] = True

    def alloc_c(size, top=False):
        if dry:
            return 0
        r = arena.alloc(size, top, seen[0])
        while r is None and in_backward[0] and outstanding:
            cancel_last_prefetch()
            r = arena.alloc(size, top, seen[0])
        if r is None:
            raise Budget("arena too small")
        off, tag = r
        if tag > seen[0]:
            emit(KWAIT, S_COMPUTE, S.d2h_event[tag])
            seen[0] = tag
        return off

    def free_c(off, size):
        if not dry:
            arena.free(off, size, -1)

    def release_fwd(t):
        if t == 0:
            return
        if t not in klass:
            free_c(loc[t], G.bytes[t])
            loc[t] = None
        elif klass[t] == SWAP:
            ev = new_event()
            emit(KREC, S_COMPUTE, ev)
            emit(KWAIT, S_D2H, ev)
            pinned_off[t] = S.swap_bytes
            S.swap_bytes += G.bytes[t]
            emit(KO, t, loc[t], pinned_off[t])
            done = new_event()
            emit(KREC, S_D2H, done)
            k = len(S.d2h_event)
            S.d2h_event.append(done)
            S.d2h_map.append(t)
            if not dry:
                arena.free(loc[t], G.bytes[t], k)
            loc[t] = None
            state[t] = "out"
        elif klass[t] == RECOMPUTE:
            free_c(loc[t], G.bytes[t])
            loc[t] = None

    def issue_swapin(t, blocking):
        start = len(cmds)
        if dry:
            off, tag = 0, -1
        else:
            r = arena.alloc(G.bytes[t], False, seen[0])
            if r is None and blocking:
                while r is None and outstanding:
                    cancel_last_prefetch()
                    r = arena.alloc(G.bytes[t], False, seen[0])
                if r is None:
                    raise Budget("arena too small for a swap-in")
                start = len(cmds)
            if r is None:
                return False
            off, tag = r
        loc[t] = off
        alloc_tag[t] = tag
        ev = new_event()
        emit(KREC, S_COMPUTE, ev)
        emit(KWAIT, S_H2D, ev)
        if tag > seen[0]:
            emit(KWAIT, S_H2D, S.d2h_event[tag])
        emit(KWAIT, S_H2D, S.d2h_event[S.d2h_map.index(t)])
        emit(KI, t, off, pinned_off[t])
        arr = new_event()
        emit(KREC, S_H2D, arr)
        S.arrive_event[t] = arr
        state[t] = "flight"
        if not blocking:
            outstanding.append((t, start, len(cmds)))
        return True

    def touch(t, step):
        if t not in first_touch:
            first_touch[t] = step
            touch_seq.append(t)
        last_touch[t] = step

    def ensure(t, step):
        touch(t, step)
        if t == 0:
            return
        if loc[t] is not None:
            if state.get(t) == "flight":
                for k, o in enumerate(outstanding):
                    if o[0] == t:
                        del outstanding[k]
                        break
                emit(KWAIT, S_COMPUTE, S.arrive_event[t])
                state[t] = "in"
            return
        if t in klass and klass[t] == SWAP:
            if t in pending:
                pending.remove(t)
            issue_swapin(t, True)
            emit(KWAIT, S_COMPUTE, S.arrive_event[t])
            state[t] = "in"
            return
        ins = _uniq(G.finputs[t])
        # forward-transient inputs (no feature maps) that this call has to regenerate are dropped again after
        # use; one that is already there belongs to an outer recomputation that still reads it
        made = [u for u in ins if u != 0 and u not in klass and loc[u] is None]
        for u in ins:
            ensure(u, step)
        loc[t] = alloc_c(G.bytes[t])
        raw = G.finputs[t]
        emit(KR, t, loc[t], loc[raw[0]], loc[raw[1]] if len(raw) > 1 else OFF_NONE)
        S.n_refwd += 1
        for u in made:
            free_c(loc[u], G.bytes[u])
            loc[u] = None

    # ---------------- forward
    for i in range(1, n):
        ins = G.finputs[i]
        if G.ops[i] == "dead":
            continue
        if G.ops[i] == "softmax_ce" or G.apply_into[i] >= 0:
            # no output tensor: the loss, and a BN that is applied inside its consumer (statistics only)
            emit(KF, i, OFF_NONE, loc[ins[0]], OFF_NONE)
        else:
            top = i in klass and klass[i] == KEEP
            loc[i] = alloc_c(G.bytes[i], top)
            emit(KF, i, loc[i], loc[ins[0]], loc[ins[1]] if len(ins) > 1 else OFF_NONE)
        for t in _uniq(ins):
            if G.last_consumer[t] == i:
                release_fwd(t)

    # ---------------- backward
    in_backward[0] = True
    shared = {}     # gradient buffer offset -> node that still has to read it while another tensor owns it
    if not dry:
        for t in info["touch_seq"]:
            if t in klass and klass[t] == SWAP:
                pending.append(t)
        free_at = {}
        for t, s in info["last_touch"].items():
            free_at.setdefault(s, []).append(t)
        steps = info["bwd_steps"]
        next_step = {steps[k]: steps[k + 1] for k in range(len(steps) - 1)}

    def try_prefetch():
        while pending and not blocked[0]:
            if issue_swapin(pending[0], False):
                pending.popleft()
            else:
                break

    for i in range(n - 1, 0, -1):
        op = G.ops[i]
        if op != "softmax_ce" and gloc[i] is None:
            continue
        bwd_steps.append(i)
        blocked[0] = False
        if not dry and ahead:
            try_prefetch()
        for t in G.needs[i]:
            ensure(t, i)
        if not dry and not ahead and i in next_step:
            nxt = next_step[i]
            for t in list(pending):
                if info["first_touch"][t] == nxt and not blocked[0]:
                    if issue_swapin(t, False):
                        pending.remove(t)
        need_off = loc[G.needs[i][0]] if G.needs[i] else OFF_NONE
        ins = G.inputs[i]
        dy = gloc[i] if op != "softmax_ce" else OFF_NONE
        outs = []
        transferred = False
        if op in ("relu", "bn", "bnrelu"):
            x = ins[0]
            if x == 0:
                outs.append((OFF_NONE, M_NONE))
            elif gloc[x] is None and dy not in shared:
                gloc[x] = dy
                transferred = True
                outs.append((dy, M_TRANSFER))
            elif gloc[x] is None:
                # dy is also another tensor's gradient (see _shared_reader): leave it untouched
                gloc[x] = alloc_c(G.gbytes[x])
                outs.append((gloc[x], M_WRITE))
            else:
                outs.append((gloc[x], M_ACC))
        elif op in ("add", "addrelu") and _shared_reader(G, i, gloc) is not None:
            # both inputs take the (masked) dy buffer over: one of them only reads it, before anything
            # is accumulated into the other's gradient -- no copy
            shared[dy] = ins[_shared_reader(G, i, gloc)]
            for u in ins:
                gloc[u] = dy
                outs.append((dy, M_TRANSFER))
            transferred = True
        elif op in ("add", "addrelu"):
            for u in ins:
                if u == 0:
                    outs.append((OFF_NONE, M_NONE))
                elif gloc[u] is None and not transferred:
                    gloc[u] = dy
                    transferred = True
                    outs.append((dy, M_TRANSFER))
                elif gloc[u] is None:
                    gloc[u] = alloc_c(G.gbytes[u])
                    outs.append((gloc[u], M_WRITE))
                else:
                    outs.append((gloc[u], M_ACC))
        else:
            x = ins[0]
            if x == 0:
                outs.append((OFF_NONE, M_NONE))
            elif gloc[x] is None:
                gloc[x] = alloc_c(G.gbytes[x])
                outs.append((gloc[x], M_WRITE))
            else:
                outs.append((gloc[x], M_ACC))
        while len(outs) < 2:
            outs.append((OFF_NONE, M_NONE))
        emit(KB, i, dy, need_off, outs[0][0], outs[0][1], outs[1][0], outs[1][1])
        if op != "softmax_ce":
            if shared.get(dy) == i:
                del shared[dy]          # its other owner keeps the buffer
            elif not transferred:
                free_c(dy, G.gbytes[i])
            gloc[i] = None
        if not dry:
            for t in free_at.get(i, []):
                if t != 0 and loc[t] is not None:
                    arena.free(loc[t], G.bytes[t], -1)
                    loc[t] = None

    if dry:
        return {"first_touch": first_touch, "last_touch": last_touch, "touch_seq": touch_seq, "bwd_steps": bwd_steps}
    S.cmds = [c for c in cmds if c is not None]
    S.peak = arena.peak
    S.extent = 0 if arena.lo is None else arena.hi - arena.lo
    return S


def _shared_reader(G, i, gloc):
    """Backward of z = a + b hands dy to both inputs.  When one input u is consumed by this add alone,
    is produced after the other input t and after every other consumer of t, does not read t itself
    (its backward would add to t's gradient while still reading dy), and its own backward never needs
    to modify dy, then u's backward has read dy before anything is accumulated into t's gradient:
    both gradients can be the one dy buffer.  Returns the position of u in the inputs, or None."""
    ins = G.inputs[i]
    if len(ins) != 2 or ins[0] == ins[1] or 0 in ins or gloc[ins[0]] is not None or gloc[ins[1]] is not None:
        return None
    for ju in (0, 1):
        u, t = ins[ju], ins[1 - ju]
        if G.consumers[u] != [i] or G.ops[u] in ("add", "addrelu") or t > u or t in G.inputs[u]:
            continue
        if any(c != i and c > u for c in G.consumers[t]):
            continue
        return ju
    return None


# ------------------------------------------------------------------ timeline simulation

class Profile:
    """durations in ms: per node forward / backward / re-forward, per feature map out / in"""

    def __init__(self, t_fwd, t_bwd, t_refwd, t_out, t_in):
        self.t_fwd, self.t_bwd, self.t_refwd, self.t_out, self.t_in = t_fwd, t_bwd, t_refwd, t_out, t_in


def simulate(G, S, P):
    """three serial resources; a command starts when its stream is free and every event it
    waited for has been recorded.  Returns (step time, L_O, L_I) with L_O / L_I as sets of
    tensor ids: maps whose swap-out / swap-in was not hidden by computation."""
    t = [0.0, 0.0, 0.0]
    ev = {}
    d2h_index_of_event = {e: k for k, e in enumerate(S.d2h_event)}
    arrive_map = {e: m for m, e in S.arrive_event.items()}
    done_time = {}
    fwd_end = 0.0
    LO, LI = set(), set()
    for c in S.cmds:
        k = c[0]
        if k == KF:
            t[0] = t[0] + P.t_fwd[c[1]]
            fwd_end = t[0]
        elif k == KR:
            t[0] = t[0] + P.t_refwd[c[1]]
        elif k == KB:
            t[0] = t[0] + P.t_bwd[c[1]]
        elif k == KO:
            t[1] = t[1] + P.t_out[G.fidx[c[1]]]
            done_time[c[1]] = t[1]
        elif k == KI:
            t[2] = t[2] + P.t_in[G.fidx[c[1]]]
        elif k == KREC:
            ev[c[2]] = t[c[1]]
        else:
            s, e = c[1], c[2]
            if ev[e] > t[s]:
                if e in d2h_index_of_event:
                    for j in range(d2h_index_of_event[e] + 1):
                        m = S.d2h_map[j]
                        if done_time[m] > t[s]:
                            LO.add(m)
                elif e in arrive_map and s == S_COMPUTE:
                    LI.add(arrive_map[e])
                t[s] = ev[e]
    for m, d in done_time.items():
        if d > fwd_end:
            LO.add(m)
    return max(t), LO, LI


# ------------------------------------------------------------------ classification search

def _splitmix64(state):
    """one step of the splitmix64 generator: (new state, 64-bit output)"""
    m = (1 << 64) - 1
    state = (state + 0x9E3779B97F4A7C15) & m
    z = state
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return state, z ^ (z >> 31)


class Planner:
    def __init__(self, G, P, cap, pinned_cap=None, max_bits=10, restarts=8, seed=None):
        self.G, self.P, self.cap, self.pinned_cap, self.max_bits = G, P, cap, pinned_cap, max_bits
        self.restarts = restarts
        # refine mode only (not in the paper): a classification made earlier, e.g. from a coarser
        # profile, that competes with the two-step plan as the starting point of the local search
        self.seed = seed
        self.evals = 0
        self.LO, self.LI = set(), set()

    def evaluate(self, cls, ahead=True, cap=None):
        """simulated step time of a classification, or None if it does not fit"""
        self.evals += 1
        try:
            S = build_schedule(self.G, cls, self.cap if cap is None else cap, ahead, self.pinned_cap)
        except Budget:
            return None
        return simulate(self.G, S, self.P)[0]

    def plan(self, mode):
        G = self.G
        nf = len(G.fmaps)
        if mode == "incore":
            cls = [KEEP] * nf
            T = self.evaluate(cls)
            if T is None:
                raise Budget("in-core does not fit")
            return cls, T
        if mode == "superneurons":
            return self.superneurons()
        allswap = [SWAP] * nf
        if mode == "swapall_nosched":
            T = self.evaluate(allswap, ahead=False)
            if T is None:
                raise Budget("all-swap does not fit")
            return allswap, T
        T = self.evaluate(allswap)
        if T is None:
            raise Budget("all-swap does not fit")
        if mode == "swapall":
            return allswap, T
        cls, T = self.step1(allswap, T)
        if mode == "swapopt":
            return cls, T
        cls, T = self.step2(cls, T)
        if mode == "pooch":
            return cls, T
        if self.seed is not None and len(self.seed) == nf:
            Ts = self.evaluate(list(self.seed))
            if Ts is not None and Ts < T:
                cls, T = list(self.seed), Ts
        return self.refine(cls, T)

    def superneurons(self):
        """the static policy the paper compares against (section 5.2): keep maps from the output
        layer backwards while they fit; of the rest, convolution outputs swap and all others
        are recomputed; each swap-in starts with the preceding backward computation"""
        G = self.G
        cls = [SWAP if G.ops[t] == "conv" else RECOMPUTE for t in G.fmaps]
        T = self.evaluate(cls, ahead=False)
        if T is None:
            raise Budget("the static policy does not fit")
        for k in range(len(cls) - 1, -1, -1):
            trial = list(cls)
            trial[k] = KEEP
            Tt = self.evaluate(trial, ahead=False)
            if Tt is None:
                break
            cls, T = trial, Tt
        return cls, T

    def step1(self, allswap, T_all):
        """keep/swap search (section 4.4.2)"""
        G = self.G
        S = build_schedule(G, allswap, self.cap, True, self.pinned_cap)
        _, LO, LI = simulate(G, S, self.P)
        self.LO, self.LI = set(LO), set(LI)
        # cap on the exponential part: brute-force the max_bits maps of L_I with the largest
        # tensor ids (closest to the output); the rest joins the greedy list
        li = sorted(LI)
        if len(li) > self.max_bits:
            overflow, li = li[:len(li) - self.max_bits], li[len(li) - self.max_bits:]
        else:
            overflow = []
        greedy = sorted((LO - LI) | set(overflow), reverse=True)     # from the output layer
        best_T, best = T_all, list(allswap)
        for mask in range(1 << len(li)):
            cur = list(allswap)
            for b, t in enumerate(li):
                if (mask >> b) & 1:
                    cur[G.fidx[t]] = KEEP
            if mask != 0:
                T = self.evaluate(cur)
                if T is None:
                    continue
                if T < best_T:
                    best_T, best = T, list(cur)
            for t in greedy:
                trial = list(cur)
                trial[G.fidx[t]] = KEEP
                T = self.evaluate(trial)
                if T is None:
                    break       # section 4.4.2: kept from the output layer while they still fit; the scan ends at the first map that does not
                cur = trial
                if T < best_T:
                    best_T, best = T, list(cur)
        return best, best_T

    def step2(self, cls, T0):
        """swap/recompute classification by r(X) (section 4.4.3, equation 1)"""
        G = self.G
        cls = list(cls)
        L = [k for k in range(len(cls)) if cls[k] == SWAP]
        while L:
            ratios = {}
            for k in L:
                res = list(cls)
                res[k] = KEEP
                # reference: X resident in an arena enlarged by X's size -- or by 2, 4, 8 times that,
                # then without limit, when the allocator cannot place the plan in the smallest one
                T_res = None
                for f in (1, 2, 4, 8, None):
                    T_res = self.evaluate(res, cap=(self.cap + f * G.bytes[G.fmaps[k]]) if f else (1 << 46))
                    if T_res is not None:
                        break
                rec = list(cls)
                rec[k] = RECOMPUTE
                T_rec = self.evaluate(rec)
                if T_res is None or T_rec is None:
                    # the flip does not fit now; it may once other maps have moved: X stays in L
                    # but cannot be picked in this round
                    ratios[k] = None
                    continue
                swap_ov = T0 - T_res
                rec_ov = T_rec - T_res
                ratios[k] = float("inf") if swap_ov <= 0.0 else rec_ov / swap_ov
            L = [k for k in L if ratios[k] is None or ratios[k] < 1.0]
            cand = [k for k in L if ratios[k] is not None]
            if not cand:
                break
            kmin = cand[0]
            for k in cand:
                if ratios[k] < ratios[kmin]:
                    kmin = k
            cls[kmin] = RECOMPUTE
            L.remove(kmin)
            T0 = self.evaluate(cls)
        return cls, T0

    def _descend(self, cls, T0):
        """each round evaluates every single-map change of class and applies the one with the
        smallest simulated step time (first in (map, class) order on ties) if it is strictly
        faster; stops when no change helps"""
        cls = list(cls)
        while True:
            best = None
            for k in range(len(cls)):
                for v in (KEEP, SWAP, RECOMPUTE):
                    if v == cls[k]:
                        continue
                    trial = list(cls)
                    trial[k] = v
                    T = self.evaluate(trial)
                    if T is None:
                        continue
                    if T < (T0 if best is None else best[0]):
                        best = (T, k, v)
            if best is None:
                return cls, T0
            T0, k, v = best
            cls[k] = v

    def refine(self, cls, T0):
        """Not in the paper: an iterated local search on top of its two steps, with the same
        simulator and the same three classes.  Descend from the two-step plan; then `restarts`
        times: give 6 maps drawn by splitmix64 (seed 1907050130) a drawn class each, descend
        again if that plan fits, and keep the result if it is strictly faster than the best."""
        best, best_T = self._descend(cls, T0)
        state = 1907050130
        nf = len(best)
        for _ in range(self.restarts):
            trial = list(best)
            for _ in range(6):
                state, a = _splitmix64(state)
                state, b = _splitmix64(state)
                trial[a % nf] = b % 3
            T = self.evaluate(trial)
            if T is None:
                continue
            trial, T = self._descend(trial, T)
            if T < best_T:
                best, best_T = trial, T
        return best, best_T
