// Static schedule, timeline simulation and classification search (paper section 4).
//
//  * The feature-map set: every tensor some backward computation reads (section 2.2), the
//    network input excepted (caller data, resident).  Only these are classified (4.1.1).
//  * build_schedule(): one step as an ordered command list with fixed arena offsets.
//    Swap-out follows the last forward use, swap-in precedes the first backward use (3.1);
//    a recompute-class map is dropped after its last forward use and regenerated from its
//    producer's inputs, recursively (3.2).  Swap-ins are issued as early as the arena has
//    room (4.3) or together with the preceding backward computation (the unscheduled variant measured in section 5.1).
//    Because the problem is identical every iteration, allocation order is static: the
//    paper profiles malloc/free order at run time (4.2); here it is decided once, and every
//    cross-stream hazard is an explicit event wait, so a plan that builds can never run out
//    of memory or race, whatever the timings.
//  * simulate(): three serial resources (compute, device-to-host, host-to-device) advanced
//    over that list with profiled durations (4.1.2); also returns L_O / L_I (4.4.2).
//  * Planner: the two-step heuristic search (4.4.2, 4.4.3, equation 1).
#include "core.hpp"

#include <algorithm>
#include <map>
#include <deque>

namespace pooch {

namespace {

int64_t round_up(int64_t n) { return (n + ALIGN - 1) / ALIGN * ALIGN; }

struct BudgetFail {
    const char *why;
};

// Free list over [0, cap).  A free block's tag is the index of the swap-out that must have
// completed before the block may be overwritten (-1: none).  Swap-outs complete in issue
// order, so a stream that has waited for swap-out k may take any block with tag <= k.
struct Arena {
    struct Block {
        int64_t off, size;
        int tag;
    };
    std::vector<Block> B;
    int64_t used = 0, peak = 0, lo = -1, hi = -1;
    explicit Arena(int64_t cap)
    {
        if (cap > 0) B.push_back({0, cap, -1});
    }
    void normalize(int seen)
    {
        for (auto &b : B)
            if (b.tag <= seen) b.tag = -1;
        size_t w = 0;
        for (size_t r = 0; r < B.size(); ++r) {
            if (w > 0 && B[w - 1].off + B[w - 1].size == B[r].off && B[w - 1].tag == B[r].tag) B[w - 1].size += B[r].size;
            else B[w++] = B[r];
        }
        B.resize(w);
    }
    // Among all runs of adjacent free blocks holding `size` bytes take the one whose largest
    // tag is smallest; ties: lowest address (bottom) / highest address (top).
    bool alloc(int64_t size, bool top, int seen, int64_t &off, int &tag_out)
    {
        if (size == 0) {
            off = 0;
            tag_out = -1;
            return true;
        }
        normalize(seen);
        const int nb = (int)B.size();
        int bi = -1, bj = -1, btag = 0;
        if (!top) {
            for (int i = 0; i < nb; ++i) {
                int64_t total = 0;
                int tag = -1, j = i;
                for (;;) {
                    total += B[j].size;
                    tag = std::max(tag, B[j].tag);
                    if (total >= size) break;
                    if (j + 1 < nb && B[j].off + B[j].size == B[j + 1].off) ++j;
                    else {
                        j = -1;
                        break;
                    }
                }
                if (j < 0) continue;
                if (bi < 0 || tag < btag) {
                    bi = i;
                    bj = j;
                    btag = tag;
                }
            }
            if (bi < 0) return false;
            off = B[bi].off;
            const int64_t end = off + size;
            const int64_t rest = B[bj].off + B[bj].size - end;
            const Block tail = {end, rest, B[bj].tag};
            B.erase(B.begin() + bi, B.begin() + bj + 1);
            if (rest > 0) B.insert(B.begin() + bi, tail);
        } else {
            for (int i = nb - 1; i >= 0; --i) {
                int64_t total = 0;
                int tag = -1, j = i;
                for (;;) {
                    total += B[j].size;
                    tag = std::max(tag, B[j].tag);
                    if (total >= size) break;
                    if (j - 1 >= 0 && B[j - 1].off + B[j - 1].size == B[j].off) --j;
                    else {
                        j = -1;
                        break;
                    }
                }
                if (j < 0) continue;
                if (bi < 0 || tag < btag) {
                    bi = i;
                    bj = j;
                    btag = tag;
                }
            }
            if (bi < 0) return false;
            const int64_t end = B[bi].off + B[bi].size;
            off = end - size;
            const int64_t rest = off - B[bj].off;
            const Block head = {B[bj].off, rest, B[bj].tag};
            B.erase(B.begin() + bj, B.begin() + bi + 1);
            if (rest > 0) B.insert(B.begin() + bj, head);
        }
        tag_out = btag;
        used += size;
        peak = std::max(peak, used);
        lo = lo < 0 ? off : std::min(lo, off);
        hi = std::max(hi, off + size);
        return true;
    }
    void release(int64_t off, int64_t size, int tag)
    {
        if (size == 0) return;
        used -= size;
        size_t k = 0;
        while (k < B.size() && B[k].off < off) ++k;
        B.insert(B.begin() + k, Block{off, size, tag});
        if (k + 1 < B.size() && B[k].off + B[k].size == B[k + 1].off && B[k].tag == B[k + 1].tag) {
            B[k].size += B[k + 1].size;
            B.erase(B.begin() + k + 1);
        }
        if (k > 0 && B[k - 1].off + B[k - 1].size == B[k].off && B[k - 1].tag == B[k].tag) {
            B[k - 1].size += B[k].size;
            B.erase(B.begin() + k);
        }
    }
};

struct DryInfo {
    std::vector<int> first_touch, last_touch;  // per tensor, -1 if never touched
    std::vector<int> touch_seq, bwd_steps;
};

constexpr int64_t LOC_NONE = INT64_MIN;
enum { ST_NONE = 0, ST_OUT, ST_FLIGHT, ST_IN };

struct Walker {
    const Graph &G;
    const std::vector<uint8_t> &cls;
    const bool ahead, dry;
    const DryInfo *info;
    Arena arena;
    Schedule &S;
    std::vector<Cmd> &cmds;
    std::vector<char> dead;  // cancelled commands
    std::vector<int64_t> loc, gloc, pinned_off;
    std::vector<int> state, alloc_tag;
    int seen = -1;
    std::deque<int> pending;
    struct Outst {
        int t;
        size_t a, b;
    };
    std::vector<Outst> outstanding;
    bool in_backward = false, blocked = false;
    DryInfo rec;

    Walker(const Graph &g, const std::vector<uint8_t> &c, int64_t cap, bool ahead_, const DryInfo *inf, Schedule &s)
        : G(g), cls(c), ahead(ahead_), dry(inf == nullptr), info(inf), arena(inf ? cap : 0), S(s), cmds(s.cmds)
    {
        const int n = G.n();
        loc.assign(n, LOC_NONE);
        gloc.assign(n, LOC_NONE);
        pinned_off.assign(n, 0);
        state.assign(n, ST_NONE);
        alloc_tag.assign(n, -1);
        S.arrive_event.assign(n, -1);
        rec.first_touch.assign(n, -1);
        rec.last_touch.assign(n, -1);
        loc[0] = OFF_INPUT;
    }

    int klass(int t) const { return G.fidx[t] < 0 ? -1 : (int)cls[G.fidx[t]]; }
    int new_event() { return S.n_events++; }
    void emit(int kind, int id, int64_t a0 = 0, int64_t a1 = 0, int64_t a2 = 0, int64_t a3 = 0, int64_t a4 = 0, int64_t a5 = 0)
    {
        cmds.push_back(Cmd{kind, id, {a0, a1, a2, a3, a4, a5}});
        dead.push_back(0);
    }

    void cancel_last_prefetch()
    {
        const Outst o = outstanding.back();
        outstanding.pop_back();
        for (size_t k = o.a; k < o.b; ++k) dead[k] = 1;
        arena.release(loc[o.t], G.bytes[o.t], alloc_tag[o.t]);
        loc[o.t] = LOC_NONE;
        state[o.t] = ST_OUT;
        pending.push_front(o.t);
        blocked = true;
    }

    int64_t alloc_c(int64_t size, bool top = false)
    {
        if (dry) return 0;
        int64_t off;
        int tag;
        bool ok = arena.alloc(size, top, seen, off, tag);
        while (!ok && in_backward && !outstanding.empty()) {
            cancel_last_prefetch();
            ok = arena.alloc(size, top, seen, off, tag);
        }
        if (!ok) throw BudgetFail{"arena too small"};
        if (tag > seen) {
            emit(K_WAIT, S_COMPUTE, S.d2h_event[tag]);
            seen = tag;
        }
        return off;
    }
    void free_c(int64_t off, int64_t size)
    {
        if (!dry) arena.release(off, size, -1);
    }

    void release_fwd(int t)
    {
        if (t == 0) return;
        const int k = klass(t);
        if (k < 0 || k == CLS_RECOMPUTE) {
            free_c(loc[t], G.bytes[t]);
            loc[t] = LOC_NONE;
        } else if (k == CLS_SWAP) {
            const int ev = new_event();
            emit(K_REC, S_COMPUTE, ev);
            emit(K_WAIT, S_D2H, ev);
            pinned_off[t] = S.swap_bytes;
            S.swap_bytes += G.bytes[t];
            emit(K_OUT, t, loc[t], pinned_off[t]);
            const int done = new_event();
            emit(K_REC, S_D2H, done);
            const int idx = (int)S.d2h_event.size();
            S.d2h_event.push_back(done);
            S.d2h_map.push_back(t);
            if (!dry) arena.release(loc[t], G.bytes[t], idx);
            loc[t] = LOC_NONE;
            state[t] = ST_OUT;
        }
    }

    int d2h_index_of(int t) const
    {
        for (size_t k = 0; k < S.d2h_map.size(); ++k)
            if (S.d2h_map[k] == t) return (int)k;
        return -1;
    }

    bool issue_swapin(int t, bool blocking)
    {
        size_t start = cmds.size();
        int64_t off = 0;
        int tag = -1;
        if (!dry) {
            bool ok = arena.alloc(G.bytes[t], false, seen, off, tag);
            if (!ok && blocking) {
                while (!ok && !outstanding.empty()) {
                    cancel_last_prefetch();
                    ok = arena.alloc(G.bytes[t], false, seen, off, tag);
                }
                if (!ok) throw BudgetFail{"arena too small for a swap-in"};
                start = cmds.size();
            }
            if (!ok) return false;
        }
        loc[t] = off;
        alloc_tag[t] = tag;
        const int ev = new_event();
        emit(K_REC, S_COMPUTE, ev);
        emit(K_WAIT, S_H2D, ev);
        if (tag > seen) emit(K_WAIT, S_H2D, S.d2h_event[tag]);
        emit(K_WAIT, S_H2D, S.d2h_event[d2h_index_of(t)]);
        emit(K_IN, t, off, pinned_off[t]);
        const int arr = new_event();
        emit(K_REC, S_H2D, arr);
        S.arrive_event[t] = arr;
        state[t] = ST_FLIGHT;
        if (!blocking) outstanding.push_back(Outst{t, start, cmds.size()});
        return true;
    }

    void touch(int t, int step)
    {
        if (rec.first_touch[t] < 0) {
            rec.first_touch[t] = step;
            rec.touch_seq.push_back(t);
        }
        rec.last_touch[t] = step;
    }

    static std::vector<int> uniq(const std::vector<int> &v)
    {
        std::vector<int> o;
        for (int x : v)
            if (std::find(o.begin(), o.end(), x) == o.end()) o.push_back(x);
        return o;
    }

    void ensure(int t, int step)
    {
        touch(t, step);
        if (t == 0) return;
        if (loc[t] != LOC_NONE) {
            if (state[t] == ST_FLIGHT) {
                for (size_t k = 0; k < outstanding.size(); ++k)
                    if (outstanding[k].t == t) {
                        outstanding.erase(outstanding.begin() + k);
                        break;
                    }
                emit(K_WAIT, S_COMPUTE, S.arrive_event[t]);
                state[t] = ST_IN;
            }
            return;
        }
        if (klass(t) == CLS_SWAP) {
            auto it = std::find(pending.begin(), pending.end(), t);
            if (it != pending.end()) pending.erase(it);
            issue_swapin(t, true);
            emit(K_WAIT, S_COMPUTE, S.arrive_event[t]);
            state[t] = ST_IN;
            return;
        }
        const std::vector<int> ins = uniq(G.finputs[t]);
        // forward-transient inputs (no feature maps) that this call has to regenerate are dropped again after
        // use; one that is already there belongs to an outer recomputation that still reads it
        std::vector<int> made;
        for (int u : ins)
            if (u != 0 && G.fidx[u] < 0 && loc[u] == LOC_NONE) made.push_back(u);
        for (int u : ins) ensure(u, step);
        loc[t] = alloc_c(G.bytes[t]);
        const std::vector<int> &raw = G.finputs[t];
        emit(K_REFWD, t, loc[t], loc[raw[0]], raw.size() > 1 ? loc[raw[1]] : OFF_NONE);
        S.n_refwd++;
        for (int u : made) {
            free_c(loc[u], G.bytes[u]);
            loc[u] = LOC_NONE;
        }
    }

    void try_prefetch()
    {
        while (!pending.empty() && !blocked) {
            if (issue_swapin(pending.front(), false)) pending.pop_front();
            else break;
        }
    }

    void run()
    {
        const int n = G.n();
        for (int i = 1; i < n; ++i) {
            const std::vector<int> &ins = G.finputs[i];
            if (G.nodes[i].op == OP_DEAD) continue;
            if (G.nodes[i].op == OP_LOSS || G.apply_into[i] >= 0) {
                // no output tensor: the loss, and a BN that is applied inside its consumer (statistics only)
                emit(K_FWD, i, OFF_NONE, loc[ins[0]], OFF_NONE);
            } else {
                const bool top = klass(i) == CLS_KEEP;
                loc[i] = alloc_c(G.bytes[i], top);
                emit(K_FWD, i, loc[i], loc[ins[0]], ins.size() > 1 ? loc[ins[1]] : OFF_NONE);
            }
            for (int t : uniq(ins))
                if (G.last_consumer[t] == i) release_fwd(t);
        }

        in_backward = true;
        // gradient buffer offset -> node that still has to read it while another tensor owns it
        std::map<int64_t, int> shared;
        // Backward of z = a + b hands dy to both inputs.  When one input u is consumed by this add
        // alone, is produced after the other input t and after every other consumer of t, and its
        // own backward never needs to modify dy, then u's backward has read dy before anything is
        // accumulated into t's gradient: both gradients can be the one dy buffer.  Position of u, or -1.
        auto shared_reader = [&](int i) -> int {
            const std::vector<int> &in2 = G.inputs[i];
            if (in2.size() != 2 || in2[0] == in2[1] || in2[0] == 0 || in2[1] == 0) return -1;
            if (gloc[in2[0]] != LOC_NONE || gloc[in2[1]] != LOC_NONE) return -1;
            for (int ju = 0; ju < 2; ++ju) {
                const int u = in2[ju], t = in2[1 - ju];
                if (G.consumers[u].size() != 1 || G.consumers[u][0] != i) continue;
                if (G.nodes[u].op == OP_ADD || G.nodes[u].op == OP_ADDRELU || t > u) continue;
                // u must not read t itself: its backward would add to t's gradient while still reading dy
                if (std::find(G.inputs[u].begin(), G.inputs[u].end(), t) != G.inputs[u].end()) continue;
                bool late = false;
                for (int c : G.consumers[t]) late = late || (c != i && c > u);
                if (late) continue;
                return ju;
            }
            return -1;
        };
        std::vector<std::vector<int>> free_at;
        std::vector<int> next_step;
        if (!dry) {
            for (int t : info->touch_seq)
                if (klass(t) == CLS_SWAP) pending.push_back(t);
            free_at.assign(n, {});
            // ascending tensor id within a step (the order a dictionary built from ascending
            // keys would give is insertion order of last_touch; use touch order of the dry pass)
            for (int t : info->touch_seq)
                if (info->last_touch[t] >= 0) free_at[info->last_touch[t]].push_back(t);
            next_step.assign(n, -1);
            for (size_t k = 0; k + 1 < info->bwd_steps.size(); ++k) next_step[info->bwd_steps[k]] = info->bwd_steps[k + 1];
        }

        for (int i = n - 1; i >= 1; --i) {
            const Op op = G.nodes[i].op;
            if (op != OP_LOSS && gloc[i] == LOC_NONE) continue;
            rec.bwd_steps.push_back(i);
            blocked = false;
            if (!dry && ahead) try_prefetch();
            for (int t : G.needs[i]) ensure(t, i);
            if (!dry && !ahead && next_step[i] >= 0) {
                const int nxt = next_step[i];
                const std::vector<int> snapshot(pending.begin(), pending.end());
                for (int t : snapshot)
                    if (info->first_touch[t] == nxt && !blocked)
                        if (issue_swapin(t, false)) pending.erase(std::find(pending.begin(), pending.end(), t));
            }
            const int64_t need_off = G.needs[i].empty() ? OFF_NONE : loc[G.needs[i][0]];
            const std::vector<int> &ins = G.inputs[i];
            const int64_t dy = op != OP_LOSS ? gloc[i] : OFF_NONE;
            int64_t o[2] = {OFF_NONE, OFF_NONE};
            int m[2] = {M_NONE, M_NONE};
            bool transferred = false;
            const int reader = (op == OP_ADD || op == OP_ADDRELU) ? shared_reader(i) : -1;
            if (op == OP_RELU || op == OP_BN || op == OP_BNRELU) {
                const int x = ins[0];
                if (x == 0) {
                } else if (gloc[x] == LOC_NONE && !shared.count(dy)) {
                    gloc[x] = dy;
                    transferred = true;
                    o[0] = dy;
                    m[0] = M_TRANSFER;
                } else if (gloc[x] == LOC_NONE) {
                    // dy is also another tensor's gradient (see shared_reader): leave it untouched
                    gloc[x] = alloc_c(G.gbytes[x]);
                    o[0] = gloc[x];
                    m[0] = M_WRITE;
                } else {
                    o[0] = gloc[x];
                    m[0] = M_ACC;
                }
            } else if (reader >= 0) {
                // both inputs take the (masked) dy buffer over: one of them only reads it, before
                // anything is accumulated into the other's gradient -- no copy
                shared[dy] = ins[reader];
                for (int j = 0; j < 2; ++j) {
                    gloc[ins[j]] = dy;
                    o[j] = dy;
                    m[j] = M_TRANSFER;
                }
                transferred = true;
            } else if (op == OP_ADD || op == OP_ADDRELU) {
                for (int j = 0; j < 2; ++j) {
                    const int u = ins[j];
                    if (u == 0) continue;
                    if (gloc[u] == LOC_NONE && !transferred) {
                        gloc[u] = dy;
                        transferred = true;
                        o[j] = dy;
                        m[j] = M_TRANSFER;
                    } else if (gloc[u] == LOC_NONE) {
                        gloc[u] = alloc_c(G.gbytes[u]);
                        o[j] = gloc[u];
                        m[j] = M_WRITE;
                    } else {
                        o[j] = gloc[u];
                        m[j] = M_ACC;
                    }
                }
            } else {
                const int x = ins[0];
                if (x == 0) {
                } else if (gloc[x] == LOC_NONE) {
                    gloc[x] = alloc_c(G.gbytes[x]);
                    o[0] = gloc[x];
                    m[0] = M_WRITE;
                } else {
                    o[0] = gloc[x];
                    m[0] = M_ACC;
                }
            }
            emit(K_BWD, i, dy, need_off, o[0], m[0], o[1], m[1]);
            if (op != OP_LOSS) {
                const auto sh = shared.find(dy);
                if (sh != shared.end() && sh->second == i) shared.erase(sh);   // its other owner keeps the buffer
                else if (!transferred) free_c(dy, G.gbytes[i]);
                gloc[i] = LOC_NONE;
            }
            if (!dry)
                for (int t : free_at[i])
                    if (t != 0 && loc[t] != LOC_NONE) {
                        arena.release(loc[t], G.bytes[t], -1);
                        loc[t] = LOC_NONE;
                    }
        }
    }
};

}  // namespace

std::string Graph::analyze()
{
    const int n = this->n();
    if (n < 2) return "graph needs an input and at least one layer";
    if (nodes[0].op != OP_INPUT) return "node 0 must be the input";
    if (nodes[n - 1].op != OP_LOSS) return "the last node must be softmax_ce";
    inputs.assign(n, {});
    bytes.assign(n, 0);
    gbytes.assign(n, 0);
    consumers.assign(n, {});
    finputs.assign(n, {});
    fconsumers.assign(n, {});
    needs.assign(n, {});
    fused_into.assign(n, -1);
    apply_into.assign(n, -1);
    for (int i = 0; i < n; ++i) {
        const Node &nd = nodes[i];
        if (i > 0 && nd.op == OP_INPUT) return "only one input node is supported";
        if (nd.op == OP_LOSS && i != n - 1) return "softmax_ce must be the terminal node";
        if (nd.op == OP_BNRELU || nd.op == OP_ADDRELU || nd.op == OP_DEAD) return "graph was already analysed";
        for (int j = 0; j < nd.nin; ++j) {
            if (nd.in[j] < 0 || nd.in[j] >= i) return "layer input does not precede it";
            if (nodes[nd.in[j]].op == OP_LOSS) return "the loss has no consumers";
        }
    }
    if (fuse) {
        std::vector<std::vector<int>> raw(n);
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < nodes[i].nin; ++j) {
                const int t = nodes[i].in[j];
                if (std::find(raw[t].begin(), raw[t].end(), i) == raw[t].end()) raw[t].push_back(i);
            }
        for (int i = 0; i < n; ++i) {
            if ((nodes[i].op != OP_BN && nodes[i].op != OP_ADD) || raw[i].size() != 1 || nodes[raw[i][0]].op != OP_RELU) continue;
            Node &r = nodes[raw[i][0]];
            Node &b = nodes[i];
            r.op = b.op == OP_BN ? OP_BNRELU : OP_ADDRELU;
            r.nin = b.nin;
            r.in[0] = b.in[0];
            r.in[1] = b.in[1];
            r.eps = b.eps;
            fused_into[i] = raw[i][0];
            b.op = OP_DEAD;
            b.nin = 0;
        }
        for (int a = 0; a < n; ++a) {
            if (nodes[a].op != OP_ADDRELU) continue;
            for (int j = 0; j < nodes[a].nin; ++j) {
                const int b = nodes[a].in[j];
                if (nodes[b].op == OP_BN && raw[b].size() == 1 && fused_into[raw[b][0]] == a) apply_into[b] = a;
            }
        }
    }
    for (int i = 0; i < n; ++i) {
        const Node &nd = nodes[i];
        for (int j = 0; j < nd.nin; ++j) {
            inputs[i].push_back(nd.in[j]);
            finputs[i].push_back(apply_into[nd.in[j]] == i ? nodes[nd.in[j]].in[0] : nd.in[j]);
        }
        bytes[i] = (nd.op == OP_LOSS || nd.op == OP_DEAD || apply_into[i] >= 0) ? 0 : round_up(4 * nd.numel());
        gbytes[i] = (nd.op == OP_LOSS || nd.op == OP_DEAD) ? 0 : round_up(4 * nd.numel());
        for (int t : inputs[i])
            if (std::find(consumers[t].begin(), consumers[t].end(), i) == consumers[t].end()) consumers[t].push_back(i);
        for (int t : finputs[i])
            if (std::find(fconsumers[t].begin(), fconsumers[t].end(), i) == fconsumers[t].end()) fconsumers[t].push_back(i);
        switch (nd.op) {
        case OP_CONV: case OP_BN: case OP_BNRELU: case OP_MAXPOOL: case OP_FC: case OP_LOSS: needs[i] = {inputs[i][0]}; break;
        case OP_RELU: case OP_ADDRELU: needs[i] = {i}; break;
        default: break;
        }
    }
    mask_only.assign(n, 0);
    if (masks) {
        std::vector<char> read_by_other(n, 0);
        for (int i = 0; i < n; ++i)
            for (int t : needs[i])
                if (t != i) read_by_other[t] = 1;
        for (int i = 0; i < n; ++i)
            if ((nodes[i].op == OP_RELU || nodes[i].op == OP_ADDRELU) && !read_by_other[i]) {
                mask_only[i] = 1;
                needs[i].clear();
            }
    }
    last_consumer.assign(n, -1);
    for (int t = 0; t < n; ++t) {
        if (t != n - 1 && consumers[t].empty() && nodes[t].op != OP_DEAD) return "a layer output is never consumed";
        for (int c : fconsumers[t]) last_consumer[t] = std::max(last_consumer[t], c);
    }
    std::vector<char> needed(n, 0);
    for (int i = 0; i < n; ++i)
        for (int t : needs[i]) needed[t] = 1;
    needed[0] = 0;
    fmaps.clear();
    fidx.assign(n, -1);
    for (int t = 0; t < n; ++t)
        if (needed[t]) {
            fidx[t] = (int)fmaps.size();
            fmaps.push_back(t);
        }
    return "";
}

bool build_schedule(const Graph &G, const std::vector<uint8_t> &cls, int64_t cap, bool ahead, int64_t pinned_cap,
                    Schedule &out, std::string *why)
{
    Schedule drys;
    Walker d(G, cls, 0, ahead, nullptr, drys);
    d.run();  // dry pass: who touches what, when (never fails)
    int64_t total_swap = 0;
    for (size_t k = 0; k < G.fmaps.size(); ++k)
        if (cls[k] == CLS_SWAP) total_swap += G.bytes[G.fmaps[k]];
    if (pinned_cap >= 0 && total_swap > pinned_cap) {
        if (why) *why = "pinned buffer too small";
        return false;
    }
    out = Schedule();
    Walker w(G, cls, cap, ahead, &d.rec, out);
    try {
        w.run();
    } catch (const BudgetFail &f) {
        if (why) *why = f.why;
        return false;
    }
    std::vector<Cmd> kept;
    kept.reserve(out.cmds.size());
    for (size_t k = 0; k < out.cmds.size(); ++k)
        if (!w.dead[k]) kept.push_back(out.cmds[k]);
    out.cmds.swap(kept);
    out.peak = w.arena.peak;
    out.extent = w.arena.lo < 0 ? 0 : w.arena.hi - w.arena.lo;
    return true;
}

SimResult simulate(const Graph &G, const Schedule &S, const Profile &P)
{
    double t[3] = {0.0, 0.0, 0.0};
    std::vector<double> ev(S.n_events, 0.0);
    std::vector<int> d2h_index_of_event(S.n_events, -1), arrive_map(S.n_events, -1);
    for (size_t k = 0; k < S.d2h_event.size(); ++k) d2h_index_of_event[S.d2h_event[k]] = (int)k;
    for (size_t m = 0; m < S.arrive_event.size(); ++m)
        if (S.arrive_event[m] >= 0) arrive_map[S.arrive_event[m]] = (int)m;
    const int n = G.n();
    std::vector<double> done_time(n, -1.0);
    std::vector<char> inLO(n, 0), inLI(n, 0);
    double fwd_end = 0.0;
    for (const Cmd &c : S.cmds) {
        switch (c.kind) {
        case K_FWD: t[0] = t[0] + P.t_fwd[c.id]; fwd_end = t[0]; break;
        case K_REFWD: t[0] = t[0] + P.t_refwd[c.id]; break;
        case K_BWD: t[0] = t[0] + P.t_bwd[c.id]; break;
        case K_OUT: t[1] = t[1] + P.t_out[G.fidx[c.id]]; done_time[c.id] = t[1]; break;
        case K_IN: t[2] = t[2] + P.t_in[G.fidx[c.id]]; break;
        case K_REC: ev[c.a[0]] = t[c.id]; break;
        default: {
            const int s = c.id;
            const int e = (int)c.a[0];
            if (ev[e] > t[s]) {
                if (d2h_index_of_event[e] >= 0) {
                    for (int j = 0; j <= d2h_index_of_event[e]; ++j) {
                        const int m = S.d2h_map[j];
                        if (done_time[m] > t[s]) inLO[m] = 1;
                    }
                } else if (arrive_map[e] >= 0 && s == S_COMPUTE) {
                    inLI[arrive_map[e]] = 1;
                }
                t[s] = ev[e];
            }
        }
        }
    }
    for (int m : S.d2h_map)
        if (done_time[m] > fwd_end) inLO[m] = 1;
    SimResult r;
    r.T = std::max(t[0], std::max(t[1], t[2]));
    for (int m = 0; m < n; ++m) {
        if (inLO[m]) r.LO.push_back(m);
        if (inLI[m]) r.LI.push_back(m);
    }
    return r;
}

double Planner::evaluate(const std::vector<uint8_t> &cls, bool ahead, int64_t cap_override)
{
    ++evals;
    Schedule S;
    if (!build_schedule(G, cls, cap_override >= 0 ? cap_override : cap, ahead, pinned_cap, S)) return -1.0;
    return simulate(G, S, P).T;
}

bool Planner::plan(int mode, std::vector<uint8_t> &cls, double &T, bool &ahead)
{
    const size_t nf = G.fmaps.size();
    ahead = true;
    if (mode == MODE_INCORE) {
        cls.assign(nf, CLS_KEEP);
        T = evaluate(cls);
        return T >= 0.0;
    }
    if (mode == MODE_SUPERNEURONS) {
        // the static policy of section 5.2: keep from the output layer backwards while it fits; of the
        // rest convolution outputs swap, all others are recomputed; swap-ins are not moved up
        ahead = false;
        cls.resize(nf);
        for (size_t k = 0; k < nf; ++k) cls[k] = G.nodes[G.fmaps[k]].op == OP_CONV ? CLS_SWAP : CLS_RECOMPUTE;
        T = evaluate(cls, false);
        if (T < 0.0) return false;
        for (int k = (int)nf - 1; k >= 0; --k) {
            std::vector<uint8_t> trial = cls;
            trial[k] = CLS_KEEP;
            const double Tt = evaluate(trial, false);
            if (Tt < 0.0) break;
            cls = trial;
            T = Tt;
        }
        return true;
    }
    const std::vector<uint8_t> allswap(nf, CLS_SWAP);
    if (mode == MODE_SWAPALL_NOSCHED) {
        cls = allswap;
        ahead = false;
        T = evaluate(cls, false);
        return T >= 0.0;
    }
    T = evaluate(allswap);
    if (T < 0.0) return false;
    cls = allswap;
    if (mode == MODE_SWAPALL) return true;
    std::vector<uint8_t> best;
    double best_T;
    step1(allswap, T, best, best_T);
    cls = best;
    T = best_T;
    if (mode == MODE_SWAPOPT) return true;
    step2(cls, T);
    if (mode == MODE_POOCH) return true;
    if (seed && seed->size() == cls.size()) {
        const double Ts = evaluate(*seed);
        if (Ts >= 0.0 && Ts < T) {
            cls = *seed;
            T = Ts;
        }
    }
    refine(cls, T);
    return true;
}

// keep/swap search (section 4.4.2)
void Planner::step1(const std::vector<uint8_t> &allswap, double T_all, std::vector<uint8_t> &best, double &best_T)
{
    Schedule S;
    build_schedule(G, allswap, cap, true, pinned_cap, S);
    const SimResult sr = simulate(G, S, P);
    LO = sr.LO;
    LI = sr.LI;
    // cap on the exponential part: brute-force the max_bits maps of L_I closest to the output,
    // the rest joins the greedy list
    std::vector<int> li = LI, overflow;
    if ((int)li.size() > max_bits) {
        overflow.assign(li.begin(), li.end() - max_bits);
        li.erase(li.begin(), li.end() - max_bits);
    }
    std::vector<int> greedy;
    for (int t : LO)
        if (!std::binary_search(LI.begin(), LI.end(), t)) greedy.push_back(t);
    for (int t : overflow) greedy.push_back(t);
    std::sort(greedy.begin(), greedy.end());
    greedy.erase(std::unique(greedy.begin(), greedy.end()), greedy.end());
    std::reverse(greedy.begin(), greedy.end());  // from the output layer
    best_T = T_all;
    best = allswap;
    for (uint64_t mask = 0; mask < ((uint64_t)1 << li.size()); ++mask) {
        std::vector<uint8_t> cur = allswap;
        for (size_t b = 0; b < li.size(); ++b)
            if ((mask >> b) & 1) cur[G.fidx[li[b]]] = CLS_KEEP;
        if (mask != 0) {
            const double T = evaluate(cur);
            if (T < 0.0) continue;
            if (T < best_T) {
                best_T = T;
                best = cur;
            }
        }
        for (int t : greedy) {
            std::vector<uint8_t> trial = cur;
            trial[G.fidx[t]] = CLS_KEEP;
            const double T = evaluate(trial);
            if (T < 0.0) break;   // section 4.4.2: maps are kept from the output layer while they still fit, so the scan ends at the first that does not
            cur = trial;
            if (T < best_T) {
                best_T = T;
                best = cur;
            }
        }
    }
}

// swap/recompute classification by r(X) = recompute_overhead / swap_overhead (equation 1)
void Planner::step2(std::vector<uint8_t> &cls, double &T0)
{
    const double INF = 1e300;
    std::vector<int> L;
    for (size_t k = 0; k < cls.size(); ++k)
        if (cls[k] == CLS_SWAP) L.push_back((int)k);
    while (!L.empty()) {
        std::vector<double> ratio(cls.size(), INF);
        std::vector<char> fits(cls.size(), 1);
        for (int k : L) {
            std::vector<uint8_t> res = cls;
            res[k] = CLS_KEEP;
            // reference: X resident, in an arena enlarged by X's size -- or by more (2, 4, 8 times, then
            // without limit) when the allocator cannot place that plan in the smallest enlargement
            double T_res = -1.0;
            for (int f = 1; f <= 16 && T_res < 0.0; f *= 2)
                T_res = evaluate(res, true, f <= 8 ? cap + f * G.bytes[G.fmaps[k]] : ((int64_t)1 << 46));
            std::vector<uint8_t> rc = cls;
            rc[k] = CLS_RECOMPUTE;
            const double T_rec = evaluate(rc);
            if (T_res < 0.0 || T_rec < 0.0) {
                // does not fit now; it may once other maps have moved: stays in L, not pickable
                fits[k] = 0;
                continue;
            }
            const double swap_ov = T0 - T_res, rec_ov = T_rec - T_res;
            ratio[k] = swap_ov <= 0.0 ? INF : rec_ov / swap_ov;
        }
        std::vector<int> L2, cand;
        for (int k : L)
            if (!fits[k] || ratio[k] < 1.0) L2.push_back(k);
        L.swap(L2);
        for (int k : L)
            if (fits[k]) cand.push_back(k);
        if (cand.empty()) break;
        int kmin = cand[0];
        for (int k : cand)
            if (ratio[k] < ratio[kmin]) kmin = k;
        cls[kmin] = CLS_RECOMPUTE;
        L.erase(std::find(L.begin(), L.end(), kmin));
        T0 = evaluate(cls);
    }
}

// best strictly-improving single class change per round, first in (map, class) order; until none helps
void Planner::descend(std::vector<uint8_t> &cls, double &T0)
{
    for (;;) {
        double best_T = T0;
        int best_k = -1, best_v = 0;
        for (size_t k = 0; k < cls.size(); ++k)
            for (int v = CLS_KEEP; v <= CLS_RECOMPUTE; ++v) {
                if (v == cls[k]) continue;
                std::vector<uint8_t> trial = cls;
                trial[k] = (uint8_t)v;
                const double T = evaluate(trial);
                if (T < 0.0) continue;
                if (T < best_T) {
                    best_T = T;
                    best_k = (int)k;
                    best_v = v;
                }
            }
        if (best_k < 0) return;
        T0 = best_T;
        cls[best_k] = (uint8_t)best_v;
    }
}

namespace {
uint64_t splitmix64(uint64_t &state)
{
    state += 0x9E3779B97F4A7C15ull;
    uint64_t z = state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
}  // namespace

// Not in the paper: iterated local search on top of the two steps, judged by the same simulation.
// Descend from the two-step plan; then `restarts` times give 6 drawn maps a drawn class each
// (splitmix64, fixed seed), descend again if that plan fits, keep it if strictly faster.
void Planner::refine(std::vector<uint8_t> &cls, double &T0)
{
    descend(cls, T0);
    uint64_t state = 1907050130ull;
    const uint64_t nf = cls.size();
    for (int r = 0; r < restarts; ++r) {
        std::vector<uint8_t> trial = cls;
        for (int j = 0; j < 6; ++j) {
            const uint64_t a = splitmix64(state);
            const uint64_t b = splitmix64(state);
            trial[a % nf] = (uint8_t)(b % 3);
        }
        double T = evaluate(trial);
        if (T < 0.0) continue;
        descend(trial, T);
        if (T < T0) {
            cls = trial;
            T0 = T;
        }
    }
}

}  // namespace pooch
