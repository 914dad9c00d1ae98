"""The library's planner (C++) against the plan oracle (oracle/plan.py), on the CPU.

Integer work must agree exactly: feature-map set, command lists (kinds, ids, arena and
pinned offsets, events), peak bytes, L_O / L_I, the classification every mode picks, the
number of simulations.  Simulated times are sums of the same doubles in the same order, so
they agree to the last bit as well.  The library's command lists also go through the
independent schedule validator."""
import json
import os

import numpy as np
import pytest

import schedule_check
import workloads
from oracle import plan as P
from paper_1907_05013_amd import binding as B

BIG = 1 << 44
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def nets():
    return {
        "tiny": workloads.tiny_cnn(),
        "res": workloads.resnet50(batch=2, size=32, nclasses=5, blocks=(2, 1), width=4),
        "c3d": workloads.cnn3d(size=8, channels=(2, 3, 4), nclasses=2, batch=2),
        "bott": workloads.bottleneck_stage(batch=2, ch=16, size=8, blocks=2),
        "fork": workloads.late_fork(),
    }


def lib_ctx(net, dyn_cap, fuse=True, masks=False):
    probe = B.Context(net, 1 << 40, device=None, fuse=fuse, masks=masks)
    res = probe.resident_bytes()
    return B.Context(net, res + dyn_cap, device=None, fuse=fuse, masks=masks), res


def rand_profile(G, rng, link=1.0):
    nf = len(G.fmaps)
    tf = rng.uniform(0.2, 3.0, G.n)
    return [tf, rng.uniform(0.2, 5.0, G.n), tf * rng.uniform(0.3, 1.0, G.n),
            rng.uniform(0.1, 4.0, nf) * link, rng.uniform(0.1, 4.0, nf) * link]


def as_rows(S):
    rows = []
    for c in S.cmds:
        r = list(c) + [0] * (8 - len(c))
        rows.append(r)
    return np.array(rows, np.int64).reshape(-1, 8)


@pytest.mark.parametrize("fuse", [False, True])
@pytest.mark.parametrize("name", ["tiny", "res", "c3d", "bott", "fork"])
def test_feature_maps_and_command_lists_identical(name, fuse):
    net = nets()[name]
    G = P.Graph(net, fuse=fuse)
    nf = len(G.fmaps)
    incore = P.build_schedule(G, [P.KEEP] * nf, BIG)
    c, _ = lib_ctx(net, BIG, fuse)
    assert [(G.bytes[t], t) for t in G.fmaps] == c.fmaps()
    assert [c.node_fused(i) for i in range(G.n)] == [
        f if f >= 0 else a for f, a in zip(G.fused_into, G.apply_into)]
    assert any(v >= 0 for v in G.fused_into) == fuse
    rng = np.random.default_rng(21)
    prof = rand_profile(G, rng)
    oprof = P.Profile(*[list(v) for v in prof])
    ncmp = 0
    for trial in range(40):
        cls = [int(v) for v in rng.integers(0, 3, nf)] if trial else [P.KEEP] * nf
        cap = BIG if trial == 0 else int(incore.peak * rng.uniform(0.35, 1.2)) // 256 * 256
        c, _ = lib_ctx(net, cap, fuse)
        c.set_profile(*prof)
        for ahead in (True, False):
            try:
                S = P.build_schedule(G, cls, cap, ahead)
            except P.Budget:
                with pytest.raises(B.BudgetError):
                    c.set_plan(cls, ahead)
                continue
            c.set_plan(cls, ahead)
            rows = c.commands()
            assert np.array_equal(rows, as_rows(S))
            st = c.stats()
            assert (st.peak_bytes, st.extent_bytes, st.n_refwd) == (S.peak, S.extent, S.n_refwd)
            T, peak = c.simulate(cls, ahead)
            assert T == P.simulate(G, S, oprof)[0] and peak == S.peak
            schedule_check.check(G, [tuple(int(v) for v in r) for r in rows], cap)
            ncmp += 1
    assert ncmp > 20


def test_budget_of_an_odd_number_of_bytes_counts_in_whole_units():
    """ranges carved from the top of the dynamic region sit at (capacity - size): with a budget that is no multiple of
    256 they would be misaligned; the library uses the whole 256-byte units of the budget and plans as the oracle
    does for that many"""
    net = workloads.tiny_cnn()
    G = P.Graph(net, fuse=True)
    incore = P.build_schedule(G, [P.KEEP] * len(G.fmaps), BIG, True)
    cap = int(incore.peak * 0.7) // 256 * 256
    res = B.Context(net, 1 << 40, device=None).resident_bytes()
    c = B.Context(net, res + cap + 131, device=None)
    c.set_profile(*rand_profile(G, np.random.default_rng(5)))
    rng = np.random.default_rng(11)
    done = 0
    for trial in range(30):
        cls = [int(v) for v in rng.integers(0, 3, len(G.fmaps))]
        try:
            S = P.build_schedule(G, cls, cap, True)
        except P.Budget:
            continue
        c.set_plan(cls, True)
        rows = c.commands()
        assert np.array_equal(rows, as_rows(S))
        schedule_check.check(G, [tuple(int(v) for v in r) for r in rows], cap)      # (asserts 256-byte offsets)
        done += 1
    assert done >= 5
    assert c.stats().arena_bytes == res + cap


@pytest.mark.parametrize("seed", range(6))
def test_every_mode_picks_the_oracles_plan(seed):
    rng = np.random.default_rng(100 + seed)
    net = list(nets().values())[seed % 4]
    fuse = seed % 2 == 0
    G = P.Graph(net, fuse=fuse)
    nf = len(G.fmaps)
    incore = P.build_schedule(G, [P.KEEP] * nf, BIG)
    cap = int(incore.peak * rng.uniform(0.45, 0.95)) // 256 * 256
    prof = rand_profile(G, rng, link=float(rng.choice([0.2, 1.0, 4.0])))
    oprof = P.Profile(*[list(v) for v in prof])
    c, _ = lib_ctx(net, cap, fuse)
    c.set_profile(*prof)
    bits = 5
    for mode in ("swapall_nosched", "swapall", "swapopt", "pooch", "refine", "superneurons"):
        pl = P.Planner(G, oprof, cap, max_bits=bits, restarts=3)
        try:
            ocls, oT = pl.plan(mode)
        except P.Budget:
            with pytest.raises(B.BudgetError):
                c.plan(mode, bits, restarts=3)
            continue
        cls, T = c.plan(mode, bits, restarts=3)
        assert list(cls) == list(ocls)
        assert T == oT
        assert c.plan_evaluations() == pl.evals
        if mode == "swapopt":
            lo, li = c.overhead_sets()
            assert {G.fmaps[k] for k in range(nf) if lo[k]} == pl.LO
            assert {G.fmaps[k] for k in range(nf) if li[k]} == pl.LI


@pytest.mark.parametrize("seed", range(4))
def test_refine_after_a_profile_change_starts_from_the_installed_plan_too(seed):
    """plan under one profile, replace the profile, plan again in refine mode: the library tries the
    installed plan as a starting point exactly as the oracle does when given it as `seed`"""
    rng = np.random.default_rng(500 + seed)
    net = list(nets().values())[seed % 4]
    G = P.Graph(net, fuse=True)
    nf = len(G.fmaps)
    incore = P.build_schedule(G, [P.KEEP] * nf, BIG)
    prof1 = rand_profile(G, rng, link=1.0)
    prof2 = [np.asarray(v) * rng.uniform(0.5, 1.5, size=len(v)) for v in prof1]
    for frac in (rng.uniform(0.5, 0.8), 0.9, 0.97):       # the smallest of these arenas that all-swap fits
        cap = int(incore.peak * frac) // 256 * 256
        c, _ = lib_ctx(net, cap, True)
        c.set_profile(*prof1)
        try:
            cls1, _ = c.plan("refine", 4, restarts=2)
            break
        except B.BudgetError:
            continue
    else:
        pytest.fail("no arena below the in-core peak admits the all-swap plan")
    c.set_profile(*prof2)
    cls2, T2 = c.plan("refine", 4, restarts=2)
    pl = P.Planner(G, P.Profile(*[list(v) for v in prof2]), cap, max_bits=4, restarts=2, seed=list(cls1))
    ocls, oT = pl.plan("refine")
    assert list(cls2) == list(ocls) and T2 == oT and c.plan_evaluations() == pl.evals
    # and without a profile change in between there is no seed: same as a fresh planner
    cls3, T3 = c.plan("refine", 4, restarts=2)
    pl0 = P.Planner(G, P.Profile(*[list(v) for v in prof2]), cap, max_bits=4, restarts=2)
    ocls0, oT0 = pl0.plan("refine")
    assert list(cls3) == list(ocls0) and T3 == oT0 and c.plan_evaluations() == pl0.evals


def test_paper_eight_layer_example_through_the_library():
    """section 4.4.2's worked example: L_O = {5,6,7}, L_I = {4,6,7} on the all-swap timeline"""
    with open(os.path.join(GOLD, "eight_layer_example.json")) as f:
        gold = json.load(f)
    net = workloads.Net()
    t = net.input((4, 8, 16, 16))
    for _ in range(8):
        t = net.relu(t)
    net.softmax_ce(net.gavgpool(t))
    c, _ = lib_ctx(net, BIG)
    assert c.n_fmaps == 9
    t_fwd = [0.0] + gold["t_fwd"] + [0.0, 0.0]
    t_bwd = [0.0] + gold["t_bwd"] + [0.0, 0.0]
    c.set_profile(t_fwd, t_bwd, t_fwd, gold["t_out"] + [0.0], gold["t_in"] + [0.0])
    lo, li = c.overhead_sets()
    assert [k for k in range(8) if lo[k]] == gold["L_O"]
    assert [k for k in range(8) if li[k]] == gold["L_I"]
    cls, T = c.plan("swapopt", 16)
    assert list(cls[:4]) == [B.SWAP] * 4                       # hidden both ways: swap at once
    n_li = int(li.sum())                                       # the pooled vector may join the sets
    n_g = int((lo & ~li & 1).sum())
    assert c.plan_evaluations() <= 2 + (1 << n_li) * (1 + n_g)  # 2^|L_I| leaves x |L_O \ L_I| greedy


def _relu_chain(n, shape=(4, 8, 16, 16)):
    net = workloads.Net()
    t = net.input(shape)
    for _ in range(n):
        t = net.relu(t)
    net.softmax_ce(net.gavgpool(t))
    return net


def test_library_simulator_against_independent_timeline():
    """the library's simulated step time and L_O / L_I (through the C ABI) against the timeline schedule_check builds
    from the library's own command list by the definitions -- no oracle code between the two"""
    rng = np.random.default_rng(77)
    n = 0
    for name, net in nets().items():
        G = P.Graph(net, fuse=True)          # static facts only (sizes, which map a command names)
        nf = len(G.fmaps)
        probe, _ = lib_ctx(net, BIG)
        _, peak = probe.simulate([B.KEEP] * nf, want_time=False)
        for trial in range(25):
            cls = [int(v) for v in rng.integers(0, 3, nf)] if trial % 3 else [B.SWAP] * nf
            cap = int(peak * rng.uniform(0.4, 1.2)) // 256 * 256
            prof = rand_profile(G, rng, link=float(rng.choice([0.2, 1.0, 4.0])))
            c, _ = lib_ctx(net, cap)
            c.set_profile(*prof)
            for ahead in (True, False):
                try:
                    c.set_plan(cls, ahead)
                except B.BudgetError:
                    continue
                rows = [tuple(int(v) for v in r) for r in c.commands()]
                _, T, LO, LI = schedule_check.timeline(G, rows, *prof)
                assert abs(c.simulate(cls, ahead)[0] - T) <= 1e-9 * max(T, 1.0)
                if ahead and all(v == B.SWAP for v in cls):
                    lo, li = c.overhead_sets()
                    assert {G.fmaps[k] for k in range(nf) if lo[k]} == LO
                    assert {G.fmaps[k] for k in range(nf) if li[k]} == LI
                n += 1
    assert n >= 40


def test_hand_computed_timelines_through_the_library():
    """the two timelines worked out by hand in tests/test_oracle_plan.py, through the C ABI: one swapped map feeding a
    recomputation chain two deep (step times 27 / 29 / 30), and the two overheads of section 4.4.3's ratio in the exact tie"""
    net = _relu_chain(4)
    c, _ = lib_ctx(net, BIG)
    assert [p for _, p in c.fmaps()] == [1, 2, 3, 4, 5]
    cls = [B.SWAP, B.RECOMPUTE, B.RECOMPUTE, B.KEEP, B.KEEP]
    for t_out, t_in, T_want in ((5.0, 4.0, 27.0), (5.0, 7.0, 29.0), (7.0, 7.0, 30.0)):
        c.set_profile([0.0] + [2.0] * 4 + [1.0, 1.0], [0.0] + [3.0] * 4 + [1.0, 1.0], [0.0] + [1.5] * 4 + [1.0, 1.0],
                      [t_out] * 4 + [0.0], [t_in] * 4 + [0.0])
        assert c.simulate(cls)[0] == T_want
    c.set_plan(cls)
    rows = c.commands()
    assert [(int(r[0]), int(r[1])) for r in rows if r[0] <= 4] == [
        (0, 1), (0, 2), (3, 1), (0, 3), (0, 4), (0, 5), (0, 6), (4, 1), (2, 6), (2, 5), (2, 4), (1, 2), (1, 3), (2, 3), (2, 2), (2, 1)]
    # the two overheads of the tie, exactly (what step 2 does with them is compared with the oracle's step 2, which
    # has the tie test, by test_every_mode_picks_the_oracles_plan)
    net = _relu_chain(3)
    for t_re in (1.5, 1.5 - 2.0 ** -20, 1.5 + 2.0 ** -20):
        c, _ = lib_ctx(net, BIG)
        c.set_profile([0.0] + [1.0] * 3 + [1.0, 1.0], [0.0] + [2.0] * 3 + [1.0, 1.0], [0.0, 1.0, t_re, 1.0, 1.0, 1.0],
                      [0.25] * 3 + [0.0], [5.5] * 3 + [0.0])
        keep = c.simulate([B.KEEP] * 4)[0]
        assert c.simulate([B.KEEP, B.SWAP, B.KEEP, B.KEEP])[0] - keep == 1.5
        assert c.simulate([B.KEEP, B.RECOMPUTE, B.KEEP, B.KEEP])[0] - keep == t_re


def test_one_bit_relu_masks_shrink_the_feature_map_set_alike():
    """one-bit ReLU masks (off by default): a relu / add + relu whose output no other layer's backward reads keeps a mask and
    its output stops being a feature map -- the same nodes in oracle and library, the same command lists under random plans,
    valid by the independent checker; the configured networks lose exactly the ReLU in front of the global pool"""
    expect = {"tiny": 0, "res": 1, "bott": 1, "fork": None}      # tiny: that ReLU is fused into a BN + ReLU, which reads the BN's input
    ncmp = 0
    cases = [(k, nets()[k]) for k in ("tiny", "res", "bott", "fork")] + [("rand%d" % s, workloads.random_net(s, residual=s >= 80)) for s in (3, 15, 61, 85, 97, 110)]
    for name, net in cases:
        rng = np.random.default_rng(77)
        for fuse in (True, False):
            G0 = P.Graph(net, fuse=fuse)
            G = P.Graph(net, fuse=fuse, masks=True)
            kept = [i for i in range(G.n) if G.mask_only[i]]
            assert len(G.fmaps) == len(G0.fmaps) - len([i for i in kept if i in G0.fmaps])
            assert all(G.ops[i] in ("relu", "addrelu") and i not in G.fmaps for i in kept)
            if fuse and expect.get(name) is not None:
                assert len(kept) == expect[name], (name, kept)
            nf = len(G.fmaps)
            incore = P.build_schedule(G, [P.KEEP] * nf, BIG)
            c, _ = lib_ctx(net, BIG, fuse, masks=True)
            assert [(G.bytes[t], t) for t in G.fmaps] == c.fmaps()
            assert [c.node_keeps_mask(i) for i in range(G.n)] == [bool(v) for v in G.mask_only]
            c0, _ = lib_ctx(net, BIG, fuse)
            assert not any(c0.node_keeps_mask(i) for i in range(G.n))
            # the masks live in the resident region: one bit per element, in 256-byte units
            extra = sum((int(np.prod(G.shape[i])) + 31) // 32 * 4 for i in kept)
            assert 0 <= c.resident_bytes() - c0.resident_bytes() - extra < 256 * max(len(kept), 1)
            for trial in range(6):
                cls = [int(v) for v in rng.integers(0, 3, nf)] if trial else [P.KEEP] * nf
                cap = BIG if trial == 0 else int(incore.peak * rng.uniform(0.45, 1.2)) // 256 * 256
                c, _ = lib_ctx(net, cap, fuse, masks=True)
                for ahead in (True, False):
                    try:
                        S = P.build_schedule(G, cls, cap, ahead)
                    except P.Budget:
                        with pytest.raises(B.BudgetError):
                            c.set_plan(cls, ahead)
                        continue
                    c.set_plan(cls, ahead)
                    rows = c.commands()
                    assert np.array_equal(rows, as_rows(S)), (name, fuse, trial, ahead)
                    schedule_check.check(G, S.cmds, cap)
                    ncmp += 1
    assert ncmp > 100


def test_random_graphs_command_lists_identical_and_valid():
    """random layer graphs (forks, joins, chains of layers whose outputs are no feature maps): the oracle's and
    the library's command lists agree and pass the validator, fused and not, under random plans.  Seeds 15 and 61
    hold a transient tensor read twice inside one recomputation, which a nested recomputation must not drop."""
    ncmp = 0
    for seed in list(range(120)) + [136]:     # 136: add(maxpool(t), t), whose branch reads the skip tensor itself
        net = workloads.random_net(seed, residual=80 <= seed < 120)
        rng = np.random.default_rng(1000 + seed)
        for fuse in (True, False):
            G = P.Graph(net, fuse=fuse)
            nf = len(G.fmaps)
            incore = P.build_schedule(G, [P.KEEP] * nf, BIG)
            for trial in range(4):
                cls = [int(v) for v in rng.integers(0, 3, nf)] if trial else [P.KEEP] * nf
                cap = BIG if trial == 0 else int(incore.peak * rng.uniform(0.5, 1.2)) // 256 * 256
                c, _ = lib_ctx(net, cap, fuse)
                for ahead in (True, False):
                    try:
                        S = P.build_schedule(G, cls, cap, ahead)
                    except P.Budget:
                        with pytest.raises(B.BudgetError):
                            c.set_plan(cls, ahead)
                        continue
                    c.set_plan(cls, ahead)
                    rows = c.commands()
                    assert np.array_equal(rows, as_rows(S)), (seed, fuse, trial, ahead)
                    schedule_check.check(G, S.cmds, cap)
                    ncmp += 1
    assert ncmp > 900


def test_resnet50_b640_plan_fits_16gib():
    """the paper's headline case as a planning problem: 105 maps, > 50 GB, 16 GiB arena"""
    net = workloads.resnet50(batch=640)
    c = B.Context(net, 16 << 30, device=None)
    G = P.Graph(net, fuse=True)
    rng = np.random.default_rng(9)
    prof = rand_profile(G, rng)
    c.set_profile(*prof)
    cls, T = c.plan("pooch", 4)
    st = c.stats()
    assert st.resident_bytes + st.extent_bytes <= 16 << 30
    assert st.n_keep + st.n_swap + st.n_recompute == 105
    rows = c.commands()
    schedule_check.check(G, [tuple(int(v) for v in r) for r in rows], (16 << 30) - st.resident_bytes)
    with pytest.raises(B.BudgetError):
        c.plan("incore")                                        # in-core fails (section 5.2)
