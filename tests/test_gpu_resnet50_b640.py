"""ResNet-50, batch 640, fp32, 16 GiB arena: the configuration bench.py times, at full size.

The CPU oracle cannot run 14.8 TFLOP with 51 GB of saved maps in a test, so parity here is
  * bit-exact equality of the loss and of all 161 gradients between the in-core run (53 GB
    arena) and the run under the 16 GiB budget with the plan the library's own profiling pass
    and classification produce (sections 3.1, 3.2: swapping copies bits, recomputing re-executes
    the same function),
  * sampled outputs of the stem convolution (8.0 M GEMM rows) against the oracle's conv,
    computed one by one from the seeded input,
  * properties that hold at any size: the first BN's batch statistics against the moments of
    the captured conv output; every conv that feeds a BN has a filter gradient orthogonal to
    its filter, channel by channel (the loss does not change when a filter is rescaled, because
    BN divides the scale out); the FC bias gradient sums to zero (softmax rows sum to one).
ResNet-50 at full resolution against the whole oracle is in test_gpu_parity.py at batch 4."""
import numpy as np
import pytest

import workloads
from oracle import layers as OL
from paper_1907_05013_amd import binding as B

from parity_util import say

pytestmark = pytest.mark.gpu


def incore_arena(net):
    c = B.Context(net, 1 << 46, device=None)
    keep = [B.KEEP] * c.n_fmaps
    _, peak = c.simulate(keep, want_time=False)
    res, dyn = c.resident_bytes(), peak
    while True:
        try:
            B.Context(net, res + dyn, device=None).simulate(keep, want_time=False)
            return res + dyn
        except B.BudgetError:
            dyn = int(dyn * 1.02) // 256 * 256 + 256


def test_resnet50_b640_under_16gib_matches_incore_bit_for_bit():
    net, seed = workloads.load("resnet50_b640")
    params = workloads.make_params(net, seed)
    x, t = workloads.make_batch(net, seed)
    pshapes = workloads.param_shapes(net)
    shapes = [s for _, _, s in pshapes]

    say("[b640] in-core run")
    c = B.Context(net, incore_arena(net))
    c.set_params(params)
    c.set_batch(x, t)
    c.set_plan([B.KEEP] * c.n_fmaps)
    stem = np.empty(workloads.shapes(net)[1], np.float32)
    c.capture(1, stem)
    loss0 = c.step()
    c.capture(1, None)
    grads0 = c.get_grads(shapes)
    mean, istd = c.bn_stats(2, 64)
    c.close()
    del c
    assert np.isfinite(loss0) and 6.0 < loss0 < 10.0        # near ln(1000) at initialisation

    # sampled stem outputs against the oracle's convolution, one output pixel at a time
    rng = np.random.default_rng(5)
    w = params[0]
    N, _, H, W = x.shape
    worst = 0.0
    for s in range(160):
        n = int(rng.integers(N))
        oh, ow = (int(rng.integers(112)), int(rng.integers(112))) if s >= 16 else ((0, 111)[s & 1], (0, 111)[(s >> 1) & 1])
        patch = np.zeros((1, 3, 7, 7), np.float32)
        for r in range(7):
            for q in range(7):
                ih, iw = 2 * oh - 3 + r, 2 * ow - 3 + q
                if 0 <= ih < H and 0 <= iw < W:
                    patch[0, :, r, q] = x[n, :, ih, iw]
        ref = OL.conv_fwd(patch, w, (1, 1), (0, 0)).reshape(-1)
        got = stem[n, :, oh, ow]
        worst = max(worst, float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-6)))
    assert worst <= 1e-3, worst
    # first BN: batch statistics over 8.0 M rows against the moments of the captured tensor
    m = stem.mean(axis=(0, 2, 3), dtype=np.float64)
    v = stem.var(axis=(0, 2, 3), dtype=np.float64)
    assert np.abs(mean - m).max() <= 1e-3 * np.sqrt(v).max()
    assert np.abs(istd * np.sqrt(v + net[2]["eps"]) - 1.0).max() <= 1e-3
    say("[b640] stem samples worst %.2e; BN statistics ok" % worst)
    del stem

    # scale invariance: <dW_k, W_k> = 0 for every conv feeding a BN; sum of FC bias gradient = 0
    worst_inv = 0.0
    for k, (node, name, shp) in enumerate(pshapes):
        if name == "W" and net[node]["op"] == "conv":
            g = grads0[k].reshape(shp[0], -1).astype(np.float64)
            wk = params[k].reshape(shp[0], -1).astype(np.float64)
            cosine = np.abs((g * wk).sum(1)) / (np.linalg.norm(g, axis=1) * np.linalg.norm(wk, axis=1) + 1e-300)
            worst_inv = max(worst_inv, float(cosine.max()))
    assert worst_inv <= 1e-3, worst_inv
    db = grads0[-1].astype(np.float64)
    assert abs(db.sum()) <= 1e-5 * np.abs(db).sum()
    say("[b640] filter-gradient / filter cosine worst %.2e" % worst_inv)

    say("[b640] run under 16 GiB")
    fm = sum(b for b, _ in B.Context(net, 1 << 46, device=None).fmaps())
    c = B.Context(net, 16 << 30, pinned_bytes=fm + 4096)
    c.set_params(params)
    c.set_batch(x, t)
    c.profile(warmup=1, iters=3)

    def profile_summary(tag):
        tf, tb, tr, to, ti = (np.asarray(v, np.float64) for v in c.get_profile())
        fb = np.array([b for b, _ in c.fmaps()], np.float64)
        say("[b640] %s: sum of layer times fwd %.1f bwd %.1f re-forward %.1f ms; copies out %.1f GB/s in %.1f GB/s (per map: out %.1f - %.1f, in %.1f - %.1f)"
            % (tag, tf.sum(), tb.sum(), tr.sum(), fb.sum() / to.sum() / 1e6, fb.sum() / ti.sum() / 1e6,
               (fb / to / 1e6).min(), (fb / to / 1e6).max(), (fb / ti / 1e6).min(), (fb / ti / 1e6).max()))
        d2h, h2d = c.measure_link(1 << 30)
        say("[b640] %s: link alone %.1f GB/s out, %.1f GB/s in" % (tag, d2h, h2d))

    profile_summary("profile")

    def run_and_compare(tag, predicted):
        loss1 = c.step()
        st = c.stats()
        grads1 = c.get_grads(shapes)
        say("[b640] %s: keep/swap/recompute %d/%d/%d, %d re-forwards, swapped %.1f GB each way, predicted %.0f ms, measured %.0f ms"
            % (tag, st.n_keep, st.n_swap, st.n_recompute, st.n_refwd, st.swap_out_bytes / 1e9, predicted, st.step_ms))
        assert st.resident_bytes + st.extent_bytes <= 16 << 30
        assert st.n_swap + st.n_recompute > 0
        assert np.float32(loss0).tobytes() == np.float32(loss1).tobytes(), (tag, loss0, loss1)
        for k, (a, b) in enumerate(zip(grads0, grads1)):
            assert a.tobytes() == b.tobytes(), (tag, "gradient", k, pshapes[k])
        # the timeline simulation predicts the measured step (section 4.1.2): best of three steps within 10 %
        measured = []
        for _ in range(3):
            c.step()
            measured.append(c.stats().step_ms)
        say("[b640] %s: simulated %.1f ms, measured %s ms" % (tag, predicted, ", ".join("%.1f" % v for v in measured)))
        r = c.step_timed()
        bwd, bwf = np.asarray(r[2]), np.asarray(r[4])
        top = np.argsort(-bwd)[:4]
        say("[b640] %s: longest backward commands: %s" % (tag, ", ".join("node %d %s %.2f ms (filter gradient %.2f)" % (i, net[i]["op"], bwd[i], bwf[i]) for i in top)))
        assert abs(min(measured) - predicted) <= 0.10 * predicted, (tag, "simulated vs measured", measured, predicted)

    # the paper's two steps (section 4.4).  The prediction is as good as the profile it is made from, so a miss is logged
    # and the profile retaken once; a second miss fails.  (The misses seen so far -- 12 and 18 % in full-suite runs, none
    # alone -- had one cause, since removed: the context's streams came from torch's pool and two of them shared a
    # hardware queue after many contexts in one process, so swap copies sat in front of kernels.  The profile summary
    # and the longest backward commands stay in the log: 219 ms of backward layer time instead of 127, and a 40 ms
    # "filter gradient", are how that showed.)
    cls, predicted = c.plan("pooch", 8)
    try:
        run_and_compare("two-step plan", predicted)
    except AssertionError as e:
        if "simulated" not in str(e):
            raise
        say("[b640] prediction missed: %s; profiling again" % (str(e)[:200],))
        c.profile(warmup=1, iters=3)
        profile_summary("second profile")
        cls, predicted = c.plan("pooch", 8)
        run_and_compare("two-step plan (second profile)", predicted)
    # the plan bench.py times: two steps + local search with its settings (4 bits, 300 restarts), the layers
    # re-timed under that plan, classified once more
    c.plan("refine", 4, restarts=300)
    c.refine_profile(2)
    cls, predicted = c.plan("refine", 4, restarts=300)
    run_and_compare("refined plan (bench.py's)", predicted)
    # the static policy of section 5.2 does not fit this arena at batch 640 (the paper reports the same of its own
    # implementation of that policy); the refusal leaves the installed plan in place
    with pytest.raises(B.BudgetError):
        c.plan("superneurons")
    assert np.array_equal(c.get_plan(), cls)
    assert np.float32(c.step()).tobytes() == np.float32(loss0).tobytes()
    c.close()
