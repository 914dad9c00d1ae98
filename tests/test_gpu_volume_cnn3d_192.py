"""Configuration 5 at full size: the 3-d CNN on one 1 x 1 x 192^3 volume (section 1 names batch-1 3-d inputs as
the case data parallelism cannot help), fp32.

  * in-core GPU step against the whole CPU oracle: every forward tensor, the loss, all gradients (1e-3, L2 and
    element-wise; discrete decisions -- ReLU signs, max-pool maxima -- taken in the kernel's precision on both sides);
  * then the three phases of section 4.1.2 under budgets that bind: profile, classify, step, same bits as in-core.
    The configured 24 GB budget does not bind (all layer outputs total 7.4 GB), so the arena is set to fractions of
    the in-core peak instead.  A layer of the first level needs its 0.9 GB input, output and gradient at once, so
    nothing below about 55 % of the in-core peak can hold a step whatever the plan; the two smallest arenas of a
    fixed list that admit the all-swap profiling run are used.

The oracle needs minutes for the 2.9 TFLOP of this step, so the comparison is split over three tests that hand
their state on (run them in file order); each prints its steps."""
import numpy as np
import pytest

import workloads
from oracle.net import OracleNet
from paper_1907_05013_amd import binding as B
from parity_util import RTOL, say, close, rel

pytestmark = pytest.mark.gpu

STATE = {}


def _sizes(net):
    c = B.Context(net, 1 << 44, device=None)
    _, peak = c.simulate([B.KEEP] * c.n_fmaps, want_time=False)
    return c.resident_bytes(), peak, sum(b for b, _ in c.fmaps())


def test_a_forward_and_loss_vs_oracle():
    net, seed = workloads.load("cnn3d")
    assert net[0]["shape"] == (1, 1, 192, 192, 192)
    params = workloads.make_params(net, seed)
    x, t = workloads.make_batch(net, seed)
    say("[cnn3d 192^3] oracle forward")
    o = OracleNet(net, params, np.float32)
    ol = o.forward(x, t)
    say("[cnn3d 192^3] oracle forward done, loss %.7f; GPU in-core step" % ol)
    res, peak, _ = _sizes(net)
    c = B.Context(net, res + peak + (peak // 4) // 256 * 256)
    c.set_params(params)
    c.set_batch(x, t)
    c.set_plan([B.KEEP] * c.n_fmaps)
    shp = workloads.shapes(net)
    go = {}
    for i in range(1, len(net) - 1):
        if c.node_fused(i) < 0:
            go[i] = np.full(shp[i], np.nan, np.float32)
            c.capture(i, go[i])
    gl = c.step()
    gg = c.get_grads([s for _, _, s in workloads.param_shapes(net)])
    c.close()
    say("[cnn3d 192^3] GPU step done, loss %.7f" % gl)
    assert abs(gl - ol) <= RTOL * abs(ol), ("loss", gl, ol)
    worst, flips = 0.0, 0
    for i in sorted(go):
        worst = max(worst, close(("cnn3d 192^3 forward of layer", i, net[i]["op"]), go[i], o.out[i]))
        if net[i]["op"] == "relu":
            diff = (go[i] > 0) != (o.out[i] > 0)
            f = int(diff.sum())
            if f:
                pre = o.out[net[i]["x"]]
                rms = float(np.sqrt(np.mean(pre.astype(np.float64) ** 2)))
                assert float(np.abs(pre[diff]).max()) <= 5e-3 * rms, ("layer", i, "decision differs away from a tie")
                flips += f
    say("[ok] cnn3d 192^3 forward: loss gpu %.7f oracle %.7f; worst forward error %.2e (bar %.0e); %d ReLU decisions differ, all near-ties"
        % (gl, ol, worst, RTOL, flips))
    STATE.update(net=net, params=params, x=x, t=t, oracle=o, go=go, gl=gl, gg=gg)


def test_b_gradients_vs_oracle():
    if "oracle" not in STATE:
        pytest.skip("needs the state test_a leaves behind")
    net, o, go, gg = STATE["net"], STATE["oracle"], STATE["go"], STATE["gg"]
    decide = {i: go[i] for i in go if net[i]["op"] == "relu"}
    for i, L in enumerate(net):
        if L["op"] == "maxpool":
            decide[i] = go[L["x"]]
    say("[cnn3d 192^3] oracle backward (GPU's decisions)")
    og, _ = o.backward(decide)
    say("[cnn3d 192^3] oracle backward done")
    names = workloads.param_shapes(net)
    worst = 0.0
    for k, (a, b) in enumerate(zip(gg, og)):
        worst = max(worst, close(("cnn3d 192^3 gradient of parameter", k, names[k]), a, b))
    say("[ok] cnn3d 192^3 gradients: worst error %.2e (L2 and element-wise, bar %.0e)" % (worst, RTOL))
    del STATE["oracle"], STATE["go"]


def test_c_profile_plan_step_under_binding_budgets():
    if "gg" not in STATE:
        pytest.skip("needs the state test_a leaves behind")
    net, params, x, t, loss0, grads0 = (STATE[k] for k in ("net", "params", "x", "t", "gl", "gg"))
    shapes = [s for _, _, s in workloads.param_shapes(net)]
    res, peak, fm = _sizes(net)
    fits = []
    for frac in (0.50, 0.55, 0.60, 0.65, 0.70, 0.75, 0.80, 0.90):
        cap = int(peak * frac) // 256 * 256
        try:
            p = B.Context(net, res + cap, device=None)
            p.simulate([B.SWAP] * p.n_fmaps, want_time=False)
            fits.append((frac, cap))
        except B.BudgetError:
            continue
    assert len(fits) >= 2 and fits[0][0] <= 0.6, fits
    for frac, cap in fits[:2]:
        c = B.Context(net, res + cap, pinned_bytes=fm + 4096)
        c.set_params(params)
        c.set_batch(x, t)
        c.profile(warmup=1, iters=2)
        for mode in ("pooch", "refine"):
            cls, predicted = c.plan(mode, 6, restarts=8)
            l1 = c.step()
            st = c.stats()
            g1 = c.get_grads(shapes)
            assert st.resident_bytes + st.extent_bytes <= st.arena_bytes
            assert st.n_swap + st.n_recompute > 0
            assert np.float32(l1).tobytes() == np.float32(loss0).tobytes(), (frac, mode, l1, loss0)
            for k, (a, b) in enumerate(zip(grads0, g1)):
                assert a.tobytes() == b.tobytes(), (frac, mode, "gradient", k, rel(b, a))
            c.step()
            say("[ok] cnn3d 192^3 under %.0f %% of the in-core peak (%.2f GiB arena), %s: keep/swap/recompute %d/%d/%d, "
                "%d re-forwards, swapped %.2f GB each way, simulated %.1f ms, measured %.1f ms; same bits as in-core"
                % (100 * frac, (res + cap) / 2 ** 30, mode, st.n_keep, st.n_swap, st.n_recompute, st.n_refwd,
                   st.swap_out_bytes / 1e9, predicted, c.stats().step_ms))
        c.close()
    STATE.clear()
