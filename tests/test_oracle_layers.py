"""Pins for the CPU oracle's layer arithmetic: each function is checked against something
other than itself -- an independent formulation on a library routine, a closed form, an
invariant of the mathematics, or central finite differences in float64."""
import numpy as np
import pytest
from numpy.lib.stride_tricks import sliding_window_view

from oracle import layers as L
from oracle.net import OracleNet
import workloads

RNG = np.random.default_rng(12345)


def rnd(*shape, dtype=np.float64):
    return RNG.standard_normal(shape).astype(dtype)


def conv_ref(x, w, stride, pad):
    """independent formulation: zero-pad, take all windows with numpy's strided view,
    subsample by the stride, contract with einsum"""
    nsp = w.ndim - 2
    xp = np.pad(x, [(0, 0), (0, 0)] + [(p, p) for p in pad])
    win = sliding_window_view(xp, w.shape[2:], axis=tuple(range(2, 2 + nsp)))
    sl = (slice(None), slice(None)) + tuple(slice(None, None, s) for s in stride)
    win = win[sl]
    if nsp == 2:
        return np.einsum("nchwab,kcab->nkhw", win, w)
    return np.einsum("ncdhwabe,kcabe->nkdhw", win, w)


CONV_CASES = [
    ((2, 3, 7, 6), (4, 3, 3, 3), (1, 1), (1, 1)),
    ((1, 2, 9, 8), (3, 2, 3, 3), (2, 2), (1, 1)),
    ((2, 3, 11, 11), (2, 3, 7, 7), (2, 2), (3, 3)),
    ((2, 5, 6, 6), (4, 5, 1, 1), (2, 2), (0, 0)),
    ((1, 2, 5, 6, 7), (3, 2, 3, 3, 3), (1, 1, 1), (1, 1, 1)),
    ((1, 2, 6, 5, 7), (2, 2, 2, 3, 1), (2, 1, 2), (0, 1, 0)),
]


@pytest.mark.parametrize("xs,ws,stride,pad", CONV_CASES)
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_conv_fwd_vs_windowed_einsum(xs, ws, stride, pad, dtype):
    x, w = rnd(*xs, dtype=dtype), rnd(*ws, dtype=dtype)
    y = L.conv_fwd(x, w, stride, pad)
    ref = conv_ref(x.astype(np.float64), w.astype(np.float64), stride, pad)
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12 if dtype == np.float64 else 2e-5)


def test_conv_1x1_is_matmul_and_box_sum():
    x = rnd(2, 5, 4, 3)
    w = rnd(7, 5, 1, 1)
    y = L.conv_fwd(x, w, (1, 1), (0, 0))
    ref = np.einsum("kc,nchw->nkhw", w[:, :, 0, 0], x)
    np.testing.assert_allclose(y, ref, atol=1e-12)
    ones = np.ones((1, 1, 3, 3))
    xb = rnd(1, 1, 6, 6)
    yb = L.conv_fwd(xb, ones, (1, 1), (0, 0))
    for i in range(4):
        for j in range(4):
            assert abs(yb[0, 0, i, j] - xb[0, 0, i:i + 3, j:j + 3].sum()) < 1e-12


@pytest.mark.parametrize("xs,ws,stride,pad", CONV_CASES)
def test_conv_adjoint_identities(xs, ws, stride, pad):
    """<conv(x;w), dy> == <x, dgrad(dy;w)> == <w, wgrad(dy;x)> (bilinearity)"""
    x, w = rnd(*xs), rnd(*ws)
    y = L.conv_fwd(x, w, stride, pad)
    dy = rnd(*y.shape)
    lhs = float((y * dy).sum())
    dx = L.conv_dgrad(dy, w, x.shape, stride, pad)
    dw = L.conv_wgrad(dy, x, w.shape, stride, pad)
    assert abs(lhs - float((x * dx).sum())) < 1e-9 * max(1.0, abs(lhs))
    assert abs(lhs - float((w * dw).sum())) < 1e-9 * max(1.0, abs(lhs))


def fd_grad(f, a, eps=1e-6):
    g = np.zeros_like(a)
    flat, gf = a.reshape(-1), g.reshape(-1)
    for i in range(flat.size):
        old = flat[i]
        flat[i] = old + eps
        fp = f()
        flat[i] = old - eps
        fm = f()
        flat[i] = old
        gf[i] = (fp - fm) / (2 * eps)
    return g


def test_conv_gradients_finite_difference():
    x, w = rnd(1, 2, 5, 4), rnd(3, 2, 3, 2)
    stride, pad = (2, 1), (1, 0)
    dy = rnd(*L.conv_fwd(x, w, stride, pad).shape)
    f = lambda: float((L.conv_fwd(x, w, stride, pad) * dy).sum())
    np.testing.assert_allclose(L.conv_dgrad(dy, w, x.shape, stride, pad), fd_grad(f, x), atol=1e-7)
    np.testing.assert_allclose(L.conv_wgrad(dy, x, w.shape, stride, pad), fd_grad(f, w), atol=1e-7)


def test_bn_forward_invariants_and_stats():
    x = rnd(4, 3, 5, 6) * np.array([1.0, 3.0, 0.2]).reshape(1, 3, 1, 1) + np.array([0.5, -2.0, 10.0]).reshape(1, 3, 1, 1)
    eps = 2e-5
    y, mean, istd = L.bn_fwd(x, np.ones(3), np.zeros(3), eps)
    mu = x.mean(axis=(0, 2, 3))
    var = x.var(axis=(0, 2, 3))  # numpy's var is the biased one
    np.testing.assert_allclose(mean, mu, atol=1e-12)
    np.testing.assert_allclose(istd, 1 / np.sqrt(var + eps), rtol=1e-12)
    np.testing.assert_allclose(y.mean(axis=(0, 2, 3)), 0, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=(0, 2, 3)), var / (var + eps), rtol=1e-10)
    g, b = np.array([2.0, -1.0, 0.5]), np.array([0.1, 0.2, -0.3])
    y2, _, _ = L.bn_fwd(x, g, b, eps)
    np.testing.assert_allclose(y2, y * g.reshape(1, 3, 1, 1) + b.reshape(1, 3, 1, 1), atol=1e-12)


def test_bn_backward_invariants_and_fd():
    x, dy = rnd(3, 2, 4, 3), rnd(3, 2, 4, 3)
    g, b, eps = np.array([1.5, -0.7]), np.array([0.2, 0.1]), 1e-3
    _, mean, istd = L.bn_fwd(x, g, b, eps)
    dx, dg, db = L.bn_bwd(x, dy, g, mean, istd)
    xh = (x - mean.reshape(1, 2, 1, 1)) * istd.reshape(1, 2, 1, 1)
    np.testing.assert_allclose(dx.sum(axis=(0, 2, 3)), 0, atol=1e-12)
    # sum dx*xh = gamma*istd*dgamma*(1 - sum xh^2/m) = gamma*istd*dgamma*eps/(var+eps)
    var = x.var(axis=(0, 2, 3))
    np.testing.assert_allclose((dx * xh).sum(axis=(0, 2, 3)), g * istd * dg * eps / (var + eps), atol=1e-12)
    np.testing.assert_allclose(db, dy.sum(axis=(0, 2, 3)), atol=1e-12)
    f = lambda: float((L.bn_fwd(x, g, b, eps)[0] * dy).sum())
    np.testing.assert_allclose(dx, fd_grad(f, x), atol=1e-6)
    np.testing.assert_allclose(dg, fd_grad(f, g), atol=1e-6)
    np.testing.assert_allclose(db, fd_grad(f, b), atol=1e-6)


def test_relu():
    x = np.array([-1.0, 0.0, 2.0, -0.0, 3.5])
    y = L.relu_fwd(x)
    np.testing.assert_array_equal(y, [0, 0, 2, 0, 3.5])
    np.testing.assert_array_equal(L.relu_bwd(y, np.ones(5)), [0, 0, 1, 0, 1])


def test_maxpool_ramp_ties_and_routing():
    # strictly increasing ramp: the last in-bounds element of each window is the maximum
    x = np.arange(36, dtype=np.float64).reshape(1, 1, 6, 6)
    y = L.maxpool_fwd(x, (3, 3), (2, 2), (1, 1))
    assert y.shape == (1, 1, 3, 3)
    for i in range(3):
        for j in range(3):
            assert y[0, 0, i, j] == x[0, 0, min(2 * i + 1, 5), min(2 * j + 1, 5)]
    # ties: a constant map sends every window's gradient to its FIRST in-bounds element
    c = np.zeros((1, 1, 4, 4))
    dy = np.arange(1, 5, dtype=np.float64).reshape(1, 1, 2, 2)
    dx = L.maxpool_bwd(c, dy, (3, 3), (2, 2), (1, 1))
    exp = np.zeros((4, 4))
    exp[0, 0] += 1  # window (0,0) covers rows -1..1, cols -1..1 -> first in-bounds (0,0)
    exp[0, 1] += 2  # window (0,1): rows -1..1, cols 1..3 -> (0,1)
    exp[1, 0] += 3
    exp[1, 1] += 4
    np.testing.assert_array_equal(dx[0, 0], exp)
    # 3-d, 2x2x2 stride 2: disjoint windows, gradient lands on the brute-force argmax
    x3 = rnd(1, 2, 4, 4, 4)
    y3 = L.maxpool_fwd(x3, (2, 2, 2), (2, 2, 2), (0, 0, 0))
    ref = x3.reshape(1, 2, 2, 2, 2, 2, 2, 2).transpose(0, 1, 2, 4, 6, 3, 5, 7).reshape(1, 2, 2, 2, 2, 8).max(-1)
    np.testing.assert_array_equal(y3, ref)
    d3 = rnd(*y3.shape)
    dx3 = L.maxpool_bwd(x3, d3, (2, 2, 2), (2, 2, 2), (0, 0, 0))
    up = lambda a: a.repeat(2, 2).repeat(2, 3).repeat(2, 4)
    np.testing.assert_array_equal(dx3, np.where(x3 == up(y3), up(d3), 0.0))


def test_maxpool_fd_overlapping():
    x = rnd(1, 2, 7, 7)
    dy = rnd(*L.maxpool_fwd(x, (3, 3), (2, 2), (1, 1)).shape)
    f = lambda: float((L.maxpool_fwd(x, (3, 3), (2, 2), (1, 1)) * dy).sum())
    np.testing.assert_allclose(L.maxpool_bwd(x, dy, (3, 3), (2, 2), (1, 1)), fd_grad(f, x, 1e-7), atol=1e-6)


def test_gavgpool_closed_form():
    x = rnd(2, 3, 4, 5)
    np.testing.assert_allclose(L.gavgpool_fwd(x), x.mean(axis=(2, 3)), atol=1e-13)
    dy = rnd(2, 3)
    np.testing.assert_allclose(L.gavgpool_bwd(dy, x.shape), np.broadcast_to(dy[:, :, None, None] / 20, x.shape), atol=1e-15)


def test_fc_vs_matmul():
    x, w, b, dy = rnd(3, 5), rnd(4, 5), rnd(4), rnd(3, 4)
    np.testing.assert_allclose(L.fc_fwd(x, w, b), x @ w.T + b, atol=1e-13)
    dx, dw, db = L.fc_bwd(x, w, dy)
    np.testing.assert_allclose(dx, dy @ w, atol=1e-13)
    np.testing.assert_allclose(dw, dy.T @ x, atol=1e-13)
    np.testing.assert_allclose(db, dy.sum(0), atol=1e-13)


@pytest.mark.parametrize("K", [2, 10, 1000])
def test_softmax_ce_closed_forms(K):
    z = np.zeros((4, K))
    t = np.array([0, K - 1, 1, 0], np.int32)
    loss, dz = L.softmax_ce(z, t)
    assert abs(loss - np.log(K)) < 1e-12
    z = rnd(4, K) * 5 + 300.0  # large offset: needs the max subtraction
    loss, dz = L.softmax_ce(z, t)
    np.testing.assert_allclose(dz.sum(1), 0, atol=1e-13)
    p = np.exp(z - z.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    assert abs(loss + np.log(p[np.arange(4), t]).mean()) < 1e-10
    f = lambda: L.softmax_ce(z, t)[0]
    if K <= 10:
        np.testing.assert_allclose(dz, fd_grad(f, z, 1e-5), atol=1e-8)


def _softmax_ce_decimal(z, t):
    """loss and dz of softmax cross-entropy by the definition -log(exp(z_t) / sum_j exp(z_j)) in 60-digit decimal
    arithmetic (no max subtraction, no log1p: at this precision the plain definition needs neither)"""
    import decimal
    D = decimal.Decimal
    with decimal.localcontext() as ctx:
        ctx.prec = 60
        N, K = z.shape
        loss = D(0)
        dz = np.empty((N, K), object)
        for n in range(N):
            # shifted by an integer so that exp stays in Decimal's exponent range; exact in decimal
            shift = D(int(np.floor(float(z[n].max()))))
            e = [(D(float(v)) - shift).exp() for v in z[n]]
            tot = sum(e)
            loss += -(e[t[n]] / tot).ln()
            for j in range(K):
                dz[n, j] = (e[j] / tot - (1 if j == t[n] else 0)) / N
        return float(loss / N), np.array([[float(v) for v in row] for row in dz])


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_softmax_ce_confident_samples(dtype):
    """a labelled class that leads by a wide margin: loss and gradient are tiny and must not be lost to rounding.
    Closed form -- one class M above K - 1 equal ones: loss = log1p((K-1) e^-M), dz_t = -(K-1) e^-M / (1 + (K-1) e^-M) / N
    -- and random logits scaled by 50 against the definition in 60-digit decimal arithmetic."""
    import math
    K, N = 1000, 3
    for M in (10.0, 40.0, 80.0):
        z = np.full((N, K), -1.5, dtype)
        t = np.array([0, 7, K - 1], np.int32)
        z[np.arange(N), t] += dtype(M)
        loss, dz = L.softmax_ce(z, t)
        q = (K - 1) * math.exp(-M)
        assert abs(loss - math.log1p(q)) <= 1e-12 * math.log1p(q), (M, loss, math.log1p(q))
        want_t = -q / (1 + q) / N
        got_t = dz[np.arange(N), t].astype(np.float64)
        assert np.all(np.abs(got_t - want_t) <= 2e-7 * abs(want_t)), (M, got_t, want_t)   # dz is stored in `dtype`
    rng = np.random.default_rng(3)
    z = (rng.standard_normal((4, 12)) * 50).astype(dtype)
    t = np.array([int(np.argmax(z[0])), int(np.argmax(z[1])), 3, int(np.argmin(z[3]))], np.int32)
    loss, dz = L.softmax_ce(z, t)
    want_loss, want_dz = _softmax_ce_decimal(z.astype(np.float64), t)
    assert abs(loss - want_loss) <= 1e-12 * abs(want_loss)
    tol = 2e-7 if dtype == np.float32 else 1e-12
    floor = 1e-37 if dtype == np.float32 else 1e-300          # below the storage type's normal range
    assert np.all(np.abs(dz.astype(np.float64) - want_dz) <= tol * np.abs(want_dz) + floor)


def _net_fd(net, seed, nsample=40):
    params = [p.astype(np.float64) for p in workloads.make_params(net, seed, perturb=True)]
    x, t = workloads.make_batch(net, seed)
    x = x.astype(np.float64)
    on = OracleNet(net, params, np.float64)
    loss, grads, dx = on.step(x, t)
    rng = np.random.default_rng(seed)
    plist = [on.params[i][j] for i in sorted(on.params) for j in range(len(on.params[i]))]
    worst = 0.0
    for arr, g in list(zip(plist, grads)) + [(on.out[0], dx)]:
        flat, gf = arr.reshape(-1), g.reshape(-1)
        for idx in rng.choice(flat.size, size=min(nsample, flat.size), replace=False):
            old = flat[idx]
            eps = 1e-6
            flat[idx] = old + eps
            lp = on.forward(on.out[0], t)
            flat[idx] = old - eps
            lm = on.forward(on.out[0], t)
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            worst = max(worst, abs(fd - gf[idx]) / max(1e-4, abs(fd)))
    return loss, worst


def test_whole_net_fd_tiny_cnn():
    net, seed = workloads.load("tiny")
    loss, worst = _net_fd(net, seed, nsample=12)
    assert np.isfinite(loss) and worst < 1e-4, worst


def test_whole_net_fd_residual_and_pools():
    """a small ResNet-shaped net (stem, overlapping maxpool, projection and identity
    bottlenecks, strided 1x1) and a small 3-d net: covers forks, adds and both pools"""
    net = workloads.resnet50(batch=2, size=20, nclasses=5, blocks=(2, 1), width=4)
    loss, worst = _net_fd(net, 77, nsample=6)
    assert np.isfinite(loss) and worst < 1e-4, worst
    net3 = workloads.cnn3d(size=8, channels=(2, 3), nclasses=2, batch=2)
    loss, worst = _net_fd(net3, 78, nsample=6)
    assert np.isfinite(loss) and worst < 1e-4, worst


def test_f32_build_tracks_f64():
    net, seed = workloads.load("tiny")
    params = workloads.make_params(net, seed, perturb=True)
    x, t = workloads.make_batch(net, seed)
    l32, g32, _ = OracleNet(net, params, np.float32).step(x, t)
    l64, g64, _ = OracleNet(net, params, np.float64).step(x, t)
    assert abs(l32 - l64) < 1e-5 * abs(l64)
    for a, b in zip(g32, g64):
        assert np.linalg.norm(a - b) <= 1e-4 * max(np.linalg.norm(b), 1e-12)


def test_bn_running_averages_closed_form():
    """k forward passes over one batch: a geometric series towards numpy's mean and unbiased
    variance (np.var, ddof=1) of the layer's input, from (0, 1); decay 0 keeps the batch's own
    statistics (tied to the saved mean / istd of the forward pass), decay 1 never moves"""
    net = workloads.resnet50(batch=3, size=16, nclasses=4, blocks=(1, 1), width=4)
    params = workloads.make_params(net, 5, perturb=True)
    x, t = workloads.make_batch(net, 5)
    bns = [i for i, l in enumerate(net) if l["op"] == "bn"]
    d, k = 0.8, 3
    on = OracleNet(net, params, np.float64, decay=d)
    for _ in range(k):
        on.forward(x, t)
    assert sorted(on.running) == bns
    for i in bns:
        v = on.out[net[i]["x"]]
        axes = (0,) + tuple(range(2, v.ndim))
        rm, rv = on.running[i]
        np.testing.assert_allclose(rm, (1 - d ** k) * np.mean(v, axis=axes), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(rv, d ** k + (1 - d ** k) * np.var(v, axis=axes, ddof=1), rtol=1e-12)
    last = OracleNet(net, params, np.float64, decay=0.0)
    last.forward(x, t)
    frozen = OracleNet(net, params, np.float64, decay=1.0)
    frozen.forward(x, t)
    for i in bns:
        mean, istd = last.aux[i]
        m = last.out[net[i]["x"]].size // mean.size
        np.testing.assert_allclose(last.running[i][0], mean, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(last.running[i][1], (1.0 / istd ** 2 - net[i]["eps"]) * m / (m - 1), rtol=1e-9)
        assert (frozen.running[i][0] == 0).all() and (frozen.running[i][1] == 1).all()
    # a single value per channel: the variance term is 0 and the factor m / max(m - 1, 1) is 1
    one = workloads.Net()
    h = one.bn(one.input((1, 3, 1, 1)))
    one.softmax_ce(one.fc(one.gavgpool(h), 2))
    o1 = OracleNet(one, workloads.make_params(one, 1), np.float64, decay=0.5)
    xb, tb = workloads.make_batch(one, 1)
    o1.forward(xb, tb)
    np.testing.assert_allclose(o1.running[1][0], 0.5 * xb.reshape(3))
    np.testing.assert_allclose(o1.running[1][1], 0.5)


def test_backward_with_decisions_handed_in():
    """OracleNet.backward(decide_from=...): with the forward pass's own tensors nothing changes (same bits); with an
    all-zero tensor for one ReLU nothing passes it, so every gradient upstream of it is exactly zero and the
    ones downstream are untouched; a max-pool handed another input routes by that input's maxima."""
    net = workloads.Net()
    t = net.input((2, 3, 8, 8))
    t = net.relu(net.bn(net.conv(t, 4, (3, 3), (1, 1), (1, 1))))      # relu = 3
    t = net.maxpool(t, (2, 2), (2, 2), (0, 0))                         # maxpool = 4
    t = net.relu(net.bn(net.conv(t, 5, (3, 3), (1, 1), (1, 1))))      # relu = 7
    net.softmax_ce(net.fc(net.gavgpool(t), 3))
    params = workloads.make_params(net, 3, perturb=True)
    x, lab = workloads.make_batch(net, 3)
    o = OracleNet(net, params, np.float64)
    loss, g0, dx0 = o.step(x.astype(np.float64), lab)
    g1, dx1 = o.backward({3: o.out[3], 7: o.out[7], 4: o.out[3]})
    assert all(a.tobytes() == b.tobytes() for a, b in zip(g0, g1)) and dx0.tobytes() == dx1.tobytes()
    g2, dx2 = o.backward({7: np.zeros_like(o.out[7])})
    names = workloads.param_shapes(net)
    for (node, _, _), a, b in zip(names, g0, g2):
        if node < 7:
            assert not a.any() or not b.any()          # upstream of the blocked ReLU: exactly zero now
            assert not b.any()
        else:
            assert a.tobytes() == b.tobytes()
    assert not dx2.any()
    # the max-pool decides from the tensor it is handed: reversing every 2x2 window's contents moves the gradient
    flipped = np.ascontiguousarray(o.out[3][:, :, ::-1, ::-1])
    g3, _ = o.backward({4: flipped})
    dy_pool = np.ones_like(o.out[4])
    want = L.maxpool_bwd(flipped, dy_pool, (2, 2), (2, 2), (0, 0))
    own = L.maxpool_bwd(o.out[3], dy_pool, (2, 2), (2, 2), (0, 0))
    assert not np.array_equal(want, own)
    assert any(a.tobytes() != b.tobytes() for a, b in zip(g0[:3], g3[:3]))
    assert all(a.tobytes() == b.tobytes() for a, b in zip(g0[3:], g3[3:]))
