"""Seeded synthetic workloads: layer lists, parameters and batches.

This module serves both the CPU oracle and the HIP library's tests/bench.  It
holds configuration and random-number generation only -- none of the method's
arithmetic (no layer maths, no scheduling, no planning).  Every input is synthetic:
the paper measures throughput only (section 5.1: images per second = batch size /
time per iteration) and never says which images it fed, so N(0,1) tensors of the
paper's shapes stand in for them.

A network is a list of layer dicts; a layer's id is its list index and insertion
order is execution order:
    {"op": "input", "shape": (N, C, H, W) or (N, C, D, H, W)}
    {"op": "conv", "x": id, "cout": K, "k": (..), "stride": (..), "pad": (..)}
    {"op": "bn", "x": id, "eps": 2e-5}
    {"op": "relu", "x": id}
    {"op": "add", "a": id, "b": id}
    {"op": "maxpool", "x": id, "k": (..), "stride": (..), "pad": (..)}
    {"op": "gavgpool", "x": id}
    {"op": "fc", "x": id, "nout": O}
    {"op": "softmax_ce", "x": id}
Parameters, in layer order: conv -> W[K,C,*k]; bn -> gamma[C], beta[C];
fc -> W[O,I], b[O].
"""
import numpy as np

SEED_BASE = 190705013
BN_EPS = 2e-5


class Net(list):
    """list of layer dicts with small builder helpers (no arithmetic)."""

    def _push(self, **kw):
        self.append(kw)
        return len(self) - 1

    def input(self, shape):
        return self._push(op="input", shape=tuple(int(v) for v in shape))

    def conv(self, x, cout, k, stride, pad):
        return self._push(op="conv", x=x, cout=int(cout), k=tuple(k), stride=tuple(stride), pad=tuple(pad))

    def bn(self, x, eps=BN_EPS):
        return self._push(op="bn", x=x, eps=float(eps))

    def relu(self, x):
        return self._push(op="relu", x=x)

    def add(self, a, b):
        return self._push(op="add", a=a, b=b)

    def maxpool(self, x, k, stride, pad):
        return self._push(op="maxpool", x=x, k=tuple(k), stride=tuple(stride), pad=tuple(pad))

    def gavgpool(self, x):
        return self._push(op="gavgpool", x=x)

    def fc(self, x, nout):
        return self._push(op="fc", x=x, nout=int(nout))

    def softmax_ce(self, x):
        return self._push(op="softmax_ce", x=x)


def layer_inputs(layer):
    if layer["op"] == "input":
        return []
    if layer["op"] == "add":
        return [layer["a"], layer["b"]]
    return [layer["x"]]


def shapes(net):
    """Logical NC(D)HW output shape of every layer (sizes only, for sizing buffers)."""
    out = []
    for L in net:
        op = L["op"]
        if op == "input":
            s = L["shape"]
        elif op in ("conv", "maxpool"):
            i = out[L["x"]]
            sp = tuple((i[2 + d] + 2 * L["pad"][d] - L["k"][d]) // L["stride"][d] + 1
                       for d in range(len(L["k"])))
            s = (i[0], L["cout"] if op == "conv" else i[1]) + sp
        elif op in ("bn", "relu"):
            s = out[L["x"]]
        elif op == "add":
            s = out[L["a"]]
        elif op == "gavgpool":
            s = out[L["x"]][:2]
        elif op == "fc":
            s = (out[L["x"]][0], L["nout"])
        elif op == "softmax_ce":
            s = ()
        else:
            raise ValueError(op)
        out.append(tuple(int(v) for v in s))
    return out


def param_shapes(net):
    """[(layer id, name, shape)] in parameter order."""
    sh = shapes(net)
    ps = []
    for i, L in enumerate(net):
        if L["op"] == "conv":
            ps.append((i, "W", (L["cout"], sh[L["x"]][1]) + tuple(L["k"])))
        elif L["op"] == "bn":
            c = sh[L["x"]][1]
            ps.append((i, "gamma", (c,)))
            ps.append((i, "beta", (c,)))
        elif L["op"] == "fc":
            nin = int(np.prod(sh[L["x"]][1:]))
            ps.append((i, "W", (L["nout"], nin)))
            ps.append((i, "b", (L["nout"],)))
    return ps


def make_params(net, seed, perturb=False):
    """He-normal filters / FC weights (std = sqrt(2/fan_in), fan_in = Cin * prod(kernel)),
    gamma = 1, beta = 0, bias = 0.  perturb=True draws gamma, beta and biases at random
    too, so that tests exercise terms that vanish at the default initialisation."""
    rng = np.random.default_rng(seed)
    out = []
    for _, name, shp in param_shapes(net):
        if name == "W":
            fan_in = int(np.prod(shp[1:]))
            out.append((rng.standard_normal(shp) * np.sqrt(2.0 / fan_in)).astype(np.float32))
        elif name == "gamma":
            g = 1.0 + 0.3 * rng.standard_normal(shp) if perturb else np.ones(shp)
            out.append(g.astype(np.float32))
        else:
            b = 0.2 * rng.standard_normal(shp) if perturb else np.zeros(shp)
            out.append(b.astype(np.float32))
    return out


def make_batch(net, seed, nclasses=None):
    """x ~ N(0,1) float32 of the input shape; labels uniform over the classes, int32."""
    rng = np.random.default_rng(seed + 7919)
    shp = net[0]["shape"]
    x = rng.standard_normal(shp, dtype=np.float32)
    if nclasses is None:
        nclasses = next(L["nout"] for L in reversed(net) if L["op"] == "fc")
    t = rng.integers(0, nclasses, size=shp[0]).astype(np.int32)
    return x, t


# ---------------------------------------------------------------- the five configurations

def tiny_cnn(batch=2, size=16, ch=8, nclasses=10):
    """4 x [conv3x3 ch, stride 1, pad 1 + BN + ReLU], global average pool, FC, softmax-CE."""
    net = Net()
    t = net.input((batch, 3, size, size))
    for _ in range(4):
        t = net.conv(t, ch, (3, 3), (1, 1), (1, 1))
        t = net.bn(t)
        t = net.relu(t)
    t = net.gavgpool(t)
    t = net.fc(t, nclasses)
    net.softmax_ce(t)
    return net


def _bottleneck(net, x, mid, out, stride, project):
    """ResNet bottleneck in the original form: the stride sits on the first 1x1."""
    s = (stride, stride)
    t = net.relu(net.bn(net.conv(x, mid, (1, 1), s, (0, 0))))
    t = net.relu(net.bn(net.conv(t, mid, (3, 3), (1, 1), (1, 1))))
    t = net.bn(net.conv(t, out, (1, 1), (1, 1), (0, 0)))
    sc = net.bn(net.conv(x, out, (1, 1), s, (0, 0))) if project else x
    return net.relu(net.add(t, sc))


def bottleneck_stage(batch=32, ch=256, size=56, blocks=3, nclasses=10):
    """3 identity bottleneck blocks (1x1 64, 3x3 64, 1x1 256) on a batch x 256 x 56 x 56 input;
    the configuration names no loss, so a global-average-pool + FC 256->10 + softmax-CE
    head is attached to give the step a scalar to differentiate."""
    net = Net()
    t = net.input((batch, ch, size, size))
    for _ in range(blocks):
        t = _bottleneck(net, t, ch // 4, ch, 1, False)
    t = net.gavgpool(t)
    t = net.fc(t, nclasses)
    net.softmax_ce(t)
    return net


def late_fork(batch=2, ch=8, size=8, nclasses=3):
    """Test shape: a residual add whose skip tensor t gets one more consumer after the branch was built, so
    that the add's backward cannot hand a single gradient buffer to both inputs (the branch's gradient needs
    a buffer of its own); the late consumer's result joins a second add whose inputs are both normalised."""
    net = Net()
    t = net.input((batch, 3, size, size))
    t = net.relu(net.bn(net.conv(t, ch, (3, 3), (1, 1), (1, 1))))
    u = net.bn(net.conv(t, ch, (3, 3), (1, 1), (1, 1)))
    v = net.bn(net.conv(t, ch, (1, 1), (1, 1), (0, 0)))
    z = net.relu(net.add(t, u))
    w = net.relu(net.add(net.bn(net.conv(z, ch, (1, 1), (1, 1), (0, 0))), v))
    net.softmax_ce(net.fc(net.gavgpool(w), nclasses))
    return net


def random_net(seed, batch=2, ch=4, size=6, nclasses=3, residual=False):
    """Test shape: a random directed acyclic graph of shape-preserving layers (3x3 and 1x1 convolutions, batch
    normalisation, ReLU, 3x3 stride-1 max-pool, adds of two different earlier tensors), every tensor consumed,
    closed by a global pool, FC and the loss.  Exercises forks, joins and chains of layers whose outputs are no
    feature maps in orders no configured network has.  residual: also draws whole conv-bn-relu groups and
    residual joins relu(bn(conv(a)) + b), relu(bn(conv(a)) + bn(conv(b))), the patterns the fused kernels serve."""
    rng = np.random.default_rng(seed)
    net = Net()
    ts = [net.input((batch, ch, size, size))]
    consumed = set()
    for _ in range(int(rng.integers(4, 14))):
        ops = ("conv3", "conv1", "bn", "relu", "add", "pool", "bn", "relu", "add")
        if residual:
            ops = ops + ("cbr", "join", "join", "join2")
        op = ops[int(rng.integers(0, len(ops)))]
        a = ts[int(rng.integers(max(0, len(ts) - 4), len(ts)))]
        if op in ("cbr", "join", "join2"):
            b = ts[int(rng.integers(0, len(ts)))]
            u = net.bn(net.conv(a, ch, (3, 3), (1, 1), (1, 1)))
            if op == "cbr":
                t = net.relu(u)
            elif op == "join" and b != 0:
                t = net.relu(net.add(u, b) if rng.integers(0, 2) else net.add(b, u))
                consumed.add(b)
            else:
                t = net.relu(net.add(u, net.bn(net.conv(b, ch, (1, 1), (1, 1), (0, 0)))))
                consumed.add(b)
            consumed.add(a)
            ts.append(t)
            continue
        if op == "conv3":
            t = net.conv(a, ch, (3, 3), (1, 1), (1, 1))
        elif op == "conv1":
            t = net.conv(a, ch, (1, 1), (1, 1), (0, 0))
        elif op == "bn":
            t = net.bn(a)
        elif op == "relu":
            t = net.relu(a)
        elif op == "pool":
            t = net.maxpool(a, (3, 3), (1, 1), (1, 1))
        else:
            b = ts[int(rng.integers(0, len(ts)))]
            if b == a:
                continue
            t = net.add(a, b)
            consumed.add(b)
        consumed.add(a)
        ts.append(t)
    t = ts[-1]
    for u in ts[1:-1]:
        if u not in consumed:
            t = net.add(t, u)
    net.softmax_ce(net.fc(net.gavgpool(t), nclasses))
    return net


def resnet50(batch=64, size=224, nclasses=1000, blocks=(3, 4, 6, 3), width=64):
    """ResNet-50, original form: 7x7/2 stem, 3x3/2 maxpool pad 1, bottleneck 3-4-6-3 with a
    projection shortcut in the first block of each stage, 1000-way FC."""
    net = Net()
    t = net.input((batch, 3, size, size))
    t = net.relu(net.bn(net.conv(t, width, (7, 7), (2, 2), (3, 3))))
    t = net.maxpool(t, (3, 3), (2, 2), (1, 1))
    mid = width
    for si, nb in enumerate(blocks):
        for b in range(nb):
            stride = 2 if (b == 0 and si > 0) else 1
            t = _bottleneck(net, t, mid, mid * 4, stride, b == 0)
        mid *= 2
    t = net.gavgpool(t)
    t = net.fc(t, nclasses)
    net.softmax_ce(t)
    return net


def cnn3d(size=192, channels=(32, 64, 128, 256, 512), nclasses=2, batch=1):
    """5 levels of [conv3d 3x3x3 + BN + ReLU] x 2, 2x2x2 maxpool between levels,
    global average pool, FC."""
    net = Net()
    t = net.input((batch, 1, size, size, size))
    for li, c in enumerate(channels):
        if li > 0:
            t = net.maxpool(t, (2, 2, 2), (2, 2, 2), (0, 0, 0))
        for _ in range(2):
            t = net.relu(net.bn(net.conv(t, c, (3, 3, 3), (1, 1, 1), (1, 1, 1))))
    t = net.gavgpool(t)
    t = net.fc(t, nclasses)
    net.softmax_ce(t)
    return net


CONFIGS = {
    "tiny": (tiny_cnn, {}, SEED_BASE + 1),
    "bottleneck": (bottleneck_stage, {}, SEED_BASE + 2),
    "resnet50_b64": (resnet50, {"batch": 64}, SEED_BASE + 3),
    "resnet50_b640": (resnet50, {"batch": 640}, SEED_BASE + 4),
    "cnn3d": (cnn3d, {}, SEED_BASE + 5),
}


def load(name, **override):
    """(net, seed) of a named configuration; keyword overrides shrink it for tests."""
    fn, kw, seed = CONFIGS[name]
    kw = dict(kw)
    kw.update(override)
    return fn(**kw), seed
