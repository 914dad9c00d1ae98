"""One back-propagation step on a layer list, the plain way (paper section 2.1).

Forward runs the layers in insertion order and keeps every output; backward walks them
in reverse and hands each layer the gradient of its output.  There is no memory budget,
no swapping and no recomputation here: the out-of-core method reproduces exactly the
in-core result (swapping copies bits, recomputing re-executes the same function --
sections 3.1 and 3.2), so the definition of the in-core step is the oracle for any plan.

A tensor consumed by several layers receives the sum of their gradients, added in the
order the backward pass reaches the consumers (reverse insertion order).

Each forward pass also moves every batch normalisation's running averages (the statistics a
trained network normalises with; part of the training loop of section 2.1, used by no step):
mean <- d mean + (1 - d) batch mean, var <- d var + (1 - d) batch variance m / max(m - 1, 1),
m values per channel, from mean 0 and variance 1, d = 0.9 -- the convention of the framework
the paper's implementation sits in (section 5).  Kept in float64 whatever the step's dtype.

Where floating point decides something discrete -- which elements a ReLU lets through, which element of a
window is the maximum -- two correct fp32 evaluations may decide differently for values within rounding of a tie,
and the backward pass then differs by that element's whole gradient.  A comparison can therefore hand backward()
the other side's decisions (`decide_from`): the backward of a ReLU then masks with that side's output instead of
this forward pass's, and the backward of a max-pool picks its maxima in that side's input.  Everything else,
the forward pass included, is unchanged.

Test infrastructure only; imports nothing from the HIP library or its binding.
"""
import numpy as np

from . import layers as L


def _inputs(layer):
    if layer["op"] == "input":
        return []
    if layer["op"] == "add":
        return [layer["a"], layer["b"]]
    return [layer["x"]]


class OracleNet:
    def __init__(self, net, params, dtype=np.float32, decay=0.9):
        self.net = net
        self.dtype = np.dtype(dtype)
        self.decay = float(decay)
        self.running = {}       # bn layer -> [mean, var], float64
        self.params = {}
        it = iter(params)
        for i, layer in enumerate(net):
            if layer["op"] == "conv":
                self.params[i] = [np.ascontiguousarray(next(it), self.dtype)]
            elif layer["op"] in ("bn", "fc"):
                self.params[i] = [np.ascontiguousarray(next(it), self.dtype),
                                  np.ascontiguousarray(next(it), self.dtype)]
        self.out = None

    def forward(self, x, labels):
        net, out, self.aux = self.net, [], {}
        for i, layer in enumerate(net):
            op = layer["op"]
            if op == "input":
                y = np.ascontiguousarray(x, self.dtype)
            elif op == "conv":
                y = L.conv_fwd(out[layer["x"]], self.params[i][0], layer["stride"], layer["pad"])
            elif op == "bn":
                g, b = self.params[i]
                y, mean, istd = L.bn_fwd(out[layer["x"]], g, b, layer["eps"])
                self.aux[i] = (mean, istd)
                self._update_running(i, out[layer["x"]])
            elif op == "relu":
                y = L.relu_fwd(out[layer["x"]])
            elif op == "add":
                y = out[layer["a"]] + out[layer["b"]]
            elif op == "maxpool":
                y = L.maxpool_fwd(out[layer["x"]], layer["k"], layer["stride"], layer["pad"])
            elif op == "gavgpool":
                y = L.gavgpool_fwd(out[layer["x"]])
            elif op == "fc":
                w, b = self.params[i]
                y = L.fc_fwd(out[layer["x"]], w, b)
            elif op == "softmax_ce":
                loss, dz = L.softmax_ce(out[layer["x"]], labels)
                self.aux[i] = dz
                y = loss
            else:
                raise ValueError(op)
            out.append(y)
        self.out = out
        return out[-1]

    def _update_running(self, i, x):
        cn = x.shape[1]
        v = np.moveaxis(np.asarray(x, np.float64), 1, 0).reshape(cn, -1)
        m = v.shape[1]
        mu = v.sum(axis=1) / m
        var = ((v - mu[:, None]) ** 2).sum(axis=1) / m
        rm, rv = self.running.get(i, (np.zeros(cn), np.ones(cn)))
        d = self.decay
        self.running[i] = [d * rm + (1.0 - d) * mu, d * rv + (1.0 - d) * var * (m / max(m - 1, 1))]

    def backward(self, decide_from=None):
        """returns (param grads in parameter order, gradient of the loss w.r.t. the input).
        decide_from: {relu layer: an output tensor of it, max-pool layer: an input tensor of it} whose signs /
        maxima replace this forward pass's own where the layer's backward takes its discrete decision."""
        net, out = self.net, self.out
        decide_from = decide_from or {}
        g = [None] * len(net)

        def acc(i, v):
            g[i] = v if g[i] is None else g[i] + v

        pgrads = {}
        for i in range(len(net) - 1, -1, -1):
            layer = net[i]
            op = layer["op"]
            if op == "softmax_ce":
                acc(layer["x"], self.aux[i])
                continue
            if op == "input" or g[i] is None:
                continue
            dy = np.ascontiguousarray(g[i])
            if op == "conv":
                x, w = out[layer["x"]], self.params[i][0]
                pgrads[i] = [L.conv_wgrad(dy, x, w.shape, layer["stride"], layer["pad"])]
                acc(layer["x"], L.conv_dgrad(dy, w, x.shape, layer["stride"], layer["pad"]))
            elif op == "bn":
                mean, istd = self.aux[i]
                dx, dg, db = L.bn_bwd(out[layer["x"]], dy, self.params[i][0], mean, istd)
                pgrads[i] = [dg, db]
                acc(layer["x"], dx)
            elif op == "relu":
                acc(layer["x"], L.relu_bwd(np.ascontiguousarray(decide_from.get(i, out[i]), self.dtype), dy))
            elif op == "add":
                acc(layer["a"], dy)
                acc(layer["b"], dy)
            elif op == "maxpool":
                xin = np.ascontiguousarray(decide_from.get(i, out[layer["x"]]), self.dtype)
                acc(layer["x"], L.maxpool_bwd(xin, dy, layer["k"], layer["stride"], layer["pad"]))
            elif op == "gavgpool":
                acc(layer["x"], L.gavgpool_bwd(dy, out[layer["x"]].shape))
            elif op == "fc":
                dx, dw, db = L.fc_bwd(out[layer["x"]], self.params[i][0], dy)
                pgrads[i] = [dw, db]
                acc(layer["x"], dx)
            g[i] = None if i != 0 else g[i]
        flat = []
        for i in sorted(pgrads):
            flat.extend(pgrads[i])
        return flat, g[0]

    def step(self, x, labels, decide_from=None):
        loss = self.forward(x, labels)
        grads, dx = self.backward(decide_from)
        return loss, grads, dx
