"""Pin for WHERE the oracle's bf16-storage mode rounds (the benchmark's "bf16 conv inputs with
fp32 accumulate and master weights, fp32 BN statistics and updates"; the paper fixes no number
format).

The rounding points, stated once, here, as a list:
  input     the module input as it is stored in the delay ring
  weights   conv weights as the convolution operand (master weights stay unrounded)
  z         every conv output, before its batch statistics are taken
  act       every post-ReLU activation and every block output
  dz        the gradient w.r.t. a conv output (after the BN backward)
  dact      the gradient w.r.t. a stored activation inside a block, before its ReLU mask
  dproj     the projection branch's gradient w.r.t. the block input, before the sum
  dblock    the gradient w.r.t. a block input (the sum of the two branches)
  delta_in  the error gradient received from the module above
  dhead     the head's gradient w.r.t. its input
Statistics, dgamma/dbeta, dW, the loss and the update are never rounded.

The comparator does not repeat the oracle's formulas: it is the network of tests/torch_ref.py
(PyTorch float64 library ops + autograd) with two autograd functions spliced in at exactly the
points of the list, one that rounds a value on the way forward and one that rounds a gradient on
the way back. Both sides compute in float64 and round through float32 to bf16, so the only
difference left is the order of float64 sums (1e-16 relative): a stored value could differ by
one bf16 ulp only if a float64 sum fell within 1e-16 of a rounding boundary, which no element
of these seeded cases does. Bound asserted: relative L2 error <= 1e-9 on the module output,
the gradient passed down and every parameter gradient. Leaving out ANY single point of the list
on the comparator's side must break that bound by orders of magnitude (second test): a
rounding point moved, added or dropped in the oracle cannot go unnoticed.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wk
from workloads import BLOCK_STEM, BLOCK_BASIC, BLOCK_BOTTLENECK, BLOCK_HEAD
from oracle import ddg_oracle as orc
from tests import torch_ref

POINTS = ("input", "weights", "z", "act", "dz", "dact", "dproj", "dblock", "delta_in", "dhead")


def _bf16(t):
    return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)


class _RoundValue(torch.autograd.Function):
    """Rounds on the way forward; the gradient passes unchanged."""
    @staticmethod
    def forward(ctx, x):
        return _bf16(x)

    @staticmethod
    def backward(ctx, g):
        return g


class _RoundGrad(torch.autograd.Function):
    """Identity on the way forward; rounds the gradient on the way back."""
    @staticmethod
    def forward(ctx, x):
        return x.view_as(x)

    @staticmethod
    def backward(ctx, g):
        return _bf16(g)


class Rounded:
    """tests/torch_ref.py's network with the rounding points spliced in; `skip` names points to
    leave out."""
    def __init__(self, skip=()):
        self.skip = set(skip)

    def rv(self, point, x):
        return x if point in self.skip else _RoundValue.apply(x)

    def rg(self, point, x):
        return x if point in self.skip else _RoundGrad.apply(x)

    def unit(self, x, p, name, stride, eps):
        w = self.rv("weights", p[name + ".W"])
        z = F.conv2d(x, w, stride=stride, padding=1 if w.shape[-1] == 3 else 0)
        z = self.rg("dz", self.rv("z", z))
        return F.batch_norm(z, None, None, p[name + ".bn.gamma"], p[name + ".bn.beta"], True, 0.0, eps)

    def stored_act(self, y):
        return self.rg("dact", self.rv("act", F.relu(y)))

    def forward(self, blocks, params, x, labels=None, eps=1e-5):
        for b, p in zip(blocks, params):
            if b.kind == BLOCK_HEAD:
                x = self.rg("dhead", x)
                logits = x.mean((2, 3)) @ p["fc.W"].t() + p["fc.b"]
                return F.cross_entropy(logits, torch.as_tensor(labels, dtype=torch.long))
            x = self.rg("dblock", x)
            if b.kind == BLOCK_STEM:
                x = self.rv("act", F.relu(self.unit(x, p, "conv1", b.stride, eps)))
                continue
            if b.kind == BLOCK_BASIC:
                o = self.stored_act(self.unit(x, p, "conv1", b.stride, eps))
                z = self.unit(o, p, "conv2", 1, eps)
            else:
                o = self.stored_act(self.unit(x, p, "conv1", 1, eps))
                o = self.stored_act(self.unit(o, p, "conv2", b.stride, eps))
                z = self.unit(o, p, "conv3", 1, eps)
            sc = self.unit(self.rg("dproj", x), p, "proj", b.stride, eps) if b.projection else x
            x = self.rv("act", F.relu(z + sc))
        return x


def _rel(a, b):
    a, b = np.asarray(a, np.float64).ravel(), np.asarray(b, np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


# (blocks of the module, k, K, batch, input CHW, classes)
MID = ([wk.Block(BLOCK_BASIC, 8, 0, 8, 1, 0), wk.Block(BLOCK_BASIC, 8, 0, 16, 2, 1),
        wk.Block(BLOCK_BOTTLENECK, 16, 4, 16, 1, 0), wk.Block(BLOCK_BOTTLENECK, 16, 8, 32, 2, 1)], 2, 3, 3, (8, 9, 9), 0)
TOP = ([wk.Block(BLOCK_BASIC, 8, 0, 8, 1, 0), wk.Block(BLOCK_BASIC, 8, 0, 16, 2, 1), wk.Block(BLOCK_HEAD, 16, 0, 5, 1, 0)],
       2, 2, 4, (8, 8, 8), 5)
FIRST = ([wk.Block(BLOCK_STEM, 3, 0, 8, 1, 0), wk.Block(BLOCK_BASIC, 8, 0, 8, 1, 0)], 1, 2, 3, (3, 8, 8), 0)


def _oracle_pass(case, seed):
    """One delayed backward pass of the oracle in bf16-storage mode on unrounded seeded inputs:
    (theta, h_in, delta or labels, h_out, delta_out, grad)."""
    blocks, k, K, N, chw, classes = case
    net = orc.OracleNet(K, [[b.as_tuple() for b in blocks]], N, chw, classes, 0.9, 0.0, 1e-5, "f64", k_first=k,
                        store_bf16=True)
    n = net.param_count(k)
    theta = wk.normal(seed, 1, n) * 0.3 + 0.1
    net.set_params(k, theta)
    delay = K - k
    h_ins = [wk.normal(seed, 10 + t, N * int(np.prod(chw))).reshape((N,) + chw) for t in range(delay + 1)]
    out = None
    for t in range(delay + 1):
        h = net.forward(k, t, h_ins[t])
        if t == 0:
            out = h
        oshape = net.out_shape(k)
        if classes:
            top = (np.arange(N) * 3 % classes).astype(np.int32)
            did, dout, loss = net.backward_delayed(k, t, None, top, in_shape=h_ins[0].shape)
        else:
            top = wk.normal(seed, 50, int(np.prod(oshape))).reshape(oshape)
            did, dout, loss = net.backward_delayed(k, t, top, None, in_shape=h_ins[0].shape)
        assert bool(did) == (t == delay)
        if did:
            g = net.get_grad(k).copy()
        net.update(k, 0.0)
    # with a delay the backward pass re-forwards h_ins[0] (weights unchanged: step size 0)
    return theta, h_ins[0], top, out, dout, g, (loss if classes else None)


def _torch_pass(case, theta, h_in, top, skip=()):
    blocks, k, K, N, chw, classes = case
    net = Rounded(skip)
    params = torch_ref.unflatten(blocks, theta, classes)
    x = torch.tensor(h_in, dtype=torch.float64)
    x = net.rv("input", x).requires_grad_(k > 1)
    if classes:
        loss = net.forward(blocks, params, x, top)
        loss.backward()
        out = loss.item()
    else:
        h = net.forward(blocks, params, x)
        d = net.rv("delta_in", torch.tensor(top, dtype=torch.float64))
        (h * d).sum().backward()
        out = h.detach().numpy()
    dx = x.grad.numpy() if k > 1 else None
    return out, dx, torch_ref.flatten_grads(params)


@pytest.mark.parametrize("name,case", [("mid", MID), ("top", TOP), ("first", FIRST)])
def test_rounding_points_of_the_bf16_storage_mode(name, case):
    theta, h_in, top, h_out, dout, g, loss = _oracle_pass(case, seed=41)
    out, dx, gref = _torch_pass(case, theta, h_in, top)
    if case[5]:
        assert abs(out - loss) <= 1e-12 * abs(loss)
    else:
        assert _rel(h_out, out) <= 1e-9
    if dx is not None:
        assert _rel(dout, dx) <= 1e-9
    assert _rel(g, gref) <= 1e-9
    # and the mode is not a no-op: the unrounded network is measurably elsewhere
    out0, dx0, g0 = _torch_pass(case, theta, h_in, top, skip=POINTS)
    assert _rel(g, g0) > 1e-3


@pytest.mark.parametrize("point", POINTS)
def test_every_rounding_point_is_distinguished(point):
    """Leaving out one point on the comparator's side moves the result far beyond the bound in
    at least one of the three modules (each point occurs in at least one of them)."""
    worst = 0.0
    for case in (MID, TOP, FIRST):
        theta, h_in, top, h_out, dout, g, loss = _oracle_pass(case, seed=41)
        out, dx, gref = _torch_pass(case, theta, h_in, top, skip=(point,))
        e = [_rel(g, gref)]
        if not case[5]:
            e.append(_rel(h_out, out))
        if dx is not None:
            e.append(_rel(dout, dx))
        worst = max(worst, max(e))
    assert worst > 1e-5, (point, worst)
