"""Why the gradient-like tensors of a bf16-storage implementation cannot meet 2e-2 against the
UNROUNDED oracle, shown by counting (CPU only).

Storing a conv output in bf16 moves a pre-activation that lies near zero across zero for a small
share of the elements; each such element switches its ReLU derivative between 0 and 1. This test
counts those elements and checks three things on residual blocks of the benchmark's kind:

  1. the relative L2 distance between the gradient of the rounded network and that of the
     unrounded one is the one the counts predict, sqrt(sum over ReLUs of flipped / active), within
     30 % (independent, equally distributed gradient elements: a flipped element
     removes or adds one element's worth of energy at its layer);
  2. with the ReLU decisions of the rounded network taken from the unrounded one (nothing else
     changed: every tensor is still rounded where the storage mode rounds it) the distance falls
     to the level of plain rounding noise, several times below the tolerance of 2e-2: the
     decisions, not the arithmetic, are what separates the two;
  3. the oracle's own two modes (store_bf16 on / off) are exactly that far apart (its rounded mode
     is pinned to the comparator used here by test_oracle_bf16_placement.py).

The comparator is the PyTorch float64 network with explicit casts of test_oracle_bf16_placement.py.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wk
from workloads import BLOCK_BASIC
from oracle import ddg_oracle as orc
from tests import torch_ref
from tests.test_oracle_bf16_placement import POINTS, Rounded, _rel


class Probed(Rounded):
    """Rounded network that records the input of every ReLU, and can take the ReLU decisions
    from a list recorded earlier (`masks`) instead of from its own pre-activations."""
    def __init__(self, skip=(), masks=None):
        super().__init__(skip)
        self.pre, self.masks, self._i = [], masks, 0

    def relu(self, y):
        self.pre.append(y.detach().clone())
        if self.masks is None:
            return F.relu(y)
        m = self.masks[self._i]
        self._i += 1
        return y * m      # forward value and derivative follow the given decision

    def stored_act(self, y):
        return self.rg("dact", self.rv("act", self.relu(y)))

    def forward(self, blocks, params, x, labels=None, eps=1e-5):
        for b, p in zip(blocks, params):
            assert b.kind == BLOCK_BASIC and not b.projection
            x = self.rg("dblock", x)
            o = self.stored_act(self.unit(x, p, "conv1", b.stride, eps))
            z = self.unit(o, p, "conv2", 1, eps)
            x = self.rv("act", self.relu(z + x))
        return x


def _run(blocks, theta, h_in, delta, skip=(), masks=None):
    net = Probed(skip, masks)
    params = torch_ref.unflatten(blocks, theta, 0)
    x = net.rv("input", torch.tensor(h_in, dtype=torch.float64)).requires_grad_(True)
    h = net.forward(blocks, params, x)
    d = net.rv("delta_in", torch.tensor(delta, dtype=torch.float64))
    (h * d).sum().backward()
    return net.pre, h.detach().numpy(), x.grad.numpy(), torch_ref.flatten_grads(params)


@pytest.mark.parametrize("nblocks,seed", [(1, 5), (2, 6), (4, 7)])
def test_gradient_distance_is_the_counted_relu_flips(nblocks, seed):
    C, N, HW = 16, 8, 16
    blocks = [wk.Block(BLOCK_BASIC, C, 0, C, 1, 0) for _ in range(nblocks)]
    nparam = sum(int(np.prod(s)) for b in blocks for _, s in wk.block_param_shapes(b, 0))
    rng_theta = wk.normal(seed, 1, nparam)
    # He-scaled conv weights, gamma near 1, beta near 0 (the benchmark's initialisation, perturbed)
    theta, off = np.empty(nparam), 0
    for b in blocks:
        for name, shp in wk.block_param_shapes(b, 0):
            n = int(np.prod(shp))
            v = rng_theta[off:off + n]
            if name.endswith(".W"):
                theta[off:off + n] = v * np.sqrt(2.0 / (shp[1] * shp[2] * shp[3]))
            elif name.endswith("gamma"):
                theta[off:off + n] = 1.0 + 0.1 * v
            else:
                theta[off:off + n] = 0.1 * v
            off += n
    h_in = np.maximum(wk.normal(seed, 2, N * C * HW * HW).reshape(N, C, HW, HW), 0.0)   # a post-ReLU activation
    delta = wk.normal(seed, 3, N * C * HW * HW).reshape(N, C, HW, HW) * 1e-2

    pre_p, h_p, dx_p, g_p = _run(blocks, theta, h_in, delta, skip=POINTS)     # nothing rounded
    pre_r, h_r, dx_r, g_r = _run(blocks, theta, h_in, delta)                  # bf16 storage
    flipped = [int(((a > 0) != (b > 0)).sum()) for a, b in zip(pre_p, pre_r)]
    active = [int((a > 0).sum()) for a in pre_p]
    assert len(flipped) == 2 * nblocks and all(f > 0 for f in flipped), flipped
    share = [f / a.numel() for f, a in zip(flipped, pre_p)]
    # a few elements in a thousand per ReLU, growing with depth as the forward error accumulates
    assert all(1e-4 < s < 2e-2 for s in share), share

    predicted = float(np.sqrt(sum(f / a for f, a in zip(flipped, active))))
    d_dx, d_g = _rel(dx_r, dx_p), _rel(g_r, g_p)
    # 1. the distance is the one the counts predict
    # (measured: 0.061 / 0.114 / 0.177 predicted, 0.053 / 0.105 / 0.146 found for 1 / 2 / 4 blocks)
    assert 0.7 * predicted <= d_dx <= 1.3 * predicted, (predicted, d_dx, flipped, active)
    assert 0.6 * predicted <= d_g <= 1.3 * predicted, (predicted, d_g)
    # ... and is beyond the tolerance although the forward output is well inside it
    assert d_dx > 2e-2 and _rel(h_r, h_p) < 1e-2, (d_dx, _rel(h_r, h_p))

    # 2. same rounding everywhere, ReLU decisions of the unrounded network: rounding noise only
    masks = [(a > 0).to(torch.float64) for a in pre_p]
    _, h_m, dx_m, g_m = _run(blocks, theta, h_in, delta, masks=masks)
    # (measured 4.1e-3 / 5.3e-3 / 6.9e-3 on the gradient passed down)
    assert _rel(dx_m, dx_p) < 0.15 * d_dx and _rel(dx_m, dx_p) < 1e-2, (_rel(dx_m, dx_p), d_dx)
    assert _rel(g_m, g_p) < 0.15 * d_g and _rel(g_m, g_p) < 1e-2, (_rel(g_m, g_p), d_g)

    # 3. the oracle's two modes are that far apart
    def oracle(store):
        net = orc.OracleNet(2, [[b.as_tuple() for b in blocks]], N, (C, HW, HW), 0, 0.9, 0.0, 1e-5, "f64", k_first=2,
                            store_bf16=store)
        net.set_params(2, theta)
        net.forward(2, 0, h_in)
        did, dout, _ = net.backward_delayed(2, 0, delta, None, in_shape=h_in.shape)
        assert did
        return dout, net.get_grad(2).copy()
    dx_op, g_op = oracle(False)
    dx_or, g_or = oracle(True)
    assert _rel(dx_op, dx_p) <= 1e-9 and _rel(dx_or, dx_r) <= 1e-9
    assert abs(_rel(dx_or, dx_op) - d_dx) <= 1e-6 * d_dx and abs(_rel(g_or, g_op) - d_g) <= 1e-6 * d_g
