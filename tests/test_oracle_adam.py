"""Pins for the oracle's Adam-DDG update (Algorithm 2).

  * On a network held in one module (K=1, no delay) it is Adam: agrees with torch.optim.Adam.
  * The first executed update moves every weight by lr * g / (|g| + eps) (both moments start at
    zero, so the bias-corrected first moment is g and the second is g^2): a closed form that
    also fixes how the bias-correction exponent counts: a module's warm-up iterations, in which
    it has no gradient, execute no update and do not advance it.
  * With eps = 0 the update does not change when the gradient is scaled.
"""
import numpy as np
import torch

import workloads as wk
from oracle import ddg_oracle as orc
from tests import torch_ref
from tests.test_oracle_ddg import tiny, make_net, all_params


def test_adam_matches_torch_optimizer_when_K_is_1():
    wl = tiny()
    wl.weight_decay = 5e-4
    net = make_net(wl)
    net.set_adam(True, 0.9, 0.999, 1e-8)
    blocks = [b for m in wl.modules for b in m.blocks]
    flat = np.concatenate(all_params(net))
    params = torch_ref.unflatten(blocks, flat, wl.num_classes)
    opt = torch.optim.Adam([p for d in params for p in d.values()], lr=1e-3, betas=(0.9, 0.999), eps=1e-8,
                           weight_decay=5e-4)
    for t in range(4):
        x, y = wk.minibatch(wl, t)
        net.bp_step(x, y, 1e-3)
        opt.zero_grad()
        torch_ref.forward_blocks(blocks, params, torch.tensor(x), y, wl.bn_eps).backward()
        opt.step()
    got = np.concatenate(all_params(net))
    ref = np.concatenate([p.detach().numpy().ravel() for d in params for p in d.values()])
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-12)


def test_first_executed_update_has_the_closed_form_also_after_warm_up():
    wl = tiny(K_cuts=(1, 2))           # K = 3: module 1 gets its first gradient at t = 2
    net = make_net(wl)
    lr, eps = 1e-3, 1e-8
    net.set_adam(True, 0.9, 0.999, eps)
    before = {k: net.get_params(k).copy() for k in net.ks()}
    first_seen = {}
    for t in range(4):
        x, y = wk.minibatch(wl, t)
        net.ddg_step(x, y, lr)
        for k in net.ks():
            g = net.get_grad(k)
            if g is not None and k not in first_seen:
                first_seen[k] = t
                step = before[k] - net.get_params(k)
                np.testing.assert_allclose(step, lr * g / (np.abs(g) + eps), rtol=1e-10, atol=1e-18)
                assert net.get_updates(k) == 1
            elif g is None:
                assert np.array_equal(net.get_params(k), before[k]) and net.get_updates(k) == 0
            before[k] = net.get_params(k).copy()
    assert first_seen == {1: 2, 2: 1, 3: 0}     # delays K - k


def test_update_is_invariant_to_the_gradient_scale_when_eps_is_zero():
    """One module (k=1 of K=2) driven through forward / backward_delayed / update with a
    synthetic error gradient: the backward pass is linear in it, so scaling it by 64 scales
    the gradient, the first moment (x64) and the second (x4096) exactly, and m/sqrt(v) does
    not move: the weights must come out bit-identical."""
    wl = tiny()
    m1 = wl.modules[0]
    results = []
    for scale in (1.0, 64.0):
        net = orc.OracleNet(wl.K, [[b.as_tuple() for b in m1.blocks]], wl.batch, (m1.in_c, m1.in_h, m1.in_w), 0,
                            0.9, 0.0, wl.bn_eps, "f64", k_first=1, store_bf16=False)
        net.set_params(1, wk.init_module_params(wl, m1))
        net.set_adam(True, 0.9, 0.999, 0.0)
        for t in range(4):
            x, _ = wk.minibatch(wl, t)
            net.forward(1, t, x)
            delta = wk.synthetic_delta(wl, m1, t) * scale
            net.backward_delayed(1, t, delta, None, in_shape=x.shape)
            net.update(1, 1e-3)
        assert net.get_updates(1) == 3                  # t = 0 is warm-up for a delay of 1
        results.append(net.get_params(1))
    assert np.array_equal(results[0], results[1])
    assert not np.array_equal(results[0], wk.init_module_params(wl, m1))
