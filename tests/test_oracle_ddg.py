"""Pins for the oracle's DDG driver (Section 3, Eq. 6-9, Algorithm 1).

  * K=1 is plain backpropagation (Section 3.2).
  * Module k uses the error gradient of iteration t-K+k, and no gradient while
    t-K+k < 0 (Eq. 8).
  * In stale-Jacobian mode g_k^t is the gradient of the whole network on
    minibatch t-K+k at the weights of iteration t-K+k (Eq. 8-9).
  * The whole-network gradient agrees with PyTorch float64 autograd.
"""
import numpy as np
import pytest
import torch

import workloads as wk
from workloads.configs import custom_cifar, custom_bottleneck
from oracle import ddg_oracle as orc
from tests import torch_ref


def tiny(K_cuts=(2,), batch=4, hw=8, classes=10):
    wl = wk.get_workload("tiny_k2")
    blocks = [b for m in wl.modules for b in m.blocks]
    from workloads.configs import _split
    wl.modules = _split(blocks, list(K_cuts), 3, hw, hw)
    wl.K = len(K_cuts) + 1
    wl.batch = batch
    return wl


def make_net(wl, perturb_bn=True, **kw):
    kw.setdefault("store_bf16", False)
    net = orc.OracleNet.from_workload(wl, **kw)
    for m in wl.modules:
        net.set_params(m.k, wk.init_module_params(wl, m, perturb_bn=perturb_bn))
    return net


def all_params(net):
    return [net.get_params(k).copy() for k in net.ks()]


def test_parameter_counts_follow_the_block_shapes():
    for name in wk.WORKLOADS:
        wl = wk.get_workload(name)
        net = orc.OracleNet.from_workload(wl, batch=1)
        for m in wl.modules:
            assert net.param_count(m.k) == wk.module_param_count(m, wl.num_classes)
    # ResNet-110 conv weights: 1.72 M parameters in total
    wl = wk.get_workload("resnet110_k4")
    total = sum(wk.module_param_count(m, wl.num_classes) for m in wl.modules)
    assert 1.72e6 < total < 1.75e6


def test_whole_network_gradient_matches_torch_autograd():
    """Everything at once: conv/BN/ReLU/add/projection/GAP/FC/CE forward and backward."""
    wl = custom_cifar(1, [2], batch=3, num_classes=7, hw=8)   # has stride-2 projection blocks
    net = make_net(wl)
    x, y = wk.minibatch(wl, 0)
    loss = net.bp_step(x, y, 0.0, update=False)
    blocks = [b for m in wl.modules for b in m.blocks]
    flat = np.concatenate([net.get_params(k) for k in net.ks()])
    params = torch_ref.unflatten(blocks, flat, wl.num_classes)
    xt = torch.tensor(x, dtype=torch.float64)
    ref = torch_ref.forward_blocks(blocks, params, xt, y, wl.bn_eps)
    ref.backward()
    assert abs(loss - ref.item()) < 1e-12 * max(1, abs(ref.item()))
    g = np.concatenate([net.get_grad(k) for k in net.ks()])
    gref = torch_ref.flatten_grads(params)
    np.testing.assert_allclose(g, gref, rtol=1e-9, atol=1e-12)


def test_bottleneck_module_matches_torch_autograd():
    wl = custom_bottleneck(2, batch=2, c=16, mid=4, hw=5)
    net = make_net(wl)
    m = wl.modules[0]
    k = m.k
    h_in = wk.normal(3, 1, 2 * 16 * 5 * 5).reshape(2, 16, 5, 5)
    delta = wk.synthetic_delta(wl, m, 0, 1.0)
    params = torch_ref.unflatten(m.blocks, net.get_params(k), 0)
    xt = torch.tensor(h_in, dtype=torch.float64, requires_grad=True)
    out = torch_ref.forward_blocks(m.blocks, params, xt, None, wl.bn_eps)
    (out * torch.tensor(delta)).sum().backward()
    # delay K-k = 2: forward t=0,1,2; the first backward happens at t=2 on the input of t=0
    for t in range(3):
        h = net.forward(k, t, h_in if t == 0 else h_in * (t + 1))
        did, dout, _ = net.backward_delayed(k, t, delta, None, in_shape=h_in.shape)
        assert did == (1 if t == 2 else 0)
        if t == 0:
            np.testing.assert_allclose(h, out.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dout, xt.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(net.get_grad(k), torch_ref.flatten_grads(params), rtol=1e-9, atol=1e-12)


def test_module_backward_matches_finite_differences():
    """Central differences through a whole module (BN in training mode, head included)."""
    wl = tiny(batch=2, hw=4)
    net = make_net(wl)
    x, y = wk.minibatch(wl, 0)
    net.bp_step(x, y, 0.0, update=False)
    rng = np.random.default_rng(0)
    for k in net.ks():
        g = net.get_grad(k)
        theta = net.get_params(k).copy()
        for i in rng.choice(theta.size, 12, replace=False):
            vals = []
            for sgn in (+1, -1):
                th = theta.copy()
                th[i] += sgn * 1e-5
                net.set_params(k, th)
                vals.append(net.bp_step(x, y, 0.0, update=False))
            net.set_params(k, theta)
            fd = (vals[0] - vals[1]) / 2e-5
            assert abs(fd - g[i]) <= 1e-6 * max(1.0, abs(g[i])), (k, i, fd, g[i])


def test_momentum_sgd_matches_torch_optimizer():
    wl = tiny()
    wl.weight_decay = 5e-4
    net = make_net(wl)
    blocks = [b for m in wl.modules for b in m.blocks]
    flat = np.concatenate(all_params(net))
    params = torch_ref.unflatten(blocks, flat, wl.num_classes)
    opt = torch.optim.SGD([p for d in params for p in d.values()], lr=0.1, momentum=0.9,
                          weight_decay=5e-4)
    for t in range(3):
        x, y = wk.minibatch(wl, t)
        net.bp_step(x, y, 0.1)
        opt.zero_grad()
        torch_ref.forward_blocks(blocks, params, torch.tensor(x), y, wl.bn_eps).backward()
        opt.step()
    got = np.concatenate(all_params(net))
    ref = np.concatenate([p.detach().numpy().ravel() for d in params for p in d.values()])
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-12)


def test_K1_is_backpropagation():
    """One module holding every layer: the DDG driver equals plain BP + SGD bit for bit."""
    wl1 = tiny(K_cuts=())
    wl2 = tiny()
    ddg = make_net(wl1)
    bp = make_net(wl2)
    # identical weights: concatenate the two modules' vectors for the one-module network
    ddg.set_params(1, np.concatenate(all_params(bp)))
    for t in range(4):
        x, y = wk.minibatch(wl2, t)
        l1 = ddg.ddg_step(x, y, 0.1)
        l2 = bp.bp_step(x, y, 0.1)
        assert l1 == l2
    assert np.array_equal(ddg.get_params(1), np.concatenate(all_params(bp)))
    assert np.array_equal(ddg.get_velocity(1), np.concatenate([bp.get_velocity(k) for k in bp.ks()]))


@pytest.mark.parametrize("cuts", [(2,), (1, 2), (1, 2, 3)])
def test_frozen_weights_gradients_are_delayed_backprop(cuts):
    """With step size 0 every g_k^t and delta equals plain BP on minibatch t-K+k."""
    wl = tiny(K_cuts=cuts)
    K = wl.K
    ddg = make_net(wl)
    bp = make_net(wl)
    T = K + 2
    ref_g, ref_d = {}, {}
    for s in range(T):
        x, y = wk.minibatch(wl, s)
        bp.bp_step(x, y, 0.0, update=False)
        for k in bp.ks():
            ref_g[(k, s)] = bp.get_grad(k).copy()
            if k < K:
                ref_d[(k, s)] = bp.get_delta(k)[0].copy()
    for t in range(T):
        x, y = wk.minibatch(wl, t)
        ddg.ddg_step(x, y, 0.0)
        for k in ddg.ks():
            s = t - K + k
            g = ddg.get_grad(k)
            if s < 0:
                assert g is None
            else:
                assert np.array_equal(g, ref_g[(k, s)]), (t, k)
            if k < K:
                d, ts = ddg.get_delta(k)
                # the gradient written during iteration t by module k+1 belongs to t-K+k+1
                s_out = t - K + k + 1
                if s_out < 0:
                    assert d is None
                else:
                    assert ts == s_out and np.array_equal(d, ref_d[(k, s_out)]), (t, k)


@pytest.mark.parametrize("cuts", [(2,), (1, 2, 3)])
def test_stale_jacobian_mode_is_the_paper_closed_form(cuts):
    """g_k^t equals the full-network gradient on minibatch s at the weights w^s, s=t-K+k."""
    wl = tiny(K_cuts=cuts)
    K = wl.K
    ddg = make_net(wl, stale_jacobian=True)
    probe = make_net(wl)
    history = []
    for t in range(K + 3):
        history.append(all_params(ddg))   # w^t before the update of iteration t
        x, y = wk.minibatch(wl, t)
        ddg.ddg_step(x, y, 0.05)
        for k in ddg.ks():
            s = t - K + k
            if s < 0:
                assert ddg.get_grad(k) is None
                continue
            for kk, th in zip(probe.ks(), history[s]):
                probe.set_params(kk, th)
            xs, ys = wk.minibatch(wl, s)
            probe.bp_step(xs, ys, 0.0, update=False)
            np.testing.assert_allclose(ddg.get_grad(k), probe.get_grad(k), rtol=1e-12, atol=1e-15)


def test_reforward_mode_differs_from_closed_form_only_through_the_module_own_weights():
    """Default mode: Jacobians of module k are taken at (stored input, current weights)."""
    wl = tiny()
    ddg = make_net(wl)
    lit = make_net(wl, stale_jacobian=True)
    diffs = []
    for t in range(3):
        x, y = wk.minibatch(wl, t)
        ddg.ddg_step(x, y, 0.1)
        lit.ddg_step(x, y, 0.1)
        diffs.append(np.abs(ddg.get_params(1) - lit.get_params(1)).max())
    # K=2, module 1 (delay 1): no update at t=0, so w^1 = w^0 and the update of t=1 (s=0)
    # is the same either way; at t=2 the stored input of s=1 meets w^2 != w^1.
    assert diffs[0] == 0 and diffs[1] == 0 and diffs[2] > 0
    # the last module has no delay: both modes agree there until module 1 diverges
    assert np.array_equal(ddg.get_h(2).shape, lit.get_h(2).shape)


def test_warm_up_and_fifo_depth():
    wl = tiny(K_cuts=(1, 2, 3))
    K = wl.K
    ddg = make_net(wl)
    init = all_params(ddg)
    for t in range(K + 2):
        x, y = wk.minibatch(wl, t)
        ddg.ddg_step(x, y, 0.1)
        for k in ddg.ks():
            changed = not np.array_equal(ddg.get_params(k), init[k - 1])
            assert changed == (t >= K - k), (t, k)          # first update at t = K-k
            assert ddg.fifo_depth(k) == min(t + 1, K - k), (t, k)
            if t < K - k:
                assert np.all(ddg.get_velocity(k) == 0)


def test_module_calls_compose_into_the_driver():
    """forward / backward_delayed / update per module, with the mailbox kept by the caller,
    reproduces ddg_step bit for bit."""
    wl = tiny(K_cuts=(1, 2))
    K = wl.K
    a = make_net(wl)
    b = make_net(wl)
    mailbox = {}
    for t in range(5):
        x, y = wk.minibatch(wl, t)
        la = a.ddg_step(x, y, 0.1)
        h = x
        for k in b.ks():
            h = b.forward(k, t, h)
        staged = {}
        lb = None
        for k in b.ks():
            did, dout, loss = b.backward_delayed(k, t, mailbox.get(k), y)
            assert did == (1 if t - K + k >= 0 else 0)
            if did and k > 1:
                staged[k - 1] = dout
            if k == K:
                lb = loss
        mailbox.update(staged)
        for k in b.ks():
            b.update(k, 0.1)
        assert la == lb
    for k in a.ks():
        assert np.array_equal(a.get_params(k), b.get_params(k))


# ---- storage-precision mode (bf16 operands / stored tensors, arithmetic unchanged) ----------

def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(5)
    v = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-6, 6, 4096),
                        [0.0, -0.0, 1.0, 1.00390625, 1.005859375, 1.001953125, 3.0e38, 1e-40]])
    got = orc.round_bf16(v)
    ref = torch.tensor(v, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, ref)
    assert np.array_equal(orc.round_bf16(got), got)          # idempotent
    # ties go to the even significand: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert orc.round_bf16(np.array([1.00390625]))[0] == 1.0
    assert orc.round_bf16(np.array([1.01171875]))[0] == 1.015625


def test_bf16_storage_mode_keeps_invariants_and_stays_close():
    wl = tiny()
    plain = make_net(wl)
    rounded = make_net(wl, store_bf16=True)
    for t in range(3):
        x, y = wk.minibatch(wl, t)
        x = orc.round_bf16(x).reshape(x.shape)
        lp = plain.ddg_step(x, y, 0.05)
        lr_ = rounded.ddg_step(x, y, 0.05)
        assert abs(lp - lr_) < 2e-2 * abs(lp)
    for k in plain.ks():
        a, b = plain.get_params(k), rounded.get_params(k)
        assert 0 < np.linalg.norm(a - b) < 2e-2 * np.linalg.norm(a)
        # master weights are never rounded
        assert not np.array_equal(b, orc.round_bf16(b))
    # the forward output of a rounded module is representable in bf16
    h = rounded.get_h(1)
    assert np.array_equal(h, orc.round_bf16(h).reshape(h.shape))
    # K=1 == BP also holds with rounding (same code path, same rounding points)
    wl1 = tiny(K_cuts=())
    ddg1 = make_net(wl1, store_bf16=True)
    bp = make_net(wl, store_bf16=True)
    ddg1.set_params(1, np.concatenate(all_params(bp)))
    for t in range(3):
        x, y = wk.minibatch(wl, t)
        assert ddg1.ddg_step(x, y, 0.1) == bp.bp_step(x, y, 0.1)
    assert np.array_equal(ddg1.get_params(1), np.concatenate(all_params(bp)))
