"""Pins for the oracle's running batch-norm estimates and its evaluation forward.

The paper reports test error (Section 5) and leaves batch normalisation at test time to its
citations; the reading taken (running estimates with weight 0.1 for the newest batch statistic,
unbiased variance, moved by the forward pass on the current minibatch only) is the convention
of the library routine these pins compare against, torch.nn.functional.batch_norm:

  * after training forwards, the estimates equal the ones the library routine keeps;
  * repeating one minibatch n times gives the closed form (1-(1-rho)^n)*stat + (1-rho)^n*r0;
  * the re-forward of a stored input inside the delayed backward does not move them;
  * the evaluation forward equals the library routine with training=False (module output,
    logits, loss), and changes no training state.
"""
import numpy as np
import torch

import workloads as wk
from workloads.configs import custom_cifar, custom_bottleneck
from oracle import ddg_oracle as orc
from tests import torch_ref


def make_net(wl, **kw):
    kw.setdefault("store_bf16", False)
    net = orc.OracleNet.from_workload(wl, **kw)
    for m in wl.modules:
        net.set_params(m.k, wk.init_module_params(wl, m, perturb_bn=True))
    return net


def torch_side(wl):
    blocks = [b for m in wl.modules for b in m.blocks]
    flat = np.concatenate([wk.init_module_params(wl, m, perturb_bn=True) for m in wl.modules])
    params = torch_ref.unflatten(blocks, flat, wl.num_classes)
    return blocks, params, torch_ref.new_running(blocks, params)


def oracle_running(net):
    return np.concatenate([net.get_running(k) for k in net.ks()])


def test_running_estimates_match_the_library_routine():
    """Whole network (stem, identity and stride-2 projection blocks), three different
    minibatches through the forward of plain backpropagation (K=1)."""
    wl = custom_cifar(1, [], batch=5, num_classes=7, hw=8)
    net = make_net(wl)
    blocks, params, running = torch_side(wl)
    start = oracle_running(net)
    np.testing.assert_array_equal(start, torch_ref.flatten_running(blocks, running))   # means 0, variances 1
    for t in range(3):
        x, y = wk.minibatch(wl, t)
        net.bp_step(x, y, 0.0, update=False)
        with torch.no_grad():
            torch_ref.forward_blocks(blocks, params, torch.tensor(x), y, wl.bn_eps, running=running, training=True)
        np.testing.assert_allclose(oracle_running(net), torch_ref.flatten_running(blocks, running), rtol=1e-11, atol=1e-13)
    assert np.abs(oracle_running(net) - start).max() > 1e-3


def test_repeating_a_minibatch_gives_the_closed_form():
    wl = custom_bottleneck(1, batch=3, c=16, mid=8, hw=5, K=1, k=1)
    m = wl.modules[0]
    net = make_net(wl)
    rho = 0.25
    net.set_bn_momentum(rho)
    shape = (wl.batch, m.in_c, m.in_h, m.in_w)
    h = wk.normal(3, 1, int(np.prod(shape))).reshape(shape)
    r0 = net.get_running(m.k).copy()
    net.forward(m.k, 0, h)
    r1 = net.get_running(m.k).copy()
    stat = (r1 - (1 - rho) * r0) / rho            # what one pass mixes in
    n = 6
    for t in range(1, n):
        net.forward(m.k, t, h)
    expect = (1 - (1 - rho) ** n) * stat + (1 - rho) ** n * r0
    np.testing.assert_allclose(net.get_running(m.k), expect, rtol=1e-12, atol=1e-14)
    # the statistic is that of the conv outputs: unbiased variance, here checked for the first unit
    params = torch_ref.unflatten(m.blocks, net.get_params(m.k), 0)
    z = torch.nn.functional.conv2d(torch.tensor(h), params[0]["conv1.W"].detach())
    c = z.shape[1]
    np.testing.assert_allclose(stat[:c], z.mean((0, 2, 3)).numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(stat[c:2 * c], z.transpose(0, 1).reshape(c, -1).var(1, unbiased=True).numpy(), rtol=1e-10)


def test_the_reforward_of_a_stored_input_does_not_move_the_estimates():
    """K=2 with step size 0 (weights fixed): after n iterations module 1 has seen n minibatches
    in its forward pass and n-1 of them again in the re-forward of its delayed backward; its
    estimates must be those of n forward passes."""
    wl = custom_cifar(1, [2], batch=4, num_classes=5, hw=8)
    net = make_net(wl)
    blocks, params, running = torch_side(wl)
    n = 4
    for t in range(n):
        x, y = wk.minibatch(wl, t)
        net.ddg_step(x, y, 0.0)
        with torch.no_grad():
            torch_ref.forward_blocks(blocks, params, torch.tensor(x), y, wl.bn_eps, running=running, training=True)
    np.testing.assert_allclose(oracle_running(net), torch_ref.flatten_running(blocks, running), rtol=1e-11, atol=1e-13)


def test_evaluation_forward_matches_the_library_routine_and_touches_nothing():
    wl = custom_cifar(1, [2], batch=4, num_classes=5, hw=8)
    net = make_net(wl)
    blocks, params, running = torch_side(wl)
    for t in range(3):                               # move the estimates away from (0, 1)
        x, y = wk.minibatch(wl, t)
        net.ddg_step(x, y, 0.0)
        with torch.no_grad():
            torch_ref.forward_blocks(blocks, params, torch.tensor(x), y, wl.bn_eps, running=running, training=True)
    x, y = wk.minibatch(wl, 7)
    before = (oracle_running(net).copy(), [net.fifo_depth(k) for k in net.ks()], [net.get_params(k).copy() for k in net.ks()])
    h1 = net.forward_eval(1, x)
    loss, logits = net.forward_eval(2, h1, y)
    with torch.no_grad():
        nb1 = len(wl.modules[0].blocks)
        ref_h1 = torch_ref.forward_blocks(blocks[:nb1], params[:nb1], torch.tensor(x), None, wl.bn_eps,
                                          running=running[:nb1], training=False)
        ref_loss, ref_logits = torch_ref.forward_blocks(blocks, params, torch.tensor(x), y, wl.bn_eps, running=running,
                                                        training=False, want_logits=True)
    np.testing.assert_allclose(h1, ref_h1.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(logits, ref_logits.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(loss, float(ref_loss), rtol=1e-10)
    # evaluation differs from a training-mode forward on the same input (batch statistics)
    with torch.no_grad():
        train_h1 = torch_ref.forward_blocks(blocks[:nb1], params[:nb1], torch.tensor(x), None, wl.bn_eps)
    assert np.abs(train_h1.numpy() - h1).max() > 1e-3
    after = (oracle_running(net), [net.fifo_depth(k) for k in net.ks()], [net.get_params(k) for k in net.ks()])
    np.testing.assert_array_equal(before[0], after[0])
    assert before[1] == after[1]
    for a, b in zip(before[2], after[2]):
        np.testing.assert_array_equal(a, b)
    # and training continues as if it had not happened
    twin = make_net(wl)
    for t in range(3):
        xx, yy = wk.minibatch(wl, t)
        twin.ddg_step(xx, yy, 0.0)
    xx, yy = wk.minibatch(wl, 3)
    assert net.ddg_step(xx, yy, 0.05) == twin.ddg_step(xx, yy, 0.05)
    for k in net.ks():
        np.testing.assert_array_equal(net.get_params(k), twin.get_params(k))
