"""Checkpoint and resume of a running DDG pipeline: weights, velocity (second moment, update
count), running estimates, every module's delay ring, the error gradients in flight between the
modules and the iteration counter are read out between two iterations, written into a NEW
pipeline, and the run continued there. Every tensor of the continued run (loss, module outputs,
mailboxes, gradients, weights, velocities, running estimates) must equal, bit for bit, that of
the uninterrupted run: the same kernels run on the same bits. A checkpoint without the ring
would have to replay the warm-up (Eq. 8 of the paper: no gradient for the first K-k iterations)
and would not."""
import sys

import numpy as np
import pytest

import workloads as wk
from workloads.configs import custom_cifar

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def H():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from tests import gpu_harness
    return gpu_harness


def _build(H, wl, adam):
    import torch
    import paper_1804_10574_amd as ddg
    st = [torch.cuda.Stream() for _ in range(wl.K)]
    pipe = ddg.Pipeline(H.descs_for(wl), [s.cuda_stream for s in st])
    if adam:
        pipe.set_optimizer(ddg.DDG_OPT_ADAM, 0.9, 0.999, 1e-8)
    return pipe, st


def _step(H, wl, pipe, t, loss_dev):
    import torch
    x, y = wk.minibatch(wl, t)
    xd = H.to_dev_nhwc(x, wl)
    yd = torch.from_numpy(y).to("cuda")
    pipe.step(xd, yd, wl.lr, loss_dev)
    pipe.sync()
    return float(loss_dev.item())


def _observe(pipe, K):
    out = {}
    for k in range(1, K + 1):
        m = pipe.module(k)
        out[f"w{k}"] = m.get_params(); out[f"v{k}"] = m.get_velocity(); out[f"r{k}"] = m.get_running()
        g = m.get_grad()
        if g is not None:
            out[f"g{k}"] = g
        if k < K:
            out[f"h{k}"] = pipe.get_h(k)
            d, it = pipe.get_delta(k)
            out[f"d{k}_iteration"] = np.array([it])
            if d is not None:
                out[f"d{k}"] = d
    return out


@pytest.mark.parametrize("case", ["tiny_k2_f32_sgd", "cifar_k3_bf16_sgd", "cifar_k3_bf16_adam"])
def test_resumed_run_continues_bit_for_bit(H, case):
    import torch
    import paper_1804_10574_amd as ddg
    if case.startswith("tiny"):
        wl = wk.get_workload("tiny_k2")
    else:
        wl = custom_cifar(2, [3, 5], batch=8, num_classes=10, hw=32, dtype="bf16", name="cifar_k3")
    adam = case.endswith("adam")
    K = wl.K
    T1, T2 = K + 3, 4          # the checkpoint is taken in steady state, every ring full
    _say(f"case {case}: {T1} iterations, checkpoint, {T2} more")
    loss_dev = torch.zeros(1, dtype=torch.float32, device="cuda")
    thetas = {m.k: wk.init_module_params(wl, m, perturb_bn=True).astype(np.float32) for m in wl.modules}

    # the uninterrupted run
    pa, sa = _build(H, wl, adam)
    for k in range(1, K + 1):
        pa.module(k).set_params(thetas[k])
    ref = []
    for t in range(T1 + T2):
        loss = _step(H, wl, pa, t, loss_dev)
        if t >= T1:
            ref.append((loss, _observe(pa, K)))
    pa.close()

    # the same run, stopped after T1 iterations
    pb, sb = _build(H, wl, adam)
    for k in range(1, K + 1):
        pb.module(k).set_params(thetas[k])
    for t in range(T1):
        _step(H, wl, pb, t, loss_dev)
    ck = {"t": pb.time(), "mods": {}, "mail": {}}
    assert ck["t"] == T1
    for k in range(1, K + 1):
        m = pb.module(k)
        ck["mods"][k] = {"w": m.get_params(), "v": m.get_velocity(), "r": m.get_running(),
                         "m2": m.get_moment2() if adam else None, "n": m.get_update_count(),
                         "ring": [m.get_ring_slot(i) for i in range(m.ring_slots())]}
        assert m.ring_slots() == K - k + 1 and m.get_time() == T1
    for k in range(1, K):
        ck["mail"][k] = pb.get_mail(k)
        assert ck["mail"][k][1] == T1 - K + k, (k, ck["mail"][k][1])
    pb.close()

    # a new pipeline takes the checkpoint and continues
    pc, sc = _build(H, wl, adam)
    for k in range(1, K + 1):
        m, c = pc.module(k), ck["mods"][k]
        m.set_params(c["w"]); m.set_velocity(c["v"]); m.set_running(c["r"])
        if adam:
            m.set_moment2(c["m2"]); m.set_update_count(c["n"])
        for i, slot in enumerate(c["ring"]):
            m.set_ring_slot(i, slot)
    pc.set_time(ck["t"])
    for k in range(1, K):
        pc.set_mail(k, *ck["mail"][k])
    bad = []
    for i, t in enumerate(range(T1, T1 + T2)):
        loss = _step(H, wl, pc, t, loss_dev)
        obs = _observe(pc, K)
        rl, ro = ref[i]
        if loss != rl:
            bad.append(f"t={t} loss {loss!r} != {rl!r}")
        if sorted(obs) != sorted(ro):
            bad.append(f"t={t} tensors {sorted(obs)} != {sorted(ro)}")
            continue
        for name in obs:
            if not np.array_equal(obs[name], ro[name]):
                bad.append(f"t={t} {name}: {int((obs[name] != ro[name]).sum())} of {obs[name].size} elements differ")
    pc.close()
    assert not bad, "\n".join(bad[:20])
    # and the ring matters: a pipeline that takes the weights and velocities only starts with the
    # warm-up of Eq. 8 again (no gradient for module 1 in its first iteration), the resumed one did not
    assert "g1" in ref[0][1]
    pd, sd = _build(H, wl, adam)
    for k in range(1, K + 1):
        pd.module(k).set_params(ck["mods"][k]["w"]); pd.module(k).set_velocity(ck["mods"][k]["v"])
    _step(H, wl, pd, 0, loss_dev)
    assert pd.module(1).get_grad() is None
    assert not np.array_equal(pd.module(K).get_params(), ref[0][1][f"w{K}"])
    pd.close()
