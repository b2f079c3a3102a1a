"""The evaluation forward that allocates nothing (ddg_forward_eval_static: every intermediate in
the library's static device array) against ddg_forward_eval (the module's own forward buffers)
and against the oracle, through the C boundary. Two calls in a row share the one array: a
CIFAR-shaped bf16 module first, then a smaller fp32 module that ends in the head, which finds
the first call's contents in the scratch."""
import numpy as np
import pytest

import workloads as wk
from workloads.configs import custom_cifar

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _train_forward_passes(H, wl, mod, oracle, m, steps):
    """Forward passes in training mode (warm-up iterations: no gradient yet) so that the running
    estimates the evaluation normalises with have moved away from their start values."""
    import torch
    shape_in = (wl.batch, m.in_c, m.in_h, m.in_w)
    for t in range(steps):
        h_in = wk.normal(23, 500 + t, int(np.prod(shape_in))).reshape(shape_in)
        hd = H.to_dev_nhwc(h_in, wl)
        if wl.dtype == "bf16":
            h_in = H.from_dev_nhwc(hd)
        h_out = None
        if m.blocks[-1].kind != wk.BLOCK_HEAD:
            h_out = torch.empty((wl.batch, m.out_h, m.out_w, m.out_c), dtype=H.tdtype(wl), device="cuda")
        mod.forward(t, hd, h_out)
        oracle.forward(m.k, t, h_in)
        assert not mod.backward_delayed(t, delta_in=None, delta_out=None)
        mod.update(t, 0.0)
        oracle.backward_delayed(m.k, t, None, None, in_shape=shape_in)
        oracle.update(m.k, 0.0)
    mod.sync()


def test_static_scratch_evaluation_matches_the_allocating_one():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_1804_10574_amd as ddg
    from oracle import ddg_oracle as orc
    from tests import gpu_harness as H

    # ---- first call: module 1 of K=3, bf16, 32x32: stem, identity blocks at 16 channels (the
    # fold of a block's output into the next conv), a stride-2 projection block, 32 channels
    wl = custom_cifar(3, [5, 9], batch=24, num_classes=10, hw=32, dtype="bf16", name="static_eval_a")
    m = wl.modules[0]
    mod = ddg.Module(H.descs_for(wl)[0])
    oracle = orc.OracleNet.from_workload(wl, dtype="f64")
    H.init_both(wl, {mm.k: (mod if mm.k == m.k else _Sink()) for mm in wl.modules}, oracle)
    _say("case static evaluation: module 1 of K=3, bf16, batch 24")
    _train_forward_passes(H, wl, mod, oracle, m, 2)
    shape_in = (wl.batch, m.in_c, m.in_h, m.in_w)
    x = wk.normal(23, 600, int(np.prod(shape_in))).reshape(shape_in)
    xd = H.to_dev_nhwc(x, wl)
    x = H.from_dev_nhwc(xd)
    ref = torch.empty((wl.batch, m.out_h, m.out_w, m.out_c), dtype=torch.bfloat16, device="cuda")
    got = torch.full_like(ref, float("nan"))
    mod.forward_eval(xd, ref)
    mod.forward_eval_static(xd, got)
    mod.sync()
    assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
    e = H.rel_err(H.from_dev_nhwc(got), oracle.forward_eval(m.k, x))
    _say(f"static evaluation, first call: identical to ddg_forward_eval; rel err vs oracle {e:.2e}")
    assert e <= 2e-2
    running = mod.get_running().copy()

    # ---- second call, smaller: the last module of a small fp32 network (ends in the head)
    wl2 = custom_cifar(1, [2], batch=6, num_classes=7, hw=10, dtype="f32", name="static_eval_b")
    m2 = wl2.modules[-1]
    mod2 = ddg.Module(H.descs_for(wl2)[m2.k - 1])
    oracle2 = orc.OracleNet.from_workload(wl2, dtype="f64")
    H.init_both(wl2, {mm.k: (mod2 if mm.k == m2.k else _Sink()) for mm in wl2.modules}, oracle2)
    _say("case static evaluation: head module, fp32, batch 6 (after the larger call)")
    shape2 = (wl2.batch, m2.in_c, m2.in_h, m2.in_w)
    x2 = wk.normal(23, 700, int(np.prod(shape2))).reshape(shape2)
    x2d = H.to_dev_nhwc(x2, wl2)
    y2 = (np.arange(wl2.batch) % wl2.num_classes).astype(np.int32)
    y2d = torch.from_numpy(y2).to("cuda")
    ref_logits = torch.zeros((wl2.batch, wl2.num_classes), dtype=torch.float32, device="cuda")
    got_logits = torch.full_like(ref_logits, float("nan"))
    ref_loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    got_loss = torch.full_like(ref_loss, float("nan"))
    mod2.forward_eval(x2d, None, y2d, ref_loss, ref_logits)
    mod2.forward_eval_static(x2d, None, y2d, got_loss, got_logits)
    mod2.sync()
    assert torch.equal(got_logits, ref_logits) and torch.equal(got_loss, ref_loss)
    o_loss, o_logits = oracle2.forward_eval(m2.k, x2, y2)
    assert H.rel_err(got_logits.cpu().numpy(), o_logits) <= 1e-4
    assert abs(float(got_loss.cpu()[0]) - o_loss) <= 1e-4 * abs(o_loss)

    # ---- and the first module again: same bits as before, estimates untouched
    got.fill_(float("nan"))
    mod.forward_eval_static(xd, got)
    mod.sync()
    assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
    np.testing.assert_array_equal(mod.get_running(), running)
    mod.close()
    mod2.close()


class _Sink:
    """Stands in for the modules of a workload that a single-module test does not build."""
    def set_params(self, th):
        pass
