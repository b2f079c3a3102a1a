"""Host-only checks of the C boundary: the library loads, exports every symbol that
include/ddg.h declares, and rejects bad arguments / call orders before any device work
(dry_run modules allocate nothing and launch nothing)."""
import os
import re

import pytest

import workloads as wk
import paper_1804_10574_amd as ddg
from paper_1804_10574_amd.ddg import make_desc, EXPORTS
from tests.gpu_harness import descs_for

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "ddg.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ddg_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = ddg.load_library()
    names = declared_symbols()
    assert len(names) >= 25
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(EXPORTS) == names
    assert "gfx950" in ddg.version()


def test_dry_run_state_machine():
    wl = wk.get_workload("tiny_k2")
    d = descs_for(wl, dry_run=True)
    m = ddg.Module(d[0])   # k=1 of K=2: delay 1
    assert m.param_count() == wk.module_param_count(wl.modules[0])
    assert m.out_shape() == (16, 8, 8)
    fake = 4096  # never dereferenced in dry_run
    with pytest.raises(ddg.DDGError) as e:
        m.backward_delayed(0, delta_in=fake)
    assert e.value.status == 3
    with pytest.raises(ddg.DDGError) as e:
        m.forward(1, fake, fake)           # must start at t = 0
    assert e.value.status == 3
    m.forward(0, fake, fake)
    with pytest.raises(ddg.DDGError):
        m.forward(1, fake, fake)           # backward(0) missing
    with pytest.raises(ddg.DDGError):
        m.update(0, 0.1)
    assert m.backward_delayed(0, delta_in=fake) is False   # s = -1: warm-up
    m.update(0, 0.1)
    m.forward(1, fake, fake)
    with pytest.raises(ddg.DDGError) as e:
        m.backward_delayed(1, delta_in=None)               # s = 0 needs delta_in
    assert e.value.status == 1
    assert m.backward_delayed(1, delta_in=fake) is True
    m.update(1, 0.1)
    with pytest.raises(ddg.DDGError) as e:
        m.forward(2, 4097, fake)                           # misaligned
    assert e.value.status == 1


def test_evaluation_calls_follow_the_state_machine():
    """ddg_forward_eval runs between iterations only, needs labels for a loss, and is refused in
    stale-Jacobian mode; the running estimates count two values per BN channel; the weight of
    the newest batch statistic can only be set before the first iteration."""
    wl = wk.get_workload("tiny_k2")
    d = descs_for(wl, dry_run=True)
    m = ddg.Module(d[0])
    channels = sum(co for b in wl.modules[0].blocks for _, _, co, _, _ in wk.configs.conv_units(b))
    assert m.running_count() == 2 * channels
    fake = 4096
    m.set_bn_momentum(0.2)
    with pytest.raises(ddg.DDGError) as e:
        m.set_bn_momentum(1.5)
    assert e.value.status == 1
    m.forward_eval(fake, fake)                 # before iteration 0: allowed
    with pytest.raises(ddg.DDGError) as e:
        m.forward_eval(fake, None)             # a module without a head needs h_out
    assert e.value.status == 1
    m.forward(0, fake, fake)
    with pytest.raises(ddg.DDGError) as e:
        m.forward_eval(fake, fake)             # in the middle of iteration 0
    assert e.value.status == 3
    m.backward_delayed(0, delta_in=fake)
    m.update(0, 0.1)
    m.forward_eval(fake, fake)
    with pytest.raises(ddg.DDGError) as e:
        m.set_bn_momentum(0.1)                 # the run has begun
    assert e.value.status == 3
    head = ddg.Module(d[1])
    with pytest.raises(ddg.DDGError) as e:
        head.forward_eval(fake, None, labels=None, loss_out=fake)
    assert e.value.status == 1
    head.forward_eval(fake, None, labels=fake, loss_out=fake, logits_out=fake)
    stale = ddg.Module(descs_for(wl, dry_run=True, stale_jacobian=True)[0])
    with pytest.raises(ddg.DDGError) as e:
        stale.forward_eval(fake, fake)
    assert e.value.status == 3


def test_head_module_argument_rules():
    wl = wk.get_workload("tiny_k2")
    d = descs_for(wl, dry_run=True)
    m = ddg.Module(d[1])
    fake = 4096
    m.forward(0, fake, None)
    with pytest.raises(ddg.DDGError):
        m.backward_delayed(0, delta_in=fake, labels=fake, delta_out=fake)
    with pytest.raises(ddg.DDGError):
        m.backward_delayed(0, labels=None, delta_out=fake)
    with pytest.raises(ddg.DDGError):
        m.backward_delayed(0, labels=fake, delta_out=None)   # k > 1 needs delta_out
    assert m.backward_delayed(0, labels=fake, delta_out=fake) is True


@pytest.mark.parametrize("mutate,status", [
    (dict(K=0), 1), (dict(k=3), 1), (dict(compute=7), 1), (dict(batch=0), 2),
    (dict(momentum=1.5), 1), (dict(bn_eps=0.0), 1),
])
def test_create_rejects_bad_descriptors(mutate, status):
    wl = wk.get_workload("tiny_k2")
    m0 = wl.modules[0]
    args = dict(K=2, k=1, batch=4, in_chw=(m0.in_c, m0.in_h, m0.in_w),
                blocks=[b.as_tuple() for b in m0.blocks], num_classes=0, compute=0, momentum=0.9,
                weight_decay=0.0, bn_eps=1e-5, dry_run=True)
    args.update(mutate)
    with pytest.raises(ddg.DDGError) as e:
        ddg.Module(make_desc(**args))
    assert e.value.status == status


def test_create_rejects_bad_block_lists():
    S, B, H = wk.BLOCK_STEM, wk.BLOCK_BASIC, wk.BLOCK_HEAD
    def mk(blocks, k=1, K=2, classes=0, in_c=3):
        return make_desc(K, k, 4, (in_c, 8, 8), blocks, classes, 0, 0.9, 0.0, 1e-5, dry_run=True)
    for blocks, kw in [
        ([(S, 3, 0, 16, 1, 0), (B, 32, 0, 32, 1, 0)], {}),              # channel mismatch
        ([(S, 3, 0, 16, 1, 0), (B, 16, 0, 32, 2, 0)], {}),              # needs projection
        ([(S, 3, 0, 24, 1, 0)], {}),                                    # cout not a power of two
        ([(S, 3, 0, 16, 3, 0)], {}),                                    # stride 3
        ([(S, 3, 0, 16, 1, 0), (H, 16, 0, 10, 1, 0)], dict(classes=10)),  # head but k != K
        ([(S, 3, 0, 16, 1, 0)], dict(classes=10)),                      # classes without head
    ]:
        with pytest.raises(ddg.DDGError) as e:
            ddg.Module(mk(blocks, **kw))
        assert e.value.status == 2, (blocks, str(e.value))


def test_maximum_sizes_are_checked_on_the_host():
    """The kernels index pixels and elements with 32 bits: a module whose largest tensor would not
    fit is refused when it is created (DDG_ERR_SHAPE), the largest one that fits is accepted
    (dry run: nothing is allocated), and the smallest shapes (batch 1, one 8x8 image) plan too."""
    S, B = wk.BLOCK_STEM, wk.BLOCK_BASIC
    blocks = [(S, 3, 0, 16, 1, 0), (B, 16, 0, 16, 1, 0)]
    def mk(batch, hw):
        return make_desc(2, 1, batch, (3, hw, hw), blocks, 0, 1, 0.9, 0.0, 1e-5, dry_run=True)
    # 16 channels x 32 x 32 x batch elements must stay below 2^31
    limit = (2 ** 31 - 1) // (16 * 32 * 32)
    ddg.Module(mk(limit, 32)).close()
    with pytest.raises(ddg.DDGError) as e:
        ddg.Module(mk(limit + 1, 32))
    assert e.value.status == 2 and "32-bit" in str(e.value)
    m = ddg.Module(mk(1, 8))
    assert m.out_shape() == (16, 8, 8)
    m.close()


def test_a_module_may_be_the_head_alone():
    """A split point after the last conv layer leaves only the classifier in the last module."""
    H = wk.BLOCK_HEAD
    m = ddg.Module(make_desc(2, 2, 4, (16, 8, 8), [(H, 16, 0, 10, 1, 0)], 10, 0, 0.9, 0.0, 1e-5, dry_run=True))
    assert m.param_count() == 16 * 10 + 10
    m.close()


def test_dry_run_pipeline_schedule():
    wl = wk.get_workload("resnet110_k4")
    p = ddg.Pipeline(descs_for(wl, dry_run=True))
    fake = 4096
    for t in range(6):
        p.step(fake, fake, 0.01)
        for k in range(1, 4):
            _, it = p.get_delta(k)
            # module k+1 wrote, during iteration t, the gradient of iteration t-K+k+1
            s = t - 4 + k + 1
            assert it == (s if s >= 0 else -1), (t, k, it)
    for k in range(1, 5):
        assert p.module(k).param_count() == wk.module_param_count(wl.modules[k - 1], wl.num_classes)


def test_static_scratch_evaluation_checks_its_size_on_the_host():
    """ddg_forward_eval_static refuses, before any device work, a module whose evaluation pass
    does not fit the 64 MiB static scratch, and runs the same argument and state checks as
    ddg_forward_eval (dry-run modules: nothing is launched)."""
    fake = 4096
    wl = wk.get_workload("resnet110_k4")
    m = ddg.Module(descs_for(wl, dry_run=True)[0])              # batch 256: 2 x 8 MiB outputs + 2 x 16 MiB convs
    m.forward_eval_static(fake, fake)
    with pytest.raises(ddg.DDGError) as e:
        m.forward_eval_static(None, fake)
    assert e.value.status == 1
    m.forward(0, fake, fake)
    with pytest.raises(ddg.DDGError) as e:                      # between iterations only
        m.forward_eval_static(fake, fake)
    assert e.value.status == 3
    big = ddg.Module(descs_for(wl, dry_run=True, batch=512)[0])
    with pytest.raises(ddg.DDGError) as e:
        big.forward_eval_static(fake, fake)
    assert e.value.status == 2 and "static scratch" in str(e.value)
    big.forward_eval(fake, fake)                                # the allocating one has no such limit


def test_checkpoint_calls_follow_the_state_machine():
    """The ring and the time of a module, and the time and the gradients in flight of a pipeline, can be
    read and set between iterations only; slot indices and the iteration of a restored gradient
    are checked; stale-Jacobian mode has no checkpoint (dry run: nothing is copied)."""
    import numpy as np
    wl = wk.get_workload("resnet110_k4")
    d = descs_for(wl, dry_run=True)
    m = ddg.Module(d[1])                                   # k = 2 of K = 4: delay 2, three slots
    assert m.ring_slots() == 3 and m.get_time() == 0
    nbytes = 256 * 32 * 32 * 16 * 2
    assert m.get_ring_slot(0).size == nbytes
    with pytest.raises(ddg.DDGError) as e:
        m.get_ring_slot(3)
    assert e.value.status == 1
    fake = 4096
    m.forward(0, fake, fake)
    with pytest.raises(ddg.DDGError) as e:                 # in the middle of iteration 0
        m.set_time(5)
    assert e.value.status == 3
    with pytest.raises(ddg.DDGError) as e:
        m.set_ring_slot(0, np.zeros(nbytes, np.uint8))
    assert e.value.status == 3
    m.backward_delayed(0, delta_in=fake, delta_out=fake); m.update(0, 0.1)
    m.set_time(7)
    assert m.get_time() == 7
    with pytest.raises(ddg.DDGError):
        m.forward(1, fake, fake)
    m.forward(7, fake, fake)                               # continues at the restored iteration
    assert m.backward_delayed(7, delta_in=fake, delta_out=fake) is True    # 7 - 2 >= 0: a gradient is due
    m.update(7, 0.1)
    m.close()
    ms = ddg.Module(descs_for(wl, dry_run=True, stale_jacobian=True)[1])
    with pytest.raises(ddg.DDGError) as e:
        ms.set_time(3)
    assert e.value.status == 3
    ms.close()

    p = ddg.Pipeline(d)
    assert p.time() == 0
    assert p.get_mail(1) == (None, -1)
    p.set_time(9)
    assert p.time() == 9 and p.module(3).get_time() == 9
    # the gradient in flight to module k at time t belongs to iteration t - K + k
    with pytest.raises(ddg.DDGError) as e:
        p.set_mail(2, np.zeros(256 * 16 * 16 * 32 * 2, np.uint8), 9 - 4 + 2 - 1)
    assert e.value.status == 1
    p.set_mail(2, np.zeros(256 * 16 * 16 * 32 * 2, np.uint8), 9 - 4 + 2)
    _, it = p.get_mail(2)
    assert it == 7
    p.step(fake, fake, 0.01)
    assert p.time() == 10
    _, it = p.get_delta(1)
    assert it == 9 - 4 + 2                                  # module 2 wrote, during iteration 9, the gradient of 9-K+k+1
    p.close()


def _order_hooks():
    import ctypes as C
    lib = ddg.load_library()
    lib.ddg_internal_pipeline_waits.restype = C.c_long
    lib.ddg_internal_pipeline_waits.argtypes = [C.c_void_p]
    lib.ddg_internal_pipeline_drop_wait.restype = None
    lib.ddg_internal_pipeline_drop_wait.argtypes = [C.c_void_p, C.c_long]
    return lib


def _dry_pipeline(K, own_forward_streams, stale=False):
    from workloads.configs import custom_cifar
    cuts = {1: [], 2: [4], 3: [3, 5], 4: [2, 4, 6], 5: [1, 3, 5, 7]}[K]
    wl = custom_cifar(2, cuts, batch=2, num_classes=10, hw=8, dtype="f32", name=f"dry_k{K}")
    assert wl.K == K
    streams = [4096 * (i + 1) for i in range(K)]                 # handles are never used in a dry run
    fstreams = [4096 * (i + 101) for i in range(K)] if own_forward_streams else None
    return ddg.Pipeline(descs_for(wl, streams=streams, fstreams=fstreams, dry_run=True, stale_jacobian=stale), streams)


@pytest.mark.parametrize("K", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("mode", ["streams", "forward_streams", "stale_jacobian"])
def test_events_order_every_tensor_the_streams_share(K, mode):
    """The pipeline's model of its own stream ordering (vector clocks over the event records and
    waits it issues; every call's reads and writes of the exchanged activations, mailbox slots,
    ring slots, tapes, weights and gradients declared) finds no access that the events leave
    unordered, for K = 1..5 modules on K streams, with a forward stream per module, and in
    stale-Jacobian mode."""
    p = _dry_pipeline(K, mode == "forward_streams", stale=(mode == "stale_jacobian"))
    fake = 4096
    for t in range(3 * K + 6):
        p.step(fake, fake, 0.01)
    p.close()


@pytest.mark.parametrize("own_forward_streams", [False, True])
def test_a_missing_wait_is_found(own_forward_streams):
    """Leaving out any single wait of a K = 3 schedule, in the model only: the model must report
    a hazard for the waits that order two streams' accesses to a shared tensor, and name it."""
    lib = _order_hooks()
    K, steps = 3, 12
    fake = 4096
    p = _dry_pipeline(K, own_forward_streams)
    for t in range(steps):
        p.step(fake, fake, 0.01)
    total = lib.ddg_internal_pipeline_waits(p._h)
    p.close()
    assert total > 4 * steps
    found, kinds = 0, set()
    for n in range(total):
        p = _dry_pipeline(K, own_forward_streams)
        lib.ddg_internal_pipeline_drop_wait(p._h, n)
        try:
            for t in range(steps):
                p.step(fake, fake, 0.01)
        except ddg.DDGError as e:
            assert e.status == 3 and "hazard" in str(e), str(e)
            found += 1
            tensor = str(e).split("touches ")[1].split(" ")[0].split("/")[0].rstrip("0123456789")
            kinds.add(str(e).split(" hazard")[0].split(": ")[-1] + " " + tensor)
        p.close()
    print(found, "of", total, sorted(kinds))
    # most waits are the only thing that orders their pair of accesses
    assert found >= total // 2, (found, total)
    want = {"read-after-write h", "read-after-write mail", "write-after-read h"}
    if own_forward_streams:
        want |= {"read-after-write w", "write-after-read w", "write-after-read mail"}
    assert want <= kinds, kinds


def test_bench_names_kernels_as_the_profiler_does():
    """bench.py's label of the kernel behind a profile kind agrees with the kind the profile
    summaries derive from that kernel's name, for the bf16 and the fp32 instances."""
    import sys
    sys.path.insert(0, ROOT)
    import bench
    from paper_1804_10574_amd import profile_summary as ps
    for kind in ("conv_fprop.tiled_c16_w32", "conv_dgrad.tiled_c32_w16", "conv_bwd_pair.tiled_c64_w8",
                 "conv_wgrad.tiled_c16_w32", "conv_wgrad.tiled_c64_w8"):
        for dtype in ("bf16", "f32"):
            label = bench.hip_kernel_label(kind, dtype)
            assert ("_f32_" in label) == (dtype == "f32"), label
            concrete = label.replace("2|0", "2").replace("XF", "0").replace("ddg::", "void ddg::") + "(args)"
            assert ps.kind_of(concrete) == kind, (label, ps.kind_of(concrete))
    assert bench.hip_kernel_label("bn_apply", "f32").endswith("<float, U>")
    assert bench.hip_kernel_label("sgd", "bf16") == bench.HIP_KERNEL_OF.get("sgd", "sgd")
