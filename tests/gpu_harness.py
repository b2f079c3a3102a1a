"""Helpers for the GPU parity tests: build the HIP modules / pipeline from a workload,
move seeded inputs to the device in the boundary's layout, and compare with the oracle.

PyTorch is used for device memory and streams only."""
import numpy as np
import torch

import workloads as wk
import paper_1804_10574_amd as ddg
from paper_1804_10574_amd.ddg import make_desc
from oracle import ddg_oracle as orc


def tdtype(wl):
    return torch.bfloat16 if wl.dtype == "bf16" else torch.float32


def compute_enum(wl):
    return ddg.DDG_BF16 if wl.dtype == "bf16" else ddg.DDG_F32


def to_dev_nhwc(a_nchw, wl):
    """float64 NCHW numpy -> device NHWC tensor in the workload's activation type."""
    t = torch.from_numpy(np.ascontiguousarray(a_nchw.transpose(0, 2, 3, 1))).to(torch.float32)
    return t.to("cuda").to(tdtype(wl)).contiguous()


def from_dev_nhwc(t):
    """device NHWC tensor -> float64 NCHW numpy"""
    return t.to(torch.float32).cpu().numpy().astype(np.float64).transpose(0, 3, 1, 2)


def nhwc_np_to_nchw(a):
    return np.asarray(a, np.float64).transpose(0, 3, 1, 2)


def descs_for(wl, streams=None, dry_run=False, batch=None, fstreams=None, stale_jacobian=False):
    out = []
    for i, m in enumerate(wl.modules):
        out.append(make_desc(wl.K, m.k, batch or wl.batch, (m.in_c, m.in_h, m.in_w),
                             [b.as_tuple() for b in m.blocks],
                             wl.num_classes if m.blocks[-1].kind == wk.BLOCK_HEAD else 0,
                             compute_enum(wl), wl.momentum, wl.weight_decay, wl.bn_eps,
                             stream=(streams[i] if streams else None), dry_run=dry_run,
                             forward_stream=(fstreams[i] if fstreams else None),
                             stale_jacobian=stale_jacobian))
    return out


def rel_err(a, b):
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-12))


def split_params(wl, m, flat):
    """-> list of (name, array) per parameter tensor of module m."""
    out, off = [], 0
    for bi, b in enumerate(m.blocks):
        for name, shp in wk.block_param_shapes(b, wl.num_classes):
            n = int(np.prod(shp))
            out.append((f"m{m.k}.b{bi}.{name}", np.asarray(flat[off:off + n])))
            off += n
    assert off == len(flat)
    return out


def compare_params(wl, m, got, ref, tol, what, report):
    worst = 0.0
    for (name, g), (_, r) in zip(split_params(wl, m, got), split_params(wl, m, ref)):
        if np.linalg.norm(r) < 1e-10 and np.linalg.norm(g) < 1e-7:
            continue
        e = rel_err(g, r)
        worst = max(worst, e)
        if e > tol:
            report.append(f"{what} {name}: rel err {e:.3e} > {tol:g}")
    return worst


def init_both(wl, pipe_or_mods, oracle, perturb_bn=True):
    """Same seeded initial parameters into the oracle and the HIP modules. With bf16 conv
    operands the fp32 master weights are identical on both sides."""
    for m in wl.modules:
        th = wk.init_module_params(wl, m, perturb_bn=perturb_bn).astype(np.float32)
        oracle.set_params(m.k, th.astype(np.float64))
        pipe_or_mods[m.k].set_params(th)


DERIV_KINDS = ("grad", "delta")          # contain the ReLU derivative (discontinuous)
SMOOTH_KINDS = ("loss", "h", "params", "velocity")


def run_pipeline_parity(wl, steps, tol, streams=True, perturb_bn=True, teacher_forced=True,
                        loose=0.25, deriv_tol=None, say=None, forward_streams=False, adam=None, lr_of=None,
                        stale_jacobian=False):
    """Run `steps` DDG iterations on the HIP pipeline and on the float64 oracle with the same
    seeded inputs and compare per tensor (relative L2 error).

    teacher_forced: before every iteration the GPU's weights and velocities are set to the
    oracle's, so each iteration's error is the kernels' own and not the accumulated divergence
    of two trajectories. The mailboxes and input rings stay the GPU's own.

    Returns (failures, stats). Criteria (relative L2 error per tensor):
      * loss and forward outputs h: every iteration within tol.
      * gradients g, error gradients delta, and what the update makes of them (velocity,
        updated weights) contain the ReLU derivative, a discontinuous function of the
        pre-activations: one whose sign is decided within rounding distance of zero may fall
        on either side in any finite-precision implementation, which changes that element's
        derivative by O(1). For these the median over (iteration, tensor) must be within
        `deriv_tol` (default: tol) and every single value within `loose`: a wrong kernel is
        wrong in every iteration, a sign event is rare and bounded.
      * without teacher forcing everything is held to tol at every iteration.
    """
    K = wl.K
    st = [torch.cuda.Stream() for _ in range(K)] if streams else None
    fst = [torch.cuda.Stream() for _ in range(K)] if (streams and forward_streams) else None
    pipe = ddg.Pipeline(descs_for(wl, fstreams=[s.cuda_stream for s in fst] if fst else None,
                                  stale_jacobian=stale_jacobian),
                        [s.cuda_stream for s in st] if st else None)
    mods = {k: pipe.module(k) for k in range(1, K + 1)}
    oracle = orc.OracleNet.from_workload(wl, dtype="f64", stale_jacobian=stale_jacobian)
    init_both(wl, mods, oracle, perturb_bn)
    if adam:   # (beta1, beta2, eps): Algorithm 2 instead of momentum SGD, on both sides
        oracle.set_adam(True, *adam)
        pipe.set_optimizer(ddg.DDG_OPT_ADAM, *adam)
    errs = {k: [] for k in ("loss", "h", "params", "velocity", "grad", "delta")}
    report = []
    loss_dev = torch.zeros(1, dtype=torch.float32, device="cuda")
    for t in range(steps):
        lr = lr_of(t) if lr_of else wl.lr       # the step-size schedule is the caller's
        x, y = wk.minibatch(wl, t)
        xd = to_dev_nhwc(x, wl)
        yd = torch.from_numpy(y).to("cuda")
        if wl.dtype == "bf16":
            x = from_dev_nhwc(xd)          # both sides see the same rounded images
        if teacher_forced and t > 0:
            for m in wl.modules:
                mods[m.k].set_params(oracle.get_params(m.k).astype(np.float32))
                mods[m.k].set_velocity(oracle.get_velocity(m.k).astype(np.float32))
                if adam:
                    mods[m.k].set_moment2(oracle.get_moment2(m.k).astype(np.float32))
                    mods[m.k].set_update_count(oracle.get_updates(m.k))
        torch.cuda.synchronize()
        pipe.step(xd, yd, lr, loss_dev)
        pipe.sync()
        ref_loss = oracle.ddg_step(x, y, lr)
        got_loss = float(loss_dev.cpu()[0])
        errs["loss"].append((abs(got_loss - ref_loss) / max(abs(ref_loss), 1e-12), f"t={t} loss"))
        for m in wl.modules:
            g, r = mods[m.k].get_grad(), oracle.get_grad(m.k)
            if (g is None) != (r is None):
                report.append(f"t={t} module {m.k}: gradient present on one side only")
                continue
            if g is None:
                continue
            if adam and mods[m.k].get_update_count() != oracle.get_updates(m.k):
                report.append(f"t={t} module {m.k}: update count {mods[m.k].get_update_count()} vs {oracle.get_updates(m.k)}")
            extra = (("velocity", mods[m.k].get_moment2(), oracle.get_moment2(m.k)),) if adam else ()
            for kind, a, b in (("grad", g, r), ("params", mods[m.k].get_params(), oracle.get_params(m.k)),
                               ("velocity", mods[m.k].get_velocity(), oracle.get_velocity(m.k))) + extra:
                for (name, av), (_, bv) in zip(split_params(wl, m, a), split_params(wl, m, b)):
                    if np.linalg.norm(bv) < 1e-9 and np.linalg.norm(av) < 1e-6:
                        continue
                    errs[kind].append((rel_err(av, bv), f"t={t} {kind} {name}"))
        for k in range(1, K):
            errs["h"].append((rel_err(nhwc_np_to_nchw(pipe.get_h(k)), oracle.get_h(k)), f"t={t} h_{k}"))
            d_ref, ts_ref = oracle.get_delta(k)
            d_got, ts_got = pipe.get_delta(k)
            if ts_ref != ts_got:
                report.append(f"t={t} delta_{k}: iteration {ts_got} vs oracle {ts_ref}")
            elif ts_ref >= 0:
                errs["delta"].append((rel_err(nhwc_np_to_nchw(d_got), d_ref), f"t={t} delta_{k}"))
    pipe.close()
    stats = {}
    for kind, lst in errs.items():
        if not lst:
            continue
        v = np.array([e for e, _ in lst])
        stats[kind] = {"median": float(np.median(v)), "max": float(v.max()), "n": len(lst)}
        strict = kind in ("loss", "h") or not teacher_forced
        dtol = tol if kind == "params" or deriv_tol is None else deriv_tol
        if strict:
            for e, name in lst:
                if not e <= tol:
                    report.append(f"{name}: rel err {e:.3e} > {tol:g}")
        else:
            if not np.median(v) <= dtol:
                report.append(f"{kind}: median rel err {np.median(v):.3e} > {dtol:g}")
            for e, name in lst:
                if not e <= loose:
                    report.append(f"{name}: rel err {e:.3e} > loose bound {loose:g}")
    if say:
        say(f"{wl.name} {wl.dtype} steps={steps} teacher_forced={teacher_forced}: " +
            ", ".join(f"{k} med {v['median']:.2e} max {v['max']:.2e}" for k, v in stats.items()))
    return report, stats


def run_pipeline_envelope(wl, steps, tol, factor=2.0, say=None):
    """Parity for networks too deep for a fixed tolerance on derivative-like tensors (fp32: the
    "rounded" oracle below is the oracle computing in fp32, and every h is held to tol).

    Three runs of the same DDG iterations from the same weights: the HIP pipeline, the oracle in
    its bf16-storage mode, and the oracle in plain fp64 (no rounding anywhere: the exact result).
    Both rounded runs are measured against the exact one. The HIP path passes when, per kind of
    tensor, its median distance from the exact result is at most `factor` times the bf16-mode
    oracle's own distance plus tol: it is then as close to the truth as a straightforward bf16
    implementation of the same arithmetic is. Loss and the first module's output are also held
    to tol against the bf16-mode oracle directly. Weights and velocities of all three are reset
    to the bf16-mode oracle's after every iteration."""
    K = wl.K
    st = [torch.cuda.Stream() for _ in range(K)]
    pipe = ddg.Pipeline(descs_for(wl), [s.cuda_stream for s in st])
    mods = {k: pipe.module(k) for k in range(1, K + 1)}
    if wl.dtype == "bf16":
        rounded = orc.OracleNet.from_workload(wl, dtype="f64", store_bf16=True)
    else:
        rounded = orc.OracleNet.from_workload(wl, dtype="f32", store_bf16=False)
    exact = orc.OracleNet.from_workload(wl, dtype="f64", store_bf16=False)
    init_both(wl, mods, rounded, perturb_bn=False)
    for m in wl.modules:
        exact.set_params(m.k, rounded.get_params(m.k).astype(np.float64))
    gpu_e = {k: [] for k in ("h", "grad", "delta")}
    orc_e = {k: [] for k in ("h", "grad", "delta")}
    report = []
    loss_dev = torch.zeros(1, dtype=torch.float32, device="cuda")
    for t in range(steps):
        x, y = wk.minibatch(wl, t)
        xd = to_dev_nhwc(x, wl)
        yd = torch.from_numpy(y).to("cuda")
        x = from_dev_nhwc(xd)
        if t > 0:
            for m in wl.modules:
                p, v = rounded.get_params(m.k), rounded.get_velocity(m.k)
                p, v = p.astype(np.float64), v.astype(np.float64)
                mods[m.k].set_params(p.astype(np.float32)); mods[m.k].set_velocity(v.astype(np.float32))
                exact.set_params(m.k, p); exact.set_velocity(m.k, v)
        torch.cuda.synchronize()
        pipe.step(xd, yd, wl.lr, loss_dev)
        pipe.sync()
        l_r = rounded.ddg_step(x, y, wl.lr)
        exact.ddg_step(x, y, wl.lr)
        l_g = float(loss_dev.cpu()[0])
        if not abs(l_g - l_r) <= tol * abs(l_r):
            report.append(f"t={t} loss {l_g} vs {l_r}")
        for k in range(1, 2 if wl.dtype == "bf16" else K):
            e1 = rel_err(nhwc_np_to_nchw(pipe.get_h(k)), rounded.get_h(k))
            if not e1 <= tol:
                report.append(f"t={t} h_{k}: rel err {e1:.3e} > {tol:g}")
        for k in range(1, K):
            gpu_e["h"].append(rel_err(nhwc_np_to_nchw(pipe.get_h(k)), exact.get_h(k)))
            orc_e["h"].append(rel_err(rounded.get_h(k), exact.get_h(k)))
            d_ex, ts_ex = exact.get_delta(k)
            d_ro, ts_ro = rounded.get_delta(k)
            d_g, ts_g = pipe.get_delta(k)
            if not (ts_ex == ts_ro == ts_g):
                report.append(f"t={t} delta_{k}: iterations {ts_g}/{ts_ro}/{ts_ex}")
            elif ts_ex >= 0:
                gpu_e["delta"].append(rel_err(nhwc_np_to_nchw(d_g), d_ex))
                orc_e["delta"].append(rel_err(d_ro, d_ex))
        for m in wl.modules:
            g, r, e = mods[m.k].get_grad(), rounded.get_grad(m.k), exact.get_grad(m.k)
            if (g is None) != (r is None):
                report.append(f"t={t} module {m.k}: gradient present on one side only")
            if g is None or r is None:
                continue
            for (name, gv), (_, rv), (_, ev) in zip(split_params(wl, m, g), split_params(wl, m, r),
                                                    split_params(wl, m, e)):
                if np.linalg.norm(ev) < 1e-9:
                    continue
                gpu_e["grad"].append(rel_err(gv, ev))
                orc_e["grad"].append(rel_err(rv, ev))
    pipe.close()
    stats = {}
    for kind in gpu_e:
        if not gpu_e[kind]:
            continue
        a, b = float(np.median(gpu_e[kind])), float(np.median(orc_e[kind]))
        stats[kind] = (a, b)
        if not a <= factor * b + tol:
            report.append(f"{kind}: median distance from exact {a:.3e} (HIP) vs {b:.3e} (bf16-mode oracle)")
    if say:
        say(f"{wl.name} envelope steps={steps}: " +
            ", ".join(f"{k} HIP {a:.2e} / oracle-bf16 {b:.2e}" for k, (a, b) in stats.items()))
    return report, stats
