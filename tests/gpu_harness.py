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
                        loose=2e-2, deriv_tol=None, say=None, forward_streams=False, adam=None, lr_of=None,
                        stale_jacobian=False, per_iteration=None, store_bf16=None):
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
    oracle = orc.OracleNet.from_workload(wl, dtype="f64", stale_jacobian=stale_jacobian, store_bf16=store_bf16)
    init_both(wl, mods, oracle, perturb_bn)
    if adam:   # (beta1, beta2, eps): Algorithm 2 instead of momentum SGD, on both sides
        oracle.set_adam(True, *adam)
        pipe.set_optimizer(ddg.DDG_OPT_ADAM, *adam)
    errs = {k: [] for k in ("loss", "h", "params", "velocity", "grad", "delta")}
    report = []
    loss_dev = torch.zeros(1, dtype=torch.float32, device="cuda")
    for t in range(steps):
        seen = {k: len(v) for k, v in errs.items()}
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
        if per_iteration:   # the largest relative error of each kind in this iteration
            per_iteration(f"  {wl.name} t={t}: " + ", ".join(
                f"{k} {max(e for e, _ in v[seen[k]:]):.2e}" for k, v in errs.items() if len(v) > seen[k]))
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


def run_pipeline_three_way(wl, steps, arith="f64", say=None, second_rounded=None, teacher_forced=True,
                           perturb_bn=False):
    """The HIP pipeline next to two oracles on the same seeded inputs, from the same weights:
      rounded  the oracle in the HIP path's storage precision (bf16 workloads: the bf16-storage
               mode; fp32 workloads: the oracle computing in fp32), arithmetic `arith`;
      plain    the oracle with no rounding of stored tensors (fp32 workloads: in fp64).
    second_rounded: optionally a third oracle, the rounded one in another arithmetic ("f32"): the
    distance between the two rounded oracles is how far two straightforward implementations in
    the same storage precision lie apart by the order of their sums alone.
    Weights and velocities of all sides are set to the rounded oracle's before every iteration
    (teacher_forced), so every iteration's distance is that iteration's own.

    Returns (report, dist): report lists structural failures (gradient present on one side
    only, mailbox iteration stamps); dist[kind][pair] is a list of (relative L2 error, name) with
    kind in loss / h / delta / grad / params / velocity and pair in hip_rounded, hip_plain,
    rounded_plain (and rounded2_rounded); dist[kind]["norm_ratio"] lists |HIP| / |rounded| per
    tensor (a zero, or a wrongly scaled, result shows there even where the directions of two
    correct results have decorrelated). Assertions are the caller's."""
    K = wl.K
    st = [torch.cuda.Stream() for _ in range(K)]
    pipe = ddg.Pipeline(descs_for(wl), [s.cuda_stream for s in st])
    mods = {k: pipe.module(k) for k in range(1, K + 1)}
    bf = wl.dtype == "bf16"
    rounded = orc.OracleNet.from_workload(wl, dtype=arith if bf else "f32", store_bf16=bf)
    plain = orc.OracleNet.from_workload(wl, dtype=arith if bf else "f64", store_bf16=False)
    others = {"plain": plain}
    if second_rounded:
        others["rounded2"] = orc.OracleNet.from_workload(wl, dtype=second_rounded, store_bf16=bf)
    init_both(wl, mods, rounded, perturb_bn=perturb_bn)
    for o in others.values():
        for m in wl.modules:
            o.set_params(m.k, rounded.get_params(m.k))
    kinds = ("loss", "h", "delta", "grad", "params", "velocity")
    pairs = ("hip_rounded", "hip_plain", "rounded_plain") + (("rounded2_rounded",) if second_rounded else ())
    dist = {k: {p: [] for p in pairs + ("norm_ratio",)} for k in kinds}
    report = []
    loss_dev = torch.zeros(1, dtype=torch.float32, device="cuda")

    def book(kind, name, hip, rnd, pln, rnd2=None):
        dist[kind]["norm_ratio"].append((float(np.linalg.norm(np.asarray(hip, np.float64).ravel()) /
                                               max(np.linalg.norm(np.asarray(rnd, np.float64).ravel()), 1e-300)), name))
        dist[kind]["hip_rounded"].append((rel_err(hip, rnd), name))
        dist[kind]["hip_plain"].append((rel_err(hip, pln), name))
        dist[kind]["rounded_plain"].append((rel_err(rnd, pln), name))
        if rnd2 is not None:
            dist[kind]["rounded2_rounded"].append((rel_err(rnd2, rnd), name))

    for t in range(steps):
        x, y = wk.minibatch(wl, t)
        xd = to_dev_nhwc(x, wl)
        yd = torch.from_numpy(y).to("cuda")
        if bf:
            x = from_dev_nhwc(xd)
        if teacher_forced and t > 0:
            for m in wl.modules:
                p, v = rounded.get_params(m.k), rounded.get_velocity(m.k)
                mods[m.k].set_params(p.astype(np.float32)); mods[m.k].set_velocity(v.astype(np.float32))
                for o in others.values():
                    o.set_params(m.k, p); o.set_velocity(m.k, v)
        torch.cuda.synchronize()
        pipe.step(xd, yd, wl.lr, loss_dev)
        pipe.sync()
        l_r = rounded.ddg_step(x, y, wl.lr)
        l_o = {n: o.ddg_step(x, y, wl.lr) for n, o in others.items()}
        l_g = float(loss_dev.cpu()[0])
        if say:
            say(f"  {wl.name} t={t}: loss HIP {l_g:.6f} rounded {l_r:.6f} plain {l_o['plain']:.6f}")
        book("loss", f"t={t} loss", [l_g], [l_r], [l_o["plain"]], [l_o["rounded2"]] if second_rounded else None)
        for k in range(1, K):
            book("h", f"t={t} h_{k}", nhwc_np_to_nchw(pipe.get_h(k)), rounded.get_h(k), plain.get_h(k),
                 others["rounded2"].get_h(k) if second_rounded else None)
            d_g, ts_g = pipe.get_delta(k)
            d_r, ts_r = rounded.get_delta(k)
            d_p, ts_p = plain.get_delta(k)
            if not (ts_g == ts_r == ts_p):
                report.append(f"t={t} delta_{k}: iterations {ts_g}/{ts_r}/{ts_p}")
            elif ts_r >= 0:
                book("delta", f"t={t} delta_{k}", nhwc_np_to_nchw(d_g), d_r, d_p,
                     others["rounded2"].get_delta(k)[0] if second_rounded else None)
        for m in wl.modules:
            g, r, e = mods[m.k].get_grad(), rounded.get_grad(m.k), plain.get_grad(m.k)
            if (g is None) != (r is None):
                report.append(f"t={t} module {m.k}: gradient present on one side only")
            if g is None or r is None:
                continue
            r2 = others["rounded2"] if second_rounded else None
            for kind, a, b, c, d in (("grad", g, r, e, r2.get_grad(m.k) if r2 else None),
                                     ("params", mods[m.k].get_params(), rounded.get_params(m.k), plain.get_params(m.k),
                                      r2.get_params(m.k) if r2 else None),
                                     ("velocity", mods[m.k].get_velocity(), rounded.get_velocity(m.k), plain.get_velocity(m.k),
                                      r2.get_velocity(m.k) if r2 else None)):
                sp = [split_params(wl, m, v) if v is not None else None for v in (a, b, c, d)]
                for i, (name, av) in enumerate(sp[0]):
                    if np.linalg.norm(sp[2][i][1]) < 1e-9:
                        continue
                    book(kind, f"t={t} {kind} {name}", av, sp[1][i][1], sp[2][i][1], sp[3][i][1] if sp[3] else None)
    pipe.close()
    if say:
        for kind in kinds:
            if not dist[kind]["hip_rounded"]:
                continue
            say(f"{wl.name} {wl.dtype} steps={steps} {kind}: " + ", ".join(
                f"{p} med {np.median([e for e, _ in dist[kind][p]]):.2e} max {max(e for e, _ in dist[kind][p]):.2e}"
                for p in pairs))
    return report, dist


def med(lst):
    return float(np.median([e for e, _ in lst])) if lst else 0.0


def worst(lst):
    return max((e for e, _ in lst), default=0.0)
