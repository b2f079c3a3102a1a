#!/usr/bin/env python3
"""Throughput of the DDG module-step path on one MI355X.

A step is one DDG iteration of the whole pipeline (forward of all K modules, delayed
backward with re-forward, momentum-SGD update) on one synthetic minibatch that is already
resident in HBM. Prints ONE JSON line: images/sec, plus the roofline position of the kernel
family that takes the most time and the CPU oracle timed on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet110_k4]
"""
from __future__ import annotations

import argparse
import json
import re
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


# profile kind -> the HIP kernel it times (as rocprofv3 names it)
HIP_KERNEL_OF = {
    "conv_fprop.tiled_c16_w32": "ddg::conv3x3_tiled_kernel<16, 32, 1, XF>",
    "conv_fprop.tiled_c32_w16": "ddg::conv3x3_tiled_kernel<32, 16, 1, XF>",
    "conv_fprop.tiled_c64_w8": "ddg::conv3x3_tiled_kernel<64, 8, 1, XF>",
    "conv_dgrad.tiled_c16_w32": "ddg::conv3x3_tiled_kernel<16, 32, 2|0, XF>",
    "conv_dgrad.tiled_c32_w16": "ddg::conv3x3_tiled_kernel<32, 16, 2|0, XF>",
    "conv_dgrad.tiled_c64_w8": "ddg::conv3x3_tiled_kernel<64, 8, 2|0, XF>",
    "conv_bwd_pair.tiled_c16_w32": "ddg::bwd_pair_kernel<16, 32, 2|0, XF>",
    "conv_bwd_pair.tiled_c32_w16": "ddg::bwd_pair_kernel<32, 16, 2|0, XF>",
    "conv_bwd_pair.tiled_c64_w8": "ddg::bwd_pair_kernel<64, 8, 2|0, XF>",
    "bn_apply": "ddg::bn_apply_chunk_kernel<bf16_t, U>",
    "conv_wgrad.tiled_c16_w32": "ddg::wgrad_tiled_kernel<16, 16, 32, 1, 3>",
    "conv_wgrad.tiled_c32_w16": "ddg::wgrad_tiled_kernel<32, 32, 16, 1, 3>",
    "conv_wgrad.tiled_c64_w8": "ddg::wgrad_tiled_kernel<64, 64, 8, 1, 3>",
    "conv_wgrad.tiled_stride2": "ddg::wgrad_tiled_kernel<Cin, 2*Cin, W, 2, R>",
    "conv_fprop.wide": "ddg::conv_wide_kernel<1, XFORM, BK, R>",
    "conv_dgrad.wide": "ddg::conv_wide_kernel<0|2, false, BK, R>",
    "conv_wgrad.wide": "ddg::wgrad_wide_kernel",
    "conv_fprop.generic": "ddg::conv_mfma_kernel<T, MB, NB, false, VEC>",
    "conv_dgrad.generic": "ddg::conv_mfma_kernel<T, MB, NB, true, VEC>",
    "conv_wgrad.generic": "ddg::wgrad_mfma_vec_kernel<T> / wgrad_mfma_kernel<T>",
}


def hip_kernel_label(kind, dtype):
    """The HIP kernel a profile kind times, as rocprofv3 names it (the fp32 instances of the
    LDS-tiled kernels have names of their own)."""
    name = HIP_KERNEL_OF.get(kind, kind)
    if dtype == "f32":
        m = re.match(r"conv_(fprop|dgrad|bwd_pair|wgrad)\.tiled_c(\d+)_w(\d+)$", kind)
        if m:
            what, c, w = m.groups()
            name = {"fprop": f"ddg::conv3x3_tiled_f32_kernel<{c}, {w}, 1, XF>",
                    "dgrad": f"ddg::conv3x3_tiled_f32_kernel<{c}, {w}, 2|0, XF>",
                    "bwd_pair": f"ddg::bwd_pair_f32_kernel<{c}, {w}, 2|0, XF>",
                    "wgrad": f"ddg::wgrad_tiled_f32_kernel<{c}, {w}>"}[what]
        name = name.replace("bf16_t", "float")
    return name


def build_pipeline(wl, serial=False, forward_streams=False, stale_jacobian=False):
    import torch
    import numpy as np
    import workloads as wk
    import paper_1804_10574_amd as ddg
    from paper_1804_10574_amd.ddg import make_desc
    streams = [torch.cuda.Stream() for _ in range(wl.K)]
    # optional: forward passes on streams of their own
    fstreams = [torch.cuda.Stream() for _ in range(wl.K)] if (forward_streams and not serial) else None
    descs = []
    for m in wl.modules:
        descs.append(make_desc(wl.K, m.k, wl.batch, (m.in_c, m.in_h, m.in_w),
                               [b.as_tuple() for b in m.blocks],
                               wl.num_classes if m.blocks[-1].kind == wk.BLOCK_HEAD else 0,
                               ddg.DDG_BF16 if wl.dtype == "bf16" else ddg.DDG_F32,
                               wl.momentum, wl.weight_decay, wl.bn_eps,
                               forward_stream=fstreams[m.k - 1].cuda_stream if fstreams else None,
                               stale_jacobian=stale_jacobian))
    pipe = ddg.Pipeline(descs, None if serial else [s.cuda_stream for s in streams])
    for m in wl.modules:
        pipe.module(m.k).set_params(wk.init_module_params(wl, m).astype(np.float32))
    return pipe, streams


class SingleModule:
    """One module on its own (the ImageNet-shaped bottleneck slice): its input and the delayed
    error gradient are synthetic tensors resident in HBM; a step is ddg_forward +
    ddg_backward_delayed + ddg_update. Presents the calls the timing loop uses on a pipeline."""

    def __init__(self, wl, stale_jacobian=False, forward_stream=False):
        import torch
        import numpy as np
        import workloads as wk
        import paper_1804_10574_amd as ddg
        from paper_1804_10574_amd.ddg import make_desc
        m = wl.modules[0]
        self.wl, self.m = wl, m
        self.stream = torch.cuda.Stream()
        self.fstream = torch.cuda.Stream() if forward_stream else None
        tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        desc = make_desc(wl.K, m.k, wl.batch, (m.in_c, m.in_h, m.in_w), [b.as_tuple() for b in m.blocks], 0,
                         ddg.DDG_BF16 if wl.dtype == "bf16" else ddg.DDG_F32, wl.momentum, wl.weight_decay,
                         wl.bn_eps, stream=self.stream.cuda_stream, stale_jacobian=stale_jacobian,
                         forward_stream=self.fstream.cuda_stream if self.fstream else None)
        self.mod = ddg.Module(desc)
        self.mod.set_params(wk.init_module_params(wl, m).astype(np.float32))
        shape_in = (wl.batch, m.in_c, m.in_h, m.in_w)
        def dev(a):
            return torch.from_numpy(np.ascontiguousarray(a.transpose(0, 2, 3, 1))).to(torch.float32).cuda().to(tdt).contiguous()
        self.h = [dev(wk.normal(wl.seed, 100 + i, int(np.prod(shape_in))).reshape(shape_in)) for i in range(4)]
        self.delta = [dev(wk.synthetic_delta(wl, m, i)) for i in range(4)]
        self.h_out = torch.empty((wl.batch, m.out_h, m.out_w, m.out_c), dtype=tdt, device="cuda")
        self.d_out = torch.empty_like(self.h[0])
        self.t = 0

    def step(self, i):
        self.mod.forward(self.t, self.h[i % 4], self.h_out)
        self.mod.backward_delayed(self.t, delta_in=self.delta[i % 4], delta_out=self.d_out)
        self.mod.update(self.t, self.wl.lr)
        self.t += 1

    def set_optimizer(self, *a):
        self.mod.set_optimizer(*a)

    def modules(self):
        return [self.mod]

    def sync(self):
        self.mod.sync()

    def close(self):
        self.mod.close()


def cpu_baseline_single(wl_name, sample_batch):
    """The CPU oracle on the single-module workload at a reduced batch: K warm-up iterations
    (fill the ring), then one steady-state forward + delayed backward + update."""
    import numpy as np
    import workloads as wk
    from oracle import ddg_oracle as orc
    wl = wk.get_workload(wl_name, batch=sample_batch)
    m = wl.modules[0]
    net = orc.OracleNet.from_workload(wl, dtype="f32", store_bf16=False)
    net.set_params(m.k, wk.init_module_params(wl, m))
    shape_in = (wl.batch, m.in_c, m.in_h, m.in_w)
    h = wk.normal(wl.seed, 100, int(np.prod(shape_in))).reshape(shape_in)
    delta = wk.synthetic_delta(wl, m, 0)
    def one(t):
        net.forward(m.k, t, h)
        net.backward_delayed(m.k, t, delta, None, in_shape=shape_in)
        net.update(m.k, wl.lr)
    for t in range(wl.K):
        one(t)
    t0 = time.perf_counter()
    one(wl.K)
    dt = time.perf_counter() - t0
    return {"value": sample_batch / dt, "unit": "images/sec", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{wl_name} at batch {sample_batch} (of {wk.get_workload(wl_name).batch}), "
                      f"1 steady-state step after {wl.K} warm-up steps, fp32 oracle"}


def cpu_baseline(wl_name, sample_batch, timed_steps=1):
    """The CPU oracle (fp32 instance, as it stands) on a bounded sample of the workload:
    the same network and module split at a reduced batch, K warm-up iterations to fill the
    delay rings, then `timed_steps` steady-state iterations."""
    import workloads as wk
    from oracle import ddg_oracle as orc
    wl = wk.get_workload(wl_name, batch=sample_batch)
    net = orc.OracleNet.from_workload(wl, dtype="f32", store_bf16=False)
    for m in wl.modules:
        net.set_params(m.k, wk.init_module_params(wl, m))
    x, y = wk.minibatch(wl, 0)
    for _ in range(wl.K):
        net.ddg_step(x, y, wl.lr)
    t0 = time.perf_counter()
    for _ in range(timed_steps):
        net.ddg_step(x, y, wl.lr)
    dt = time.perf_counter() - t0
    return {"value": sample_batch * timed_steps / dt, "unit": "images/sec", "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": f"{wl_name} at batch {sample_batch} (of {wk.get_workload(wl_name).batch}), "
                      f"{timed_steps} steady-state step(s) after {wl.K} warm-up steps, fp32 oracle"}


def measure(wl, args, steps, warmup):
    """Times `steps` steps of workload wl after K + warmup untimed ones and, unless switched off,
    runs the per-launch event pass. Returns the fields of the bench line that describe this
    workload (value, ms_per_step, config, roofline, kernels, ...)."""
    import numpy as np
    import torch
    import workloads as wk
    single = SingleModule(wl, args.stale_jacobian, args.forward_streams) if wl.single_module else None
    if single:
        pipe = single
    else:
        pipe, streams = build_pipeline(wl, args.serial, args.forward_streams, args.stale_jacobian)
    if args.optimizer == "adam":
        import paper_1804_10574_amd as ddg
        pipe.set_optimizer(ddg.DDG_OPT_ADAM, 0.9, 0.999, 1e-8)
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    # a few distinct minibatches, resident in HBM before the timed region
    nbuf = 4
    xs, ys = [], []
    for i in range(0 if single else nbuf):
        x, y = wk.minibatch(wl, i)
        xs.append(torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 3, 1))).to(torch.float32).cuda().to(tdt).contiguous())
        ys.append(torch.from_numpy(y).cuda())
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    def step(i):
        if single:
            single.step(i)
        else:
            pipe.step(xs[i % nbuf], ys[i % nbuf], wl.lr, loss)

    it = 0
    for _ in range(wl.K + warmup):      # fill the delay rings, then warm up
        step(it); it += 1
    pipe.sync(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(it); it += 1
    pipe.sync(); torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    final_loss = float(loss.cpu()[0])
    ms = dt / steps * 1e3
    out = {
        "value": wl.batch * steps / dt, "unit": "images/sec", "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "dtype": wl.dtype,
        "config": {"workload": wl.name, "network": wl.notes, "K": wl.K, "global_batch": wl.batch,
                   "image": "3x32x32", "classes": wl.num_classes, "streams": (2 if args.forward_streams else 1) if (args.serial or single) else (2 * wl.K - 1 if args.forward_streams else wl.K),
                   "optimizer": args.optimizer,
                   "gradient": "stale Jacobian (Eq. 6-7 as printed)" if args.stale_jacobian else "re-forward with current weights",
                   "parallelism": "K modules as HIP streams on one GPU"},
        "final_loss": final_loss,
    }
    if single:
        m = wl.modules[0]
        out["config"].update({"image": None, "classes": None, "module": f"k={m.k} of K={wl.K} (delay {wl.K - m.k})",
                              "module_input": f"{m.in_c}x{m.in_h}x{m.in_w}",
                              "parallelism": "one module, one HIP stream; synthetic input and delayed error gradient"})
        out.pop("final_loss")

    if not args.no_roofline:
        # second pass with per-launch HIP events on each module's stream
        mods = single.modules() if single else [pipe.module(k) for k in range(1, wl.K + 1)]
        for m in mods:
            m.profile_reset(); m.profile_enable(True)
        psteps = max(2, min(5, steps))
        for _ in range(psteps):
            step(it); it += 1
        pipe.sync()
        fam = {}
        per_module = []      # summed kernel time and launches of each module's stream, per step
        for m in mods:
            tot_ms, tot_n = 0.0, 0
            for name, (n, tms, nbytes, flops) in m.profile_read().items():
                a = fam.setdefault(name, [0, 0.0, 0.0, 0.0])
                a[0] += n; a[1] += tms; a[2] += nbytes; a[3] += flops
                tot_ms += tms; tot_n += n
            per_module.append({"kernel_ms_per_step": tot_ms / psteps, "launches_per_step": tot_n / psteps})
            m.profile_enable(False)
        peak_tf = MFMA_PEAK_TFLOPS[wl.dtype]

        def entry(n, tms, nbytes, flops):
            e = {"launches_per_step": n / psteps, "avg_us": tms / n * 1e3, "ms_per_step": tms / psteps}
            if nbytes > 0 and tms > 0:
                e["algorithmic_MB_per_launch"] = nbytes / n / 1e6
                e["GBps"] = nbytes / 1e9 / (tms / 1e3)
            if flops > 0 and tms > 0:
                e["TFLOPs"] = flops / 1e12 / (tms / 1e3)
            if nbytes > 0 and tms > 0:
                # the roof that binds this kind: the time its algorithmic bytes need at the HBM
                # peak against the time its flops need at the MFMA peak of its operand type; the
                # fraction is that time over the measured one
                t_hbm = nbytes / (HBM_PEAK_GBS * 1e9)
                t_mfma = flops / (peak_tf * 1e12)
                e["bound"] = "mfma" if t_mfma > t_hbm else "hbm"
                e["frac_of_min_roof"] = max(t_hbm, t_mfma) / (tms / 1e3)
                if flops > 0:
                    e["mfma_frac"] = e["TFLOPs"] / peak_tf
                e["hbm_frac"] = e["GBps"] / HBM_PEAK_GBS
            return e

        # the library books one kind per kernel ("family.instance"); families are their sums
        kernels = {name: entry(*v) for name, v in fam.items() if v[0]}
        famsum = {}
        for name, v in fam.items():
            a = famsum.setdefault(name.split(".")[0], [0, 0.0, 0.0, 0.0])
            for i in range(4):
                a[i] += v[i]
        families = {name: entry(*v) for name, v in famsum.items() if v[0]}
        dom = max((k for k in kernels if "GBps" in kernels[k]), key=lambda k: kernels[k]["ms_per_step"])
        d = kernels[dom]
        n, tms, nbytes, flops = fam[dom]
        ai = flops / nbytes if nbytes else 0.0
        ridge = peak_tf * 1e12 / (HBM_PEAK_GBS * 1e9)
        if flops and ai >= ridge:
            roof = {"bound": "mfma", "achieved": d["TFLOPs"], "peak": peak_tf, "unit": "TFLOP/s"}
        else:
            roof = {"bound": "hbm", "achieved": d["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        # measured HBM bytes per launch of this kernel: from the committed counter summary of the
        # same workload (two rocprofv3 --pmc passes, calibrated by the library's copy kernel);
        # traffic_stale: the kernel sources have changed since that summary was taken
        roof["traffic"] = None
        here = os.path.dirname(os.path.abspath(__file__))
        tpath = os.path.join(here, "profiles", f"hbm_traffic_{wl.name}_{wl.dtype}.txt")
        if os.path.exists(tpath):
            from paper_1804_10574_amd.profile_summary import read_traffic_table, read_source_digest, source_digest
            roof["traffic"] = read_traffic_table(tpath).get(dom)
            roof["traffic_source"] = os.path.relpath(tpath, here)
            roof["traffic_stale"] = read_source_digest(tpath) != source_digest()
        roof["kernel"] = dom
        roof["hip_kernel"] = hip_kernel_label(dom, wl.dtype)
        roof["avg_launch_us"] = d["avg_us"]
        roof["launches_per_step"] = d["launches_per_step"]
        roof["algorithmic_bytes_per_launch"] = nbytes / n
        if flops:
            roof["arithmetic_intensity_flop_per_byte"] = ai
            roof["mfma_frac"] = d["TFLOPs"] / peak_tf
        out["roofline"] = roof
        out["per_module"] = per_module
        out["kernels"] = kernels
        out["families"] = families
        convs = [k for k in ("conv_fprop", "conv_dgrad", "conv_wgrad", "conv_bwd_pair") if k in families]
        conv_ms = sum(famsum[k][1] for k in convs)
        out["conv_mfma_util"] = sum(famsum[k][3] for k in convs) / 1e12 / (conv_ms / 1e3) / peak_tf if conv_ms else None
        out["conv_hbm_frac"] = sum(famsum[k][2] for k in convs) / 1e9 / (conv_ms / 1e3) / HBM_PEAK_GBS if conv_ms else None
        # all conv kinds against the roof that binds each of them
        out["conv_frac_of_min_roof"] = (sum(max(fam[k][2] / (HBM_PEAK_GBS * 1e9), fam[k][3] / (peak_tf * 1e12))
                                            for k in fam if k.split(".")[0] in convs) / (conv_ms / 1e3)) if conv_ms else None
        bn = [k for k in ("bn_apply", "bn_bwd_reduce", "bn_bwd_apply") if k in families]
        bn_ms = sum(famsum[k][1] for k in bn)
        out["bn_hbm_frac"] = sum(famsum[k][2] for k in bn) / 1e9 / (bn_ms / 1e3) / HBM_PEAK_GBS if bn_ms else None
        out["algorithmic_GFLOP_per_step"] = sum(v[3] for v in fam.values()) / psteps / 1e9
        out["algorithmic_GB_per_step"] = sum(v[2] for v in fam.values()) / psteps / 1e9
    pipe.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet110_k4")
    ap.add_argument("--batch", type=int, default=0,
                    help="run the workload at another batch than the one it is specified with (0: as specified); "
                         "for the step-time-against-batch fit, not a bench line: implies --no-secondary and --no-cpu-baseline")
    ap.add_argument("--cpu-sample-batch", type=int, default=0,
                    help="batch of the oracle's timed sample (0: the workload's own batch; K warm-up + 1 timed "
                         "iteration, about 30 s of CPU work for resnet110_k4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the short measurement of the ImageNet-shaped single module that the default "
                         "run adds to its line")
    ap.add_argument("--optimizer", choices=["sgd", "adam"], default="sgd",
                    help="momentum SGD (Algorithm 1, the headline configuration) or Adam (Algorithm 2, "
                         "beta1 0.9, beta2 0.999, eps 1e-8)")
    ap.add_argument("--stale-jacobian", action="store_true",
                    help="Eq. 6-7 read literally (tapes and weight snapshots per ring slot, no re-forward); "
                         "not the headline configuration")
    ap.add_argument("--serial", action="store_true", help="all modules on one stream")
    ap.add_argument("--forward-streams", action="store_true",
                    help="give each module's forward pass a stream of its own (2K-1 streams; "
                         "slower than K streams on this GPU, kept for comparison)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (modules are concurrent streams on one "
              "device); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wk
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = wk.get_workload(args.workload)
    if args.batch and args.batch != wl.batch:
        wl = wk.get_workload(args.workload, batch=args.batch)
        wl.name = f"{wl.name}@batch{args.batch}"     # named in config.workload: not the specified configuration
        args.no_secondary = args.no_cpu_baseline = True
    res = measure(wl, args, args.steps, args.warmup)
    out = {"metric": "DDG module images/sec on 1 MI355X", "value": res.pop("value"), "unit": res.pop("unit"),
           "n_gpus": 1, "steps": res.pop("steps"), "warmup": res.pop("warmup"), "ms_per_step": res.pop("ms_per_step"),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": res.pop("dtype"),
           "data": "synthetic"}
    out.update(res)
    if wl.name == "resnet110_k4" and not args.no_secondary:
        # the benchmark's fifth configuration (one ImageNet-shaped module of 23 bottleneck blocks,
        # the GEMM-class kernels), measured in the same run: 30 timed steps as specified
        wl2 = wk.get_workload("r101_stage3_k4m2")
        r2 = measure(wl2, args, 30, 5)
        sec = {k: r2[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "dtype", "config") if k in r2}
        for k in ("roofline", "conv_mfma_util", "conv_frac_of_min_roof", "bn_hbm_frac", "algorithmic_GFLOP_per_step",
                  "algorithmic_GB_per_step"):
            if k in r2:
                sec[k] = r2[k]
        if "kernels" in r2:   # the kinds that take 3 % of the step or more
            sec["kernels"] = {k: v for k, v in r2["kernels"].items() if v["ms_per_step"] >= 0.03 * r2["ms_per_step"]}
        out["secondary"] = sec
    if not args.no_cpu_baseline:
        if wl.single_module:
            out["cpu_baseline"] = cpu_baseline_single(wl.name, min(args.cpu_sample_batch or 2, 2))
        else:
            out["cpu_baseline"] = cpu_baseline(wl.name, args.cpu_sample_batch or wl.batch, timed_steps=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
