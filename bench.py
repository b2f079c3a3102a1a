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
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def traffic_model(wl):
    """Algorithmic bytes and flops per kernel family for one steady-state step.

    Bytes: every operand read once and every result written once in its storage type
    (conv: input + weights + output; BN/elementwise: the tensors the formula names).
    Flops: 2*M*N*K per convolution pass. Returns {family: [launches, bytes, flops]}.
    """
    import workloads as wk
    from workloads.configs import conv_units
    esz = 2 if wl.dtype == "bf16" else 4
    fam = {}

    def add(name, nbytes, flops=0.0):
        f = fam.setdefault(name, [0, 0.0, 0.0])
        f[0] += 1
        f[1] += nbytes
        f[2] += flops

    N = wl.batch
    for m in wl.modules:
        passes = 2 if m.k < wl.K else 1     # forward, and re-forward when the delay is > 0
        h, w = m.in_h, m.in_w
        first = True
        for b in m.blocks:
            if b.kind == wk.BLOCK_HEAD:
                continue
            units = conv_units(b)
            nmain = len(units) - (1 if b.projection else 0)
            ho, wo = (h - 1) // b.stride + 1, (w - 1) // b.stride + 1
            uh, uw = h, w
            main_out = []
            for ui, (name, ci, co, r, st) in enumerate(units):
                if name == "proj":
                    ih, iw = h, w
                else:
                    ih, iw = uh, uw
                p, q = (ih - 1) // st + 1, (iw - 1) // st + 1
                e_in, e_out, e_w = N * ih * iw * ci, N * p * q * co, co * ci * r * r
                flops = 2.0 * N * p * q * co * ci * r * r
                for _ in range(passes):
                    add("conv_fprop", (e_in + e_out + e_w) * esz, flops)
                    add("bn_finalize", 0)
                # backward of this unit
                add("bn_bwd_reduce", 3 * e_out * esz)          # dy, mask, z
                add("bn_bwd_finalize", 0)
                add("bn_bwd_apply", 4 * e_out * esz)           # dy, mask, z -> dz
                add("conv_wgrad", (e_in + e_out) * esz + e_w * 4, flops)
                add("wgrad_reduce", e_w * 4)
                needs_dx = not (first and m.k == 1 and (ui == 0 or name == "proj"))
                if needs_dx:
                    extra = 0
                    if name != "proj" and ui == 0 and b.kind != wk.BLOCK_STEM:
                        extra = e_in * esz * (1 if b.projection else 2)   # shortcut term (+mask)
                    add("conv_dgrad", (e_in + e_out + e_w) * esz + extra, flops)
                if name != "proj":
                    uh, uw = p, q
                    main_out.append(e_out)
            # activations: z -> relu(bn(z)) between main units; the block output reads the last
            # conv output and the shortcut (or the projection's conv output)
            e_y = N * ho * wo * b.cout
            for _ in range(passes):
                for e_mid in main_out[:-1]:
                    add("bn_apply", 2 * e_mid * esz)
                add("bn_apply", (2 if b.kind == wk.BLOCK_STEM else 3) * e_y * esz)
            h, w = ho, wo
            first = False
    return fam


def build_pipeline(wl, serial=False, one_stream_per_module=False):
    import torch
    import numpy as np
    import workloads as wk
    import paper_1804_10574_amd as ddg
    from paper_1804_10574_amd.ddg import make_desc
    streams = [torch.cuda.Stream() for _ in range(wl.K)]
    fstreams = [torch.cuda.Stream() for _ in range(wl.K)]   # forward passes on streams of their own
    descs = []
    for m in wl.modules:
        descs.append(make_desc(wl.K, m.k, wl.batch, (m.in_c, m.in_h, m.in_w),
                               [b.as_tuple() for b in m.blocks],
                               wl.num_classes if m.blocks[-1].kind == wk.BLOCK_HEAD else 0,
                               ddg.DDG_BF16 if wl.dtype == "bf16" else ddg.DDG_F32,
                               wl.momentum, wl.weight_decay, wl.bn_eps,
                               forward_stream=None if (serial or one_stream_per_module) else fstreams[m.k - 1].cuda_stream))
    pipe = ddg.Pipeline(descs, None if serial else [s.cuda_stream for s in streams])
    for m in wl.modules:
        pipe.module(m.k).set_params(wk.init_module_params(wl, m).astype(np.float32))
    return pipe, streams


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet110_k4")
    ap.add_argument("--cpu-sample-batch", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-roofline", action="store_true")
    ap.add_argument("--serial", action="store_true", help="all modules on one stream")
    ap.add_argument("--one-stream-per-module", action="store_true",
                    help="forward and delayed backward of a module share one stream")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (modules are concurrent streams on one "
              "device); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as wk
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = wk.get_workload(args.workload)
    if wl.single_module:
        raise SystemExit("bench.py times full pipelines; single-module workloads are parity cases")
    pipe, streams = build_pipeline(wl, args.serial, args.one_stream_per_module)
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    # a few distinct minibatches, resident in HBM before the timed region
    nbuf = 4
    xs, ys = [], []
    for i in range(nbuf):
        x, y = wk.minibatch(wl, i)
        xs.append(torch.from_numpy(np.ascontiguousarray(x.transpose(0, 2, 3, 1))).to(torch.float32).cuda().to(tdt).contiguous())
        ys.append(torch.from_numpy(y).cuda())
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()

    def step(i):
        pipe.step(xs[i % nbuf], ys[i % nbuf], wl.lr, loss)

    it = 0
    for _ in range(wl.K + args.warmup):      # fill the delay rings, then warm up
        step(it); it += 1
    pipe.sync(); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(it); it += 1
    pipe.sync(); torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    final_loss = float(loss.cpu()[0])
    ms = dt / args.steps * 1e3
    out = {
        "metric": "DDG module images/sec on 1 MI355X", "value": wl.batch * args.steps / dt,
        "unit": "images/sec", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "network": wl.notes, "K": wl.K, "global_batch": wl.batch,
                   "image": "3x32x32", "classes": wl.num_classes, "streams": 1 if args.serial else (wl.K if args.one_stream_per_module else 2 * wl.K - 1),
                   "parallelism": "K modules as HIP streams on one GPU"},
        "final_loss": final_loss,
    }

    if not args.no_roofline:
        # second pass with per-launch HIP events on each module's stream
        mods = [pipe.module(k) for k in range(1, wl.K + 1)]
        for m in mods:
            m.profile_reset(); m.profile_enable(True)
        psteps = max(2, min(5, args.steps))
        for _ in range(psteps):
            step(it); it += 1
        pipe.sync()
        fam_t = {}
        for m in mods:
            for name, (n, tms) in m.profile_read().items():
                a = fam_t.setdefault(name, [0, 0.0]); a[0] += n; a[1] += tms
            m.profile_enable(False)
        model = traffic_model(wl)
        kernels = {}
        for name, (n, tms) in fam_t.items():
            if n == 0:
                continue
            launches = n / psteps
            avg_ms = tms / n
            e = {"launches_per_step": launches, "avg_us": avg_ms * 1e3, "ms_per_step": tms / psteps}
            if name in model and model[name][1] > 0:
                nb, fl = model[name][1], model[name][2]
                e["algorithmic_GB_per_step"] = nb / 1e9
                e["GBps"] = nb / 1e9 / (tms / psteps / 1e3)
                if fl:
                    e["TFLOPs"] = fl / 1e12 / (tms / psteps / 1e3)
            kernels[name] = e
        dom = max((k for k in kernels if "GBps" in kernels[k]), key=lambda k: kernels[k]["ms_per_step"])
        d = kernels[dom]
        nb, fl = model[dom][1], model[dom][2]
        ai = fl / nb if nb else 0.0
        ridge = MFMA_PEAK_TFLOPS[wl.dtype] * 1e12 / (HBM_PEAK_GBS * 1e9)
        if fl and ai >= ridge:
            roof = {"bound": "mfma", "achieved": d["TFLOPs"], "peak": MFMA_PEAK_TFLOPS[wl.dtype], "unit": "TFLOP/s"}
        else:
            roof = {"bound": "hbm", "achieved": d["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof["traffic"] = None
        roof["kernel"] = dom
        roof["avg_launch_us"] = d["avg_us"]
        roof["launches_per_step"] = d["launches_per_step"]
        roof["algorithmic_bytes_per_launch"] = nb / max(model[dom][0], 1)
        if fl:
            roof["mfma_frac"] = d["TFLOPs"] / MFMA_PEAK_TFLOPS[wl.dtype]
        out["roofline"] = roof
        out["kernels"] = kernels
        conv_ms = sum(kernels[k]["ms_per_step"] for k in ("conv_fprop", "conv_dgrad", "conv_wgrad") if k in kernels)
        conv_fl = sum(model[k][2] for k in ("conv_fprop", "conv_dgrad", "conv_wgrad") if k in model)
        out["conv_mfma_util"] = conv_fl / 1e12 / (conv_ms / 1e3) / MFMA_PEAK_TFLOPS[wl.dtype] if conv_ms else None
        bn = [k for k in ("bn_apply", "bn_bwd_reduce", "bn_bwd_apply") if k in kernels]
        bn_ms = sum(kernels[k]["ms_per_step"] for k in bn)
        out["bn_hbm_frac"] = sum(model[k][1] for k in bn) / 1e9 / (bn_ms / 1e3) / HBM_PEAK_GBS if bn_ms else None

    pipe.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl.name, args.cpu_sample_batch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
