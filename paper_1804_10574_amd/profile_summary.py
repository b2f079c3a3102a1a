"""Turn rocprofv3 CSV output of a bench.py run into the short text summaries kept under profiles/.

    python -m paper_1804_10574_amd.profile_summary stats  <run_kernel_stats.csv> --steps N
    python -m paper_1804_10574_amd.profile_summary traffic <fetch counter_collection.csv> \
                                                           <write counter_collection.csv>

`stats` prints per-kernel calls, average duration and share of the kernel time; N is the number
of pipeline iterations the profiled command ran (bench.py runs K + warmup + steps + 5 when the
roofline pass is on). `traffic` prints, per kernel, the FETCH_SIZE and WRITE_SIZE counters
(KiB per dispatch, averaged over the dispatches of that kernel) and the calibrated bytes per
launch. The calibration factor of each counter is known bytes / counter reading for the library's
own copy kernel (16 bytes per thread, one 16-byte load and store each, launches below the grid
cap only), taken from the same two runs.

The kernel -> kind mapping is the one the library books its per-launch measurements under
(ddg_profile_kind_name), so that bench.py can look a kernel's traffic up by kind.
"""
import argparse
import collections
import csv
import hashlib
import os
import re
import sys


def source_digest() -> str:
    """A digest of the kernel and host sources of the library (csrc/): a counter summary carries
    the digest of the sources it was taken with, so that a reader can tell when they have
    changed since."""
    csrc = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h", ".cpp")) and name != "peaks_main.hip":    # (the measuring tool is no part of the library)
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def read_source_digest(path: str):
    for line in open(path):
        if line.startswith("csrc digest:"):
            return line.split(":", 1)[1].strip()
    return None


def kind_of(kernel_name: str) -> str:
    n = kernel_name.split("(")[0].replace("void ", "").replace("ddg::", "").strip()
    m = re.match(r"conv3x3_tiled_kernel<(\d+), (\d+), (\d+)", n)
    if m:
        fam = "conv_fprop" if m.group(3) == "1" else "conv_dgrad"
        return f"{fam}.tiled_c{m.group(1)}_w{m.group(2)}"
    m = re.match(r"conv3x3_tiled_f32_kernel<(\d+), (\d+), (\d+)", n)
    if m:   # the fp32 instances book the same kinds
        fam = "conv_fprop" if m.group(3) == "1" else "conv_dgrad"
        return f"{fam}.tiled_c{m.group(1)}_w{m.group(2)}"
    m = re.match(r"bwd_pair(?:_f32)?_kernel<(\d+), (\d+), ", n)
    if m:
        return f"conv_bwd_pair.tiled_c{m.group(1)}_w{m.group(2)}"
    m = re.match(r"wgrad_tiled_f32_kernel<(\d+), (\d+)>", n)
    if m:
        return f"conv_wgrad.tiled_c{m.group(1)}_w{m.group(2)}"
    m = re.match(r"wgrad_tiled_kernel<(\d+), (\d+), (\d+), (\d+), (\d+)>", n)
    if m:   # <Cin, Cout, output width, stride, kernel size>
        return "conv_wgrad.tiled_stride2" if m.group(4) == "2" else f"conv_wgrad.tiled_c{m.group(1)}_w{m.group(3)}"
    m = re.match(r"conv_wide_kernel<(\d+), ", n)
    if m:   # <STATS, ...>: 1 = forward statistics (the forward conv); 0 / 2 = the input gradient
        return "conv_fprop.wide" if m.group(1) == "1" else "conv_dgrad.wide"
    if n.startswith("wgrad_wide_kernel"):
        return "conv_wgrad.wide"
    m = re.match(r"conv_mfma_kernel<\w+, \d+, \d+, (true|false)", n)
    if m:   # <T, MB, NB, DGRAD, VEC>
        return "conv_dgrad.generic" if m.group(1) == "true" else "conv_fprop.generic"
    table = [("wgrad_mfma_kernel", "conv_wgrad.generic"), ("wgrad_mfma_vec_kernel", "conv_wgrad.generic"), ("wgrad_reduce", "wgrad_reduce"),
             ("bn_bwd_apply_kernel", "bn_bwd_apply"), ("bn_bwd_apply_chunk_kernel", "bn_bwd_apply"), ("bn_bwd_reduce_kernel", "bn_bwd_reduce"),
             ("bn_bwd_finalize", "bn_bwd_finalize"), ("bn_apply_kernel", "bn_apply"),
             ("bn_apply_chunk_kernel", "bn_apply"), ("bn_apply_pair_kernel", "bn_apply"),
             ("running_update_kernel", "bn_running"), ("eval_vectors_kernel", "bn_running"),
             ("bn_finalize", "bn_finalize"), ("head_", "head"), ("sgd_kernel", "sgd"),
             ("pack_", "pack_weights"), ("copy_kernel", "copy")]
    for prefix, kind in table:
        if n.startswith(prefix):
            return kind
    return n


def short(kernel_name: str) -> str:
    return kernel_name.split("(")[0].replace("void ", "").replace("ddg::", "").strip()


def stats(path: str, steps: float, out=sys.stdout):
    rows = list(csv.DictReader(open(path)))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print(f"kernel time per pipeline iteration: {total / 1e6 / steps:.3f} ms "
          f"({sum(int(r['Calls']) for r in rows) / steps:.0f} launches)", file=out)
    print(f"{'kernel':<44} {'kind':<26} {'calls/it':>8} {'avg us':>8} {'ms/it':>7} {'share':>6}", file=out)
    kinds = collections.defaultdict(lambda: [0, 0.0])
    for r in rows:
        t = float(r["TotalDurationNs"])
        k = kinds[kind_of(r["Name"])]
        k[0] += int(r["Calls"]); k[1] += t
        print(f"{short(r['Name'])[:44]:<44} {kind_of(r['Name']):<26} {int(r['Calls']) / steps:8.1f} "
              f"{float(r['AverageNs']) / 1e3:8.2f} {t / 1e6 / steps:7.3f} {100 * t / total:5.1f}%", file=out)
    print("", file=out)
    print("per kind (the unit bench.py's `kernels` and `roofline` use):", file=out)
    print(f"{'kind':<28} {'calls/it':>8} {'avg us':>8} {'ms/it':>7}", file=out)
    for name, (n, t) in sorted(kinds.items(), key=lambda kv: -kv[1][1]):
        print(f"{name:<28} {n / steps:8.1f} {t / n / 1e3:8.2f} {t / 1e6 / steps:7.3f}", file=out)


def _per_kernel(path: str, counter: str):
    agg = collections.defaultdict(lambda: [0, 0.0])
    copies = []
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        v = float(r["Counter_Value"])
        a = agg[short(r["Kernel_Name"])]
        a[0] += 1
        a[1] += v
        if short(r["Kernel_Name"]) == "copy_kernel":
            threads = int(r["Grid_Size"])
            if 256 < threads < 2048 * 256:          # below the grid cap: 16 bytes per thread
                copies.append((threads * 16.0, v * 1024.0))
    return agg, copies


def traffic(fetch_csv: str, write_csv: str, out=sys.stdout):
    f_agg, f_cal = _per_kernel(fetch_csv, "FETCH_SIZE")
    w_agg, w_cal = _per_kernel(write_csv, "WRITE_SIZE")
    if not f_cal or not w_cal:
        raise SystemExit("no calibration dispatches of copy_kernel found")
    kf = sum(b for b, _ in f_cal) / sum(c for _, c in f_cal)
    kw = sum(b for b, _ in w_cal) / sum(c for _, c in w_cal)
    print(f"csrc digest: {source_digest()}", file=out)
    print(f"calibration (copy_kernel, {len(f_cal)} dispatches of known size): "
          f"bytes read = {kf:.4f} x FETCH_SIZE KiB, bytes written = {kw:.4f} x WRITE_SIZE KiB", file=out)
    print("kind | kernel | dispatches | FETCH_SIZE KiB/dispatch | WRITE_SIZE KiB/dispatch | "
          "calibrated bytes/dispatch", file=out)
    kinds = collections.defaultdict(lambda: [0, 0.0, 0.0, []])
    for name in f_agg:
        n, fs = f_agg[name]
        _, ws = w_agg.get(name, (0, 0.0))
        k = kinds[kind_of(name)]
        k[0] += n; k[1] += fs; k[2] += ws; k[3].append(name)
    for kind, (n, fs, ws, names) in sorted(kinds.items(), key=lambda kv: -(kv[1][1] * kf + kv[1][2] * kw)):
        b = (fs * kf + ws * kw) * 1024.0 / n
        print(f"{kind} | {' + '.join(sorted(names))} | {n} | {fs / n:.1f} | {ws / n:.1f} | {b:.0f}", file=out)


def mfma(util_csv: str, flops_csv: str, out=sys.stdout):
    """Matrix-core evidence per kernel kind from two counter passes: MfmaUtil (MFMA-busy cycles
    over elapsed cycles times SIMDs, in %) and MfmaFlopsBF16 (flops the MFMA instructions
    executed, zero padding included)."""
    u_agg, _ = _per_kernel(util_csv, "MfmaUtil")
    f_agg, _ = _per_kernel(flops_csv, "MfmaFlopsBF16")
    print("kind | kernel | dispatches | MfmaUtil % (mean over dispatches) | executed bf16 MFMA GFLOP/dispatch", file=out)
    kinds = collections.defaultdict(lambda: [0, 0.0, 0, 0.0, []])
    for name, (n, us) in u_agg.items():
        k = kinds[kind_of(name)]
        k[0] += n; k[1] += us; k[4].append(name)
    for name, (n, fs) in f_agg.items():
        k = kinds[kind_of(name)]
        k[2] += n; k[3] += fs
    for kind, (n, us, nf, fs, names) in sorted(kinds.items(), key=lambda kv: -kv[1][3]):
        if fs <= 0.0:
            continue                                  # no matrix-core work in this kind
        print(f"{kind} | {' + '.join(sorted(names))} | {n} | {us / max(n, 1):.2f} | {fs / max(nf, 1) / 1e9:.3f}", file=out)


def read_traffic_table(path: str) -> dict:
    """kind -> calibrated bytes per dispatch, from a summary written by `traffic`."""
    table = {}
    for line in open(path):
        parts = [p.strip() for p in line.split("|")]
        if len(parts) == 6 and parts[2].isdigit():
            table[parts[0]] = float(parts[5])
    return table


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats"); s.add_argument("csv"); s.add_argument("--steps", type=float, required=True)
    t = sub.add_parser("traffic"); t.add_argument("fetch_csv"); t.add_argument("write_csv")
    f = sub.add_parser("mfma"); f.add_argument("util_csv"); f.add_argument("flops_csv")
    a = ap.parse_args()
    if a.cmd == "stats":
        stats(a.csv, a.steps)
    elif a.cmd == "traffic":
        traffic(a.fetch_csv, a.write_csv)
    else:
        mfma(a.util_csv, a.flops_csv)


if __name__ == "__main__":
    main()
