"""Turns rocprofv3 output of `bench.py` runs into the short text summaries under profiles/.

    python -m paper_2509_13232_amd.profile_summary --workload C3 --chunk-tokens 0 [--path two_calls] \\
        --trace DIR --bench-json FILE [--fetch DIR --write DIR] [--mfma DIR] --out profiles

Writes profiles/step_<workload>_*.md for bench.py's default path (one call for loss and gradients) and
profiles/step_<workload>_two_calls_*.md for --path two_calls.

DIR are the -d directories of the rocprofv3 runs whose commands the summaries quote (run from
/tmp with TMPDIR=/tmp); FILE is the JSON line bench.py printed under the kernel-trace run.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os

from .build import source_digest

KERNELS = (("fwd_sweep", "fwd_sweep_kernel"), ("bwd_recompute", "recompute_dz_kernel"),
           ("logits_to_dz", "dz_from_logits_kernel"),
           ("bwd_dhidden", "gemm_store_kernel<false>"), ("bwd_dw", "gemm_store_kernel<true>"))
BENCH = "python3 bench.py --no-cpu-baseline --no-small --no-logits-in --no-others"


def _bench(args):
    return f"{BENCH} --path {args.path}"


def _stamp(args):
    return f"source_digest: {source_digest()}\npath: {args.path}\nchunk_tokens: {args.chunk_tokens}\n"


def _one(d, pattern):
    f = sorted(glob.glob(os.path.join(d, "**", pattern), recursive=True))
    if not f:
        raise SystemExit(f"no {pattern} under {d}")
    return f[0]


def _short(name):
    return name.split("(")[0].replace("void ", "")


def _counters(d):
    """{counter: {short kernel name: [value per dispatch, in order]}}"""
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(_one(d, "*counter_collection.csv")) as fh:
        for r in csv.DictReader(fh):
            out[r["Counter_Name"]][_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return out


def _of(table, sub):
    ks = [k for k in table if sub in k]
    return table[ks[0]] if ks else []


def kernel_trace(args, b):
    rows = list(csv.DictReader(open(_one(args.trace, "*kernel_stats.csv"))))
    o = [f"# rocprofv3 kernel-trace summary: whole SPO step, workload {args.workload}\n",
         "Command (from /tmp with TMPDIR=/tmp, on one MI355X):\n",
         f"    rocprofv3 --kernel-trace --stats -d <dir> -o p --output-format csv -- \\\n        {_bench(args)} --steps 2 --warmup 1"
         f" --workload {args.workload} --chunk-tokens {args.chunk_tokens}\n",
         _stamp(args),
         f"Workload: {b['config']['workload']}\n",
         f"bench.py under the profiler: {b['value']} tokens/s, {b['ms_per_step']} ms/step, "
         f"{b['tflops_executed']} TFLOP/s executed = {100 * b['mfma_util_executed']:.1f} % of 2500.\n",
         "Per-kernel averages measured live by bench.py with HIP events on the launch stream (same run):\n"]
    for k, v in b["roofline"]["kernels"].items():
        rate = f"{v['tflops']:7.1f} TFLOP/s" if "tflops" in v else f"{v['GBps']:7.1f} GB/s (reads + writes)"
        o.append(f"    {k:14s} {v['avg_launch_ms']:10.4f} ms/launch  x{v['launches_per_step']}/step  {rate}")
    o.append(f"\nDominant kernel by time per step: {b['roofline']['kernel']} "
             f"({b['roofline']['achieved']} TFLOP/s = {100 * b['roofline']['frac']:.1f} % of 2500).\n")
    o.append("rocprofv3 kernel stats (library kernels and the six largest others):\n")
    o.append(f"    {'kernel':58s} {'calls':>6s} {'total ms':>11s} {'avg ms':>10s} {'%':>7s}")
    n_other = 0
    for r in rows:
        if "spo::" not in r["Name"]:
            n_other += 1
            if n_other > 6:
                continue
        o.append(f"    {_short(r['Name'])[:58]:58s} {int(r['Calls']):6d} {int(r['TotalDurationNs']) / 1e6:11.3f} "
                 f"{float(r['AverageNs']) / 1e6:10.4f} {float(r['Percentage']):7.3f}")
    o.append("\ngemm_store_kernel<false> is the dHidden contraction, gemm_store_kernel<true> the dW contraction;")
    o.append("fwd_sweep_kernel<true> is the sweep that also stores a piece's logits, dz_from_logits_kernel the pass that turns")
    o.append("them into logit gradients. The batch is walked in pieces (one call) or the backward in chunks of tokens that")
    o.append("carry a gradient (two calls); per-launch averages are over all launches of a step, the last of which is")
    o.append("shorter. Kernels outside the spo namespace are torch's input generation.\n")
    return "\n".join(o)


def hbm_traffic(args, b):
    f, w = _counters(args.fetch)["FETCH_SIZE"], _counters(args.write)["WRITE_SIZE"]
    # bench.py's calibration copy is torch.add(src, 0.0, out=dst) on 2^28 floats: its three largest dispatches
    copy = [k for k in f if "CUDAFunctorOnSelf_add" in k]
    cf = sorted(x for k in copy for x in f[k])[-3:]
    cw = sorted(x for k in copy for x in w[k])[-3:]
    gib_kib = float(1 << 20)
    sf, sw = gib_kib / (sum(cf) / len(cf)), gib_kib / (sum(cw) / len(cw))
    T, H, V = b["config"]["T"], b["config"]["H"], b["config"]["V"]
    kern = b["roofline"]["kernels"]
    n_chunks = kern["bwd_dhidden"]["launches_per_step"]
    Tc = b["active_tokens"] / n_chunks          # average tokens per backward launch
    Tf = T / kern["fwd_sweep"]["launches_per_step"]   # tokens per launch of the sweep
    store = Tf * V * 2 if args.path == "one_call" else 0
    alg = {"fwd_sweep": (Tf * H * 2 + V * H * 2, Tf * 8 + store), "bwd_recompute": (Tc * H * 2 + V * H * 2, Tc * V * 2),
           "logits_to_dz": (Tc * V * 2, Tc * V * 2),
           "bwd_dhidden": (Tc * V * 2 + V * H * 2, Tc * H * 2), "bwd_dw": (Tc * V * 2 + Tc * H * 2 + V * H * 4, V * H * 4)}
    o = [f"# L2 <-> fabric traffic of the MFMA kernels of the SPO step (workload {args.workload}), rocprofv3 --pmc\n",
         "Commands (from /tmp with TMPDIR=/tmp, one counter per run):\n",
         f"    rocprofv3 --pmc FETCH_SIZE -d <dir> -o p --output-format csv -- \\\n        {_bench(args)} --steps 1 --warmup 0 --calibrate-copy"
         f" --workload {args.workload} --chunk-tokens {args.chunk_tokens}",
         f"    rocprofv3 --pmc WRITE_SIZE -d <dir> -o p --output-format csv -- \\\n        (the same bench.py command)\n",
         _stamp(args),
         "Calibration: `--calibrate-copy` runs a plain elementwise copy that reads 1 GiB and writes 1 GiB (1048576 KiB",
         f"each). The counters read FETCH_SIZE = {sum(cf) / len(cf):.0f} and WRITE_SIZE = {sum(cw) / len(cw):.0f} for it, so readings are",
         f"scaled by {sf:.3f} (fetch) and {sw:.3f} (write).\n",
         "Average per launch over all launches of the one profiled step, scaled, in GB (1e9 bytes); 'algorithmic' = operands read once +",
         "outputs written once, for the average launch:\n",
         f"    {'kernel':16s} {'launches':>8s} {'fetch GB':>10s} {'write GB':>10s} {'alg. read':>10s} {'alg. write':>11s}"]
    total = {}
    for name, sub in KERNELS:
        fv, wv = _of(f, sub), _of(w, sub)
        if not fv:
            continue
        # a launch as bench.py counts it (dW's short last round of tiles is a dispatch of its own, inside the same launch)
        nl = kern[name]["launches_per_step"] if name in kern else len(fv)
        fb, wb = sum(fv) / nl * 1024 * sf, sum(wv) / nl * 1024 * sw
        o.append(f"    {name:16s} {nl:8d} {fb / 1e9:10.2f} {wb / 1e9:10.2f} {alg[name][0] / 1e9:10.2f} {alg[name][1] / 1e9:11.2f}")
        total[name] = fb + wb
    o.append("\ntraffic_bytes_per_launch: " + " ".join(f"{k}={v:.4g}" for k, v in total.items()))
    o.append("\n(fetch + write; the line above is what bench.py quotes as roofline.traffic while the kernel sources and the")
    o.append("chunk size are the ones named here)\n")
    o.append("Reading: the contraction kernels are MFMA-bound, not HBM-bound. A 256 x 256 tile pulls 64 KiB of operands into the CU per")
    o.append("64 contraction steps whatever the cache does; the fetch column is what the eight L2s miss (operand panels are")
    o.append("shared by the 4 x 8 tiles that run together on an XCD, not across XCDs) and is served mostly by the 256 MB")
    o.append("Infinity Cache.\n")
    return "\n".join(o)


def mfma_counters(args, b):
    c = _counters(args.mfma)
    o = [f"# MFMA counters of the SPO step (workload {args.workload}), rocprofv3 --pmc\n",
         "Command (from /tmp with TMPDIR=/tmp):\n",
         "    rocprofv3 --pmc SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES GRBM_GUI_ACTIVE \\\n"
         f"        -d <dir> -o p --output-format csv -- {_bench(args)} --steps 1 --warmup 0"
         f" --workload {args.workload} --chunk-tokens {args.chunk_tokens}\n",
         _stamp(args),
         "Sums over the launches of one step. One MOPS count is 512 flop; SQ_VALU_MFMA_BUSY_CYCLES is summed over the 1024",
         "SIMDs and GRBM_GUI_ACTIVE over the 8 XCDs, so busy share = MFMA_BUSY / 1024 / (GUI_ACTIVE / 8) is the fraction of",
         "cycles a SIMD's MFMA pipe was busy, the utilisation against the peak at the clock the kernel really ran at.\n",
         f"    {'kernel':16s} {'launches':>8s} {'MOPS_BF16':>12s} {'flop = MOPS*512':>16s} {'MFMA busy share':>16s} {'cycles per XCD':>15s}"]
    for name, sub in KERNELS:
        mops, busy, gui = _of(c["SQ_INSTS_VALU_MFMA_MOPS_BF16"], sub), _of(c["SQ_VALU_MFMA_BUSY_CYCLES"], sub), _of(c["GRBM_GUI_ACTIVE"], sub)
        if not mops:
            continue
        o.append(f"    {name:16s} {b['roofline']['kernels'].get(name, {}).get('launches_per_step', len(mops)):8d} {sum(mops):12.4e} {sum(mops) * 512:16.4e} "
                 f"{sum(busy) / 1024 / (sum(gui) / 8):16.3f} {sum(gui) / 8:15.4e}")
    T, H, V, ta = b["config"]["T"], b["config"]["H"], b["config"]["V"], b["active_tokens"]
    pad = lambda x, a: (x + a - 1) // a * a
    o.append(f"\nAnalytic: forward 2 x T_pad x V_pad x H = {2.0 * pad(T, 256) * pad(V, 256) * H:.4e}; each backward contraction")
    o.append(f"2 x (active tokens, {ta}) x V_pad x H = {2.0 * ta * pad(V, 256) * H:.4e} plus the padding of each chunk to whole")
    o.append("tiles of 256 tokens.\n")
    return "\n".join(o)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--chunk-tokens", type=int, default=0)
    ap.add_argument("--path", default="one_call", choices=["one_call", "two_calls"])
    ap.add_argument("--trace")
    ap.add_argument("--bench-json", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--mfma")
    ap.add_argument("--out", default="profiles")
    args = ap.parse_args()
    b = json.loads(open(args.bench_json).read().strip().splitlines()[-1])
    stem = os.path.join(args.out, f"step_{args.workload.lower()}_" + ("" if args.path == "one_call" else "two_calls_"))
    if args.trace:
        open(stem + "kernel_trace.md", "w").write(kernel_trace(args, b))
    if args.fetch and args.write:
        open(stem + "hbm_traffic.md", "w").write(hbm_traffic(args, b))
    if args.mfma:
        open(stem + "mfma_counters.md", "w").write(mfma_counters(args, b))


if __name__ == "__main__":
    main()
