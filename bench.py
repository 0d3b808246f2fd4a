#!/usr/bin/env python3
"""Throughput of the SPO hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: prioritized
sampling -> advantages -> tracker update -> fused LM-head + clipped
policy-gradient loss forward -> backward (dHidden and dW); with --path one_call
(the default) loss and gradients come from spo_pg_loss_fwd_bwd, which forms the
logits once, with --path two_calls from spo_pg_loss_fwd followed by
spo_pg_loss_bwd, which forms them twice.  Default workload: the
Qwen3-8B head shape (H=4096, V=151936, bf16), 128 packed variable-length
responses (~280k tokens).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3|C2|C4]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E
MFMA_KERNELS = ("fwd_sweep", "bwd_recompute", "bwd_dhidden", "bwd_dw")
HBM_KERNELS = ("logits_to_dz",)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_digest() -> str:
    """Digest of the kernel sources: a traffic profile is only quoted for the kernels it was taken from."""
    from paper_2509_13232_amd.build import source_digest
    return source_digest()


def profiled_traffic(workload: str, chunk_tokens: int, one_call: bool):
    """Bytes across the L2 <-> fabric boundary per launch (reads + writes) of each heavy kernel, from the
    tracked rocprofv3 summary profiles/step_<workload>_[two_calls_]hbm_traffic.md, or None when that
    summary was taken from other kernel sources, another chunk size, or does not exist."""
    path = os.path.join(ROOT, "profiles", f"step_{workload.lower()}_{'' if one_call else 'two_calls_'}hbm_traffic.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    dig = re.search(r"^source_digest:\s*(\w+)", text, re.M)
    chunk = re.search(r"^chunk_tokens:\s*(\d+)", text, re.M)
    line = re.search(r"^traffic_bytes_per_launch:\s*(.+)$", text, re.M)
    if not (dig and chunk and line) or dig.group(1) != kernel_source_digest() or int(chunk.group(1)) != chunk_tokens:
        return None
    return {k: float(v) for k, v in (kv.split("=") for kv in line.group(1).split())}


def cpu_model() -> str:
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def run_workload(spo, wl, torch, name, steps, warmup, chunk_tokens, want_d_hidden, one_call=True):
    """Times `steps` steps of workload `name`; returns (result dict, live tensors for the follow-up legs)."""
    import ctypes as C
    dev = "cuda"
    cfg = wl.CONFIGS[name]
    t_setup = time.time()
    a0, b0 = wl.tracker_state(cfg)
    alpha, beta = torch.as_tensor(a0).to(dev), torch.as_tensor(b0).to(dev)
    tb = wl.token_batch(cfg, device=dev)
    T, H, V, B = tb.T, cfg.H, cfg.V, cfg.B
    target = torch.as_tensor(tb.target).to(dev)
    cu = torch.as_tensor(tb.cu_seqlens).to(dev)
    mask = None if tb.mask is None else torch.as_tensor(tb.mask).to(dev)
    old_logp = wl.behaviour_logp_standin(tb.hidden, tb.W, tb.target, cfg.w_std, tb.noise)
    idx0 = wl.distinct_indices(cfg, B)
    reward = torch.as_tensor(wl.rewards(cfg, idx0)).to(dev)
    kl = torch.as_tensor(wl.kl_divergences(cfg, B)).to(dev)
    M = T if tb.mask is None else int(tb.mask.sum())
    log(f"[bench] workload {cfg.name}: T={T} B={B} H={H} V={V} N={cfg.N} unmasked={M} "
        f"(setup {time.time() - t_setup:.1f}s)")

    # preallocated outputs and workspaces: nothing is allocated inside the timed region by the library
    adv_holder = torch.zeros(B, dtype=torch.float32, device=dev)
    desc = spo.make_desc(tb.hidden, tb.W, target, old_logp, mask, adv_holder, cu, cfg.eps_low, cfg.eps_high)
    ws_s = torch.empty(spo.lib().spo_sample_prompts_workspace_bytes(cfg.N, B), dtype=torch.uint8, device=dev)
    if one_call:
        ws_f = torch.empty(256, dtype=torch.uint8, device=dev)
        ws_b = torch.empty(max(256, spo.spo_pg_loss_fwd_bwd_workspace_bytes(desc, chunk_tokens)), dtype=torch.uint8, device=dev)
    else:
        ws_f = torch.empty(max(256, spo.lib().spo_pg_loss_fwd_workspace_bytes(C.byref(desc[0]))), dtype=torch.uint8, device=dev)
        ws_b = torch.empty(max(256, spo.spo_pg_loss_bwd_workspace_bytes(desc, chunk_tokens)), dtype=torch.uint8, device=dev)
    d_W = torch.empty((V, H), dtype=torch.float32, device=dev)
    log(f"[bench] workspaces: fwd {ws_f.numel() / 2**30:.2f} GiB, bwd {ws_b.numel() / 2**30:.2f} GiB")
    state = {}

    def step(it: int):
        idx = spo.spo_sample_prompts(alpha, beta, B, cfg.eps_explore, cfg.sample_seed, it, workspace=ws_s)
        _, adv, _ = spo.spo_advantages(alpha, beta, idx, reward)
        spo.spo_tracker_update(alpha, beta, idx, reward, kl, cfg.d_half, cfg.rho_min, cfg.rho_max)
        adv_holder.copy_(adv)   # the descriptor points at adv_holder
        if one_call:
            loss, logp, lse, stats, _, _ = spo.spo_pg_loss_fwd_bwd(desc, 1.0, d_W=d_W, want_d_hidden=want_d_hidden,
                                                                   chunk_tokens=chunk_tokens, workspace=ws_b)
        else:
            loss, logp, lse, stats = spo.spo_pg_loss_fwd(desc, workspace=ws_f)
            spo.spo_pg_loss_bwd(desc, logp, lse, 1.0, d_W=d_W, want_d_hidden=want_d_hidden, chunk_tokens=chunk_tokens,
                                workspace=ws_b)
        state["loss"], state["stats"] = loss, stats

    for w in range(warmup):
        step(w)
    torch.cuda.synchronize()
    spo.spo_kernel_timing_read()
    spo.spo_kernel_timing_enable(True)
    # per-step marks on the launch stream (no host synchronisation inside the timed region)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for k in range(steps):
        step(warmup + k)
        marks[k + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_ms = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(steps))
    spo.spo_kernel_timing_enable(False)
    times = spo.spo_kernel_timing_read()
    sec = (t1 - t0) / steps
    stats = state["stats"].cpu().tolist()
    log(f"[bench] {cfg.name}: {sec * 1e3:.1f} ms/step, loss {state['loss'].item():.6f}, clipped share {stats[1]:.4f}, "
        f"mean ratio {stats[2]:.4f}")

    # The forward contracts over all T tokens; the backward only over the tokens that carry a
    # gradient (unmasked and on the unclipped branch: stats[0] * (1 - stats[1]) of them).
    t_active = round(stats[0] * (1.0 - stats[1]))
    thv = {"fwd_sweep": 2.0 * T * H * V}            # flops of one contraction of a kernel class per step
    # one call without a loss mask: the contractions run over every token (rows without a gradient are scaled by 0)
    all_rows = one_call and tb.mask is None
    for k in MFMA_KERNELS[1:]:
        thv[k] = 2.0 * (T if all_rows else t_active) * H * V
    kern = {}
    for k in MFMA_KERNELS:
        ms, n = times[k]
        if n:
            kern[k] = {"ms_per_step": round(ms / steps, 3), "launches_per_step": n // steps,
                       "avg_launch_ms": round(ms / n, 4), "tflops": round(thv[k] / (ms / steps * 1e-3) / 1e12, 1)}
    executed = sum(thv[k] for k in kern)
    useful = 2.0 * T * H * V + 2 * 2.0 * t_active * H * V   # logits once, dHidden and dW of the tokens with a gradient
    # the pass from stored logits to logit gradients (one-call path): 2 V bytes read and 2 V written per active token
    V_blk = (V + 255) // 256 * 256
    for k in HBM_KERNELS:
        ms, n = times[k]
        if n:
            kern[k] = {"ms_per_step": round(ms / steps, 3), "launches_per_step": n // steps, "avg_launch_ms": round(ms / n, 4),
                       "GBps": round(4.0 * t_active * V_blk / (ms / steps * 1e-3) / 1e9, 1), "bound": "hbm"}
    res = {
        "path": "one_call (spo_pg_loss_fwd_bwd)" if one_call else "two_calls (spo_pg_loss_fwd, spo_pg_loss_bwd)",
        "tokens_per_s": round(T / sec, 1), "ms_per_step": round(sec * 1e3, 3),
        "ms_per_step_median": round(step_ms[len(step_ms) // 2], 3), "ms_per_step_min": round(step_ms[0], 3),
        "T": T, "B": B, "H": H, "V": V, "N": cfg.N, "active_tokens": t_active, "clipped_share": round(stats[1], 5),
        "workspace_bytes": {"fwd": ws_f.numel(), "bwd": ws_b.numel(), "sampler": ws_s.numel()},
        "tflops_useful": round(useful / sec / 1e12, 1), "tflops_executed": round(executed / sec / 1e12, 1),
        "mfma_util_executed": round(executed / sec / 1e12 / PEAK_BF16_TFLOPS, 4), "kernels": kern,
        "workload": f"{cfg.name}: {B} packed responses, lengths {cfg.lengths}, T={T} tokens, H={H}, V={V}, "
                    f"{cfg.N}-prompt tracker, mask {cfg.mask_frac}; old_logp is a closed-form stand-in "
                    f"(target logit - log V - s^2/2 + N(0,{cfg.noise_std}^2)), not a forward pass + noise",
    }
    live = dict(cfg=cfg, tb=tb, target=target, old_logp=old_logp, reward=reward, kl=kl, a0=a0, b0=b0, times=times,
                thv=thv, steps=steps)
    del ws_b, d_W, ws_f
    return res, live


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C3", choices=["C2", "C3", "C4"])
    ap.add_argument("--chunk-tokens", type=int, default=0, help="backward chunk (0: the library's bounded default)")
    ap.add_argument("--path", default="one_call", choices=["one_call", "two_calls"],
                    help="loss and gradients from one call (logits formed once) or from forward then backward")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-logits-in", action="store_true")
    ap.add_argument("--no-small", action="store_true", help="skip the tracker / advantage / sampler timings")
    ap.add_argument("--no-others", action="store_true", help="skip the secondary workloads (C2, C4)")
    ap.add_argument("--cpu-tokens", type=int, default=0, help="oracle sample size (0: the shortest whole response)")
    ap.add_argument("--calibrate-copy", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU: the path is built and measured on a single MI355X "
            "(across GPUs it would shard by responses). Run with --gpus 1.")
        return 2

    import numpy as np
    import torch

    from paper_2509_13232_amd import binding as spo
    from paper_2509_13232_amd import workloads as wl

    if not torch.cuda.is_available():
        log("bench.py needs a GPU")
        return 2
    spo.lib()
    torch.cuda.set_device(0)
    dev = "cuda"

    if args.calibrate_copy:
        # a plain elementwise copy of known size (1 GiB read, 1 GiB written) whose hardware
        # counters calibrate the FETCH_SIZE / WRITE_SIZE readings of the other kernels
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    one_call = args.path == "one_call"
    res, live = run_workload(spo, wl, torch, args.workload, args.steps, args.warmup, args.chunk_tokens, True, one_call)
    cfg, tb, times, thv = live["cfg"], live["tb"], live["times"], live["thv"]
    T, H, V, B = res["T"], res["H"], res["V"], res["B"]
    kern = res["kernels"]

    # ---------------------------------------------------------------- roofline of the dominant kernel
    dom = max((k for k in kern if k in MFMA_KERNELS), key=lambda k: kern[k]["ms_per_step"])
    ms_dom, n_dom = times[dom]
    flops_per_launch = thv[dom] * args.steps / n_dom
    achieved = flops_per_launch / (ms_dom / n_dom * 1e-3) / 1e12
    traffic = profiled_traffic(cfg.name, args.chunk_tokens, one_call)
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": None if traffic is None else traffic.get(dom),
                "flops_per_launch": flops_per_launch, "avg_launch_ms": round(ms_dom / n_dom, 4), "kernels": kern}

    out = {
        "metric": "tokens/sec fused LM-head+SPO PG loss fwd+bwd at H=4096,V=151936; MFMA util %",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "ms_per_step_median": res["ms_per_step_median"],
        "ms_per_step_min": res["ms_per_step_min"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": res["workload"], "T": T, "B": B, "H": H, "V": V, "N": cfg.N,
                   "eps": [cfg.eps_low, cfg.eps_high], "d_half": cfg.d_half,
                   "path": res["path"],
                   "chunk_tokens": args.chunk_tokens or "library default (what is stored of a piece, or the logit gradients of a chunk, <= 8 GiB)",
                   "workspace_bytes": res["workspace_bytes"]},
        "active_tokens": res["active_tokens"], "tflops_useful": res["tflops_useful"],
        "tflops_executed": res["tflops_executed"], "mfma_util_executed": res["mfma_util_executed"],
        "clipped_share": res["clipped_share"],
        "device": torch.cuda.get_device_name(0), "torch": torch.__version__, "roofline": roofline,
    }

    # ---------------------------------------------------------------- logits-in variant (HBM bound)
    target, old_logp = live["target"], live["old_logp"]
    if not args.no_logits_in:
        Tl = min(T, 8192)
        torch.cuda.empty_cache()
        logits = torch.empty((Tl, V), dtype=torch.bfloat16, device=dev)
        for s in range(0, Tl, 1024):
            logits[s:s + 1024] = tb.hidden[s:s + 1024] @ tb.W.t()   # input preparation, not timed
        lcu = torch.tensor([0, Tl], dtype=torch.int32, device=dev)
        ladv = torch.ones(1, dtype=torch.float32, device=dev)
        ldesc = spo.make_desc(None, None, target[:Tl], old_logp[:Tl], None, ladv, lcu, cfg.eps_low, cfg.eps_high,
                              logits=logits)
        _, llogp, llse, _ = spo.spo_pg_loss_fwd(ldesc)
        spo.spo_pg_loss_bwd(ldesc, llogp, llse, 1.0)
        torch.cuda.synchronize()
        spo.spo_kernel_timing_read()
        spo.spo_kernel_timing_enable(True)
        reps = 5
        for _ in range(reps):
            _, llogp, llse, _ = spo.spo_pg_loss_fwd(ldesc)
            dl = spo.spo_pg_loss_bwd(ldesc, llogp, llse, 1.0)
        torch.cuda.synchronize()
        spo.spo_kernel_timing_enable(False)
        lt = spo.spo_kernel_timing_read()
        fwd_ms = lt["logits_fwd"][0] / reps
        bwd_ms = lt["logits_bwd"][0] / reps
        fwd_gbps = Tl * V * 2 / (fwd_ms * 1e-3) / 1e9
        bwd_gbps = Tl * V * 4 / (bwd_ms * 1e-3) / 1e9
        out["logits_in"] = {"tokens": Tl, "bytes_per_token_fwd": V * 2, "bytes_per_token_bwd": V * 4,
                            "fwd_ms": round(fwd_ms, 3), "bwd_ms": round(bwd_ms, 3),
                            "fwd_GBps": round(fwd_gbps, 1), "bwd_GBps": round(bwd_gbps, 1),
                            "fwd_frac_hbm": round(fwd_gbps / PEAK_HBM_GBPS, 4),
                            "bwd_frac_hbm": round(bwd_gbps / PEAK_HBM_GBPS, 4),
                            "tokens_per_s_fwd_bwd": round(Tl / ((fwd_ms + bwd_ms) * 1e-3), 1)}
        del logits, dl

    # ---------------------------------------------------------------- the oracle on the host cores
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        a0, b0 = live["a0"], live["b0"]
        reward, kl = live["reward"].cpu().numpy(), live["kl"].cpu().numpy()
        cu_np = tb.cu_seqlens
        lens = np.diff(cu_np)
        b_short = int(np.argmin(lens))                       # the shortest whole response of the batch
        s0 = int(cu_np[b_short])
        n_all = int(lens[b_short]) if args.cpu_tokens <= 0 else min(args.cpu_tokens, T)
        cores_all = oracle.num_threads()
        w64 = tb.W.double().cpu().numpy()

        def oracle_path(n_tok):
            h64 = tb.hidden[s0:s0 + n_tok].double().cpu().numpy()
            tg, ol = tb.target[s0:s0 + n_tok], old_logp[s0:s0 + n_tok].double().cpu().numpy()
            ccu = np.array([0, n_tok], np.int32)
            t0c = time.perf_counter()
            eidx = oracle.sample_prompts(a0, b0, B, cfg.eps_explore, cfg.sample_seed, 0)
            _, eadv, _ = oracle.advantages(a0, b0, eidx, reward)
            oracle.tracker_update(a0, b0, eidx, reward, kl, cfg.d_half, cfg.rho_min, cfg.rho_max)
            oracle.pg_loss_fwd(h64, w64, tg, ol, None, eadv[:1], ccu, cfg.eps_low, cfg.eps_high)
            oracle.pg_loss_bwd(h64, w64, tg, ol, None, eadv[:1], ccu, cfg.eps_low, cfg.eps_high)
            return time.perf_counter() - t0c

        dt_all = oracle_path(n_all)
        n_one = max(4, min(n_all, round(n_all / cores_all / 1.5)))   # about as long again on one core
        oracle.set_num_threads(1)
        dt_one = oracle_path(n_one)
        oracle.set_num_threads(cores_all)
        out["cpu_baseline"] = {
            "value": round(n_all / dt_all, 3), "unit": "tokens/s", "cores": cores_all, "kind": "oracle",
            "sample": f"whole path on the shortest whole response of the workload ({n_all} tokens, full H={H} "
                      f"and V={V}, fp64, {dt_all:.1f} s on {cores_all} threads); one core: its first {n_one} "
                      f"tokens in {dt_one:.1f} s",
            "one_core": {"value": round(n_one / dt_one, 3), "unit": "tokens/s", "cores": 1},
            "cpu_model": cpu_model(), "host_logical_cpus": os.cpu_count()}
        del w64

    # ---------------------------------------------------------------- tracker / advantage / sampler at 2^20 prompts
    if not args.no_small:
        c5 = wl.CONFIGS["C5"]
        a5n, b5n = wl.tracker_state(c5)
        a5, b5 = torch.as_tensor(a5n).to(dev), torch.as_tensor(b5n).to(dev)
        i5n = wl.distinct_indices(c5, c5.B)
        r5n, k5n = wl.rewards(c5, i5n), wl.kl_divergences(c5, c5.B)
        r5, k5, i5 = torch.as_tensor(r5n).to(dev), torch.as_tensor(k5n).to(dev), torch.as_tensor(i5n).to(dev)
        ws5 = torch.empty(spo.lib().spo_sample_prompts_workspace_bytes(c5.N, c5.B), dtype=torch.uint8, device=dev)

        def timed(fn, reps=20):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3   # microseconds per call, launch overhead included

        us_sample = timed(lambda: spo.spo_sample_prompts(a5, b5, c5.B, c5.eps_explore, c5.sample_seed, 1, workspace=ws5))
        us_sample_r = timed(lambda: spo.spo_sample_prompts(a5, b5, c5.B, c5.eps_explore, c5.sample_seed, 1, True,
                                                           workspace=ws5))
        us_adv = timed(lambda: spo.spo_advantages(a5, b5, i5, r5))
        us_upd = timed(lambda: spo.spo_tracker_update(a5, b5, i5, r5, k5, c5.d_half, c5.rho_min, c5.rho_max))
        # advantages of a batch of 2^20 responses (ids repeat): one workgroup against the many-workgroup form
        big = 1 << 20
        ib = torch.randint(0, c5.N, (big,), dtype=torch.int32, device=dev)
        rb = (torch.rand(big, device=dev) < 0.4).float()
        ws_adv = torch.empty(spo.lib().spo_advantages_workspace_bytes(big), dtype=torch.uint8, device=dev)
        us_adv_big1 = timed(lambda: spo.spo_advantages(a5, b5, ib, rb), reps=3)
        us_adv_big = timed(lambda: spo.spo_advantages(a5, b5, ib, rb, workspace=ws_adv))
        scan_bytes = c5.N * (8 + 8 + 8)   # alpha, beta read in two passes (8 B each), 8-byte CDF written
        small = {
            "workload": f"C5: {c5.N} tracked prompts, batch {c5.B}",
            "sample_without_replacement_us": round(us_sample, 1), "sample_with_replacement_us": round(us_sample_r, 1),
            "advantages_us": round(us_adv, 1), "tracker_update_us": round(us_upd, 1),
            "advantages_1M_responses_us": {"one_workgroup": round(us_adv_big1, 1), "with_workspace": round(us_adv_big, 1)},
            "weight_scan_GBps": round(scan_bytes / (us_sample_r * 1e-6) / 1e9, 1),
            "note": "host-visible time per call on the launch stream (several small launches each); "
                    "weight_scan_GBps counts 24 B per prompt over the with-replacement call"}
        if not args.no_cpu_baseline:
            import oracle

            def host_us(fn, reps=3):
                fn()
                t0h = time.perf_counter()
                for _ in range(reps):
                    fn()
                return (time.perf_counter() - t0h) / reps * 1e6

            small["oracle_us"] = {
                "sample_without_replacement": round(host_us(lambda: oracle.sample_prompts(
                    a5n, b5n, c5.B, c5.eps_explore, c5.sample_seed, 1)), 1),
                "sample_with_replacement": round(host_us(lambda: oracle.sample_prompts(
                    a5n, b5n, c5.B, c5.eps_explore, c5.sample_seed, 1, True)), 1),
                "advantages": round(host_us(lambda: oracle.advantages(a5n, b5n, i5n, r5n)), 1),
                "tracker_update": round(host_us(lambda: oracle.tracker_update(
                    a5n, b5n, i5n, r5n, k5n, c5.d_half, c5.rho_min, c5.rho_max)), 1),
                "note": "the oracle's C routines through their ctypes wrappers (array conversion included), "
                        "sequential code except for its OpenMP loops"}
        out["small_kernels"] = small

    # ---------------------------------------------------------------- the other token workloads, fewer steps
    if not args.no_others:
        del live, tb, target, old_logp
        torch.cuda.empty_cache()
        others = {}
        for name, (st, wu) in {"C2": (20, 3), "C4": (2, 1)}.items():
            if name == args.workload:
                continue
            r, lv = run_workload(spo, wl, torch, name, st, wu, args.chunk_tokens, True, one_call)
            del lv
            torch.cuda.empty_cache()
            r["steps"], r["warmup"] = st, wu
            others[name] = r
        out["other_workloads"] = others
        # the same workload through the other way to the gradients (forward then backward, or the one call)
        r, lv = run_workload(spo, wl, torch, args.workload, 3, 1, args.chunk_tokens, True, not one_call)
        del lv
        torch.cuda.empty_cache()
        r["steps"], r["warmup"] = 3, 1
        out["other_path"] = r

    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
