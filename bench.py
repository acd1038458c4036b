#!/usr/bin/env python3
"""Throughput of one decode-attention step (the whole hot path) on one MI355X.

A step is one ``rl_decode_attn`` call over one batch of synthetic rollout
state: every sequence of every GRPO group issues one query token against its
prompt's shared prefix and its own suffix.  Inputs are resident in HBM before
the timed region; several copies of the KV tensors are rotated so that no step
finds its inputs in the memory-side cache.

Prints ONE JSON line: query-tokens/s, the HBM roofline of the kernel (bytes the
method must move / kernel time from HIP events on the launch stream), and the
fp64 CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak

# HBM bytes one launch of the K/V-streaming kernel moved, per workload, from two rocprofv3 --pmc passes
# (FETCH_SIZE, then WRITE_SIZE) over this script, each scaled by what the same counter read for kernels of
# known size in the same run: the 1 GiB loads-only probe and the 1 GiB copies of --copy-probe, which agree
# (profiles/partial_kernel_*.md).  Carried over from that profile
# run, not measured in this one: reported only while the sources the kernel is built from still hash to
# what the counters were taken on, null otherwise.
PMC_TRAFFIC = {
    "csrc_sha256": "522ad498334b8e7a34a63f9fc9aaa400c1c8eed10561e706621335119fb2564c",
    "vlm7b": {"fetch_bytes": 623717227, "write_bytes": 9341133},
    "agentic": {"fetch_bytes": 163231461, "write_bytes": 7259546},
    "highbatch": {"fetch_bytes": 735241042, "write_bytes": 21287117},
}

OTHER_WORKLOADS = ("tiny", "vlm3b", "agentic", "highbatch")     # reported beside the default one, in short form


def strip_comments(src):
    """C++ source without its comments and with runs of white space collapsed: what the compiler sees of it."""
    out, i, n = [], 0, len(src)
    while i < n:
        c = src[i]
        if c == '"' or c == "'":                                # string / character literal: copy to its end
            j = i + 1
            while j < n and src[j] != c:
                j += 2 if src[j] == "\\" else 1
            out.append(src[i:j + 1]); i = j + 1
        elif src.startswith("//", i):
            j = src.find("\n", i)
            i = n if j < 0 else j
        elif src.startswith("/*", i):
            j = src.find("*/", i + 2)
            i = n if j < 0 else j + 2
            out.append(" ")
        else:
            out.append(c); i += 1
    return " ".join("".join(out).split())


def csrc_sha256():
    """Hash of the code (comments and layout aside) the K/V-streaming kernel is built from."""
    import hashlib
    d = os.path.join(ROOT, "paper_2512_21450_amd", "csrc")
    h = hashlib.sha256()
    for f in ("rlda_internal.h", "rlda_sched.h", "rlda_shared.hip"):
        h.update(f.encode())
        h.update(strip_comments(open(os.path.join(d, f), encoding="utf-8").read()).encode())
    return h.hexdigest()


def measured_traffic(workload, plan):
    """Counter-measured HBM bytes per launch (carried over from the profile run), or None when they do
    not describe this run."""
    t = PMC_TRAFFIC.get(workload)
    if not t or plan != 2 or not t["fetch_bytes"] or csrc_sha256() != PMC_TRAFFIC["csrc_sha256"]:
        return None
    return t["fetch_bytes"] + t["write_bytes"]


def stats_us(ms):
    """median / min / p90 of a list of millisecond samples, in microseconds"""
    a = np.asarray(ms, dtype=np.float64) * 1e3
    return {"median": float(np.median(a)), "min": float(a.min()), "p90": float(np.percentile(a, 90)), "n": int(a.size)}


def streaming_read_ceiling(torch, dev, stream):
    """GB/s of a loads-only kernel with the K/V-streaming kernel's access pattern (a measurement aid built
    into a shared object of its own), over three rotating 1 GiB buffers: the rate the memory system delivers
    to this kind of reader, next to the published peak the roofline is priced against."""
    import ctypes
    path = os.path.join(ROOT, "paper_2512_21450_amd", "libbench_stream_read.so")
    if not os.path.exists(path):
        return None
    lib = ctypes.CDLL(path)
    lib.bench_stream_read.restype = ctypes.c_int
    lib.bench_stream_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    lib.bench_stream_read_bytes.restype = ctypes.c_size_t
    lib.bench_stream_read_bytes.argtypes = [ctypes.c_size_t]
    n = 1 << 30
    bufs = [torch.zeros(n, dtype=torch.uint8, device=dev) for _ in range(3)]
    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    sh = ctypes.c_void_p(stream.cuda_stream)
    moved = lib.bench_stream_read_bytes(n)

    def go(i):
        rc = lib.bench_stream_read(bufs[i % 3].data_ptr(), n, sink.data_ptr(), sh)
        if rc != 0:
            raise RuntimeError(f"bench_stream_read failed ({rc})")
    for i in range(3):
        go(i)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(15)]
    for i, (a, b) in enumerate(ev):
        a.record(stream); go(i); b.record(stream)
    torch.cuda.synchronize()
    ms = np.median([a.elapsed_time(b) for a, b in ev])
    del bufs
    return moved / (ms * 1e-3) / 1e9


def run_decode(args, torch, B, wl, dev, wname, steps, warmup, event_calls, full):
    """One workload: K timed steps (wall clock, back to back), then `event_calls` calls bracketed by HIP
    events on the launch stream (the library records one more between its two kernels), then the parity
    check on sampled rows.  `full`: also the CPU-oracle and unoptimised-GPU reference rows."""
    w = wl.WORKLOADS[wname]
    algo = {"auto": B.RLDA_ALGO_AUTO, "simple": B.RLDA_ALGO_SIMPLE, "shared": B.RLDA_ALGO_SHARED}[args.algo]

    x = wl.make_inputs(w, threads=16)
    kv8 = args.kv == "e4m3" and w.dtype == "bf16"
    if kv8:
        x = wl.kv_to_e4m3(x)
    paged = args.page_size > 0
    active = None
    x0 = x                                    # contiguous layout, kept for the CPU leg
    if paged:
        x = wl.to_pages(x, args.page_size, seed=w.seed, poison=False)
        if args.finished > 0:
            active = (np.random.default_rng(w.seed).random(w.B) >= args.finished).astype(np.uint8)
    elif args.finished > 0:
        sys.exit("bench.py: --finished needs --page-size")
    # bytes the step must move: finished sequences contribute nothing, a prompt only if one of its sequences is live
    live_b = np.ones(w.B, bool) if active is None else active.astype(bool)
    live_p = live_b.reshape(w.P, w.G).any(axis=1)
    ab = wl.algorithmic_bytes(w, np.where(live_p, x["prefix_lens"], 0), np.where(live_b, x["suffix_lens"], 0),
                              kv_elem_bytes=1 if kv8 else 0)
    # what the K/V-streaming kernel itself has to read: the K/V rows, q and the lengths (out and lse are the
    # combine kernel's; the partial results between the two kernels are scratch, not the method's bytes)
    kern_bytes = ab["prefix"] + ab["suffix"] + w.B * w.Hq * w.d * w.elem_bytes + 4 * (w.P + w.B)

    def dev_t(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
        return torch.from_numpy(a).to(dev)

    base = {k: dev_t(v) for k, v in x.items() if isinstance(v, np.ndarray)}
    act_t = None if active is None else torch.from_numpy(active).to(dev)
    sets = [base] + [{k: (v.clone() if k.startswith(("k_", "v_")) else v) for k, v in base.items()}
                     for _ in range(max(args.sets, 1) - 1)]
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device=dev)
    lse = torch.empty((w.B, w.Hq), dtype=torch.float32, device=dev)
    descs = []
    ws = None
    for s in sets:
        if paged:
            ds = B.paged_desc_from_tensors(s["q"], s["k_prefix"], s["v_prefix"], s["prefix_lens"], s["k_pages"],
                                           s["v_pages"], s["block_table"], s["suffix_lens"], w.scale, w.G, out, lse,
                                           act_t, None, algo, s.get("k_scale"), s.get("v_scale"))
        else:
            ds = B.desc_from_tensors(s["q"], s["k_prefix"], s["v_prefix"], s["prefix_lens"], s["k_suffix"],
                                     s["v_suffix"], s["suffix_lens"], w.scale, w.G, out, lse, None, algo,
                                     s.get("k_scale"), s.get("v_scale"))
        if ws is None:
            need = B.rl_decode_attn_paged_workspace_bytes(ds) if paged else B.rl_decode_attn_workspace_bytes(ds)
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
        ds.workspace, ds.workspace_bytes = ws.data_ptr(), ws.numel()
        descs.append(ds)
    plan = B.rl_decode_attn_paged_plan(descs[0]) if paged else B.rl_decode_attn_plan(descs[0])
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    def step(i, mid=None):
        d_ = descs[i % len(descs)]
        rc = B.rl_decode_attn_paged_raw(d_, sh, mid) if paged else B.rl_decode_attn_profiled(d_, sh, mid)
        if rc != 0:
            raise B.RldaError(rc)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    value = int(live_b.sum()) / (ms_per_step * 1e-3)    # one query token per live sequence and step

    # per-call timings from HIP events on the launch stream: first the whole call (two events), then the
    # K/V-streaming kernel alone (a third event, recorded by the library between its two kernels; recording
    # it lengthens the step, so the whole-call figures come from the two-event loop)
    n_ev = max(event_calls, 1)
    ev2 = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_ev)]
    for i, (a, b) in enumerate(ev2):
        a.record(stream); step(i); b.record(stream)
    torch.cuda.synchronize()
    call_ms = [a.elapsed_time(b) for a, b in ev2]
    ev3 = [tuple(torch.cuda.Event(enable_timing=True) for _ in range(3)) for _ in range(n_ev)]
    for _, m, _ in ev3:
        m.record(stream)                      # materialise the handle the library records into
    torch.cuda.synchronize()
    for i, (a, m, b) in enumerate(ev3):
        a.record(stream); step(i, m.cuda_event); b.record(stream)
    torch.cuda.synchronize()
    kern_ms = [a.elapsed_time(m) for a, m, _ in ev3]
    rest_ms = [m.elapsed_time(b) for _, m, b in ev3]

    # sanity: the timed configuration still matches the oracle on sampled rows
    rng = np.random.default_rng(0)
    n_rows = 64 if full else 24
    rows = np.stack([rng.integers(0, w.B, n_rows), rng.integers(0, w.Hq, n_rows)], 1).astype(np.int32)
    from oracle import ref

    def oracle(**kw):
        if paged:
            return ref.decode_attn_paged_ref(x["q"], x["k_prefix"], x["v_prefix"], x["prefix_lens"], x["k_pages"],
                                             x["v_pages"], x["block_table"], x["suffix_lens"], active, w.scale, w.G,
                                             k_scale=x.get("k_scale"), v_scale=x.get("v_scale"), **kw)
        return ref.decode_attn_ref(x["q"], x["k_prefix"], x["v_prefix"], x["prefix_lens"], x["k_suffix"],
                                   x["v_suffix"], x["suffix_lens"], w.scale, w.G,
                                   k_scale=x.get("k_scale"), v_scale=x.get("v_scale"), **kw)

    ro, rl = oracle(rows=rows)
    step(0)
    torch.cuda.synchronize()
    o, l = out.cpu().numpy(), lse.cpu().numpy()
    tol_o, tol_l = (1e-5, 1e-5) if w.dtype == "f32" else (1e-2, 1e-3)
    err_o = max(float(np.abs(o[b, h] - ro[b, h]).max()) for b, h in rows)
    fin = [(b, h) for b, h in rows if np.isfinite(rl[b, h])]
    err_l = max([abs(float(l[b, h]) - rl[b, h]) for b, h in fin], default=0.0)
    parity_ok = bool(err_o <= tol_o and err_l <= tol_l)

    kern = stats_us(kern_ms)
    call = stats_us(call_ms)
    gbps = lambda nbytes, us: nbytes / (us * 1e-6) / 1e9
    res = {
        "workload": w.name, "ms_per_step": ms_per_step, "value": value, "steps": steps, "plan": plan,
        "algorithmic_bytes": ab, "kernel_algorithmic_bytes": kern_bytes,
        "whole_step_GBps": gbps(ab["total"], ms_per_step * 1e3),
        "whole_step_frac_of_hbm_peak": gbps(ab["total"], ms_per_step * 1e3) / HBM_PEAK_GBS,
        "whole_call_us_by_events": call,
        "kernel_us_by_events": kern,
        "kernel_GBps": gbps(kern_bytes, kern["median"]),
        "kernel_frac_of_hbm_peak": gbps(kern_bytes, kern["median"]) / HBM_PEAK_GBS,
        "rest_of_call_us_median": float(np.median(rest_ms) * 1e3),
        "mean_suffix_len": float(x["suffix_lens"].mean()), "max_suffix_len": int(x["suffix_lens"].max()),
        "mean_prefix_len": float(x["prefix_lens"].mean()),
        "parity": {"ok": parity_ok, "max_abs_err_out": err_o, "max_abs_err_lse": err_l, "rows": len(rows)},
        "traffic": None if paged or kv8 else measured_traffic(w.name, plan),
    }
    if not full:
        del sets, base, descs, ws
        return res

    # CPU baseline: the oracle as it stands on a bounded sample (whole sequences, all heads)
    cpu = None
    if args.cpu_seqs > 0:
        n = min(args.cpu_seqs, w.B)
        seqs = np.linspace(0, w.B - 1, n).astype(np.int32)
        rws = np.stack([np.repeat(seqs, w.Hq), np.tile(np.arange(w.Hq, dtype=np.int32), n)], 1)
        passes, c0 = 0, time.perf_counter()
        while True:                           # whole passes over the sample until about 10 s of wall time
            _, _, used = ref.decode_attn_ref(x0["q"], x0["k_prefix"], x0["v_prefix"], x0["prefix_lens"],
                                             x0["k_suffix"], x0["v_suffix"], x0["suffix_lens"], w.scale, w.G,
                                             rows=rws, return_threads=True,
                                             k_scale=x0.get("k_scale"), v_scale=x0.get("v_scale"))
            passes += 1
            c1 = time.perf_counter()
            if c1 - c0 >= args.cpu_seconds:
                break
        cpu = {"value": passes * n / (c1 - c0), "unit": "query-tokens/s", "cores": int(used), "kind": "oracle",
               "sample": f"{n} of {w.B} sequences (all {w.Hq} heads, evenly spaced, contiguous layout), "
                         f"{passes} passes, {c1 - c0:.2f} s"}

        # the same oracle on one thread, on every 16th sequence of the sample
        s1 = seqs[::16]
        r1 = np.stack([np.repeat(s1, w.Hq), np.tile(np.arange(w.Hq, dtype=np.int32), len(s1))], 1)
        c0 = time.perf_counter()
        ref.decode_attn_ref(x0["q"], x0["k_prefix"], x0["v_prefix"], x0["prefix_lens"], x0["k_suffix"],
                            x0["v_suffix"], x0["suffix_lens"], w.scale, w.G, rows=r1, n_threads=1,
                            k_scale=x0.get("k_scale"), v_scale=x0.get("v_scale"))
        cpu["one_thread_value"] = len(s1) / (time.perf_counter() - c0)
        cpu["one_thread_sample"] = f"{len(s1)} sequences, one pass"

    # second reference row: the unoptimised GPU kernel (one wavefront per row, no sharing, no split)
    naive = None
    if plan == 2 and not paged and args.naive_steps > 0:
        dn = descs[0]
        keep = dn.algo
        dn.algo = B.RLDA_ALGO_SIMPLE
        try:
            def naive_step():
                rc = B.rl_decode_attn_raw(dn, sh)
                if rc != 0:
                    raise B.RldaError(rc)
            for _ in range(2):
                naive_step()
            torch.cuda.synchronize()
            n0 = time.perf_counter()
            for _ in range(args.naive_steps):
                naive_step()
            torch.cuda.synchronize()
            nms = (time.perf_counter() - n0) * 1e3 / args.naive_steps
        finally:
            dn.algo = keep
        naive = {"kernel": "simple_kernel", "ms_per_step": nms, "steps": args.naive_steps,
                 "GBps": ab["total"] / (nms * 1e-3) / 1e9}
    res["cpu_baseline"] = cpu
    res["naive_gpu_baseline"] = naive
    res["config"] = {"workload": f"{w.name}: {w.note}; suffix {w.suffix}", "P": w.P, "G": w.G, "Hq": w.Hq,
                     "Hkv": w.Hkv, "d": w.d, "algo": {1: "simple", 2: "shared"}.get(plan, str(plan)),
                     "suffix_store": f"paged, {args.page_size} rows per page" if paged else "contiguous",
                     "kv_store": "e4m3 bytes, one factor per KV head" if kv8 else w.dtype,
                     "finished_sequences": int((~live_b).sum()),
                     "kv_sets_rotated": len(sets),
                     "mean_suffix_len": float(x["suffix_lens"].mean()), "max_suffix_len": int(x["suffix_lens"].max()),
                     "mean_prefix_len": float(x["prefix_lens"].mean())}
    res["dtype"] = w.dtype
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="vlm7b", help="tiny | vlm3b | vlm7b | agentic | highbatch")
    ap.add_argument("--algo", default="auto", choices=["auto", "simple", "shared"])
    ap.add_argument("--sets", type=int, default=3, help="rotating copies of the KV tensors")
    ap.add_argument("--event-calls", type=int, default=120,
                    help="calls timed one by one with HIP events (whatever --steps is), for the median / min / p90 figures")
    ap.add_argument("--others", type=int, default=-1,
                    help="1: also run the other four workloads in short form (key other_workloads); 0: do not; "
                         "default: only when --workload is the default one")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three 1 GiB device-to-device copies (reference for scaling HBM counters)")
    ap.add_argument("--kv", default="bf16", choices=["bf16", "e4m3"],
                    help="element type of the K/V stores (e4m3: one byte per element plus a factor per KV head; "
                         "q and the arithmetic stay bf16)")
    ap.add_argument("--naive-steps", type=int, default=20,
                    help="steps of the unoptimised GPU kernel timed as a reference row (0 = skip)")
    ap.add_argument("--page-size", type=int, default=0,
                    help="0: contiguous suffix store (the headline configuration); else rows per page of a paged store")
    ap.add_argument("--finished", type=float, default=0.0,
                    help="fraction of sequences marked finished (paged store only)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="wall time given to the CPU-oracle leg")
    ap.add_argument("--cpu-seqs", type=int, default=256, help="sequences in the CPU-oracle sample (0 = skip)")
    ap.add_argument("--op", default="decode_attn", choices=["decode_attn", "token_logprob", "policy_loss", "prefill", "tree"],
                    help="decode_attn: the headline path; token_logprob: per-token log-prob / entropy / KL kernel; "
                         "policy_loss: group advantages + clipped policy loss over --rows sequences of --tokens tokens; "
                         "prefill: causal attention of the workload's prompts over themselves; "
                         "tree: rl_decode_attn_tree on a two-level agentic batch, beside the same step composed of "
                         "two rl_decode_attn calls and rl_lse_combine")
    ap.add_argument("--tokens", type=int, default=1024, help="policy_loss: token capacity per sequence")
    ap.add_argument("--rows", type=int, default=256, help="token_logprob: rows of logits (tokens)")
    ap.add_argument("--vocab", type=int, default=0, help="token_logprob: vocabulary size (default: Qwen2's 151936)")
    ap.add_argument("--no-ref", action="store_true", help="token_logprob: no reference logits (no KL)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this is a single-GPU kernel library; only --gpus 1 is supported "
              "(the path shards by prompt group with no exchange, nothing to measure across GPUs here)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_21450_amd import binding as B
    from paper_2512_21450_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    if args.op == "token_logprob":
        return bench_token_logprob(args, torch, B, wl, dev)
    if args.op == "policy_loss":
        return bench_policy_loss(args, torch, B, wl, dev)
    if args.op == "prefill":
        return bench_prefill(args, torch, B, wl, dev)
    if args.op == "tree":
        return bench_tree(args, torch, B, wl, dev)
    if args.kv == "e4m3" and wl.WORKLOADS[args.workload].dtype != "bf16":
        sys.exit("bench.py: --kv e4m3 needs a bf16 workload")
    stream = torch.cuda.current_stream()

    if args.copy_probe:                       # a plain copy of known size, for calibrating rocprofv3 byte counters
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    ceiling = streaming_read_ceiling(torch, dev, stream)
    r = run_decode(args, torch, B, wl, dev, args.workload, args.steps, args.warmup, args.event_calls, full=True)
    others = None
    default_run = args.workload == "vlm7b" and args.page_size == 0 and args.kv == "bf16" and args.algo == "auto"
    if args.others == 1 or (args.others < 0 and default_run):
        others = {}
        for name in OTHER_WORKLOADS:
            if name == args.workload:
                continue
            o = run_decode(args, torch, B, wl, dev, name, min(args.steps, 100), min(args.warmup, 10),
                           min(args.event_calls, 60), full=False)
            others[name] = {k: o[k] for k in ("ms_per_step", "value", "plan", "algorithmic_bytes", "whole_step_GBps",
                                              "whole_step_frac_of_hbm_peak", "whole_call_us_by_events",
                                              "kernel_us_by_events", "kernel_algorithmic_bytes", "kernel_frac_of_hbm_peak",
                                              "traffic", "mean_suffix_len",
                                              "max_suffix_len", "mean_prefix_len", "parity")}
            torch.cuda.empty_cache()

    kern = r["kernel_us_by_events"]
    achieved = r["kernel_GBps"]
    res = {
        "metric": "decode-attn query-tokens/sec and achieved HBM GB/s (% of MI355X peak), 7B shape",
        "value": r["value"], "unit": "query-tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": r["dtype"], "data": "synthetic",
        "config": r["config"],
        "achieved_GBps_whole_step": r["whole_step_GBps"],
        "pct_of_hbm_peak_whole_step": 100.0 * r["whole_step_frac_of_hbm_peak"],
        "whole_call_us_by_events": r["whole_call_us_by_events"],
        "algorithmic_bytes": r["algorithmic_bytes"],
        # the dominant kernel alone: the bytes it has to read / its duration (median over the event-timed calls)
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": r["traffic"],
                     "traffic_source": "rocprofv3 counters of an earlier profile run of the same sources (profiles/)",
                     "kernel": "partial_kernel" if r["plan"] == 2 else "simple_kernel",
                     "kernel_algorithmic_bytes": r["kernel_algorithmic_bytes"],
                     "kernel_us_median": kern["median"], "kernel_us_min": kern["min"], "kernel_us_p90": kern["p90"],
                     "event_timed_calls": kern["n"],
                     "rest_of_call_us_median": r["rest_of_call_us_median"],
                     "streaming_read_ceiling_GBps": ceiling},
        "cpu_baseline": r["cpu_baseline"],
        "naive_gpu_baseline": r["naive_gpu_baseline"],
        "parity": r["parity"],
        "other_workloads": others,
    }
    print(json.dumps(res))
    ok = r["parity"]["ok"] and all(o["parity"]["ok"] for o in (others or {}).values())
    if not ok:
        sys.exit(1)


def bench_tree(args, torch, B, wl, dev):
    """One step = one rl_decode_attn_tree call on a two-level agentic batch (7B shape, 16 prompts x G = 8: the
    prompt shared by the 8 samples, a first turn shared by sub-groups of 4, long-tailed own suffixes), and the
    same step composed of what existed before: one rl_decode_attn call per level and rl_lse_combine."""
    Bn, Hq, Hkv, d, G0, G1 = 128, 28, 4, 128, 8, 4
    x = wl.make_tree_inputs(1004, Bn, Hq, Hkv, d, [(G0, 1344, ("agentic", 3, 256, 64, 192)), (G1, 512, ("uniform", 512))],
                            4096, ("lognormal", 300.0, 1.0), threads=16)
    scale = 1.0 / np.sqrt(d)
    to_dev = lambda a: (torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16) if a.dtype == np.uint16
                        else torch.from_numpy(a).to(dev))
    sets = []
    for i in range(max(args.sets, 1)):
        lv = [(to_dev(k), to_dev(v), to_dev(l), g) for k, v, l, g in x["levels"]]
        sets.append(dict(q=to_dev(x["q"]), lv=lv, ks=to_dev(x["k_suffix"]), vs=to_dev(x["v_suffix"]), sl=to_dev(x["suffix_lens"])))
    out = torch.empty((Bn, Hq, d), dtype=torch.float32, device=dev)
    lse = torch.empty((Bn, Hq), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    descs, ws = [], None
    for t in sets:
        ds = B.tree_desc_from_tensors(t["q"], t["lv"], t["ks"], t["vs"], t["sl"], scale, out, lse)
        if ws is None:
            ws = torch.empty(max(B.rl_decode_attn_tree_workspace_bytes(ds), 256), dtype=torch.uint8, device=dev)
        ds.workspace, ds.workspace_bytes = ws.data_ptr(), ws.numel()
        descs.append(ds)

    def step_tree(i):
        rc = B.rl_decode_attn_tree_raw(descs[i % len(descs)], sh)
        if rc != 0:
            raise B.RldaError(rc)

    # the composition: level 0 as a prefix-only call, level 1 as the "prefix" of groups of G1 with the suffixes, then the merge
    parts_o = torch.empty((2, Bn, Hq, d), dtype=torch.float32, device=dev)
    parts_l = torch.empty((2, Bn, Hq), dtype=torch.float32, device=dev)
    no_len = torch.zeros(Bn, dtype=torch.int32, device=dev)
    comp, ws2 = [], None
    for t in sets:
        (k0, v0, l0, _), (k1, v1, l1, _) = t["lv"]
        ks0 = t["ks"][:, :, :0].contiguous()
        da = B.desc_from_tensors(t["q"], k0, v0, l0, ks0, ks0, no_len, scale, G0, parts_o[0], parts_l[0])
        db = B.desc_from_tensors(t["q"], k1, v1, l1, t["ks"], t["vs"], t["sl"], scale, G1, parts_o[1], parts_l[1])
        if ws2 is None:
            n2 = max(B.rl_decode_attn_workspace_bytes(da), B.rl_decode_attn_workspace_bytes(db), 256)
            ws2 = torch.empty(n2, dtype=torch.uint8, device=dev)
        for dd in (da, db):
            dd.workspace, dd.workspace_bytes = ws2.data_ptr(), ws2.numel()
        comp.append((da, db))
    out2 = torch.empty_like(out)
    lse2 = torch.empty_like(lse)

    def step_comp(i):
        da, db = comp[i % len(comp)]
        rc = B.rl_decode_attn_raw(da, sh) or B.rl_decode_attn_raw(db, sh)
        if rc != 0:
            raise B.RldaError(rc)
        B.rl_lse_combine(parts_o.view(2, Bn * Hq, d), parts_l.view(2, Bn * Hq), out2.view(Bn * Hq, d), lse2.view(Bn * Hq))

    def timed(step):
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / args.steps
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(args.event_calls, 1))]
        for i, (a, b) in enumerate(ev):
            a.record(stream); step(i); b.record(stream)
        torch.cuda.synchronize()
        return wall, stats_us([a.elapsed_time(b) for a, b in ev])

    ms_tree, ev_tree = timed(step_tree)
    ms_comp, ev_comp = timed(step_comp)
    row = Hkv * 2 * d * 2
    lens0, lens1 = x["levels"][0][2], x["levels"][1][2]
    nbytes = (int(lens0.sum()) + int(lens1.sum()) + int(x["suffix_lens"].sum())) * row \
        + Bn * Hq * d * 2 + Bn * Hq * d * 4 + Bn * Hq * 4 + 4 * (len(lens0) + len(lens1) + Bn)

    from oracle import ref
    rng = np.random.default_rng(0)
    rows = np.stack([rng.integers(0, Bn, 48), rng.integers(0, Hq, 48)], 1).astype(np.int32)
    c0 = time.perf_counter()
    ro, rl = ref.decode_attn_tree_ref(x["q"], x["levels"], x["k_suffix"], x["v_suffix"], x["suffix_lens"], scale, rows=rows)
    c1 = time.perf_counter()
    step_tree(0); step_comp(0)
    torch.cuda.synchronize()
    errs = {}
    for name, (o, l) in (("tree", (out, lse)), ("composition", (out2, lse2))):
        o, l = o.cpu().numpy(), l.cpu().numpy()
        errs[name] = (max(float(np.abs(o[b, h] - ro[b, h]).max()) for b, h in rows),
                      max(abs(float(l[b, h]) - rl[b, h]) for b, h in rows))
    ok = all(eo <= 1e-2 and el <= 1e-3 for eo, el in errs.values())
    achieved = nbytes / (ms_tree * 1e-3) / 1e9
    print(json.dumps({
        "metric": "prefix-tree decode-attn query-tokens/sec and achieved HBM GB/s", "value": Bn / (ms_tree * 1e-3),
        "unit": "query-tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_tree,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"two-level agentic batch: {Bn} sequences, {Hq}/{Hkv} heads, prompt shared by {G0} "
                               f"(mean {lens0.mean():.0f} keys), first turn shared by {G1} (mean {lens1.mean():.0f}), own "
                               f"suffix mean {x['suffix_lens'].mean():.0f} max {int(x['suffix_lens'].max())}",
                   "kv_sets_rotated": len(sets)},
        "algorithmic_bytes": nbytes,
        "call_us_by_events": ev_tree,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "partial_kernel (tree form) + combine_kernel, whole call"},
        "composition_of_existing_calls": {"what": "rl_decode_attn (level 0, no suffix) + rl_decode_attn (level 1 as prefix, with "
                                                  "suffixes) + rl_lse_combine: five kernels, q read twice, fp32 partials through HBM",
                                          "ms_per_step": ms_comp, "call_us_by_events": ev_comp,
                                          "speedup_of_tree_call": ms_comp / ms_tree},
        "cpu_baseline": {"value": len(rows) / Hq / (c1 - c0), "unit": "query-tokens/s", "cores": os.cpu_count(), "kind": "oracle",
                         "sample": f"{len(rows)} (sequence, head) rows of {Bn * Hq}, {c1 - c0:.2f} s"},
        "parity": {"ok": bool(ok), "max_abs_err_out_lse": errs},
    }))
    if not ok:
        sys.exit(1)


def bench_token_logprob(args, torch, B, wl, dev):
    """One step = one rl_token_logprob call over [rows, vocab] bf16 logits (+ reference logits)."""
    V = args.vocab or wl.QWEN2_VOCAB
    n, ref = args.rows, not args.no_ref
    x = wl.make_logits(n, V, seed=3001, dtype="bf16", with_ref=ref, threads=16)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    ids = torch.from_numpy(x["token_ids"]).to(dev)
    sets = [(to_dev(x["logits"]), to_dev(x["ref_logits"]) if ref else None)]
    for _ in range(max(args.sets, 1) - 1):
        sets.append(tuple(None if t is None else t.clone() for t in sets[0]))
    names = ("logprob", "lse", "entropy", "ref_logprob", "kl") if ref else ("logprob", "lse", "entropy")
    outs = {k: torch.empty(n, dtype=torch.float32, device=dev) for k in names}
    descs, ws = [], None
    for lg, rf in sets:
        ds = B.token_logprob_desc_from_tensors(lg, ids, 1.0, rf, outs)
        if ws is None:
            ws = torch.empty(max(B.rl_token_logprob_workspace_bytes(ds), 256), dtype=torch.uint8, device=dev)
        ds.workspace, ds.workspace_bytes = ws.data_ptr(), ws.numel()
        descs.append(ds)
    stream = torch.cuda.current_stream()

    def step(i):
        rc = B.rl_token_logprob_raw(descs[i % len(descs)], stream.cuda_stream)
        if rc != 0:
            raise B.RldaError(rc)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    every = 8                                               # two event records cost a few us: not on every step
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % every == 0:
            ev[i][0].record(stream); step(i); ev[i][1].record(stream)
        else:
            step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    call_us = float(np.mean([ev[i][0].elapsed_time(ev[i][1]) for i in range(0, args.steps, every)]) * 1e3)
    nbytes = n * V * 2 * (2 if ref else 1) + n * 4 * (1 + len(names))

    from oracle.token_stats_ref import token_stats_ref
    rows = np.linspace(0, n - 1, min(n, 16)).astype(np.int64)
    c0 = time.perf_counter()
    r = token_stats_ref(x["logits"][rows], x["token_ids"][rows], 1.0, x["ref_logits"][rows] if ref else None)
    c1 = time.perf_counter()
    tol = {"logprob": 2e-5, "lse": 2e-5, "ref_logprob": 2e-5, "entropy": 1e-4, "kl": 1e-4}
    errs = {k: float(np.abs(outs[k].cpu().numpy()[rows] - r[k]).max()) for k in names}
    ok = all(errs[k] <= tol[k] for k in names)
    achieved = nbytes / (call_us * 1e-6) / 1e9
    print(json.dumps({
        "metric": "token log-prob / entropy / KL rows per second and achieved HBM GB/s", "value": n / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"token_logprob: {n} rows x {V} bf16 logits" + (" + reference logits" if ref else ""),
                   "kv_sets_rotated": len(sets)},
        "algorithmic_bytes": nbytes,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "token_partial_kernel (+ final merge)",
                     "call_us_mean": call_us},
        "cpu_baseline": {"value": len(rows) / (c1 - c0), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                         "sample": f"{len(rows)} of {n} rows, {c1 - c0:.2f} s"},
        "parity": {"ok": ok, "max_abs_err": errs},
    }))
    if not ok:
        sys.exit(1)


MFMA_BF16_PEAK_TFLOPS = 2500.0     # dense bf16 matrix-core peak of MI355X


def bench_prefill(args, torch, B, wl, dev):
    """One step = rl_prefill_attn over the prompts of --workload (prefix K/V, lengths and a query per token)."""
    w = wl.WORKLOADS[args.workload]
    if w.dtype != "bf16" or w.d != 128:
        sys.exit("bench.py: --op prefill needs a bf16, d = 128 workload")
    rng = np.random.default_rng(w.seed)
    lens = wl._draw_lens(rng, w.prefix, w.P, w.Lp_cap)
    k = wl._normal_tensor(w.seed, 1, (w.P, w.Hkv, w.Lp_cap, w.d), "bf16", 1.0, 16)
    v = wl._normal_tensor(w.seed, 2, (w.P, w.Hkv, w.Lp_cap, w.d), "bf16", 1.0, 16)
    q = wl._normal_tensor(w.seed, 5, (w.P, w.Lp_cap, w.Hq, w.d), "bf16", w.q_gain, 16)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
    tl = torch.from_numpy(lens).to(dev)
    # rotating copies of q / k / v / out, so that no call finds its inputs in the 256 MB memory-side cache
    sets = []
    for i in range(max(args.sets, 1)):
        tq, tk, tv = (to_dev(q), to_dev(k), to_dev(v)) if i == 0 else (sets[0][0].clone(), sets[0][1].clone(), sets[0][2].clone())
        o_ = torch.zeros((w.P, w.Lp_cap, w.Hq, w.d), dtype=torch.float32, device=dev)
        l_ = torch.zeros((w.P, w.Lp_cap, w.Hq), dtype=torch.float32, device=dev)
        sets.append((tq, tk, tv, o_, l_, B.prefill_desc_from_tensors(tq, tk, tv, tl, w.scale, o_, l_)))
    out, lse = sets[0][3], sets[0][4]
    stream = torch.cuda.current_stream()
    calls = [0]

    def step():
        rc = B.rl_prefill_attn_raw(sets[calls[0] % len(sets)][5], stream.cuda_stream)
        calls[0] += 1
        if rc != 0:
            raise B.RldaError(rc)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    call_us = e0.elapsed_time(e1) * 1e3 / args.steps
    L = lens.astype(np.int64)
    flops = int((4 * w.d * w.Hq * (L * (L + 1) // 2)).sum())          # 2 d per (query, visible key) pair for QK^T, 2 d for PV
    tokens = int(L.sum())

    from oracle.prefill_ref import prefill_attn_ref
    c0 = time.perf_counter()
    ro, rl = prefill_attn_ref(q[:1], k[:1], v[:1], lens[:1], w.scale)
    c1 = time.perf_counter()
    o, l = out[0].cpu().numpy().astype(np.float64), lse[0].cpu().numpy().astype(np.float64)
    n0 = int(lens[0])
    err_o, err_l = float(np.abs(o[:n0] - ro[0, :n0]).max()), float(np.abs(l[:n0] - rl[0, :n0]).max())
    ok = err_o <= 1e-2 and err_l <= 1e-3
    achieved = flops / (call_us * 1e-6) / 1e12
    print(json.dumps({
        "metric": "prefill-attention prompt tokens per second and achieved matrix-core TFLOP/s", "value": tokens / (ms_per_step * 1e-3),
        "unit": "prompt-tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"prefill of {w.name}: {w.P} prompts, mean length {L.mean():.0f}, {w.Hq}/{w.Hkv} heads, d={w.d}",
                   "tensor_sets_rotated": len(sets)},
        "algorithmic_flops": flops,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "kernel": "prefill_kernel",
                     "kernel_us_mean": call_us},
        "cpu_baseline": {"value": n0 / (c1 - c0), "unit": "prompt-tokens/s", "cores": 1, "kind": "oracle",
                         "sample": f"prompt 0 of {w.P} ({n0} tokens, all heads), {c1 - c0:.2f} s"},
        "parity": {"ok": bool(ok), "max_abs_err_out": err_o, "max_abs_err_lse": err_l, "rows": n0 * w.Hq},
    }))
    if not ok:
        sys.exit(1)


def bench_policy_loss(args, torch, B, wl, dev):
    """One step = rl_group_advantage + rl_policy_loss (with KL and entropy terms and the gradient) over
    [rows, tokens] per-token tensors with lognormal response lengths."""
    n, T, G = args.rows, args.tokens, 16
    n -= n % G
    x = wl.make_rollout_tokens(n, T, G, seed=4001, lens=("lognormal", 200.0, 1.0))
    t = {k: torch.from_numpy(v).to(dev) for k, v in x.items() if isinstance(v, np.ndarray)}
    stats = torch.empty(8, dtype=torch.float32, device=dev)
    grad = torch.empty((n, T), dtype=torch.float32, device=dev)
    rewards = torch.empty(n, dtype=torch.float32, device=dev)
    adv = torch.empty(n, dtype=torch.float32, device=dev)
    da = B.make_group_advantage_desc(n // G, G, x["metrics"].shape[0], metrics=t["metrics"].data_ptr(),
                                     weights=t["weights"].data_ptr(), rewards=rewards.data_ptr(), advantages=adv.data_ptr())
    dl = B.policy_loss_desc_from_tensors(t["logprob"], t["old_logprob"], adv, t["lens"], 0.2, 0.28, stats, t["kl"],
                                         t["entropy"], grad, 0.04, 0.01, agg=B.RL_AGG_SEQ_MEAN)
    ws = torch.empty(max(B.rl_policy_loss_workspace_bytes(dl), 256), dtype=torch.uint8, device=dev)
    dl.workspace, dl.workspace_bytes = ws.data_ptr(), ws.numel()
    stream = torch.cuda.current_stream()

    def step():
        rc = B.rl_group_advantage_raw(da, stream.cuda_stream) or B.rl_policy_loss_raw(dl, stream.cuda_stream)
        if rc != 0:
            raise B.RldaError(rc)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    call_us = e0.elapsed_time(e1) * 1e3 / args.steps
    valid = int(np.clip(x["lens"], 0, T).sum())
    nbytes = valid * 4 * 4 + n * T * 4 + n * 4 * 4          # four input arrays on valid tokens, the gradient rows, per-sequence vectors

    from oracle.policy_loss_ref import AGG_SEQ_MEAN, group_advantage_ref, policy_loss_ref
    c0 = time.perf_counter()
    _, a_ref = group_advantage_ref(x["metrics"], x["weights"], G)
    r = policy_loss_ref(x["logprob"], x["old_logprob"], a_ref.astype(np.float32), x["lens"], 0.2, 0.28, kl=x["kl"],
                        entropy=x["entropy"], beta_kl=0.04, beta_ent=0.01, agg=AGG_SEQ_MEAN)
    c1 = time.perf_counter()
    got = dict(zip(B.POLICY_LOSS_STATS, stats.cpu().numpy().astype(np.float64)))
    errs = {k: abs(got[k] - r[k]) for k in ("loss", "pg", "kl", "entropy")}
    ok = all(errs[k] <= 1e-4 * abs(r[k]) + 1e-6 for k in errs) and got["n_tokens"] == r["n_tokens"]
    achieved = nbytes / (call_us * 1e-6) / 1e9
    print(json.dumps({
        "metric": "policy-loss tokens per second and achieved HBM GB/s", "value": valid / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"policy_loss: {n} sequences x {T} tokens (G={G}), lognormal lengths, {valid} valid tokens, "
                               "KL + entropy terms, gradient written"},
        "algorithmic_bytes": nbytes,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "group_advantage_kernel + policy_count_kernel + policy_loss_kernel + policy_loss_reduce_kernel",
                     "call_us_mean": call_us},
        "cpu_baseline": {"value": valid / (c1 - c0), "unit": "tokens/s", "cores": 1, "kind": "oracle",
                         "sample": f"the whole batch, one pass, {c1 - c0:.2f} s"},
        "parity": {"ok": bool(ok), "abs_err": errs},
    }))
    if not ok:
        sys.exit(1)


if __name__ == "__main__":
    main()
