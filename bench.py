#!/usr/bin/env python3
"""Benchmark of the FlexiCache decode hot path on one MI355X.

A step is one pass of the whole hot path over one batch: on rerank steps fc_rerank_topk +
fc_promote_pages, then always fc_sparse_decode_attn.  All inputs (pool, tables, MinMax cache, every
step's queries) are resident in HBM before the timed region; the host pool sits in pinned memory.
Prints one JSON line."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per whole-pass attention launch as rocprofv3 counted them (FETCH_SIZE + WRITE_SIZE, each scaled by what the
# same counter reads for a kernel of known size in the same run): stored values, not measured by this script;
# the summaries they come from are named beside them.
STORED_TRAFFIC = {
    "cfg4_ragged_b64": (3468703135, "profiles/decode_hot_path_cfg4_ragged_b64.md"),
    "cfg2_llama8b_32k": (594121102, "profiles/decode_hot_path_cfg2_llama8b_32k.md"),
    "cfg3_long_128k": (590859109, "profiles/decode_hot_path_cfg3_long_128k.md"),
    "cfg5_offload_64k": (1784639509, "profiles/decode_hot_path_cfg5_offload_64k.md"),
}
MIN_BRACKETED_LAUNCHES = 32


def attention_bytes(cfg, unstable_topk: bool = False) -> int:
    """Algorithmic bytes one fc_sparse_decode_attn call must move: per attended page its valid tokens'
    K and V (512 B per token) and its 4 B table entry (+4 B list entry for a stable head); per
    (sequence, query head) 256 B of query and 512 B of fp32 output."""
    tot = 0
    for b in range(cfg.batch):
        n = cfg.num_pages(b)
        tail = cfg.ctx[b] - 16 * (n - 1)
        for h in range(cfg.num_kv_heads):
            if cfg.stable[h] or unstable_topk:
                k = min(cfg.topk[b], n)
                # the partial last page is always a member of a stable head's set
                toks = 16 * k - ((16 - tail) if tail < 16 else 0)
                tot += 512 * toks + 8 * k
            else:
                tot += 512 * cfg.ctx[b] + 4 * n
        tot += cfg.num_q_heads * (256 + 512)
    return tot


def rerank_bytes(cfg, stable: bool = True) -> int:
    """512 B of MinMax per page of every reranking (sequence, stable head), its queries, 4 B per selected page."""
    tot = 0
    for b in range(cfg.batch):
        n = cfg.num_pages(b)
        for h in range(cfg.num_kv_heads):
            if cfg.stable[h] == stable:
                tot += 512 * n + cfg.group * 256 + 4 * min(cfg.topk[b], n)
    return tot


def cpu_baseline(cfg, wl, budget_s: float = 15.0, unstable_topk: bool = False):
    """Times the CPU oracle, as it stands, on whole decode steps of the same workload (step 0, 1, 2, ...
    with their own queries and the configuration's rerank interval) until `budget_s` seconds of work
    have been done (at least one step)."""
    import oracle
    dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, cfg.topk,
                               cfg.rerank_interval, unstable_topk=unstable_topk)
    mm = [oracle.seq_build_minmax(wl.k[b], cfg.ctx[b]) for b in range(cfg.batch)]   # untimed: an input
    t0 = time.perf_counter()
    nbytes, steps = 0, 0
    while True:
        q = wl.queries(steps)
        if unstable_topk:
            for b in range(cfg.batch):
                dec.rerank_unstable(b, q[b], mm[b])
            nbytes += rerank_bytes(cfg, stable=False)
        if cfg.is_rerank_step(steps):
            for b in range(cfg.batch):
                dec.rerank(b, q[b], mm[b])
            nbytes += rerank_bytes(cfg)
        for b in range(cfg.batch):
            dec.attend(b, q[b], wl.k[b], wl.v[b])
        nbytes += attention_bytes(cfg, unstable_topk)
        steps += 1
        el = time.perf_counter() - t0
        if el > budget_s:
            break
    res = {"value": round(nbytes / el / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
           "sample": f"{steps} whole decode step(s) of {cfg.name} (all {cfg.batch} sequences, rerank every "
                     f"{cfg.rerank_interval} steps), {el:.1f} s of oracle time", "s_per_step": round(el / steps, 4)}
    if cfg.index in (1, 2) and res["cores"] > 1:
        # the same oracle on one thread, a few plain steps (attention only, the bulk of a step), about 5 s
        all_threads = res["cores"]
        oracle.set_threads(1)
        t0, n1 = time.perf_counter(), 0
        while True:
            q = wl.queries(steps + n1)
            for b in range(cfg.batch):
                dec.attend(b, q[b], wl.k[b], wl.v[b])
            n1 += 1
            e1 = time.perf_counter() - t0
            if e1 > budget_s / 3:
                break
        oracle.set_threads(all_threads)
        res["single_thread"] = {"value": round(n1 * attention_bytes(cfg, unstable_topk) / e1 / 1e9, 3), "unit": "GB/s",
                                "s_per_step": round(e1 / n1, 4), "sample": f"{n1} attention step(s), {e1:.1f} s"}
    return res


def device_facts(torch):
    """What the runtime says about the GPU the numbers were taken on."""
    pr = torch.cuda.get_device_properties(0)
    return {"name": pr.name, "arch": getattr(pr, "gcnArchName", None), "compute_units": pr.multi_processor_count,
            "hbm_GiB": round(pr.total_memory / 2 ** 30, 1), "l2_per_xcd_MiB": round(getattr(pr, "L2_cache_size", 0) / 2 ** 20, 1),
            "lds_per_workgroup_KiB": round(getattr(pr, "shared_memory_per_block", 0) / 1024, 1),
            "wavefront": getattr(pr, "warp_size", None)}


def run_workload(args, index: int, torch, *, main_workload: bool):
    """Builds one workload, runs warm-up + exactly args.steps timed steps, then the diagnostic passes.
    Returns the full result dictionary of that workload."""
    from paper_2511_00868_amd import binding, synth
    from paper_2511_00868_amd.session import DecodeSession

    total_steps = args.warmup + args.steps
    cfg = synth.make_config(index, batch=args.batch if main_workload else None, ctx=args.ctx if main_workload else None,
                            steps=total_steps)
    diag_steps = min(args.steps, 32)     # per diagnostic pass; with --append both passes append
    if args.append:
        import dataclasses
        cfg = dataclasses.replace(cfg, append_tokens=total_steps + 3 * diag_steps, dynamics="static")
    t_gen = time.perf_counter()
    wl = synth.Workload(cfg)
    mode = binding.FC_PROMOTE_GATHER if args.promote_mode == "gather" else binding.FC_PROMOTE_MEMCPY
    sess = DecodeSession(cfg, wl, promote_mode=mode, attn_waves=args.attn_waves, unstable_topk=args.paper_unstable_topk)
    q_all = torch.stack([sess.bits_to_dev(wl.queries(t)) for t in range(total_steps)])
    new_kv = None
    if args.append:
        toks = [wl.append(t) for t in range(total_steps + 3 * diag_steps)]
        new_kv = (torch.stack([sess.bits_to_dev(k) for k, _ in toks]), torch.stack([sess.bits_to_dev(v) for _, v in toks]))
    n_appended = [0]
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    if args.no_overlap:
        sess.overlap = False
    elif args.overlap_by != "auto":      # auto: the session's own choice (riding copies for all but tiny workloads)
        sess.overlap = True if args.overlap_by == "pages" else args.overlap_by
    main = torch.cuda.current_stream()

    def run_step(t, marks=None):
        sess.q = q_all[t]
        if marks is not None:
            e = torch.cuda.Event(enable_timing=True)
            e.record(main)
            marks.append(e)
        if new_kv is not None and (t > 0 or n_appended[0] > 0):   # appends start after the cold fill: before it no page of a stable head, the partial last one included, is in HBM
            i = n_appended[0]
            sess.append_dev(new_kv[0][i], new_kv[1][i])
            n_appended[0] = i + 1
        sess.step(t)

    for t in range(args.warmup):
        run_step(t)
    torch.cuda.synchronize()
    sess.ctx.fc_check_device_state()

    # ---- timed region: exactly `steps` steps, nothing but the hot path on the stream -----------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.warmup, total_steps):
        run_step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    sess.ctx.fc_check_device_state()
    is_rer_timed = [cfg.is_rerank_step(t) and any(cfg.stable) for t in range(args.warmup, total_steps)]

    # ---- diagnostic pass 1 (untimed for `value`): per-step durations from one event per step ----------
    diag = diag_steps
    diag = diag - diag % cfg.rerank_interval or diag
    marks = []
    for t in range(diag):
        run_step(t % total_steps, marks)
    e_end = torch.cuda.Event(enable_timing=True)
    e_end.record(main)
    torch.cuda.synchronize()
    marks.append(e_end)
    step_us = [marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(diag)]
    is_rer = [cfg.is_rerank_step(t % total_steps) and any(cfg.stable) for t in range(diag)]
    rer_us = [u for u, r in zip(step_us, is_rer) if r]
    plain_us = [u for u, r in zip(step_us, is_rer) if not r]

    # ---- diagnostic pass 1b: the parts of a rerank step, from events inside the step (each recorded event holds
    # the stream up for a few microseconds, which is why the step durations above come from a pass without them)
    rr_us, pr_us, cp_us = [], [], []
    names = ("rerank_begin", "rerank_end", "recycle_end", "copies_end")
    for t in range(diag):
        tt = t % total_steps
        rer = cfg.is_rerank_step(tt) and any(cfg.stable)
        sess.events = {k: torch.cuda.Event(enable_timing=True) for k in names} if rer else None
        run_step(tt)
        if rer:
            ev = sess.events
            torch.cuda.synchronize()
            rr_us.append(ev["rerank_begin"].elapsed_time(ev["rerank_end"]) * 1e3)
            pr_us.append(ev["rerank_end"].elapsed_time(ev["recycle_end"]) * 1e3)
            cp_us.append(ev["recycle_end"].elapsed_time(ev["copies_end"]) * 1e3)
    # ... and the chain in front of the page copies as the timed region runs it: fc_rerank_promote, one call
    chain_us = []
    if sess.fused_rerank:
        for t in range(diag):
            tt = t % total_steps
            rer = cfg.is_rerank_step(tt) and any(cfg.stable)
            sess.events = {k: torch.cuda.Event(enable_timing=True) for k in ("chain_begin", "chain_end")} if rer else None
            run_step(tt)
            if rer:
                torch.cuda.synchronize()
                chain_us.append(sess.events["chain_begin"].elapsed_time(sess.events["chain_end"]) * 1e3)
    sess.events = None
    promoted_last = int(sess.total_promoted[0])

    # ---- diagnostic pass 2: the dominant kernel, every launch bracketed by HIP events on its own stream ----
    # plain steps (a whole-pass attention launch each, the launch configuration of the timed region), as many as it
    # takes for MIN_BRACKETED_LAUNCHES brackets whatever --steps was
    raw_ms = empty_ms = 0.0
    launches = 0
    if not args.no_kernel_events:
        sess.ctx.fc_profile_begin(1, main)
        n_plain = max(MIN_BRACKETED_LAUNCHES, args.kernel_launches)
        for i in range(n_plain):
            sess.q = q_all[i % total_steps]
            if args.paper_unstable_topk and not all(cfg.stable):
                sess.rerank_unstable()
            sess.attend()
        torch.cuda.synchronize()
        raw_ms, empty_ms, launches = sess.ctx.fc_profile_end()
    sess.ctx.fc_check_device_state()

    # same-box ceiling: a plain streaming read of as many bytes of the pool as one attention call moves
    a_bytes, r_bytes = attention_bytes(cfg, args.paper_unstable_topk), rerank_bytes(cfg)
    pool_bytes = sess.kv_pool.numel() * sess.kv_pool.element_size()
    ceil_bytes = min(pool_bytes, a_bytes) // 4096 * 4096
    ceil_gbs, ceil_us = sess.ctx.fc_measure_stream_read(sess.kv_pool, ceil_bytes, 16, main)

    ride = sess.overlap in ("ride", "heads-ride")
    inline = sess.overlap in ("inline", "heads-inline")
    n_rerank = sum(is_rer_timed)
    step_bytes = a_bytes * args.steps + r_bytes * n_rerank
    if args.paper_unstable_topk:
        step_bytes += rerank_bytes(cfg, stable=False) * args.steps
    value = step_bytes / elapsed / 1e9
    # `achieved` uses the raw bracket (event, kernel, event): it contains the kernel plus the bracket's own dispatch
    # latency, so it can only understate the kernel; the same bracket around an empty kernel is reported beside it
    ach = a_bytes / (raw_ms * 1e-3) / 1e9 if raw_ms > 0 else 0.0
    corr_ms = max(raw_ms - empty_ms, 0.0)
    ach_corr = a_bytes / (corr_ms * 1e-3) / 1e9 if corr_ms > 0 else 0.0
    stock_shape = args.batch is None and args.ctx is None and not args.paper_unstable_topk and not args.append
    traffic = STORED_TRAFFIC.get(cfg.name) if stock_shape or not main_workload else None
    med = lambda xs: round(float(np.median(xs)), 2) if len(xs) else None
    res = {
        "value": round(value, 1), "ms_per_step": round(elapsed / args.steps * 1e3, 4),
        "config": {"workload": cfg.name, "batch": cfg.batch, "context": max(cfg.ctx), "context_min": min(cfg.ctx),
                   "q_heads": cfg.num_q_heads, "kv_heads": cfg.num_kv_heads, "stable_heads": int(sum(cfg.stable)),
                   "topk_pages": cfg.max_topk, "rerank_interval": cfg.rerank_interval,
                   "pages_attended_per_step": cfg.pages_attended(), "shuffled_blocks": bool(cfg.shuffle_blocks),
                   "promote_mode": args.promote_mode, "append_one_token_per_step": bool(args.append),
                   "unstable_heads": "top-K every step" if args.paper_unstable_topk else "all pages",
                   "attn_wavefronts": sess.ctx.cfg.attn_waves or "auto"},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBS, 2),
        "attn_bytes_per_step": a_bytes, "rerank_bytes_per_invocation": r_bytes,
        "step_us_plain_median": med(plain_us), "step_us_rerank_median": med(rer_us),
        "step_us_plain_min": round(float(np.min(plain_us)), 2) if plain_us else None,
        "step_us_rerank_min": round(float(np.min(rer_us)), 2) if rer_us else None,
        "rerank_exposed_us_per_step_amortised": round((float(np.median(rer_us)) - float(np.median(plain_us)))
                                                      / cfg.rerank_interval, 2) if rer_us and plain_us else None,
        "attn_call_GBps_plain_step": round(a_bytes / (float(np.median(plain_us)) * 1e-6) / 1e9, 1) if plain_us else None,
        # attention and rerank alone, promotion (PCIe) left out: R attention calls and one fc_rerank_topk, from the medians
        "attn_plus_rerank_GBps_excl_promotion": round((cfg.rerank_interval * a_bytes + r_bytes)
                                                       / ((cfg.rerank_interval * float(np.median(plain_us)) + float(np.median(rr_us))) * 1e-6) / 1e9, 1)
                                                 if plain_us and rr_us else None,
        "rerank_topk_us_per_invocation": med(rr_us),
        "rerank_topk_us_per_step_amortised": round(float(np.median(rr_us)) / cfg.rerank_interval, 2) if rr_us else None,
        # fc_rerank_promote (scoring, then selection and block recycling in one kernel), bracketed by two events
        "rerank_promote_us_per_invocation": med(chain_us),
        # with the copies in line the recycling kernel and the copies are one enqueue on one stream: only their sum is
        # seen; when they ride in an attention launch, "page copies" is that whole launch (resident pages + copies)
        "recycle_us_per_invocation": med(pr_us) if pr_us and (ride or not inline) else None,
        "page_copies_us_per_invocation": med(cp_us) if cp_us and (ride or not inline) else None,
        "recycle_and_page_copies_us_per_invocation": med(np.add(pr_us, cp_us)) if pr_us else None,
        "rerank_invocations": n_rerank, "promoted_pages_last_rerank": promoted_last,
        "promoted_MB_last_rerank": round(promoted_last * 8192 / 1e6, 2),
        "rerank_step_overlap": {False: "none", True: "by page (resident, then promoted)", "heads": "by head class",
                                "inline": "by page, copies in line on the main stream, resident pages on the other stream",
                                "heads-inline": "by head class, copies in line on the main stream, unstable heads on the other stream",
                                "ride": "by page, one stream: the copies ride in the launch that attends over the resident pages",
                                "heads-ride": "by head class, one stream: the copies ride in the unstable heads' launch"}[sess.overlap],
        "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBS, 4),
                     "traffic": traffic[0] if traffic else None,
                     "traffic_source": (traffic[1] + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, stored value, not measured in this run)") if traffic else None,
                     "kernel": "fc_decode_attn_kernel<FC_HEADS_ALL>",
                     "avg_kernel_us": round(raw_ms * 1e3, 2), "launches": launches,
                     "timing": "HIP events around every whole-pass launch of a diagnostic pass, on the launch's stream; raw bracket "
                               "(kernel + the bracket's own dispatch latency)",
                     "event_bracket_us_empty_kernel": round(empty_ms * 1e3, 2),
                     "achieved_minus_empty_bracket": round(ach_corr, 1),
                     "frac_minus_empty_bracket": round(ach_corr / HBM_PEAK_GBS, 4),
                     "algorithmic_bytes_per_launch": int(a_bytes),
                     "stream_read_ceiling_GBps": round(ceil_gbs, 1), "stream_read_ceiling_us": round(ceil_us, 2),
                     "stream_read_ceiling_bytes": int(ceil_bytes),
                     "frac_of_stream_read_ceiling": round(ach / ceil_gbs, 4) if ceil_gbs > 0 else None},
        "setup_s": round(t_gen, 1),
    }
    if main_workload and not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, wl, args.cpu_budget, args.paper_unstable_topk)
    elif cfg.index == 2 and not args.no_cpu_baseline:
        # the 32k workload is small enough for a single-thread figure beside the all-cores one (a third of the budget)
        res["cpu_baseline"] = cpu_baseline(cfg, wl, args.cpu_budget / 3, args.paper_unstable_topk)
    sess.close()
    del sess, q_all, new_kv, wl
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workloads", type=str, default="4,2,3,5",
                    help="benchmark configurations to run; the first is the one `value`, `roofline` and `cpu_baseline` are "
                         "quoted on (default: the largest single-GPU one, 64 ragged sequences), the rest are reported "
                         "under `workloads`")
    ap.add_argument("--config", type=int, default=None, help="run this one configuration only (same as --workloads N)")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--ctx", type=int, default=None)
    ap.add_argument("--promote-mode", choices=["gather", "memcpy"], default="gather")
    ap.add_argument("--attn-waves", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-launches", type=int, default=48, help="whole-pass attention launches bracketed with HIP events (at least 32)")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not bracket the attention kernel with HIP events")
    ap.add_argument("--paper-unstable-topk", action="store_true",
                    help="the paper's own treatment of unstable heads: rescored every step, top-K attention")
    ap.add_argument("--append", action="store_true",
                    help="grow every context by one token per step (fc_append_kv: page write, MinMax update, offload on fill)")
    ap.add_argument("--no-overlap", action="store_true", help="run rerank, promotion and attention back to back on one stream")
    ap.add_argument("--overlap-by", choices=["auto", "pages", "heads", "inline", "heads-inline", "ride", "heads-ride"], default="auto",
                    help="how a rerank step's attention is split around the page copies")
    ap.add_argument("--cpu-budget", type=float, default=15.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards by sequence or KV head with no "
              "exchange between shards); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    indices = [args.config] if args.config is not None else [int(x) for x in args.workloads.split(",") if x]

    import torch
    main_res = run_workload(args, indices[0], torch, main_workload=True)
    out = {
        "metric": "sparse decode attention effective HBM GB/s (% of peak) + rerank µs/step",
        "value": main_res.pop("value"), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
    }
    out.update(main_res)
    others = {}
    for idx in indices[1:]:
        r = run_workload(args, idx, torch, main_workload=False)
        rf = r["roofline"]
        others[r["config"]["workload"]] = {
            "value": r["value"], "unit": "GB/s", "pct_of_hbm_peak": r["pct_of_hbm_peak"], "ms_per_step": r["ms_per_step"],
            "steps": args.steps, "warmup": args.warmup, "attn_bytes_per_step": r["attn_bytes_per_step"],
            "batch": r["config"]["batch"], "context": r["config"]["context"], "stable_heads": r["config"]["stable_heads"],
            "topk_pages": r["config"]["topk_pages"], "rerank_interval": r["config"]["rerank_interval"],
            "attn_kernel_us": rf["avg_kernel_us"], "attn_kernel_launches": rf["launches"], "attn_kernel_frac": rf["frac"],
            "attn_kernel_frac_minus_empty_bracket": rf["frac_minus_empty_bracket"],
            "frac_of_stream_read_ceiling": rf["frac_of_stream_read_ceiling"],
            "traffic": rf["traffic"], "traffic_source": rf["traffic_source"],
            "step_us_plain_median": r["step_us_plain_median"], "step_us_rerank_median": r["step_us_rerank_median"],
            "rerank_topk_us_per_invocation": r["rerank_topk_us_per_invocation"],
            "rerank_topk_us_per_step_amortised": r["rerank_topk_us_per_step_amortised"],
            "rerank_promote_us_per_invocation": r["rerank_promote_us_per_invocation"],
            "recycle_and_page_copies_us_per_invocation": r["recycle_and_page_copies_us_per_invocation"],
            "attn_plus_rerank_GBps_excl_promotion": r["attn_plus_rerank_GBps_excl_promotion"],
            "promoted_MB_last_rerank": r["promoted_MB_last_rerank"],
        }
        if "cpu_baseline" in r:
            others[r["config"]["workload"]]["cpu_baseline"] = r["cpu_baseline"]
    if others:
        out["workloads"] = others
    out["target_note"] = ("the 70 % of HBM peak the target names is for attention plus rerank: `attn_plus_rerank_GBps_excl_promotion` "
                          "(and `roofline.frac` for the attention kernel alone); `value` is the whole step and also contains the "
                          "promotion of newly selected pages over PCIe (57 GB/s), which keeps it below 70 % on the workloads whose "
                          "rerank steps move the most bytes relative to their attention")
    out["parity_coverage"] = ("tests/test_gpu_parity.py runs every workload above at full size in this launch configuration and "
                              "compares selections, tables and page bytes exactly on every rerank and attention against the fp64 "
                              "oracle on 1-3 sampled sequences over 3-4 steps (oracle cost); reduced sizes are compared in full")
    out["device"] = device_facts(torch)
    # the paper's own end-to-end figures, other hardware and a whole serving stack: context, not a comparison
    out["paper_context"] = ("FlexiCache paper, 1x NVIDIA H100 94 GB over PCIe 5.0, fp16 KV, against vLLM: up to 70 % less GPU "
                            "KV memory, 1.38-1.55x offline throughput, 1.6-2.1x lower online per-token latency; kernel level: "
                            "decode layer up to 4x faster than dense at batch 40, stability-aware rerank 2.44x")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
