"""Kernel-level micro-sweeps shaped like the paper's two microbenchmarks (Sec. 4.5):

* decode-layer latency against batch size, dense attention vs the paper's sparse variant (every head
  attends over its top-K pages; unstable heads rescored every step, stable heads every R = 16 steps),
  at token budgets of 1024 and 2048 (64 / 128 pages), 10k-token inputs, 25 % unstable heads;
* stability-aware rerank vs rescoring every head at every step.

Synthetic inputs of those shapes (the paper's prompts and model are not available); times are HIP-event
times on one MI355X, averaged over whole rerank cycles.  Run: python -m paper_2511_00868_amd.microbench
"""
from __future__ import annotations

import argparse
import dataclasses
import json

import numpy as np

from . import binding, synth
from .session import DecodeSession


def layer_config(batch: int, ctx: int, budget_pages: int, R: int, dense: bool) -> synth.DecodeConfig:
    base = synth.make_config(2, batch=batch, ctx=ctx, steps=4 * R)
    stable = (False,) * 8 if dense else (True,) * 6 + (False,) * 2
    return dataclasses.replace(base, stable=stable, topk=(budget_pages,) * batch, rerank_interval=R,
                               hot_per_head=max(1, budget_pages // 4), dynamics="static",
                               name=f"layer_b{batch}_ctx{ctx}_k{budget_pages}{'_dense' if dense else ''}")


def time_steps(sess: DecodeSession, wl: synth.Workload, steps: int, warm: int, fn) -> float:
    """Mean microseconds per step of fn(t) over `steps` steps after `warm` warm-up steps."""
    import torch
    qs = [sess.bits_to_dev(wl.queries(t)) for t in range(warm + steps)]
    for t in range(warm):
        sess.q = qs[t]
        fn(t)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for t in range(warm, warm + steps):
        sess.q = qs[t]
        fn(t)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / steps


def sweep(batches, ctx: int, R: int, budgets):
    import torch
    rows = []
    for B in batches:
        row = {"batch": B}
        cfg = layer_config(B, ctx, budgets[0], R, dense=True)
        wl = synth.Workload(cfg)
        s = DecodeSession(cfg, wl)
        row["dense_us"] = time_steps(s, wl, 2 * R, R, lambda t: s.attend())
        s.close()
        for K in budgets:
            cfg = layer_config(B, ctx, K, R, dense=False)
            wl = synth.Workload(cfg)
            s = DecodeSession(cfg, wl, unstable_topk=True)
            row[f"sparse{K * 16}_us"] = time_steps(s, wl, 2 * R, R, s.step)          # selection, promotion, attention
            # selection + attention only (what the paper's figure times): promotion left out
            def no_promote(t, s=s):
                s.rerank_unstable()
                if s.cfg.is_rerank_step(t):
                    s.rerank()
                s.attend()
            row[f"sparse{K * 16}_select_attend_us"] = time_steps(s, wl, 2 * R, R, no_promote)
            if K == budgets[0]:
                # rerank alone: every head at every step vs stability-aware
                allh = [True] * 8
                scratch_p = torch.full_like(s.topk_pages, -1)
                scratch_c = torch.zeros_like(s.topk_count)
                def naive(t, s=s):
                    s.ctx.fc_rerank_topk(q=s.q, minmax=s.minmax, context_lens=s.context_lens, stable_flag=allh,
                                         k_per_seq=s.k_per_seq, batch=B, topk_pages=scratch_p, topk_count=scratch_c,
                                         stream=s.main)
                def aware(t, s=s):
                    s.ctx.fc_rerank_topk(q=s.q, minmax=s.minmax, context_lens=s.context_lens,
                                         stable_flag=[not x for x in s.stable], k_per_seq=s.k_per_seq, batch=B,
                                         topk_pages=scratch_p, topk_count=scratch_c, stream=s.main)
                    if t % R == 0:
                        s.ctx.fc_rerank_topk(q=s.q, minmax=s.minmax, context_lens=s.context_lens,
                                             stable_flag=s.stable, k_per_seq=s.k_per_seq, batch=B,
                                             topk_pages=scratch_p, topk_count=scratch_c, stream=s.main)
                row["rerank_all_heads_every_step_us"] = time_steps(s, wl, 2 * R, R, naive)
                row["rerank_stability_aware_us"] = time_steps(s, wl, 2 * R, R, aware)
            s.close()
        rows.append(row)
        print(json.dumps({k: (round(v, 2) if isinstance(v, float) else v) for k, v in row.items()}), flush=True)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batches", type=int, nargs="+", default=[1, 8, 16, 24, 32, 40])
    ap.add_argument("--ctx", type=int, default=10000)
    ap.add_argument("--interval", type=int, default=16)
    ap.add_argument("--budgets", type=int, nargs="+", default=[64, 128], help="page budgets (16 tokens each)")
    a = ap.parse_args()
    sweep(a.batches, a.ctx, a.interval, a.budgets)


if __name__ == "__main__":
    main()
