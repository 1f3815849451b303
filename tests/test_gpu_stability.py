"""GPU parity of the offline head-stability profiling (Sec. 2.2, 2.3) against the CPU oracle."""
import dataclasses

import numpy as np
import pytest

import oracle
from paper_2511_00868_amd import binding, synth

pytestmark = pytest.mark.gpu


def _ctx():
    return binding.Context(num_q_heads=8, num_kv_heads=8, max_batch=1, max_pages_per_seq=64, max_topk=8)


def _profile(ctx, traces, num_pages, W, counts=None):
    import torch
    steps, heads, K = traces.shape
    t_d = torch.from_numpy(np.ascontiguousarray(traces, dtype=np.int32)).cuda()
    n_d = torch.from_numpy(np.ascontiguousarray(num_pages, dtype=np.int32)).cuda()
    ts = torch.zeros((steps - W + 1, heads), dtype=torch.float64, device="cuda")
    cnt = torch.zeros(heads, dtype=torch.int32, device="cuda") if counts is None else counts
    ctx.fc_stability_profile(traces=t_d, num_pages=n_d, steps=steps, heads=heads, topk=K, window=W, ts_out=ts,
                             bottom_counts=cnt)
    torch.cuda.synchronize()
    return ts.cpu().numpy(), cnt


@pytest.mark.parametrize("steps,heads,K,W,pad", [(24, 8, 6, 5, 0), (40, 256, 64, 16, 0), (20, 12, 100, 4, 7),
                                                 (9, 4, 1, 2, 0), (30, 33, 257, 16, 0)])
def test_scores_counts_and_flags_match_the_oracle(steps, heads, K, W, pad):
    import torch
    rng = np.random.default_rng(steps * 1000 + heads)
    N = rng.integers(K + 1, 4 * K + 8, size=steps).astype(np.int32)
    N[steps // 2] = K                                   # one step where every page is selected: RCO defined 0
    traces = np.full((steps, heads, K), -1, dtype=np.int32)
    base = [np.sort(rng.choice(K + 1, K - pad, replace=False)) for _ in range(heads)]
    for t in range(steps):
        for h in range(heads):
            if h % 3 == 0:                              # slowly drifting selection
                keep = base[h].copy()
                swap = rng.integers(0, len(keep))
                cand = np.setdiff1d(np.arange(N[t]), keep)
                if len(cand):
                    keep[swap] = rng.choice(cand)
                base[h] = np.sort(keep)
                sel = base[h]
            else:                                       # fresh random selection every step
                sel = np.sort(rng.choice(N[t], K - pad, replace=False))
            traces[t, h, :K - pad] = sel
    ctx = _ctx()
    try:
        ts_gpu, cnt = _profile(ctx, traces, N, W)
        ts_ref = oracle.stability(traces, N, W)
        np.testing.assert_array_equal(ts_gpu, ts_ref)           # same fp64 operations in the same order
        cnt_ref = oracle.bottom_counts(ts_ref)
        np.testing.assert_array_equal(cnt.cpu().numpy(), cnt_ref)
        ts2, cnt = _profile(ctx, traces, N, W, cnt)              # a second sample accumulates
        np.testing.assert_array_equal(cnt.cpu().numpy(), 2 * cnt_ref)
        for num, den in ((1, 4), (1, 2), (0, 1), (1, 1)):
            flags = torch.zeros(heads, dtype=torch.uint8, device="cuda")
            ctx.fc_classify_heads(cnt, heads, flags, num, den)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(flags.cpu().numpy(), oracle.classify(2 * cnt_ref, num, den))
    finally:
        ctx.close()


def test_profiling_the_librarys_own_selections_recovers_the_heads_whose_hot_pages_move():
    """End to end: fc_rerank_topk run for every head at every step on a workload in which four heads keep
    their hot pages and four get new ones each step; the profile must call the moving heads unstable."""
    import torch
    from paper_2511_00868_amd.session import DecodeSession
    steps, W = 24, 4
    cfg = dataclasses.replace(synth.make_config(2, batch=1, ctx=4096, steps=steps), name="profile_me")
    wl = synth.Workload(cfg)
    s = DecodeSession(cfg, wl)
    try:
        K, H = s.topk_pages.shape[2], cfg.num_kv_heads
        traces = np.zeros((steps, H, K), dtype=np.int32)
        for t in range(steps):
            changed = wl.advance(t)
            if changed:
                s.refresh(changed)
            s.set_queries(wl.queries(t))
            s.ctx.fc_rerank_topk(q=s.q, minmax=s.minmax, context_lens=s.context_lens, stable_flag=[True] * H,
                                 k_per_seq=s.k_per_seq, batch=1, topk_pages=s.topk_pages, topk_count=s.topk_count)
            torch.cuda.synchronize()
            traces[t] = s.topk_pages.cpu().numpy()[0]
        N = np.full(steps, cfg.num_pages(0), dtype=np.int32)
        ts_gpu, cnt = _profile(s.ctx, traces, N, W)
        np.testing.assert_array_equal(ts_gpu, oracle.stability(traces, N, W))
        moving = np.array([not x for x in cfg.stable])
        # only a quarter of each budget is hot pages, so the moving heads still overlap a lot; the gap shows in the means
        assert ts_gpu[:, moving].mean(0).max() + 0.1 < ts_gpu[:, ~moving].mean(0).min()
        flags = torch.zeros(H, dtype=torch.uint8, device="cuda")
        s.ctx.fc_classify_heads(cnt, H, flags, 1, 4)
        torch.cuda.synchronize()
        f = flags.cpu().numpy().astype(bool)
        assert f.sum() == 2 and np.all(moving[f])                          # the paper's 25 %: two of the four movers
        np.testing.assert_array_equal(flags.cpu().numpy(), oracle.classify(cnt.cpu().numpy(), 1, 4))
    finally:
        s.close()
