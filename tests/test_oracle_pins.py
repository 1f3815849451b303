"""Pins of the CPU oracle against things other than itself: textbook dense attention written in numpy,
algebraic invariants, closed forms, brute force on tiny inputs and the values the paper prints."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2511_00868_amd import synth

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_values.json")))


def widen(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def rand_bf16(rng, shape, scale=1.0):
    return synth.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


def dense_attention_numpy(q, k, v, ctx, scale):
    """Textbook softmax attention in numpy fp64 over tokens [0, ctx)."""
    qf, kf, vf = widen(q), widen(k[:ctx]), widen(v[:ctx])
    z = scale * (kf @ qf)
    w = np.exp(z - z.max())
    w /= w.sum()
    return w @ vf, float(z.max() + np.log(np.exp(z - z.max()).sum()))


# ---- P1 / P2: attention -----------------------------------------------------------------------
@pytest.mark.parametrize("ctx", [1, 5, 16, 17, 100, 256])
def test_all_pages_equals_dense_attention(ctx):
    rng = np.random.default_rng(ctx)
    D, P = 128, 16
    n = -(-ctx // P)
    k, v = rand_bf16(rng, (n * P, D)), rand_bf16(rng, (n * P, D))
    k[ctx:] = 0x7FC0   # NaN beyond the context: must never be read
    v[ctx:] = 0x7FC0
    q = rand_bf16(rng, (D,))
    scale = 1 / np.sqrt(D)
    out, lse, ws = oracle.attention(q, k, v, ctx, np.arange(n), scale)
    ref, ref_lse = dense_attention_numpy(q, k, v, ctx, scale)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    assert abs(lse - ref_lse) < 1e-12
    assert abs(ws - 1.0) < 1e-12
    vf = widen(v[:ctx])
    assert np.all(out <= vf.max(0) + 1e-12) and np.all(out >= vf.min(0) - 1e-12)  # convex hull of V rows


def test_page_subset_equals_dense_attention_over_those_tokens():
    rng = np.random.default_rng(7)
    D, P, ctx = 128, 16, 200
    n = -(-ctx // P)
    k, v, q = rand_bf16(rng, (n * P, D)), rand_bf16(rng, (n * P, D)), rand_bf16(rng, (D,))
    pages = np.array([12, 3, 7])          # order must not matter; page 12 is partial (tokens 192..199)
    toks = np.concatenate([np.arange(p * P, min((p + 1) * P, ctx)) for p in pages])
    out, lse, ws = oracle.attention(q, k, v, ctx, pages, 0.125)
    ref, ref_lse = dense_attention_numpy(q, k[toks], v[toks], len(toks), 0.125)
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-13)
    out2, lse2, _ = oracle.attention(q, k, v, ctx, np.sort(pages), 0.125)
    np.testing.assert_allclose(out, out2, rtol=1e-13, atol=1e-14)
    assert abs(lse - ref_lse) < 1e-12 and abs(ws - 1) < 1e-12


def test_one_hot_value_recovers_softmax_weight():
    """V = indicator of token j in dim 0 makes out[0] the softmax weight of token j."""
    rng = np.random.default_rng(3)
    D, P, ctx = 128, 16, 64
    k, q = rand_bf16(rng, (ctx, D)), rand_bf16(rng, (D,))
    j = 37
    v = np.zeros((ctx, D), dtype=np.uint16)
    v[j, 0] = 0x3F80  # 1.0
    out, _, _ = oracle.attention(q, k, v, ctx, np.arange(4), 0.3)
    z = 0.3 * (widen(k) @ widen(q))
    w = np.exp(z - z.max()); w /= w.sum()
    assert abs(out[0] - w[j]) < 1e-14 and np.all(out[1:] == 0)


# ---- P3: split + log-sum-exp merge --------------------------------------------------------------
def test_any_partition_of_the_page_set_merges_to_the_same_result():
    rng = np.random.default_rng(11)
    D, P, ctx = 128, 16, 333
    n = -(-ctx // P)
    k, v, q = rand_bf16(rng, (n * P, D)), rand_bf16(rng, (n * P, D)), rand_bf16(rng, (D,), 2.0)
    scale = 1 / np.sqrt(D)
    full, full_lse, _ = oracle.attention(q, k, v, ctx, np.arange(n), scale)
    for trial in range(5):
        perm = rng.permutation(n)
        cuts = np.sort(rng.choice(np.arange(1, n), size=rng.integers(1, 6), replace=False))
        parts = np.split(perm, cuts)
        outs, lses = zip(*[oracle.attention(q, k, v, ctx, p, scale)[:2] for p in parts])
        m = max(lses)
        wts = np.exp(np.array(lses) - m)
        merged = sum(w * o for w, o in zip(wts, outs)) / wts.sum()
        np.testing.assert_allclose(merged, full, rtol=1e-12, atol=1e-13)
        assert abs(m + np.log(wts.sum()) - full_lse) < 1e-12


# ---- P4 / P5: page score ------------------------------------------------------------------------
def test_minmax_is_min_and_max_over_valid_tokens():
    rng = np.random.default_rng(5)
    D, P, ctx = 128, 16, 70
    n = -(-ctx // P)
    k = rand_bf16(rng, (n * P, D))
    k[ctx:] = 0x7FC0
    mm = oracle.build_minmax(k, ctx, P)
    kf = widen(k)
    for p in range(n):
        rows = kf[p * P:min((p + 1) * P, ctx)]
        np.testing.assert_array_equal(widen(mm[p, 0]), rows.min(0))
        np.testing.assert_array_equal(widen(mm[p, 1]), rows.max(0))


def test_score_upper_bounds_every_dot_product_and_is_tight_for_single_key_pages():
    rng = np.random.default_rng(9)
    D, P, G, ctx = 128, 16, 4, 16 * 12 + 1     # last page holds exactly one key
    n = -(-ctx // P)
    k = rand_bf16(rng, (n * P, D))
    k[16:32] = k[16]                           # page 1: sixteen identical keys
    q = rand_bf16(rng, (G, D))
    mm = oracle.build_minmax(k, ctx, P)
    s = oracle.page_scores(q, mm)
    dots = widen(k[:ctx]) @ widen(q).T          # [tokens, G]
    for p in range(n):
        rows = dots[p * P:min((p + 1) * P, ctx)]
        assert s[p] >= rows.max() - 1e-9
    assert abs(s[n - 1] - dots[ctx - 1].max()) < 1e-9        # one key: bound is exact
    assert abs(s[1] - dots[16].max()) < 1e-9                 # identical keys: bound is exact
    assert np.sum(s > np.array([dots[p * P:min((p + 1) * P, ctx)].max() for p in range(n)]) + 1e-6) >= n - 2


def test_score_closed_forms_and_homogeneity():
    rng = np.random.default_rng(13)
    D, P, ctx = 128, 16, 160
    k = rand_bf16(rng, (ctx, D))
    mm = oracle.build_minmax(k, ctx, P)
    lo, hi = widen(mm[:, 0]), widen(mm[:, 1])
    qpos = synth.f32_to_bf16_bits(np.abs(rng.standard_normal((1, D))).astype(np.float32))
    qneg = qpos | np.uint16(0x8000)
    np.testing.assert_allclose(oracle.page_scores(qpos, mm), hi @ widen(qpos[0]), rtol=1e-13)
    np.testing.assert_allclose(oracle.page_scores(qneg, mm), lo @ widen(qneg[0]), rtol=1e-13)
    q = rand_bf16(rng, (1, D))
    q4 = synth.f32_to_bf16_bits(4.0 * synth.bf16_bits_to_f32(q))   # exact power-of-two scaling
    np.testing.assert_allclose(oracle.page_scores(q4, mm), 4 * oracle.page_scores(q, mm), rtol=1e-13)
    # mixed-sign definition, retyped independently as a masked sum
    qf = widen(q[0])
    ref = np.where(qf >= 0, hi * qf, lo * qf).sum(1)
    np.testing.assert_allclose(oracle.page_scores(q, mm), ref, rtol=1e-12)


def test_group_combination_is_max_over_the_group_with_sum_as_audit_mode():
    rng = np.random.default_rng(17)
    D, P, ctx, G = 128, 16, 96, 4
    k, q = rand_bf16(rng, (ctx, D)), rand_bf16(rng, (G, D))
    mm = oracle.build_minmax(k, ctx, P)
    per = np.stack([oracle.page_scores(q[g:g + 1], mm) for g in range(G)])
    np.testing.assert_array_equal(oracle.page_scores(q, mm, 0), per.max(0))
    np.testing.assert_allclose(oracle.page_scores(q, mm, 1), per.sum(0), rtol=1e-13)


# ---- P6: selection ------------------------------------------------------------------------------
@pytest.mark.parametrize("n,K,ctx_mod", [(1, 1, 0), (8, 3, 0), (8, 3, 5), (8, 8, 0), (8, 20, 3),
                                         (128, 8, 0), (300, 37, 9), (2048, 204, 0)])
def test_selection_equals_lexsort(n, K, ctx_mod):
    rng = np.random.default_rng(n * 31 + K)
    P = 16
    ctx = n * P if ctx_mod == 0 else (n - 1) * P + ctx_mod
    s = rng.standard_normal(n)
    s[rng.integers(0, n, size=n // 3)] = 0.25       # many exact ties
    got = oracle.select_topk(s, ctx, K, P)
    want = min(K, n)
    forced = [n - 1] if ctx_mod else []
    rest = [p for p in np.lexsort((np.arange(n), -s)) if p not in forced]   # score desc, index asc
    ref = sorted(forced + rest[:want - len(forced)])
    assert list(got) == ref
    assert len(got) == want and np.all(np.diff(got) > 0)


def test_planted_hot_pages_are_selected():
    cfg = synth.make_config(1)
    w = synth.Workload(cfg)
    q = w.queries(0)
    for h in range(cfg.num_kv_heads):
        mm = oracle.build_minmax(w.k[0][h], cfg.ctx[0])
        s = oracle.page_scores(q[0, h * cfg.group:(h + 1) * cfg.group], mm)
        sel = oracle.select_topk(s, cfg.ctx[0], 8)
        assert set(w.hot[(0, h)]) <= set(int(x) for x in sel)


# ---- P7: promotion bookkeeping ------------------------------------------------------------------
def test_recycle_invariants_over_random_reranks():
    rng = np.random.default_rng(23)
    n, K = 64, 8
    table = np.zeros(n, dtype=np.int32)
    host = np.arange(100, 100 + n, dtype=np.int32)
    free = list(range(1, K + 1))
    owned = sorted(free)
    old = np.empty(0, dtype=np.int32)
    for it in range(20):
        new = np.sort(rng.choice(n, size=K, replace=False)).astype(np.int32)
        before = table.copy()
        copies, free = oracle.recycle(old, new, table, host, free)
        promoted = np.setdiff1d(new, old)
        kept = np.intersect1d(new, old)
        assert len(copies) == len(promoted)
        np.testing.assert_array_equal(copies[:, 0], host[promoted])          # source = host block
        np.testing.assert_array_equal(copies[:, 1], table[promoted])         # destination = new mapping
        np.testing.assert_array_equal(table[kept], before[kept])             # kept pages do not move
        resident = np.nonzero(table)[0]
        np.testing.assert_array_equal(resident, new)                         # resident set == S_t
        assert sorted(list(table[resident]) + free) == owned                 # blocks only permuted
        assert len(set(table[resident])) == len(resident)
        old = new
    assert free == []


def test_recycle_ordering_rule_and_cold_fill():
    table = np.zeros(6, dtype=np.int32)
    host = np.array([10, 11, 12, 13, 14, 15], dtype=np.int32)
    copies, free = oracle.recycle([], [1, 4], table, host, [7, 9, 8])
    assert copies.tolist() == [[11, 7], [14, 9]] and free == [8]
    assert table.tolist() == [0, 7, 0, 0, 9, 0]
    copies, free = oracle.recycle([1, 4], [0, 4, 5], table, host, free)   # evict 1, promote 0 and 5
    assert copies.tolist() == [[10, 8], [15, 7]] and free == []
    assert table.tolist() == [8, 0, 0, 0, 9, 7]
    with pytest.raises(RuntimeError):
        oracle.recycle([0, 4, 5], [0, 1, 2, 3], table.copy(), host, [])


# ---- P8: the paper's printed numbers ------------------------------------------------------------
def test_paper_topk_bytes():
    g = GOLD["topk_kv_bytes"]
    pages = g["budget_tokens"] // 16
    page_bytes = 2 * 16 * g["head_dim"] * g["bytes_per_elem"]     # K and V of one 16-token page
    assert g["stable_heads"] * pages * page_bytes == g["expected_mib"] * 2 ** 20


def test_paper_memory_saving_curve():
    g = GOLD["gpu_memory_saving"]
    u, budget = g["unstable_fraction"], g["budget_tokens"]

    def saving(length):
        # resident pages per head counted with the oracle's own selection on arbitrary scores
        n = -(-length // 16)
        sel = oracle.select_topk(np.zeros(n), length, budget // 16)
        return 1 - (u * n + (1 - u) * len(sel)) / n

    assert abs(saving(g["length"]) - g["expected_about"]) < g["tolerance"]
    assert saving(g["length"]) > 0.70
    assert abs(saving(4_000_000) - g["asymptote"]) < 1e-3


def test_promotion_volume_of_the_synthetic_workload_against_the_papers_range():
    """Sec. 4.4 measures 23-35 % of the top-K set promoted per rerank on real prompts.  The synthetic recipe (a
    quarter of the budget planted hot pages, the rest background pages whose score order moves with the query
    noise) promotes a little less, about a fifth: stated here so that the benchmark's PCIe volume can be read
    against the paper's (the steady-state reranks only; the first one is a cold fill of the whole budget)."""
    from paper_2511_00868_amd import synth
    lo, hi = GOLD["promoted_fraction_range"]["fraction"]
    cfg = synth.make_config(2, batch=2, ctx=16384, steps=17)
    wl = synth.Workload(cfg)
    dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, cfg.topk, cfg.rerank_interval)
    mm = [oracle.seq_build_minmax(wl.k[b], cfg.ctx[b]) for b in range(cfg.batch)]
    fractions = []
    for t in range(0, 17, cfg.rerank_interval):
        q = wl.queries(t)
        for b in range(cfg.batch):
            for h, (promoted, evicted) in dec.rerank(b, q[b], mm[b]).items():
                if t == 0:
                    assert len(promoted) == cfg.topk[b] and len(evicted) == 0          # the cold fill
                else:
                    assert len(promoted) == len(evicted)                             # fixed budget, fixed context
                    fractions.append(len(promoted) / cfg.topk[b])
    mean = float(np.mean(fractions))
    assert 0.10 < mean < hi, mean
    assert mean < lo + 0.02           # at or below the paper's lower end: the benchmark moves no more than the paper did


def test_paper_placement_example():
    g = GOLD["placement_example"]
    n, P = g["logical_pages"], 16
    ctx = g["full_pages"] * P + 5
    sel = oracle.select_topk(np.array([0.3, 0.9, 0.1, -5.0]), ctx, g["topk"])
    assert len(sel) == g["stable_gpu_pages"] and (n - 1) in sel      # the partial page is a member
    assert list(sel) == [1, 3]
    assert g["host_pages"] == ctx // P and g["unstable_gpu_pages"] == n


# ---- P9: schedule -------------------------------------------------------------------------------
def _run_schedule(R, steps, K=None):
    cfg = synth.make_config(1)
    w = synth.Workload(cfg)
    topk = [K] if K else list(cfg.topk)
    dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, topk, R)
    mm = oracle.seq_build_minmax(w.k[0], cfg.ctx[0])
    hist, outs = [], []
    for t in range(steps):
        q = w.queries(t)
        if t % R == 0:
            dec.rerank(0, q[0], mm)
        hist.append(dec.sel[(0, 0)].copy())
        outs.append(dec.attend(0, q[0], w.k[0], w.v[0])[0])
    return cfg, w, hist, outs


def test_interval_one_reranks_every_step_and_long_interval_reuses_first_selection():
    cfg, w, hist, _ = _run_schedule(1, 3)
    mm = oracle.build_minmax(w.k[0][0], cfg.ctx[0])
    for t in range(3):
        s = oracle.page_scores(w.queries(t)[0, :cfg.group], mm)
        np.testing.assert_array_equal(hist[t], oracle.select_topk(s, cfg.ctx[0], 8))
    _, _, hist, _ = _run_schedule(100, 3)
    assert all(np.array_equal(hist[0], h) for h in hist)


def test_stable_head_with_full_budget_equals_dense():
    cfg, w, hist, outs = _run_schedule(2, 2, K=128)
    assert len(hist[0]) == 128
    q = w.queries(1)[0]
    for g in range(cfg.group):
        ref, _ = dense_attention_numpy(q[g], w.k[0][0], w.v[0][0], cfg.ctx[0], 1 / np.sqrt(128))
        np.testing.assert_allclose(outs[1][g], ref, rtol=1e-12, atol=1e-13)


def test_sparse_attention_of_stable_head_is_close_to_dense_when_hot_pages_dominate():
    """Sanity of the workload (not a pin): with planted hot pages, K = 8 of 128 pages keeps most of the
    softmax mass, so the sparse output is near the dense one."""
    cfg, w, hist, outs = _run_schedule(2, 1)
    q = w.queries(0)[0]
    ref, _ = dense_attention_numpy(q[0], w.k[0][0], w.v[0][0], cfg.ctx[0], 1 / np.sqrt(128))
    assert np.abs(outs[0][0] - ref).max() < 0.5


def test_paper_variant_of_unstable_heads_selects_per_step_and_reduces_to_dense_with_full_budget():
    cfg = synth.make_config(1)
    w = synth.Workload(cfg)
    mm = oracle.seq_build_minmax(w.k[0], cfg.ctx[0])
    dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, [128], 2,
                               unstable_topk=True)
    q = w.queries(0)[0]
    dec.rerank(0, q, mm)
    dec.rerank_unstable(0, q, mm)
    assert len(dec.sel[(0, 1)]) == 128                      # head 1 is the unstable one
    out, _ = dec.attend(0, q, w.k[0], w.v[0])
    for hq in range(cfg.num_q_heads):
        h = hq // cfg.group
        ref, _ = dense_attention_numpy(q[hq], w.k[0][h], w.v[0][h], cfg.ctx[0], 1 / np.sqrt(128))
        np.testing.assert_allclose(out[hq], ref, rtol=1e-12, atol=1e-13)
    # with a real budget the unstable head follows the query of the step
    dec8 = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, [8], 2,
                                unstable_topk=True)
    for t in range(2):
        qt = w.queries(t)[0]
        dec8.rerank_unstable(0, qt, mm)
        s = oracle.page_scores(qt[cfg.group:2 * cfg.group], mm[1])
        np.testing.assert_array_equal(dec8.sel[(0, 1)], oracle.select_topk(s, cfg.ctx[0], 8))


def test_appended_tokens_join_the_sequence_and_the_started_page_joins_the_selection():
    rng = np.random.default_rng(31)
    D, P, ctx0, extra = 128, 16, 30, 5           # tokens 30, 31 complete page 1; token 32 starts page 2
    k, v = rand_bf16(rng, (48, D)), rand_bf16(rng, (48, D))
    q = rand_bf16(rng, (4, D))
    dec = oracle.OracleDecoder(1, 4, 1, [ctx0], [True], [1], 100)
    mm = oracle.seq_build_minmax(k[None], ctx0)
    dec.rerank(0, q, mm)
    assert list(dec.sel[(0, 0)]) == [1]                    # the partial page is the whole budget
    started = [dec.append(0) for _ in range(extra)]
    assert started == [None, None, 2, None, None] and dec.ctx[0] == 35
    assert list(dec.sel[(0, 0)]) == [1, 2]
    out, _ = dec.attend(0, q, k[None], v[None])
    toks = np.arange(16, 35)
    for g in range(4):
        ref, _ = dense_attention_numpy(q[g], k[toks], v[toks], len(toks), 1 / np.sqrt(D))
        np.testing.assert_allclose(out[g], ref, rtol=1e-12, atol=1e-13)
    mm2 = oracle.seq_build_minmax(k[None], 35)
    dec.rerank(0, q, mm2)                                   # next rerank: budget 1 -> only the partial page stays
    assert list(dec.sel[(0, 0)]) == [2]


# ---- offline stability profiling (Sec. 2.2, 2.3) -------------------------------------------------
def test_rco_anchors_and_closed_form():
    assert oracle.rco([1, 5, 9, 12], [1, 5, 9, 12], 100) == 1.0               # identical sets
    assert oracle.rco([0, 1], [1, 2], 4) == 0.0                               # overlap 1/2 = K/N: chance level
    assert oracle.rco([0, 1], [2, 3], 4) == 0.0                               # below chance clamps to 0
    assert oracle.rco([0, 1, 2, 3], [0, 1, 2, 3], 4) == 0.0                   # K = N: defined 0
    # (I/K - K/N) / (1 - K/N) with I = 3, K = 4, N = 64
    assert abs(oracle.rco([3, 7, 20, 41], [3, 7, 41, 50], 64) - (0.75 - 0.0625) / 0.9375) < 1e-15
    assert oracle.rco([3, 7, 20, 41], [41, 3, 50, 7], 64) == oracle.rco([3, 7, 20, 41], [3, 7, 41, 50], 64)


def test_uncorrected_overlap_of_random_draws_is_at_chance_level():
    """Sec. 2.2: the correction subtracts the hypergeometric mean K/N; with the clamp at 0 the mean RCO of
    independent random selections stays small, while identical selections give 1."""
    rng = np.random.default_rng(0)
    K, N = 16, 256
    vals = [oracle.rco(np.sort(rng.choice(N, K, replace=False)), np.sort(rng.choice(N, K, replace=False)), N)
            for _ in range(400)]
    assert 0.0 <= np.mean(vals) < 0.03 and max(vals) < 0.3


def test_stability_score_counts_and_classification_against_numpy():
    rng = np.random.default_rng(4)
    steps, heads, K, W = 24, 8, 6, 5
    N = np.arange(40, 40 + steps)
    traces = np.stack([np.stack([np.sort(rng.choice(N[t], K, replace=False)) for _ in range(heads)])
                       for t in range(steps)]).astype(np.int32)
    traces[:, 2] = traces[0, 2]                        # head 2 never changes: perfectly stable
    traces[1:, 5, :4] = traces[0, 5, :4]               # head 5 keeps 4 of 6 pages (when sorted order allows)
    traces[:, 5].sort(axis=1)
    ts = oracle.stability(traces, N, W)
    assert ts.shape == (steps - W + 1, heads)
    ref = np.zeros_like(ts)
    for s in range(steps - W + 1):
        for h in range(heads):
            r = []
            for t in range(s + 1, s + W):
                inter = len(set(traces[s, h]) & set(traces[t, h]))
                c = K / N[t]
                r.append(max(0.0, (inter / K - c) / (1 - c)))
            ref[s, h] = np.mean(r)
    np.testing.assert_allclose(ts, ref, rtol=1e-14, atol=1e-16)
    assert np.all(ts[:, 2] == 1.0)
    counts = oracle.bottom_counts(ts)
    ref_counts = np.zeros(heads, dtype=np.int32)
    for w in range(len(ts)):
        order = np.lexsort((np.arange(heads), ts[w]))  # score ascending, index ascending
        ref_counts[order[:heads // 4]] += 1
    np.testing.assert_array_equal(counts, ref_counts)
    assert counts.sum() == len(ts) * (heads // 4) and counts[2] == 0
    flags = oracle.classify(counts)
    order = np.lexsort((np.arange(heads), -counts))
    ref_flags = np.zeros(heads, dtype=np.uint8)
    ref_flags[order[:heads // 4]] = 1
    np.testing.assert_array_equal(flags, ref_flags)
    assert flags.sum() == 2 and flags[2] == 0
    # counts accumulate over samples
    np.testing.assert_array_equal(oracle.bottom_counts(ts, counts), 2 * counts)


def test_ties_at_the_budget_boundary_go_to_the_lower_page_index():
    assert list(oracle.select_topk(np.zeros(10), 160, 4)) == [0, 1, 2, 3]
    s = np.array([1.0, 5.0, 1.0, 7.0, 1.0, 1.0, 0.5, 1.0])       # two clear winners, then a five-way tie for 2 seats
    assert list(oracle.select_topk(s, 128, 4)) == [0, 1, 2, 3]
    assert list(oracle.select_topk(s, 128, 5)) == [0, 1, 2, 3, 4]
    assert list(oracle.select_topk(s, 125, 4)) == [0, 1, 3, 7]   # partial last page forced in: one tied seat left
    rng = np.random.default_rng(2)
    for _ in range(20):                                          # quantised scores: the boundary always cuts a tie group
        n, K = int(rng.integers(5, 200)), int(rng.integers(1, 40))
        s = rng.integers(0, 4, size=n).astype(np.float64)
        got = oracle.select_topk(s, n * 16, K)
        ref = sorted(np.lexsort((np.arange(n), -s))[:min(K, n)])
        assert list(got) == ref


# ---- pins found missing by mutating the oracle ---------------------------------------------------
def test_selection_pads_its_output_with_minus_one():
    import ctypes as C
    s = np.array([3.0, 1.0, 2.0], dtype=np.float64)
    out = np.full(6, 77, dtype=np.int32)
    cnt = oracle.lib().fco_select_topk(s.ctypes.data_as(C.POINTER(C.c_double)), 3, 48, 16, 6,
                                       out.ctypes.data_as(C.POINTER(C.c_int32)))
    assert cnt == 3 and out.tolist() == [0, 1, 2, -1, -1, -1]
    out[:] = 77
    cnt = oracle.lib().fco_select_topk(s.ctypes.data_as(C.POINTER(C.c_double)), 3, 48, 16, 2,
                                       out.ctypes.data_as(C.POINTER(C.c_int32)))
    assert cnt == 2 and out.tolist() == [0, 2, 77, 77, 77, 77]     # writes K entries, no more


def test_recycle_leaves_the_unused_blocks_in_order_as_the_new_free_list():
    """Available blocks = the free list, then the evicted pages' blocks in ascending page order; promoted
    pages take from the front; what is left, in that order, is the new free list (Sec. 3.4)."""
    table = np.zeros(8, dtype=np.int32)
    host = np.arange(50, 58, dtype=np.int32)
    copies, free = oracle.recycle([], [2], table, host, [5, 3, 9, 4])
    assert copies.tolist() == [[52, 5]] and free == [3, 9, 4] and table.tolist() == [0, 0, 5, 0, 0, 0, 0, 0]
    copies, free = oracle.recycle([2], [2, 6, 7], table, host, free)           # nothing evicted, two promoted
    assert copies.tolist() == [[56, 3], [57, 9]] and free == [4]
    copies, free = oracle.recycle([2, 6, 7], [0], table, host, free)           # three evicted, one promoted
    assert copies.tolist() == [[50, 4]] and free == [5, 3, 9]                   # blocks of pages 2, 6, 7
    assert table.tolist() == [4, 0, 0, 0, 0, 0, 0, 0]
    copies, free = oracle.recycle([0], [], table, host, free)                  # everything evicted
    assert len(copies) == 0 and free == [5, 3, 9, 4] and not table.any()


def test_whole_sequence_drivers_equal_the_per_head_routines_and_numpy():
    rng = np.random.default_rng(77)
    Hq, Hkv, D, ctx, P = 6, 3, 128, 75, 16
    G, n, tpad = Hq // Hkv, 5, 80
    q = rand_bf16(rng, (Hq, D))
    k = rand_bf16(rng, (Hkv, tpad, D))
    v = rand_bf16(rng, (Hkv, tpad, D))
    mm = oracle.seq_build_minmax(k, ctx)
    assert mm.shape == (Hkv, n, 2, D)
    for h in range(Hkv):
        kv = widen(k[h])
        for p in range(n):
            rows = kv[16 * p:min(16 * p + 16, ctx)]
            np.testing.assert_array_equal(widen(mm[h, p, 0]), rows.min(0))
            np.testing.assert_array_equal(widen(mm[h, p, 1]), rows.max(0))
    stable = [True, False, True]
    s = oracle.seq_scores(q, mm, stable)
    qf, mf = widen(q), widen(mm)
    for h in range(Hkv):
        if not stable[h]:
            assert np.all(np.isnan(s[h]))                       # untouched
            continue
        per_q = np.maximum(qf[h * G:(h + 1) * G, None, :] * mf[h, None, :, 0, :],
                           qf[h * G:(h + 1) * G, None, :] * mf[h, None, :, 1, :]).sum(-1)
        np.testing.assert_allclose(s[h], per_q.max(0), rtol=1e-13)
    lists = [np.array([0, 2, 4]), np.arange(n), np.array([1])]
    scale = 0.2
    out, lse = oracle.seq_attention(q, k, v, ctx, lists, scale)
    for hq in range(Hq):
        h = hq // G
        tok = np.concatenate([np.arange(16 * p, min(16 * p + 16, ctx)) for p in lists[h]])
        z = scale * widen(k[h])[tok] @ widen(q[hq])
        w = np.exp(z - z.max())
        np.testing.assert_allclose(out[hq], (w / w.sum()) @ widen(v[h])[tok], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[hq], z.max() + np.log(w.sum()), rtol=1e-13)


def test_head_ranking_ties_go_to_the_lower_head_index_and_the_quota_is_a_floor():
    ts = np.array([[0.5, 0.2, 0.2, 0.9, 0.2, 0.7, 0.8, 0.6]])          # three heads tie for the bottom quartile (2 of 8)
    assert oracle.bottom_counts(ts).tolist() == [0, 1, 1, 0, 0, 0, 0, 0]
    counts = np.array([3, 5, 5, 0, 5, 1, 2, 4], dtype=np.int32)
    assert oracle.classify(counts).tolist() == [0, 1, 1, 0, 0, 0, 0, 0]       # 8 / 4 = 2 heads, ties to the lower index
    assert oracle.classify(counts[:7]).tolist() == [0, 1, 0, 0, 0, 0, 0]      # floor(7 / 4) = 1
    assert oracle.classify(counts, 3, 8).tolist() == [0, 1, 1, 0, 1, 0, 0, 0]  # floor(8 * 3 / 8) = 3
    assert oracle.classify(np.arange(10, dtype=np.int32), 3, 10).sum() == 3    # floor(10 * 3 / 10) = 3, not (10 + 3) / 10
    assert oracle.rco([0, 1, 2, 3], [0, 1, 2, 3], 4) == 0.0                     # K = N_t: chance level is 1, defined as 0
