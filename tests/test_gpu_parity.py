"""GPU parity tests: the HIP library (through its C ABI) against the CPU oracle."""
import numpy as np
import pytest

from paper_2511_00868_amd import binding, synth

pytestmark = pytest.mark.gpu


def _run(cfg, **kw):
    from parity_util import ParityRun
    r = ParityRun(cfg, **kw)
    try:
        r.run()
        return r
    finally:
        r.close()


def test_config1_tiny_full_loop():
    r = _run(synth.make_config(1))
    assert r.promoted_total >= 8          # the cold fill alone promotes K = 8 pages


@pytest.mark.parametrize("mode", [binding.FC_PROMOTE_GATHER, binding.FC_PROMOTE_MEMCPY])
def test_config2_reduced_both_promotion_modes(mode):
    # 4096-token contexts: 256 pages, K = 25; several wavefront shares per head and ragged tails
    _run(synth.make_config(2, batch=3, ctx=4096 + 7, steps=6), promote_mode=mode)


def test_config3_reduced_drift():
    _run(synth.make_config(3, batch=2, ctx=16384, steps=17))


def test_config4_reduced_ragged_shuffled():
    _run(synth.make_config(4, batch=9, ctx=6000, steps=5))


def test_config5_reduced_planted_promotions():
    r = _run(synth.make_config(5, batch=3, ctx=8192, steps=9))
    assert r.promoted_total > 3 * 5 * 32   # more than the cold fill: planted pages forced promotions


@pytest.mark.parametrize("index,kw", [(2, dict(batch=3, ctx=4096 + 7, steps=6)), (3, dict(batch=2, ctx=16384, steps=17)),
                                      (4, dict(batch=9, ctx=6000, steps=5)), (5, dict(batch=3, ctx=8192, steps=9))])
def test_reduced_configs_through_the_two_separate_calls(index, kw):
    """fc_rerank_topk followed by fc_promote_pages (the default everywhere else is the one call fc_rerank_promote,
    which selects and recycles in one kernel): same oracle, same checks."""
    _run(synth.make_config(index, **kw), fused_rerank=False)


def test_budget_of_5000_pages():
    """K = 5000 of 6251 pages: the selection runs on 1024 threads; through the two separate calls the recycling
    kernel cannot keep its three lists in LDS and takes the variant that works on the lists in global memory;
    through fc_rerank_promote the one-kernel path still applies (it needs one list of K entries in LDS)."""
    import dataclasses
    cfg = dataclasses.replace(synth.make_config(1, ctx=100000 + 5, steps=3), topk=(5000,), hot_per_head=40,
                              name="budget_5000")
    _run(cfg)
    _run(cfg, fused_rerank=False)


@pytest.mark.parametrize("ctx,K", [(1, 1), (15, 1), (16, 1), (17, 2), (33, 1), (100, 64), (1000, 5)])
def test_edge_context_lengths_and_budgets(ctx, K):
    import dataclasses
    cfg = synth.make_config(1, ctx=ctx, steps=3)
    n = -(-ctx // 16)
    cfg = dataclasses.replace(cfg, topk=(K,), hot_per_head=min(2, n), name=f"edge_{ctx}_{K}")
    _run(cfg)


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (16, 2), (32, 2)])
def test_group_sizes(Hq, Hkv):
    import dataclasses
    cfg = dataclasses.replace(synth.make_config(1, ctx=1500, steps=3), num_q_heads=Hq, num_kv_heads=Hkv,
                              name=f"group_{Hq // Hkv}")
    _run(cfg)


def test_sixty_four_kv_heads_and_the_maximum_number_of_items():
    """64 KV heads (every bit of the head masks) and 512 sequences x 8 heads = 4096 (sequence, head) items, the
    most one context accepts: the schedule's prefix sums run over 16 rounds of 256 items."""
    import dataclasses
    rng = np.random.default_rng(5)
    base = synth.make_config(1, ctx=700, batch=2, steps=3)
    _run(dataclasses.replace(base, num_q_heads=64, num_kv_heads=64, stable=tuple(bool(x) for x in rng.integers(0, 2, 64)),
                             name="heads_64"))
    ctx = tuple(int(x) for x in rng.integers(1, 90, size=512))
    _run(dataclasses.replace(synth.make_config(4, batch=512, ctx=64, steps=2), ctx=ctx,
                             topk=tuple(max(1, -(-c // 16) // 2) for c in ctx), name="items_4096"))


def test_few_wavefronts_many_items_per_wavefront():
    # 8 wavefronts over 9 sequences x 8 heads: every wavefront crosses several item boundaries
    _run(synth.make_config(4, batch=9, ctx=3000, steps=2), attn_waves=8)


def test_all_heads_stable_and_all_heads_unstable():
    import dataclasses
    base = synth.make_config(2, batch=2, ctx=3000, steps=5)
    _run(dataclasses.replace(base, stable=(True,) * 8, name="all_stable"))
    _run(dataclasses.replace(base, stable=(False,) * 8, dynamics="static", name="all_unstable"))


# ---- full benchmark sizes, launch configuration of bench.py, sampled rows ---------------------------
@pytest.mark.timeout(900)
def test_config2_full_size_sampled_rows():
    """Llama-3-8B-shaped layer at 32k context, batch 8: selections, block tables and MinMax are checked
    for every sequence; attention outputs on two sampled sequences per step."""
    from parity_util import ParityRun
    r = ParityRun(synth.make_config(2, steps=6), sample_rows=2, seed=2)
    try:
        r.run()
    finally:
        r.close()


@pytest.mark.timeout(900)
def test_config3_full_size_128k_sampled_rows():
    from parity_util import ParityRun
    r = ParityRun(synth.make_config(3, steps=9), sample_rows=1, seed=3)
    try:
        r.check_minmax()
        for t in (0, 1, 8):      # a cold-fill rerank, a plain step, and the rerank after the drift
            r.step(t)
    finally:
        r.close()


@pytest.mark.timeout(900)
def test_config4_full_size_ragged_batch64_sampled_rows():
    """64 ragged sequences (4k-32k tokens, partial last pages), blocks shuffled over one shared pool."""
    from parity_util import ParityRun
    r = ParityRun(synth.make_config(4, steps=5), sample_rows=3, seed=4)
    try:
        r.check_minmax()
        for t in (0, 1, 4):
            r.step(t)
    finally:
        r.close()


@pytest.mark.timeout(900)
def test_config5_full_size_offload_sampled_rows():
    """16 x 64k contexts, 5 of 8 heads offloaded: cold fill, then planted pages force promotions."""
    from parity_util import ParityRun
    r = ParityRun(synth.make_config(5, steps=9), sample_rows=2, seed=5)
    try:
        r.check_minmax()
        for t in (0, 1, 4, 8):
            r.step(t)
        assert r.promoted_total >= 16 * 5 * (256 + 2 * 8)
    finally:
        r.close()


# ---- the paper's own treatment of unstable heads: top-K attention, rescored at every step -----------
def test_paper_variant_unstable_heads_topk_every_step_reduced():
    _run(synth.make_config(2, batch=3, ctx=4096 + 7, steps=6), unstable_topk=True)
    _run(synth.make_config(4, batch=5, ctx=5000, steps=5), unstable_topk=True)


@pytest.mark.timeout(900)
def test_paper_variant_full_size_sampled_rows():
    from parity_util import ParityRun
    r = ParityRun(synth.make_config(2, steps=5), sample_rows=2, seed=6, unstable_topk=True)
    try:
        r.run()
    finally:
        r.close()


# ---- contexts that grow during the run: KV append, incremental MinMax, offload of pages as they fill --
@pytest.mark.parametrize("ctx,R", [(2048, 2), (2048 + 9, 2), (300, 3)])
def test_append_tiny_growing_context(ctx, R):
    import dataclasses
    cfg = dataclasses.replace(synth.make_config(1, ctx=ctx, steps=41), append_tokens=40, rerank_interval=R,
                              name=f"append_tiny_{ctx}_{R}")
    _run(cfg)


def test_append_reduced_config2_growing_context():
    import dataclasses
    cfg = dataclasses.replace(synth.make_config(2, batch=3, ctx=4096 + 7, steps=37), append_tokens=36,
                              dynamics="static", name="append_cfg2")
    r = _run(cfg)
    assert len(r.appended_pages) == 3 * 2      # tokens 4103..4138 start pages 257 and 258 in each sequence


def test_append_long_generation_many_new_pages():
    """A generation of 330 tokens on short ragged contexts: every sequence starts 20 or 21 new pages, fills
    them, offloads them and meets them again in later reranks."""
    import dataclasses
    base = synth.make_config(4, batch=3, ctx=900, steps=331)
    cfg = dataclasses.replace(base, append_tokens=330, dynamics="static", rerank_interval=5, name="append_long")
    r = _run(cfg)
    assert len(r.appended_pages) >= 3 * 20


def test_append_paper_variant_growing_context():
    import dataclasses
    cfg = dataclasses.replace(synth.make_config(2, batch=2, ctx=2048 + 15, steps=21), append_tokens=20,
                              dynamics="static", name="append_paper_variant")
    _run(cfg, unstable_topk=True)


def test_bulk_offload_copies_exact_pages_and_skips_bad_pairs():
    import torch
    from paper_2511_00868_amd.session import DecodeSession
    cfg = synth.make_config(1, ctx=1000, steps=1)
    wl = synth.Workload(cfg)
    s = DecodeSession(cfg, wl)
    try:
        # head 1 is unstable: all of its 63 pages sit in HBM; offload a shuffled subset to fresh host blocks
        bt = s.block_table.cpu().numpy()[0, 1, :63]
        rng = np.random.default_rng(1)
        pages = rng.permutation(63)[:40]
        host = torch.zeros((64, 4096), dtype=torch.bfloat16, pin_memory=True)
        pairs = np.stack([bt[pages], np.arange(1, 41)], axis=1).astype(np.int32)
        pairs = np.concatenate([pairs, np.array([[0, 50], [5, 0], [10 ** 6, 51], [3, 64]], dtype=np.int32)])  # skipped
        pd = torch.from_numpy(pairs).cuda()
        s.ctx.fc_offload_pages(s.kv_pool, s.num_pool_blocks, host, 64, pd, len(pairs))
        torch.cuda.synchronize()
        got = host.view(torch.int16).numpy().view(np.uint16)
        from parity_util import native_page
        for i, p in enumerate(pages):
            exp = native_page(wl.k[0][1, 16 * p:16 * p + 16], wl.v[0][1, 16 * p:16 * p + 16])
            if p == 62:      # the partial page: pad tokens are copied as they are, compare the valid ones
                np.testing.assert_array_equal(got[i + 1][:2048].reshape(4, 16, 32)[:, :8], exp[:2048].reshape(4, 16, 32)[:, :8])
                np.testing.assert_array_equal(got[i + 1][2048:].reshape(128, 16)[:, :8], exp[2048:].reshape(128, 16)[:, :8])
            else:
                np.testing.assert_array_equal(got[i + 1], exp)
        assert not got[41:].any() and not got[0].any()
    finally:
        s.close()


@pytest.mark.timeout(900)
def test_one_very_long_sequence_many_partials_per_item():
    """262 147 tokens in one sequence: the unstable head alone is cut into ~1000 wavefront shares, so the
    merge runs over several 256-partial chunks; K = 700 pages for the stable head."""
    import dataclasses
    cfg = dataclasses.replace(synth.make_config(1, ctx=262144 + 3, steps=3), topk=(700,), hot_per_head=64,
                              name="one_long_sequence")
    _run(cfg)


@pytest.mark.parametrize("overlap", [True, "heads", False, "inline", "heads-inline", "heads-ride"])
def test_other_ways_of_running_a_rerank_step(overlap):
    """The default splits a rerank step by page with the copies in line on the main stream and the resident
    pages on the second stream; copies on the second stream, splitting by head class (either way) and not
    splitting at all must give the same results."""
    _run(synth.make_config(5, batch=3, ctx=8192, steps=9), overlap=overlap)
    _run(synth.make_config(2, batch=2, ctx=4096 + 7, steps=5), overlap=overlap)


@pytest.mark.parametrize("seed", range(40))
def test_random_small_configurations(seed):
    """Shapes nobody chose by hand: batch, head counts, group size, ragged contexts, budgets (some above the
    page count), rerank interval, stable flags, block order, dynamics, growth, wavefront count, promotion
    mode, the way a rerank step is overlapped and the treatment of unstable heads drawn from a seed; the
    whole loop is checked against the oracle like the named configurations."""
    rng = np.random.default_rng(1000 + seed)
    batch = int(rng.integers(1, 6))
    Hkv = int(rng.choice([1, 2, 3, 5, 8, 12]))
    G = int(rng.choice([1, 2, 4, 8, 16]))
    ctx = tuple(int(x) for x in rng.integers(1, 2500 if seed < 32 else 12000, size=batch))
    topk = tuple(int(max(1, rng.integers(1, 2 + (-(-c // 16)) * 5 // 4))) for c in ctx)
    stable = tuple(bool(x) for x in rng.integers(0, 2, size=Hkv))
    dynamics = str(rng.choice(["static", "unstable_resample", "drift"]))
    grow = int(rng.choice([0, 0, 7, 40]))
    steps = 7
    cfg = synth.DecodeConfig(name=f"random_{seed}", index=1, batch=batch, num_q_heads=Hkv * G, num_kv_heads=Hkv,
                             ctx=ctx, stable=stable, topk=topk, steps=steps, rerank_interval=int(rng.integers(1, 5)),
                             hot_per_head=int(rng.integers(1, 4)), dynamics="static" if grow else dynamics,
                             dynamics_pages=1, shuffle_blocks=bool(rng.integers(0, 2)), append_tokens=grow,
                             seed=int(rng.integers(1, 1 << 30)))
    print(cfg, flush=True)
    _run(cfg, attn_waves=int(rng.choice([0, 4, 16, 64])),
         promote_mode=int(rng.choice([binding.FC_PROMOTE_GATHER, binding.FC_PROMOTE_GATHER, binding.FC_PROMOTE_MEMCPY])),
         overlap=[True, "heads", False, "inline", "heads-inline", "ride", "heads-ride"][int(rng.integers(0, 7))], unstable_topk=bool(rng.integers(0, 4) == 0),
         fused_rerank=bool(seed % 3))
