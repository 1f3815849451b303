"""GPU tests of error paths, copy/compute ordering and per-sequence rerank phases.  Every kernel exits
normally in all of them: errors are forced from the host (bad arguments, too few blocks)."""
import ctypes as C
import dataclasses

import numpy as np
import pytest

import oracle
from paper_2511_00868_amd import binding, synth
from paper_2511_00868_amd.session import DecodeSession

pytestmark = pytest.mark.gpu


def test_bad_arguments_are_rejected_before_anything_is_launched():
    import torch
    ctx = binding.Context(num_q_heads=8, num_kv_heads=2, max_batch=2, max_pages_per_seq=16, max_topk=4)
    try:
        q = torch.zeros((2, 8, 128), dtype=torch.bfloat16, device="cuda")
        out = torch.zeros((2, 8, 128), dtype=torch.float32, device="cuda")
        tbl = torch.ones((2, 2, 16), dtype=torch.int32, device="cuda")       # every page in block 1
        lens = torch.ones(2, dtype=torch.int32, device="cuda")
        pool = torch.zeros((4, 4096), dtype=torch.bfloat16, device="cuda")
        ok = dict(q=q, kv_pool=pool, num_pool_blocks=4, block_table=tbl, context_lens=lens, stable_flag=[False, False],
                  topk_pages=None, topk_count=None, batch=2, out=out)
        for bad in (dict(q=None), dict(out=None), dict(batch=0), dict(batch=3), dict(num_pool_blocks=1),
                    dict(head_subset=7), dict(stable_flag=[True, False])):       # stable head without lists
            with pytest.raises(binding.FlexiCacheError) as e:
                ctx.fc_sparse_decode_attn(**{**ok, **bad})
            assert e.value.status == binding.FC_ERR_INVALID_ARG and "fc_sparse_decode_attn" in str(e.value)
        with pytest.raises(binding.FlexiCacheError) as e:
            ctx.fc_rerank_topk(q=q, minmax=None, context_lens=lens, stable_flag=[True, False], k_per_seq=lens, batch=2,
                               topk_pages=tbl, topk_count=lens)
        assert e.value.status == binding.FC_ERR_INVALID_ARG
        s = torch.cuda.current_stream()
        with pytest.raises(binding.FlexiCacheError) as e:
            ctx.fc_promote_pages(new_pages=tbl, new_count=lens, resident_pages=tbl, resident_count=lens, block_table=tbl,
                                 host_block_table=tbl, free_blocks=tbl, free_count=lens, stable_flag=[True, False],
                                 kv_pool=pool, num_pool_blocks=4, host_pool=pool, num_host_blocks=4, batch=2,
                                 main_stream=s, side_stream=s, mode=7)
        assert e.value.status == binding.FC_ERR_INVALID_ARG
        with pytest.raises(binding.FlexiCacheError):
            ctx.fc_write_kv_pages(q, q, 17, tbl, pool, 4)                          # more pages than max_pages_per_seq
        with pytest.raises(binding.FlexiCacheError):
            ctx.fc_build_minmax(pool, 4, tbl, None, 3, 100, q)                     # n_list must equal the page count
        ctx.fc_sparse_decode_attn(**ok)                                            # the good call still works
        torch.cuda.synchronize()
        ctx.fc_check_device_state()
    finally:
        ctx.close()
    with pytest.raises(binding.FlexiCacheError):
        binding.Context(num_q_heads=8, num_kv_heads=2, max_batch=2, max_pages_per_seq=16, max_topk=4, head_dim=64)


def test_too_few_blocks_is_reported_not_faulted():
    cfg = synth.make_config(1, steps=1)
    wl = synth.Workload(cfg)
    s = DecodeSession(cfg, wl)
    try:
        s.free_count[0, 0] = 3                    # the stable head will select 8 pages but owns 3 blocks
        s.set_queries(wl.queries(0))
        s.rerank()
        s.promote()
        s.torch.cuda.synchronize()
        with pytest.raises(binding.FlexiCacheError) as e:
            s.ctx.fc_check_device_state()
        assert e.value.status == binding.FC_ERR_STATE
        s.ctx.fc_check_device_state()             # the error word was cleared by the read
        assert int(s.promoted_count[0, 0]) == 8 and int((s.block_table[0, 0] > 0).sum()) == 3
    finally:
        s.close()


def _run_steps_against_oracle(s, wl, cfg, steps, before_step=None):
    dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, cfg.topk,
                               cfg.rerank_interval)
    mm = [oracle.seq_build_minmax(wl.k[b], cfg.ctx[b]) for b in range(cfg.batch)]
    for t in range(steps):
        q = wl.queries(t)
        s.set_queries(q)
        if before_step:
            before_step(t)
        s.step(t)
        s.torch.cuda.synchronize()
        s.ctx.fc_check_device_state()
        got = s.out.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got)), "a poisoned block was read before its copy had landed"
        sel = s.selected()
        for b in range(cfg.batch):
            if cfg.is_rerank_step(t):
                dec.rerank(b, q[b], mm[b])
            ref, _ = dec.attend(b, q[b], wl.k[b], wl.v[b], override=sel)
            err = np.abs(got[b] - ref).max(axis=1) / np.abs(ref).max(axis=1)
            assert err.max() <= 2e-3


@pytest.mark.parametrize("mode,overlap", [(binding.FC_PROMOTE_GATHER, True), (binding.FC_PROMOTE_MEMCPY, True),
                                          (binding.FC_PROMOTE_GATHER, "heads"), (binding.FC_PROMOTE_GATHER, "inline"),
                                          (binding.FC_PROMOTE_GATHER, "heads-inline"), (binding.FC_PROMOTE_MEMCPY, "inline")])
def test_attention_waits_for_delayed_copies_into_poisoned_blocks(mode, overlap):
    """Every block a promoted page will land in holds NaN until its copy arrives, and the second stream is
    held back by a long sleep kernel before each rerank step: the stable heads' attention must still see
    the copied pages (a premature read would surface as NaN).  In the in-line modes the second stream
    carries the first attention call of the pair instead of the copies: the merge must wait for it."""
    import torch
    cfg = synth.make_config(5, batch=2, ctx=4096, steps=9)
    wl = synth.Workload(cfg)
    s = DecodeSession(cfg, wl, promote_mode=mode)
    s.overlap = overlap
    try:
        fb, fc = s.free_blocks.cpu().numpy(), s.free_count.cpu().numpy()
        ids = [int(x) for b in range(cfg.batch) for h in range(cfg.num_kv_heads) for x in fb[b, h, :fc[b, h]]]
        s.kv_pool[torch.tensor(ids, device="cuda")] = float("nan")

        def hold_back_copies(t):
            if cfg.is_rerank_step(t):
                with torch.cuda.stream(s.copy):
                    torch.cuda._sleep(20_000_000)        # ~10 ms at the GPU's clock
                # recycled blocks are about to be overwritten by copies: poison them as the evicted pages leave
        _run_steps_against_oracle(s, wl, cfg, 9, hold_back_copies)
    finally:
        s.close()


@pytest.mark.parametrize("split", [False, "two streams", "ride"])
def test_per_sequence_rerank_phases(split):
    """rerank_mask staggers the sequences (the paper pauses one request at a time, Sec. 3.3): sequence b
    reranks when (t + b) mod R == 0; the others keep their lists, tables and blocks untouched.  With `split`
    the attention runs as the resident / promoted pair: on two streams around in-line copies, or on one
    stream with the copies riding in the first launch."""
    import torch
    cfg = synth.make_config(2, batch=4, ctx=2048 + 5, steps=8)
    wl = synth.Workload(dataclasses.replace(cfg, dynamics="static"))
    s = DecodeSession(cfg, wl)
    try:
        R = cfg.rerank_interval
        dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, cfg.topk, R)
        mm = [oracle.seq_build_minmax(wl.k[b], cfg.ctx[b]) for b in range(cfg.batch)]
        warmed = set()
        for t in range(2 * R):
            q = wl.queries(t)
            s.set_queries(q)
            # every sequence needs one cold fill first; afterwards they take turns
            mask = [1 if (b not in warmed or (t + b) % R == 0) else 0 for b in range(cfg.batch)]
            md = torch.tensor(mask, dtype=torch.uint8, device="cuda")
            before = (s.resident_pages.clone(), s.block_table.clone(), s.free_blocks.clone())
            s.rerank(rerank_mask=md)
            if split == "ride":
                s.promote(rerank_mask=md, copy_stream=s.main, mode=binding.FC_PROMOTE_RIDE)
                s.attend(binding.FC_PAGES_RESIDENT)
                s.attend(binding.FC_PAGES_PROMOTED)
            elif split:
                s.promote(rerank_mask=md, copy_stream=s.main)
                s.attend(binding.FC_PAGES_RESIDENT, stream=s.copy)
                s.attend(binding.FC_PAGES_PROMOTED)
            else:
                s.promote(rerank_mask=md)
                s.attend()
            torch.cuda.synchronize()
            s.ctx.fc_check_device_state()
            sel = s.selected()
            got = s.out.cpu().numpy().astype(np.float64)
            for b in range(cfg.batch):
                if mask[b]:
                    dec.rerank(b, q[b], mm[b])
                    warmed.add(b)
                    for h in range(cfg.num_kv_heads):
                        if cfg.stable[h]:
                            assert set(sel[(b, h)]) == set(dec.sel[(b, h)])
                else:
                    for old, new in zip(before, (s.resident_pages, s.block_table, s.free_blocks)):
                        assert torch.equal(old[b], new[b])
                    assert int(s.promoted_count[b].sum()) == 0
                ref, _ = dec.attend(b, q[b], wl.k[b], wl.v[b])
                assert (np.abs(got[b] - ref).max(axis=1) / np.abs(ref).max(axis=1)).max() <= 2e-3
    finally:
        s.close()


def test_stream_read_measurement_reads_in_bounds_and_rejects_bad_arguments():
    """The same-box ceiling of the benchmark: a plain read of a buffer.  Odd sizes exercise the ragged tail of
    the grid-stride loop; guard words after the buffer stay untouched (the kernel only reads the buffer, its
    sink is the workspace)."""
    import torch
    ctx = binding.Context(num_q_heads=8, num_kv_heads=2, max_batch=2, max_pages_per_seq=16, max_topk=4)
    try:
        buf = torch.arange(0, (8 << 20) // 4 + 64, dtype=torch.int32, device="cuda")
        before = buf.clone()
        for nbytes in (4096, 4096 + 16, (1 << 20) + 48, 8 << 20):
            gbs, us = ctx.fc_measure_stream_read(buf, nbytes, 4)
            assert gbs > 0 and us > 0
        assert torch.equal(buf, before)
        for bad in (dict(nbytes=100), dict(nbytes=4096 + 8), dict(launches=0), dict(launches=5000)):
            kw = {"nbytes": 4096, "launches": 2, **bad}
            with pytest.raises(binding.FlexiCacheError) as e:
                ctx.fc_measure_stream_read(buf, kw["nbytes"], kw["launches"])
            assert e.value.status == binding.FC_ERR_INVALID_ARG
        ctx.fc_profile_begin(1)
        with pytest.raises(binding.FlexiCacheError) as e:
            ctx.fc_measure_stream_read(buf, 4096, 2)
        assert e.value.status == binding.FC_ERR_STATE
        ctx.fc_profile_end()
    finally:
        ctx.close()


@pytest.mark.parametrize("overlap,steps", [("inline", 24), (True, 24), ("heads", 24), ("heads-inline", 24), (False, 24),
                                           ("ride", 24), ("heads-ride", 24), ("ride", 160)])
def test_free_running_loop_without_host_synchronisation(overlap, steps):
    """The parity harness looks at every step's results, which synchronises the host with the GPU after
    every step and could hide an ordering mistake between consecutive steps (a recycle kernel handing out a
    block that the previous step's attention is still reading, a merge that starts before its partials).
    Here 24 (once 160) steps are enqueued back to back; outputs and selections of every step
    are kept on the device and checked against the oracle only afterwards."""
    import torch
    cfg = synth.make_config(5, batch=3, ctx=8192, steps=steps)
    cfg = dataclasses.replace(cfg, dynamics="static")       # the inputs stay put; the queries alone move the selection
    wl = synth.Workload(cfg)
    s = DecodeSession(cfg, wl, keep_scores=True)
    s.overlap = overlap
    try:
        from parity_util import audit_sets
        T = cfg.steps
        qs = [wl.queries(t) for t in range(T)]
        q_dev = torch.stack([s.bits_to_dev(q) for q in qs])
        outs = torch.zeros((T,) + tuple(s.out.shape), dtype=torch.float32, device="cuda")
        sel_pages = torch.zeros((T,) + tuple(s.resident_pages.shape), dtype=torch.int32, device="cuda")
        sel_count = torch.zeros((T,) + tuple(s.resident_count.shape), dtype=torch.int32, device="cuda")
        for t in range(T):
            s.q = q_dev[t]
            if t % 3 == 1:                      # shift the two streams against each other now and then
                with torch.cuda.stream(s.copy):
                    torch.cuda._sleep(150_000)  # ~70 us
            if t % 5 == 2:
                torch.cuda._sleep(100_000)
            s.step(t)
            outs[t].copy_(s.out, non_blocking=True)
            sel_pages[t].copy_(s.resident_pages, non_blocking=True)
            sel_count[t].copy_(s.resident_count, non_blocking=True)
        torch.cuda.synchronize()
        s.ctx.fc_check_device_state()
        outs, sel_pages, sel_count = outs.cpu().numpy().astype(np.float64), sel_pages.cpu().numpy(), sel_count.cpu().numpy()
        assert np.all(np.isfinite(outs))
        dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, cfg.topk,
                                   cfg.rerank_interval)
        mm = [oracle.seq_build_minmax(wl.k[b], cfg.ctx[b]) for b in range(cfg.batch)]
        swaps = 0
        for t in range(T):
            sel = {(b, h): sel_pages[t, b, h, :sel_count[t, b, h]] for b in range(cfg.batch)
                   for h in range(cfg.num_kv_heads) if cfg.stable[h]}
            for b in range(cfg.batch):
                if cfg.is_rerank_step(t):
                    dec.rerank(b, qs[t][b], mm[b])
                for h in range(cfg.num_kv_heads):
                    if cfg.stable[h]:
                        # the selection itself: identical, except where the oracle's own fp64 scores show a near-tie at
                        # the budget boundary (the rule of the parity harness; an ordering race between scoring and
                        # selection would show up here as a swap that no near-tie explains); between reranks the
                        # list must not move at all
                        g, o = sel[(b, h)], dec.sel[(b, h)]
                        assert np.all(np.diff(g) > 0)
                        if cfg.is_rerank_step(t):
                            audit_sets(g, o, dec.last_scores[(b, h)], -1)
                            if set(g.tolist()) != set(o.tolist()):
                                swaps += 1
                                dec.sel[(b, h)] = np.array(sorted(g.tolist()), dtype=np.int32)   # follow the legal swap
                        else:
                            np.testing.assert_array_equal(g, o)
                ref, _ = dec.attend(b, qs[t][b], wl.k[b], wl.v[b])
                err = np.abs(outs[t, b] - ref).max(axis=1) / np.abs(ref).max(axis=1)
                assert err.max() <= 2e-3, (t, b, err.max())
        print(f"free-running {overlap}: near-tie swaps {swaps}")
    finally:
        s.close()


def test_riding_copies_that_no_pair_carries_are_launched_on_their_own():
    """FC_PROMOTE_RIDE leaves the copies to the next attention launch.  If that launch is a whole pass
    (FC_HEADS_ALL) instead of the first call of a pair, or another fc_promote_pages comes first, the
    library launches them on their own before it; an attention call on another stream is refused."""
    import torch
    cfg = synth.make_config(5, batch=2, ctx=4096, steps=9)
    wl = synth.Workload(cfg)
    s = DecodeSession(cfg, wl)
    try:
        dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, cfg.topk,
                                   cfg.rerank_interval)
        mm = [oracle.seq_build_minmax(wl.k[b], cfg.ctx[b]) for b in range(cfg.batch)]
        for t in range(3):
            q = wl.queries(t)
            s.set_queries(q)
            s.rerank()
            s.promote(copy_stream=s.main, mode=binding.FC_PROMOTE_RIDE)
            if t == 1:       # a second promotion with the same lists before any attention: nothing more to promote
                s.promote(copy_stream=s.main, mode=binding.FC_PROMOTE_RIDE)
            if t == 2:
                with pytest.raises(binding.FlexiCacheError) as e:
                    s.attend(stream=s.copy)
                assert e.value.status == binding.FC_ERR_INVALID_ARG
            s.attend()
            torch.cuda.synchronize()
            s.ctx.fc_check_device_state()
            got = s.out.cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(got))
            sel = s.selected()
            for b in range(cfg.batch):
                dec.rerank(b, q[b], mm[b])
                ref, _ = dec.attend(b, q[b], wl.k[b], wl.v[b], override=sel)
                assert (np.abs(got[b] - ref).max(axis=1) / np.abs(ref).max(axis=1)).max() <= 2e-3
    finally:
        s.close()


def test_attention_reports_broken_tables_instead_of_answering_plausibly():
    """A block-table entry outside the pool, a list entry outside the sequence, and an attended page whose
    table entry is the null block: the attention kernel keeps every access in bounds (so it exits normally
    and the output is finite where the clamped block holds numbers) and sets the device error word, which
    fc_check_device_state turns into FC_ERR_STATE."""
    import torch
    cfg = synth.make_config(1, ctx=1000, steps=2)
    wl = synth.Workload(cfg)
    s = DecodeSession(cfg, wl)
    try:
        s.set_queries(wl.queries(0))
        s.step(0)
        torch.cuda.synchronize()
        s.ctx.fc_check_device_state()
        good_table, good_list = s.block_table.clone(), s.resident_pages.clone()

        def attend_expecting(text):
            s.attend()
            torch.cuda.synchronize()
            with pytest.raises(binding.FlexiCacheError) as e:
                s.ctx.fc_check_device_state()
            assert e.value.status == binding.FC_ERR_STATE and text in str(e.value)
            s.ctx.fc_check_device_state()            # cleared by the read
            s.block_table.copy_(good_table)
            s.resident_pages.copy_(good_list)

        s.block_table[0, 1, 7] = s.num_pool_blocks + 12345       # unstable head, beyond the pool
        attend_expecting("= 2")
        s.block_table[0, 1, 3] = -9
        attend_expecting("= 2")
        s.resident_pages[0, 0, 2] = 10 ** 6                       # stable head, a page the sequence does not have
        attend_expecting("= 2")
        s.block_table[0, 1, 11] = 0                               # an attended page without a block
        attend_expecting("= 8")
        s.attend()                                                # and with the tables restored all is well again
        torch.cuda.synchronize()
        s.ctx.fc_check_device_state()
        assert torch.isfinite(s.out).all()
    finally:
        s.close()


def test_append_without_a_free_block_keeps_the_sequence_length():
    """fc_append_kv at a page boundary for a head that owns no free block: the error word is set, nothing is
    written for that head, and the sequence's length stays where it was (the other sequence advances)."""
    import torch
    cfg = dataclasses.replace(synth.make_config(1, ctx=2048, batch=2, steps=3), append_tokens=2, name="append_no_block")
    wl = synth.Workload(cfg)
    s = DecodeSession(cfg, wl)
    try:
        s.set_queries(wl.queries(0))
        s.step(0)
        torch.cuda.synchronize()
        assert s.context_lens.cpu().tolist() == [2048, 2048]      # the next token starts page 128 in every head
        s.free_count[0, 1] = 0                                    # sequence 0, unstable head: nothing to start it in
        table_before = s.block_table.clone()
        k, v = wl.append(1)
        s.append(k, v)
        torch.cuda.synchronize()
        with pytest.raises(binding.FlexiCacheError) as e:
            s.ctx.fc_check_device_state()
        assert e.value.status == binding.FC_ERR_STATE
        assert s.context_lens.cpu().tolist() == [2048, 2049]
        assert torch.equal(s.block_table[0, 1], table_before[0, 1])
        assert int(s.block_table[1, 1, 128]) > 0
    finally:
        s.close()


def test_a_rerank_cycle_captured_in_a_hip_graph_replays_like_the_eager_loop():
    """The default single-stream path (fc_rerank_promote with riding copies, the resident / promoted attention
    pair, one merge; whole passes on the plain steps) records no event, waits for nothing on the host and
    allocates nothing, so a whole rerank cycle can be captured in a HIP graph.  Three replays, with eager work
    and synchronisations between them, must leave the outputs, lists, tables and free lists that the same
    steps give eagerly in a second session."""
    import torch
    cfg = dataclasses.replace(synth.make_config(5, batch=3, ctx=8192, steps=32), dynamics="static")
    R = cfg.rerank_interval
    wl = synth.Workload(cfg)
    eager, graphed = DecodeSession(cfg, wl), DecodeSession(cfg, wl)
    try:
        eager.overlap = graphed.overlap = "ride"
        qs = torch.stack([eager.bits_to_dev(wl.queries(t)) for t in range(4 * R)])
        stream = torch.cuda.Stream()
        graphed.main = stream
        graphed.copy = stream

        def cycle(s, c):                                 # steps c*R .. c*R + R - 1, queries copied into the session's own buffer
            for t in range(c * R, (c + 1) * R):
                s.q.copy_(qs_view[t - c * R])
                s.step(t)

        with torch.cuda.stream(stream):
            qs_view = qs[0:R]
            cycle(graphed, 0)                            # cold fill, eagerly, on the capturing stream
            torch.cuda.synchronize()
            staged = torch.zeros_like(qs[0:R])           # the graph reads its queries from here
            qs_view = staged
            g = torch.cuda.CUDAGraph()
            g.capture_begin()
            cycle(graphed, 1)
            g.capture_end()
        torch.cuda.synchronize()
        qs_view = qs[0:R]
        cycle(eager, 0)
        for c in (1, 2, 3):
            staged.copy_(qs[c * R:(c + 1) * R])          # eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            qs_view = qs[c * R:(c + 1) * R]
            cycle(eager, c)
            torch.cuda.synchronize()
            graphed.ctx.fc_check_device_state(stream)
            eager.ctx.fc_check_device_state()
            for name in ("out", "lse", "resident_pages", "resident_count", "block_table", "free_count", "promoted_count"):
                assert torch.equal(getattr(graphed, name), getattr(eager, name)), (c, name)
            assert torch.isfinite(graphed.out).all()
    finally:
        eager.close()
        graphed.close()
