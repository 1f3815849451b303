"""CPU tests of the host-side logic: workload generator, static placement, byte accounting."""
import dataclasses

import numpy as np

from paper_2511_00868_amd import synth
from paper_2511_00868_amd.session import plan_placement, pool_blocks_needed


def test_configurations_have_the_benchmark_shapes():
    c2, c3, c5 = synth.make_config(2), synth.make_config(3), synth.make_config(5)
    assert (c2.batch, c2.num_q_heads, c2.num_kv_heads, c2.ctx[0], c2.max_topk, sum(c2.stable)) == (8, 32, 8, 32768, 204, 4)
    assert c2.pages_attended() == 8 * (4 * 2048 + 4 * 204) == 72064
    assert (c3.batch, c3.ctx[0], c3.max_topk, sum(c3.stable), c3.rerank_interval) == (4, 131072, 256, 6, 8)
    assert c3.pages_attended() == 4 * (2 * 8192 + 6 * 256) == 71680
    assert (c5.batch, c5.ctx[0], c5.max_topk, sum(c5.stable)) == (16, 65536, 256, 5)
    assert c5.pages_attended() == 16 * (3 * 4096 + 5 * 256) == 217088
    c4 = synth.make_config(4)
    assert c4.batch == 64 and min(c4.ctx) >= 4096 and max(c4.ctx) <= 32768
    assert any(x % 16 for x in c4.ctx) and any(c4.stable) and not all(c4.stable)
    assert all(k == max(1, (-(-l // 16)) // 8) for k, l in zip(c4.topk, c4.ctx))


def test_generator_is_deterministic_and_order_independent():
    cfg = synth.make_config(1, ctx=300)
    a, b = synth.Workload(cfg), synth.Workload(cfg)
    for x, y in zip(a.k + a.v, b.k + b.v):
        np.testing.assert_array_equal(x, y)
    np.testing.assert_array_equal(a.queries(3), b.queries(3))
    assert a.hot == b.hot
    # pad tokens of the partial last page are NaN patterns
    assert np.all(a.k[0][:, 300:, :] == synth.Workload.PAD_BITS)


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.005859375, 1.01171875, -2.5, 3.3895313892515355e38], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    assert back[0] == 1.0
    assert back[1] == 1.0            # exactly half way between 1.0 and 1.0078125: ties to even
    assert back[2] == 1.0078125      # just above half way
    assert back[3] == 1.015625       # half way between 1.0078125 (odd) and 1.015625 (even): to even
    assert back[4] == -2.5
    assert np.all(np.abs(back[:5] - x[:5]) <= np.abs(x[:5]) * 2.0 ** -8)


def test_hot_page_dynamics_restore_original_bits():
    cfg = dataclasses.replace(synth.make_config(3, batch=1, ctx=4096, steps=20), name="drift_small")
    w = synth.Workload(cfg)
    pristine = synth.Workload(dataclasses.replace(cfg, hot_per_head=0, dynamics="static"))
    # un-planting every hot page must give back the never-planted draw exactly
    for (b, h), pages in list(w.hot.items()):
        w._retire(b, h, list(pages))
    for x, y in zip(w.k, pristine.k):
        np.testing.assert_array_equal(x, y)


def test_drift_changes_two_pages_per_rerank_and_reports_them():
    cfg = synth.make_config(3, batch=1, ctx=8192, steps=20)
    w = synth.Workload(cfg)
    before = {k: list(v) for k, v in w.hot.items()}
    assert w.advance(3) == []                        # not a rerank step
    ch = w.advance(8)
    assert {(b, h) for b, h, _ in ch} == {(0, h) for h in range(8) if cfg.stable[h]}
    for b, h, pages in ch:
        assert len(set(before[(b, h)]) - set(w.hot[(b, h)])) == 2
        assert len(set(w.hot[(b, h)]) - set(before[(b, h)])) == 2
        assert set(pages) == set(before[(b, h)]) ^ set(w.hot[(b, h)])


def test_placement_hands_out_every_block_once_and_never_block_zero():
    for idx in (1, 2, 4):
        cfg = synth.make_config(idx, batch=3 if idx != 1 else None, ctx=3000 if idx != 1 else None)
        w = synth.Workload(cfg)
        need = pool_blocks_needed(cfg)
        order = w.block_permutation(need)
        bt, hbt, fb, fc, nblk, nhost = plan_placement(cfg, order)
        assert nblk == need + 1
        used = list(bt[bt > 0]) + [int(x) for b in range(cfg.batch) for h in range(cfg.num_kv_heads)
                                   for x in fb[b, h, :fc[b, h]]]
        assert sorted(used) == list(range(1, need + 1))
        for b in range(cfg.batch):
            n = cfg.num_pages(b)
            for h in range(cfg.num_kv_heads):
                if cfg.stable[h]:
                    assert fc[b, h] == min(cfg.topk[b], n) and not bt[b, h].any()
                    assert np.all(hbt[b, h, :n] > 0) and not hbt[b, h, n:].any()
                else:
                    assert np.all(bt[b, h, :n] > 0) and not bt[b, h, n:].any() and fc[b, h] == 0
        host_used = hbt[hbt > 0]
        assert len(set(host_used.tolist())) == len(host_used) and nhost == len(host_used) + 1
    assert synth.Workload(synth.make_config(4, batch=3, ctx=3000)).block_permutation(50).tolist() != list(range(1, 51))


def test_byte_accounting_matches_the_page_arithmetic():
    import bench
    c2 = synth.make_config(2)
    pages = c2.pages_attended()
    expect = pages * 8192 + 8 * (4 * 2048 * 4 + 4 * 204 * 8) + 8 * 32 * 768
    assert bench.attention_bytes(c2) == expect
    assert abs(bench.attention_bytes(c2) / 1e6 - 590.3) < 1.0          # 72 064 pages x 8 KiB
    assert bench.rerank_bytes(c2) == 8 * 4 * (2048 * 512 + 4 * 256 + 4 * 204)
    ragged = synth.make_config(1, ctx=100)                              # 7 pages, last one holds 4 tokens
    # stable head: K = 8 > 7 pages -> all 7 pages incl. the partial one; unstable head: the same tokens
    assert bench.attention_bytes(ragged) == (512 * 100 + 8 * 7) + (512 * 100 + 4 * 7) + 8 * 768
