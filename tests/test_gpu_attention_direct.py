"""Attention on crafted inputs with closed-form answers and awkward magnitudes (through the C ABI)."""
import dataclasses

import numpy as np
import pytest

import oracle
from paper_2511_00868_amd import synth
from paper_2511_00868_amd.session import DecodeSession

pytestmark = pytest.mark.gpu


def widen(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def make(ctx, mutate, stable=(False, False), K=4, scale=0.0, batch=1):
    cfg = dataclasses.replace(synth.make_config(1, ctx=ctx, batch=batch, steps=1), stable=stable, topk=(K,) * batch,
                              hot_per_head=0, name="crafted")
    wl = synth.Workload(cfg)
    mutate(wl)
    return cfg, wl, DecodeSession(cfg, wl, softmax_scale=scale)


def attend_and_compare(cfg, wl, s, q_bits, scale=None, tol=2e-3):
    s.set_queries(q_bits)
    if any(cfg.stable):
        s.rerank()
        s.promote()
    s.attend()
    s.torch.cuda.synchronize()
    s.ctx.fc_check_device_state()
    got, lse = s.out.cpu().numpy().astype(np.float64), s.lse.cpu().numpy().astype(np.float64)
    dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, cfg.topk, 1, scale=scale)
    for b in range(cfg.batch):
        if any(cfg.stable):
            dec.rerank(b, q_bits[b], oracle.seq_build_minmax(wl.k[b], cfg.ctx[b]))
        ref, ref_lse = dec.attend(b, q_bits[b], wl.k[b], wl.v[b], override=s.selected())
        assert np.all(np.isfinite(got[b]))
        err = np.abs(got[b] - ref).max(axis=1) / np.maximum(np.abs(ref).max(axis=1), 1e-30)
        assert err.max() <= tol, err
        np.testing.assert_allclose(lse[b], ref_lse, rtol=1e-5, atol=2e-3)
    return got


def test_identical_keys_give_the_mean_of_the_values():
    def mutate(wl):
        wl.k[0][:, :, :] = wl.k[0][:, :1, :]
    cfg, wl, s = make(1000, mutate)
    try:
        got = attend_and_compare(cfg, wl, s, wl.queries(0))
        for hq in range(cfg.num_q_heads):
            mean = widen(wl.v[0][hq // cfg.group, :1000]).mean(0)
            assert np.abs(got[0, hq] - mean).max() <= 2e-3 * np.abs(mean).max() + 1e-6
    finally:
        s.close()


def test_huge_logits_do_not_overflow_and_one_key_wins():
    bits30 = synth.f32_to_bf16_bits(np.array([30.0], dtype=np.float32))[0]
    def mutate(wl):
        wl.k[0][:, :, :] = bits30 | 0x8000                 # every key = -30 ...
        wl.k[0][:, 777, :] = bits30                        # ... but one = +30
    cfg, wl, s = make(2048, mutate)
    try:
        q = np.full((1, cfg.num_q_heads, 128), bits30, dtype=np.uint16)     # logits +-115200 / sqrt(128)
        got = attend_and_compare(cfg, wl, s, q)
        for hq in range(cfg.num_q_heads):
            np.testing.assert_allclose(got[0, hq], widen(wl.v[0][hq // cfg.group, 777]), rtol=1e-6, atol=1e-6)
    finally:
        s.close()


def test_tiny_logits_and_custom_scale():
    def mutate(wl):
        wl.k[0][:] = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(wl.k[0]) * np.float32(2.0 ** -20))
    cfg, wl, s = make(513, mutate, scale=0.5)
    try:
        attend_and_compare(cfg, wl, s, wl.queries(0), scale=0.5)
    finally:
        s.close()


def test_value_outliers_are_carried_through_the_split_p_product():
    """One value of magnitude 2^100 among unit-scale values: the hi/lo split of P must keep the small
    contributions of the other dims intact and the large one accurate."""
    def mutate(wl):
        wl.v[0][0, 5, 3] = synth.f32_to_bf16_bits(np.array([2.0 ** 100], dtype=np.float32))[0]
        wl.v[0][1, 900, 64] = synth.f32_to_bf16_bits(np.array([-2.0 ** 90], dtype=np.float32))[0]
    cfg, wl, s = make(1500, mutate)
    try:
        attend_and_compare(cfg, wl, s, wl.queries(0))
    finally:
        s.close()


def test_stable_head_with_budget_one_and_batch_of_three():
    cfg, wl, s = make(333, lambda wl: None, stable=(True, True), K=1, batch=3)
    try:
        attend_and_compare(cfg, wl, s, wl.queries(0))
        assert all(len(v) == 1 for v in s.selected().values())
    finally:
        s.close()


@pytest.mark.parametrize("stable", [(False, False), (True, False)])
def test_a_sequence_without_tokens_gets_zero_output_and_minus_infinity_lse(stable):
    """An idle slot of the batch (context length 0) has no pages: its rows are defined (zeros, lse = -inf),
    the rerank gives it an empty list, nothing is promoted for it, and its neighbours are untouched."""
    cfg, wl, s = make(333, lambda wl: None, stable=stable, K=3, batch=3)
    try:
        q = wl.queries(0)
        s.set_queries(q)
        s.context_lens[1] = 0
        s.out.fill_(7.0)
        s.lse.fill_(7.0)
        if any(stable):
            s.rerank()
            s.promote()
        s.attend()
        s.torch.cuda.synchronize()
        s.ctx.fc_check_device_state()
        out, lse = s.out.cpu().numpy().astype(np.float64), s.lse.cpu().numpy().astype(np.float64)
        assert not out[1].any() and np.all(np.isneginf(lse[1]))
        if any(stable):
            assert int(s.topk_count[1, 0]) == 0 and int(s.resident_count[1, 0]) == 0
            assert int(s.promoted_count[1, 0]) == 0
        dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable, cfg.topk, 1)
        for b in (0, 2):
            if any(stable):
                dec.rerank(b, q[b], oracle.seq_build_minmax(wl.k[b], cfg.ctx[b]))
            ref, ref_lse = dec.attend(b, q[b], wl.k[b], wl.v[b], override=s.selected())
            err = np.abs(out[b] - ref).max(axis=1) / np.abs(ref).max(axis=1)
            assert err.max() <= 2e-3
            np.testing.assert_allclose(lse[b], ref_lse, rtol=1e-5, atol=2e-3)
    finally:
        s.close()
