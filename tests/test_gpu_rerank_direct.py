"""fc_rerank_topk called directly on crafted MinMax rows: exact ties, negative scores, degenerate sizes.
Values are small integers, so fp32 (GPU) and fp64 (oracle) sums are both exact and the selections must
be identical, tie-break included."""
import numpy as np
import pytest

import oracle
from paper_2511_00868_amd import binding, synth

pytestmark = pytest.mark.gpu


def bf16(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def run_case(q_vals, kmin_vals, kmax_vals, ctx, K, Hq=4, Hkv=1):
    """q_vals [Hq, 128], kmin/kmax [Hkv, n, 128] (small integers).  Returns (gpu list, oracle list, scores)."""
    import torch
    n = kmin_vals.shape[1]
    assert n == -(-ctx // 16)
    c = binding.Context(num_q_heads=Hq, num_kv_heads=Hkv, max_batch=1, max_pages_per_seq=n, max_topk=max(1, min(K, n)))
    try:
        mm = np.stack([bf16(kmin_vals), bf16(kmax_vals)], axis=2)               # [Hkv, n, 2, 128]
        qb = bf16(q_vals)[None]                                                  # [1, Hq, 128]
        dev = lambda a, dt: torch.from_numpy(a.view(np.int16) if a.dtype == np.uint16 else a).cuda().view(dt)
        q_d, mm_d = dev(qb, torch.bfloat16), dev(mm[None], torch.bfloat16)
        lens = torch.tensor([ctx], dtype=torch.int32, device="cuda")
        kk = torch.tensor([K], dtype=torch.int32, device="cuda")
        Kmax = max(1, min(K, n))
        pages = torch.full((1, Hkv, Kmax), -7, dtype=torch.int32, device="cuda")
        cnt = torch.zeros((1, Hkv), dtype=torch.int32, device="cuda")
        sc = torch.zeros((1, Hkv, n), dtype=torch.float32, device="cuda")
        c.fc_rerank_topk(q=q_d, minmax=mm_d, context_lens=lens, stable_flag=[True] * Hkv, k_per_seq=kk, batch=1,
                         topk_pages=pages, topk_count=cnt, scores_out=sc)
        torch.cuda.synchronize()
        G = Hq // Hkv
        out = []
        for h in range(Hkv):
            s = oracle.page_scores(qb[0, h * G:(h + 1) * G], mm[h])
            np.testing.assert_array_equal(sc.cpu().numpy()[0, h], s)            # exact: small integers
            ref = oracle.select_topk(s, ctx, K)
            got = pages.cpu().numpy()[0, h]
            k = int(cnt[0, h])
            assert k == len(ref) == min(K, n)
            np.testing.assert_array_equal(got[:k], ref)
            assert np.all(got[k:] == -1)
            out.append((got[:k], ref, s))
        return out
    finally:
        c.close()


def ints(rng, shape, lo, hi):
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


def test_all_scores_equal_selects_the_lowest_page_indices():
    n, K = 300, 37
    kmin = np.full((1, n, 128), -1.0, dtype=np.float32)
    kmax = np.full((1, n, 128), 2.0, dtype=np.float32)
    q = np.ones((4, 128), dtype=np.float32)
    (got, _, s), = run_case(q, kmin, kmax, n * 16, K)
    assert list(got) == list(range(K)) and np.all(s == 256.0)
    # with a partially filled last page, that page is a member and the rest are the lowest indices
    (got, _, _), = run_case(q, kmin, kmax, n * 16 - 5, K)
    assert list(got) == list(range(K - 1)) + [n - 1]


@pytest.mark.parametrize("n,K", [(1, 1), (2, 1), (16, 16), (17, 3), (64, 64), (1000, 1), (1000, 999), (2048, 204),
                                 (8192, 256), (20000, 1500), (65536, 4096)])
def test_quantised_scores_with_many_exact_ties(n, K):
    rng = np.random.default_rng(n * 7 + K)
    # few distinct integer rows -> few distinct scores -> long runs of exact ties across the K boundary
    protos_lo = ints(rng, (5, 128), -3, 0)
    protos_hi = protos_lo + ints(rng, (5, 128), 0, 3)
    which = rng.integers(0, 5, size=n)
    kmin, kmax = protos_lo[which][None], protos_hi[which][None]
    q = ints(rng, (4, 128), -2, 2)
    for ctx in (n * 16, n * 16 - 9):
        run_case(q, kmin, kmax, ctx, K)


def test_negative_and_mixed_sign_scores_order_correctly():
    rng = np.random.default_rng(5)
    n = 500
    lo = ints(rng, (1, n, 128), 1, 4)                  # all keys positive ...
    hi = lo + ints(rng, (1, n, 128), 0, 3)
    q = -ints(rng, (4, 128), 0, 3)                      # ... all queries non-positive: every score is <= 0
    (got, ref, s), = run_case(q, lo, hi, n * 16, 50)
    assert s.max() <= 0 and s.min() < -100
    # mixed: half of the pages get negated keys, so scores straddle zero
    lo2, hi2 = lo.copy(), hi.copy()
    lo2[0, ::2], hi2[0, ::2] = -hi[0, ::2], -lo[0, ::2]
    (got, ref, s), = run_case(q, lo2, hi2, n * 16, 50)
    assert s.max() > 0 > s.min()
    assert set(got) <= set(range(0, n, 2))              # the positive scores are the negated pages


def test_group_maximum_and_several_heads():
    rng = np.random.default_rng(9)
    n, Hkv, G = 130, 3, 4
    lo = ints(rng, (Hkv, n, 128), -3, 0)
    hi = lo + ints(rng, (Hkv, n, 128), 0, 4)
    q = ints(rng, (Hkv * G, 128), -2, 2)
    res = run_case(q, lo, hi, n * 16 - 1, 20, Hq=Hkv * G, Hkv=Hkv)
    for h, (_, _, s) in enumerate(res):
        per_query = [oracle.page_scores(bf16(q[h * G + g:h * G + g + 1]), np.stack([bf16(lo[h]), bf16(hi[h])], axis=1))
                     for g in range(G)]
        np.testing.assert_array_equal(s, np.max(per_query, axis=0))


@pytest.mark.parametrize("n,K,distinct,outlier", [(3000, 500, 400, 99840.0), (8000, 700, 512, 99840.0), (2000, 150, 200, 30000.0),
                                                  (6000, 3000, 512, -99840.0), (1900, 37, 60, 3.0e38)])
def test_outliers_crowd_the_scores_into_a_few_bins(n, K, distinct, outlier):
    """Integer scores 0..distinct-1 (each shared by several pages: exact ties) plus a handful of far outliers: the
    linear bins between minimum and maximum then hold dozens of distinct values each, so the bin with the K-th
    largest score is crowded (ranked through LDS, or refined again when it holds more than 512 candidates), and
    the ties inside it must still go to the lower page indices."""
    rng = np.random.default_rng(n + K)
    val = rng.integers(0, distinct, size=n)
    row = np.zeros((1, n, 128), dtype=np.float32)
    row[0, :, 0] = val % 256                     # exact in bf16
    row[0, :, 1] = (val // 256) * 256
    far = rng.choice(n, size=7, replace=False)
    row[0, far, 2] = outlier
    q = np.zeros((4, 128), dtype=np.float32)
    q[:, :3] = 1.0
    for ctx in (n * 16, n * 16 - 3):
        (got, ref, s), = run_case(q, row, row, ctx, K)
        assert len(np.unique(s)) >= min(distinct, 50)


@pytest.mark.parametrize("seed", range(12))
def test_more_tied_candidates_than_threads(seed):
    """Up to 2048 pages the selection runs on 256 threads; with four or five distinct scores the bin that holds the
    K-th largest has 300-512 equal candidates, more than one per thread, gathered in an order that differs from run
    to run: whichever slot the boundary candidate lands in, the threshold and the tie count must come out right."""
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(1300, 2049))
    levels = int(rng.integers(4, 6))
    K = int(rng.integers(20, n - 20))
    protos_lo = ints(rng, (levels, 128), -3, 0)
    protos_hi = protos_lo + ints(rng, (levels, 128), 0, 3)
    which = rng.integers(0, levels, size=n)
    q = ints(rng, (4, 128), -2, 2)
    run_case(q, protos_lo[which][None], protos_hi[which][None], n * 16 - int(rng.integers(0, 2)) * 7, K)
