"""Shared driver of the GPU parity tests: runs the HIP path and the CPU oracle side by side on one
seeded workload and compares them (attention within 2e-3 of the row's largest magnitude, top-K sets
exactly except audited near-ties, block tables and page contents bit for bit)."""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import numpy as np

import oracle
from paper_2511_00868_amd import binding, synth
from paper_2511_00868_amd.session import DecodeSession

ATTN_TOL = 2e-3          # max |gpu - ref| / max |ref| per (sequence, query head)
ATTN_ELEM_ATOL = 1e-4    # element by element: |gpu - ref| <= ATTN_TOL * |ref| + ATTN_ELEM_ATOL * max |ref| of the row
TIE_TOL = 1e-5           # relative score gap below which a top-K swap is a legal near-tie
SCORE_TOL = 2e-5         # fp32 accumulation of 256 exact products vs fp64


def widen(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def native_page(k_page: np.ndarray, v_page: np.ndarray) -> np.ndarray:
    """The documented block layout, restated: K half = four chunks of 32 dims, [chunk][token][32];
    V half dim-major [128][16]."""
    return np.concatenate([k_page.reshape(16, 4, 32).transpose(1, 0, 2).reshape(-1), v_page.T.reshape(-1)])


def audit_sets(gpu_set, ora_set, scores, forced: int) -> None:
    g, o = set(int(x) for x in gpu_set), set(int(x) for x in ora_set)
    assert len(g) == len(gpu_set) == len(ora_set), "duplicate or missing pages in the GPU selection"
    if g == o:
        return
    kth = min(scores[p] for p in o if p != forced)
    for p in g ^ o:
        assert p != forced, "the partially filled last page must always be selected"
        gap = abs(scores[p] - kth) / max(abs(scores[p]), abs(kth))
        assert gap < TIE_TOL, f"page {p}: score {scores[p]!r} vs boundary {kth!r} is not a near-tie (gap {gap:.3e})"


def check_attention(out_gpu: np.ndarray, out_ref: np.ndarray, what: str) -> float:
    worst = 0.0
    for idx in np.ndindex(out_ref.shape[:-1]):
        ref, got = out_ref[idx], out_gpu[idx]
        assert np.all(np.isfinite(got)), f"{what}{idx}: non-finite output"
        scale = np.abs(ref).max()
        err = np.abs(got - ref).max() / scale
        worst = max(worst, err)
        assert err <= ATTN_TOL, f"{what}{idx}: relative error {err:.3e} > {ATTN_TOL}"
        # the row-wise figure alone would let small components be wrong by far more than 2e-3 of themselves
        slack = ATTN_TOL * np.abs(ref) + ATTN_ELEM_ATOL * scale
        bad = np.abs(got - ref) > slack
        assert not bad.any(), f"{what}{idx}: element {int(np.argmax(bad))} off by {np.abs(got - ref)[bad].max():.3e}"
    return worst


class ParityRun:
    def __init__(self, cfg: synth.DecodeConfig, *, promote_mode=binding.FC_PROMOTE_GATHER, attn_waves=0,
                 sample_rows: Optional[int] = None, seed: int = 0, unstable_topk: bool = False, overlap="ride",
                 fused_rerank: bool = True):
        self.cfg = cfg
        self.wl = synth.Workload(cfg)
        self.sess = DecodeSession(cfg, self.wl, promote_mode=promote_mode, attn_waves=attn_waves, keep_scores=True,
                                  unstable_topk=unstable_topk)
        self.unstable_topk = unstable_topk
        self.sess.overlap = overlap
        self.sess.fused_rerank = fused_rerank       # fc_rerank_promote, or fc_rerank_topk + fc_promote_pages
        self.dec = oracle.OracleDecoder(cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.ctx, cfg.stable,
                                        cfg.topk, cfg.rerank_interval, unstable_topk=unstable_topk)
        self.mm = [oracle.seq_build_minmax(self.wl.k[b], cfg.ctx[b]) for b in range(cfg.batch)]
        self.appended_pages = []          # (b, page) pages started by appended tokens
        # oracle-side block bookkeeping, from the same initial placement
        self.o_table = self.sess._bt0.copy()
        fb = self.sess.free_blocks.cpu().numpy()
        fc = self.sess.free_count.cpu().numpy()
        self.o_free = {(b, h): [int(x) for x in fb[b, h, :fc[b, h]]] for b in range(cfg.batch)
                       for h in range(cfg.num_kv_heads)}
        self.sample_rows = sample_rows
        self.rng = np.random.default_rng(seed)
        self.worst = 0.0
        self.near_tie_swaps = 0
        self.promoted_total = 0

    def pages_now(self, b: int) -> int:
        return -(-self.wl.cur_len[b] // 16)

    def check_minmax(self):
        mm_gpu = self.sess.minmax.cpu().view(self.sess.torch.int16).numpy().view(np.uint16)
        for b in range(self.cfg.batch):
            n = self.pages_now(b)
            np.testing.assert_array_equal(widen(mm_gpu[b, :, :n]), widen(self.mm[b]))

    def append_token(self, t: int):
        """Both sides append the token of step t; tables, free lists, MinMax rows, page bytes and the
        host copy of pages that just filled are compared."""
        cfg, wl, sess, dec = self.cfg, self.wl, self.sess, self.dec
        k, v = wl.append(t)
        sess.append(k, v)
        sess.torch.cuda.synchronize()
        sess.ctx.fc_check_device_state()
        filled = []
        for b in range(cfg.batch):
            page = dec.append(b)
            if page is not None:
                for h in range(cfg.num_kv_heads):
                    self.o_table[b, h, page] = self.o_free[(b, h)].pop()      # the last block of the free list
                self.appended_pages.append((b, page))
            if wl.cur_len[b] % 16 == 0:
                filled.append((b, wl.cur_len[b] // 16 - 1))
            self.mm[b] = oracle.seq_build_minmax(wl.k[b], wl.cur_len[b])
        assert sess.context_lens.cpu().tolist() == wl.cur_len == dec.ctx
        np.testing.assert_array_equal(sess.block_table.cpu().numpy(), self.o_table)
        fb, fc = sess.free_blocks.cpu().numpy(), sess.free_count.cpu().numpy()
        for (b, h), fl in self.o_free.items():
            assert fc[b, h] == len(fl) and list(fb[b, h, :len(fl)]) == fl
        sel = sess.selected()
        for (b, h), pages in sel.items():
            np.testing.assert_array_equal(pages, dec.sel[(b, h)])
        self.check_minmax()
        # the page being appended to: valid tokens bit for bit, in every head's HBM block
        i16 = sess.torch.int16
        for b in range(cfg.batch):
            p = (wl.cur_len[b] - 1) // 16
            ntok = wl.cur_len[b] - 16 * p
            blocks = sess.torch.tensor(self.o_table[b, :, p].astype(np.int64), device=sess.kv_pool.device)
            got = sess.kv_pool[blocks].cpu().view(i16).numpy().view(np.uint16)
            for h in range(cfg.num_kv_heads):
                kp, vp = wl.k[b][h, 16 * p:16 * p + 16], wl.v[b][h, 16 * p:16 * p + 16]
                np.testing.assert_array_equal(got[h][:2048].reshape(4, 16, 32)[:, :ntok], kp.reshape(16, 4, 32).transpose(1, 0, 2)[:, :ntok])
                np.testing.assert_array_equal(got[h][2048:].reshape(128, 16)[:, :ntok], vp.T[:, :ntok])
        # pages that just filled: the stable heads' host copy holds exactly that page
        host = sess.host_pool.view(i16).numpy().view(np.uint16)
        for b, p in filled:
            for h in range(cfg.num_kv_heads):
                if cfg.stable[h]:
                    hb = sess._hbt[b, h, p]
                    exp = native_page(wl.k[b][h, 16 * p:16 * p + 16], wl.v[b][h, 16 * p:16 * p + 16])
                    np.testing.assert_array_equal(host[hb], exp)

    def step(self, t: int, check_pool: bool = True):
        cfg, wl, sess, dec = self.cfg, self.wl, self.sess, self.dec
        # appends start after step 0: the harness begins with nothing of a stable head resident (the first
        # rerank is a cold fill), whereas after a real prefill the partial last page would already be in HBM
        if cfg.append_tokens and 1 <= t <= cfg.append_tokens:
            self.append_token(t)
        if t > 0:
            changed = wl.advance(t, sess.selected() if cfg.dynamics == "plant_nonresident" else None)
            if changed:
                sess.refresh(changed)
                for b in sorted({c[0] for c in changed}):
                    self.mm[b] = oracle.seq_build_minmax(wl.k[b], wl.cur_len[b])
        q = wl.queries(t)
        sess.set_queries(q)
        sess.step(t)
        sess.torch.cuda.synchronize()
        sess.ctx.fc_check_device_state()
        rer = cfg.is_rerank_step(t) and any(cfg.stable)
        gpu_sel = sess.selected()
        if self.unstable_topk and not all(cfg.stable):
            self.check_unstable_selection(q)
        if rer:
            scores_gpu = sess.scores.cpu().numpy()
            bt_gpu = sess.block_table.cpu().numpy()
            promoted_gpu = sess.promoted_count.cpu().numpy()
            step_promoted = 0
            for b in range(cfg.batch):
                n = self.pages_now(b)
                forced = n - 1 if wl.cur_len[b] % 16 else -1
                old = {h: dec.sel[(b, h)].copy() for h in range(cfg.num_kv_heads) if cfg.stable[h]}
                dec.rerank(b, q[b], self.mm[b])
                for h in range(cfg.num_kv_heads):
                    if not cfg.stable[h]:
                        continue
                    s64 = dec.last_scores[(b, h)]
                    np.testing.assert_allclose(scores_gpu[b, h, :n], s64, rtol=SCORE_TOL, atol=1e-4)
                    g = gpu_sel[(b, h)]
                    assert np.all(np.diff(g) > 0), "GPU list must be strictly ascending"
                    audit_sets(g, dec.sel[(b, h)], s64, forced)
                    if set(g) != set(dec.sel[(b, h)]):
                        self.near_tie_swaps += 1
                        dec.sel[(b, h)] = np.array(sorted(g), dtype=np.int32)   # follow the legal swap
                    # recycling: the oracle books the GPU's (audited) set with the same deterministic rule
                    copies, self.o_free[(b, h)] = oracle.recycle(old[h], dec.sel[(b, h)], self.o_table[b, h],
                                                                 self.sess._hbt[b, h], self.o_free[(b, h)])
                    assert promoted_gpu[b, h] == len(copies)
                    step_promoted += len(copies)
                    np.testing.assert_array_equal(bt_gpu[b, h], self.o_table[b, h])
            assert int(sess.total_promoted[0]) == step_promoted
            self.promoted_total += step_promoted
            fb = sess.free_blocks.cpu().numpy()
            fc = sess.free_count.cpu().numpy()
            for (b, h), fl in self.o_free.items():
                assert fc[b, h] == len(fl) and list(fb[b, h, :len(fl)]) == fl, (b, h, fl, fb[b, h, :fc[b, h]])
            if check_pool:
                self.check_resident_pages(bt_gpu)
        # attention, evaluated by the oracle on the (audited) selection
        out_gpu = sess.out.cpu().numpy().astype(np.float64)
        lse_gpu = sess.lse.cpu().numpy().astype(np.float64)
        rows = list(range(cfg.batch))
        if self.sample_rows is not None and self.sample_rows < cfg.batch:
            rows = sorted(self.rng.choice(cfg.batch, size=self.sample_rows, replace=False))
        for b in rows:
            ref, lse = dec.attend(b, q[b], wl.k[b], wl.v[b])
            self.worst = max(self.worst, check_attention(out_gpu[b], ref, f"step {t} seq {b} head "))
            np.testing.assert_allclose(lse_gpu[b], lse, rtol=0, atol=2e-3)

    def check_unstable_selection(self, q):
        """Paper variant: the unstable heads' every-step top-K against the oracle's (near-tie audited)."""
        cfg, sess, dec = self.cfg, self.sess, self.dec
        pages = sess.resident_pages.cpu().numpy()
        cnt = sess.resident_count.cpu().numpy()
        for b in range(cfg.batch):
            n = self.pages_now(b)
            forced = n - 1 if self.wl.cur_len[b] % 16 else -1
            dec.rerank_unstable(b, q[b], self.mm[b])
            for h in range(cfg.num_kv_heads):
                if cfg.stable[h]:
                    continue
                g = pages[b, h, :cnt[b, h]]
                assert np.all(np.diff(g) > 0)
                audit_sets(g, dec.sel[(b, h)], dec.last_scores[(b, h)], forced)
                if set(g) != set(dec.sel[(b, h)]):
                    self.near_tie_swaps += 1
                    dec.sel[(b, h)] = np.array(sorted(g), dtype=np.int32)

    def check_resident_pages(self, bt_gpu, max_pages: int = 200):
        """Every resident page of a stable head holds exactly the bytes of that page (native layout)."""
        cfg, wl = self.cfg, self.wl
        pool = self.sess.kv_pool
        todo = [(b, h, p) for (b, h), pages in self.sess.selected().items() for p in pages]
        if len(todo) > max_pages:
            idx = self.rng.choice(len(todo), size=max_pages, replace=False)
            todo = [todo[i] for i in idx]
        blocks = self.sess.torch.tensor([int(bt_gpu[b, h, p]) for b, h, p in todo], dtype=self.sess.torch.int64,
                                        device=pool.device)
        got = pool[blocks].cpu().view(self.sess.torch.int16).numpy().view(np.uint16)
        for i, (b, h, p) in enumerate(todo):
            assert bt_gpu[b, h, p] > 0
            ntok = min(16, wl.cur_len[b] - 16 * p)
            kp, vp = wl.k[b][h, 16 * p:16 * p + 16], wl.v[b][h, 16 * p:16 * p + 16]
            exp = native_page(kp, vp)
            if ntok == 16:
                np.testing.assert_array_equal(got[i], exp)
            else:      # the partially filled last page: every valid token of both halves
                np.testing.assert_array_equal(got[i][:2048].reshape(4, 16, 32)[:, :ntok], exp[:2048].reshape(4, 16, 32)[:, :ntok])
                np.testing.assert_array_equal(got[i][2048:].reshape(128, 16)[:, :ntok], exp[2048:].reshape(128, 16)[:, :ntok])

    def run(self, steps: Optional[int] = None):
        self.check_minmax()
        for t in range(steps or self.cfg.steps):
            self.step(t)
        print(f"[{self.cfg.name}] worst attention error {self.worst:.2e}, promoted {self.promoted_total}, "
              f"near-tie swaps {self.near_tie_swaps}")
        return self

    def close(self):
        self.sess.close()
