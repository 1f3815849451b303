"""Decode-loop harness over the C ABI: static placement of one workload's pages (what the paper's
block allocator would have produced after prefill and offload, Sec. 3.3), then per step
rerank -> promote -> attend.  Memory plumbing and call sequencing only; every computation is a
library call."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import binding
from .synth import DecodeConfig, Workload

PAGE_ELEMS = 2 * 16 * 128


def plan_placement(cfg: DecodeConfig, block_order: np.ndarray):
    """Host-side static placement.

    Unstable heads get one HBM block per page; a stable head of sequence b gets min(K_b, pages) HBM
    blocks (its slots, all free at the start) and one host block per page.  Returns
    (block_table [B,Hkv,Nmax], host_block_table, free_blocks [B,Hkv,Kmax], free_count [B,Hkv],
    num_pool_blocks, num_host_blocks).  Block 0 of either pool is never handed out."""
    B, H, Nmax, Kmax = cfg.batch, cfg.num_kv_heads, cfg.max_pages, list_capacity(cfg)
    bt = np.zeros((B, H, Nmax), dtype=np.int32)
    hbt = np.zeros((B, H, Nmax), dtype=np.int32)
    fb = np.zeros((B, H, Kmax), dtype=np.int32)
    fc = np.zeros((B, H), dtype=np.int32)
    nxt, hnxt = 0, 1
    for b in range(B):
        n, nf = cfg.num_pages(b), cfg.final_pages(b)
        grow = nf - n                      # pages that will be started by appended tokens
        for h in range(H):
            if cfg.stable[h]:
                k = min(cfg.topk[b], n) + grow
                fb[b, h, :k] = block_order[nxt:nxt + k]
                fc[b, h] = k
                nxt += k
                hbt[b, h, :nf] = np.arange(hnxt, hnxt + nf)
                hnxt += nf
            else:
                bt[b, h, :n] = block_order[nxt:nxt + n]
                nxt += n
                fb[b, h, :grow] = block_order[nxt:nxt + grow]
                fc[b, h] = grow
                nxt += grow
    return bt, hbt, fb, fc, nxt + 1, hnxt


def list_capacity(cfg: DecodeConfig) -> int:
    """Kmax: entries of a page list / free list: the budget plus the pages appended tokens can start
    between two reranks (they join the resident list at once and leave it at the next rerank)."""
    cur = max(cfg.num_pages(b) for b in range(cfg.batch))
    return min(min(cfg.max_topk, cur) + cfg.growth_pages + (1 if cfg.append_tokens else 0), cfg.max_pages)


def pool_blocks_needed(cfg: DecodeConfig) -> int:
    tot = 0
    for b in range(cfg.batch):
        n, grow = cfg.num_pages(b), cfg.final_pages(b) - cfg.num_pages(b)
        for h in range(cfg.num_kv_heads):
            tot += (min(cfg.topk[b], n) if cfg.stable[h] else n) + grow
    return tot


class DecodeSession:
    def __init__(self, cfg: DecodeConfig, wl: Workload, *, device: int = 0, attn_waves: int = 0,
                 promote_mode: int = binding.FC_PROMOTE_GATHER, keep_scores: bool = False,
                 unstable_topk: bool = False, softmax_scale: float = 0.0):
        import torch
        self.torch = torch
        self.cfg, self.wl = cfg, wl
        self.dev = torch.device("cuda", device)
        self.promote_mode = promote_mode
        # the paper's own treatment of unstable heads (Sec. 3.1, 3.2): rescored every step, top-K attention,
        # all pages resident; their lists are written straight into the resident arrays (nothing to promote)
        self.unstable_topk = unstable_topk
        B, H, Nmax, Kmax = cfg.batch, cfg.num_kv_heads, cfg.max_pages, list_capacity(cfg)
        self.ctx = binding.Context(num_q_heads=cfg.num_q_heads, num_kv_heads=H, max_batch=B,
                                   max_pages_per_seq=Nmax, max_topk=Kmax, device=device, attn_waves=attn_waves,
                                   softmax_scale=softmax_scale)
        order = wl.block_permutation(pool_blocks_needed(cfg))
        bt, hbt, fb, fc, nblk, nhost = plan_placement(cfg, order)
        self.num_pool_blocks, self.num_host_blocks = int(nblk), int(max(nhost, 2))
        i32 = dict(dtype=torch.int32, device=self.dev)
        self.kv_pool = torch.zeros((self.num_pool_blocks, PAGE_ELEMS), dtype=torch.bfloat16, device=self.dev)
        self.kv_pool[0].fill_(float("nan"))      # the null block must never influence a result
        self.host_pool = torch.zeros((self.num_host_blocks, PAGE_ELEMS), dtype=torch.bfloat16, pin_memory=True)
        self.block_table = torch.from_numpy(bt).to(self.dev)
        self.host_block_table = torch.from_numpy(hbt).to(self.dev)
        self.free_blocks = torch.from_numpy(fb).to(self.dev)
        self.free_count = torch.from_numpy(fc).to(self.dev)
        self._bt0, self._hbt = bt, hbt
        self.context_lens = torch.tensor(cfg.ctx, **i32)
        self.k_per_seq = torch.tensor([min(k, Kmax) for k in cfg.topk], **i32)
        self.minmax = torch.zeros((B, H, Nmax, 2, 128), dtype=torch.bfloat16, device=self.dev)
        self.topk_pages = torch.full((B, H, Kmax), -1, **i32)
        self.topk_count = torch.zeros((B, H), **i32)
        self.resident_pages = torch.full((B, H, Kmax), -1, **i32)
        self.resident_count = torch.zeros((B, H), **i32)
        self.promoted_count = torch.zeros((B, H), **i32)
        self.promoted_flags = torch.zeros((B, H, Kmax), dtype=torch.uint8, device=self.dev)
        self.total_promoted = torch.zeros(1, dtype=torch.int32, pin_memory=True)
        self.scores = torch.zeros((B, H, Nmax), dtype=torch.float32, device=self.dev) if keep_scores else None
        self.q = torch.zeros((B, cfg.num_q_heads, 128), dtype=torch.bfloat16, device=self.dev)
        self.out = torch.zeros((B, cfg.num_q_heads, 128), dtype=torch.float32, device=self.dev)
        self.lse = torch.zeros((B, cfg.num_q_heads), dtype=torch.float32, device=self.dev)
        self.main = torch.cuda.current_stream(self.dev)
        self.copy = torch.cuda.Stream(self.dev)            # second stream (default priority): page copies, or the attention that hides them
        # how a rerank step is run (see step()); splitting only pays when the attention is long enough to
        # hide something behind: below ~64 MB per pass the extra launches and the stream hand-overs cost more
        self.overlap = "ride" if cfg.pages_attended() * 8192 >= (64 << 20) else False
        if self.overlap == "ride" and promote_mode != binding.FC_PROMOTE_GATHER:
            self.overlap = "inline"        # per-page hipMemcpyAsync cannot ride in a kernel launch
        self.fused_rerank = True   # rerank + promote through fc_rerank_promote (one call) instead of the two calls
        self.events = None     # optional dict of torch events a benchmark wants recorded on a rerank step
        self.stable = list(cfg.stable)
        for b in range(B):
            self._write_sequence(b, None)
        torch.cuda.synchronize(self.dev)

    # ---- placement of page contents ---------------------------------------------------------------
    def bits_to_dev(self, a: np.ndarray):
        return self.torch.from_numpy(a.view(np.int16)).to(self.dev).view(self.torch.bfloat16)

    def _write_sequence(self, b: int, only: Optional[Dict[int, Sequence[int]]]):
        """(Re)writes pages of sequence b from the master copy: `only` = {head: pages} or None = all."""
        torch, cfg = self.torch, self.cfg
        cur = self.wl.cur_len[b]
        n = -(-cur // 16)
        kd = self.bits_to_dev(np.ascontiguousarray(self.wl.k[b][:, :n * 16]))
        vd = self.bits_to_dev(np.ascontiguousarray(self.wl.v[b][:, :n * 16]))
        sel = np.zeros((cfg.num_kv_heads, n), dtype=bool)
        if only is None:
            sel[:] = True
        else:
            for h, pages in only.items():
                sel[h, list(pages)] = True
        table_now = self._current_table(b)
        hbm_ids = np.where(sel, table_now[:, :n], 0).astype(np.int32)
        host_ids = np.where(sel, self._hbt[b][:, :n], 0).astype(np.int32)
        hbm_ids_d = torch.from_numpy(np.ascontiguousarray(hbm_ids)).to(self.dev)
        host_ids_d = torch.from_numpy(np.ascontiguousarray(host_ids)).to(self.dev)
        c = self.ctx
        c.fc_write_kv_pages(kd, vd, n, hbm_ids_d, self.kv_pool, self.num_pool_blocks, self.main)
        if any(self.stable):
            c.fc_write_kv_pages(kd, vd, n, host_ids_d, self.host_pool, self.num_host_blocks, self.main)
        # MinMax rows: from the HBM copy for unstable heads, from the host copy for stable heads
        if only is None:
            plist, nl = None, n
        else:
            pages = sorted({p for ps in only.values() for p in ps})
            plist, nl = torch.tensor(pages, dtype=torch.int32, device=self.dev), len(pages)
        unst = np.where(np.array(self.stable)[:, None], 0, table_now[:, :n]).astype(np.int32)
        c.fc_build_minmax(self.kv_pool, self.num_pool_blocks, torch.from_numpy(np.ascontiguousarray(unst)).to(self.dev),
                          plist, nl, cur, self.minmax[b], self.main)
        if any(self.stable):
            hst = torch.from_numpy(np.ascontiguousarray(self._hbt[b][:, :n])).to(self.dev)
            c.fc_build_minmax(self.host_pool, self.num_host_blocks, hst, plist, nl, cur, self.minmax[b],
                              self.main)
        torch.cuda.synchronize(self.dev)   # kd / vd die with this frame

    def _current_table(self, b: int) -> np.ndarray:
        return self.block_table[b].cpu().numpy()

    def refresh(self, changed: List[Tuple[int, int, List[int]]]):
        """Pushes master-copy changes (hot pages planted or retired) to every copy of those pages."""
        per_seq: Dict[int, Dict[int, List[int]]] = {}
        for b, h, pages in changed:
            per_seq.setdefault(b, {})[h] = pages
        for b, only in per_seq.items():
            self._write_sequence(b, only)

    # ---- the three hot-path calls -------------------------------------------------------------------
    def set_queries(self, q_bits: np.ndarray):
        self.q.copy_(self.bits_to_dev(q_bits))

    def append(self, k_bits: np.ndarray, v_bits: np.ndarray, append_mask=None):
        """One new token per sequence: page write, MinMax update, offload of pages that fill (library)."""
        kd, vd = self.bits_to_dev(k_bits), self.bits_to_dev(v_bits)
        self.append_dev(kd, vd, append_mask)
        self.torch.cuda.current_stream(self.dev).synchronize()   # kd / vd die with this frame

    def append_dev(self, kd, vd, append_mask=None):
        """Same, from bf16 device tensors [B, Hkv, D] the caller keeps alive."""
        self.ctx.fc_append_kv(k_new=kd, v_new=vd, context_lens=self.context_lens, block_table=self.block_table,
                              host_block_table=self.host_block_table, free_blocks=self.free_blocks,
                              free_count=self.free_count, resident_pages=self.resident_pages,
                              resident_count=self.resident_count, minmax=self.minmax, kv_pool=self.kv_pool,
                              num_pool_blocks=self.num_pool_blocks, host_pool=self.host_pool,
                              num_host_blocks=self.num_host_blocks, stable_flag=self.stable,
                              batch=self.cfg.batch, append_mask=append_mask, stream=self.main)

    def rerank(self, rerank_mask=None, stream=None):
        self.ctx.fc_rerank_topk(q=self.q, minmax=self.minmax, context_lens=self.context_lens,
                                stable_flag=self.stable, k_per_seq=self.k_per_seq, batch=self.cfg.batch,
                                topk_pages=self.topk_pages, topk_count=self.topk_count, rerank_mask=rerank_mask,
                                scores_out=self.scores, stream=stream or self.main)

    def rerank_unstable(self):
        """Paper variant: select the unstable heads' top-K for this step, directly into the lists the
        attention reads."""
        self.ctx.fc_rerank_topk(q=self.q, minmax=self.minmax, context_lens=self.context_lens,
                                stable_flag=[not s for s in self.stable], k_per_seq=self.k_per_seq,
                                batch=self.cfg.batch, topk_pages=self.resident_pages,
                                topk_count=self.resident_count, scores_out=self.scores, stream=self.main)

    def promote(self, rerank_mask=None, stream=None, copy_stream=None, mode=None):
        self.ctx.fc_promote_pages(new_pages=self.topk_pages, new_count=self.topk_count,
                                  resident_pages=self.resident_pages, resident_count=self.resident_count,
                                  block_table=self.block_table, host_block_table=self.host_block_table,
                                  free_blocks=self.free_blocks, free_count=self.free_count,
                                  stable_flag=self.stable, kv_pool=self.kv_pool,
                                  num_pool_blocks=self.num_pool_blocks, host_pool=self.host_pool,
                                  num_host_blocks=self.num_host_blocks, batch=self.cfg.batch,
                                  main_stream=stream or self.main, side_stream=copy_stream or self.copy,
                                  mode=self.promote_mode if mode is None else mode, rerank_mask=rerank_mask,
                                  promoted_count=self.promoted_count, promoted_flags=self.promoted_flags,
                                  total_promoted=self.total_promoted)

    def rerank_promote(self, rerank_mask=None, copy_stream=None, mode=None):
        """fc_rerank_topk + fc_promote_pages as the one call fc_rerank_promote."""
        self.ctx.fc_rerank_promote(q=self.q, minmax=self.minmax, context_lens=self.context_lens, stable_flag=self.stable,
                                   k_per_seq=self.k_per_seq, batch=self.cfg.batch, topk_pages=self.topk_pages,
                                   topk_count=self.topk_count, resident_pages=self.resident_pages,
                                   resident_count=self.resident_count, block_table=self.block_table,
                                   host_block_table=self.host_block_table, free_blocks=self.free_blocks,
                                   free_count=self.free_count, kv_pool=self.kv_pool, num_pool_blocks=self.num_pool_blocks,
                                   host_pool=self.host_pool, num_host_blocks=self.num_host_blocks, main_stream=self.main,
                                   side_stream=copy_stream or self.copy,
                                   mode=self.promote_mode if mode is None else mode, rerank_mask=rerank_mask,
                                   scores_out=self.scores, promoted_count=self.promoted_count,
                                   promoted_flags=self.promoted_flags, total_promoted=self.total_promoted)

    def attend(self, head_subset: int = binding.FC_HEADS_ALL, stream=None):
        listed = [True] * len(self.stable) if self.unstable_topk else self.stable
        self.ctx.fc_sparse_decode_attn(q=self.q, kv_pool=self.kv_pool, num_pool_blocks=self.num_pool_blocks,
                                       block_table=self.block_table, context_lens=self.context_lens,
                                       stable_flag=listed, topk_pages=self.resident_pages,
                                       topk_count=self.resident_count, batch=self.cfg.batch, out=self.out,
                                       lse=self.lse, head_subset=head_subset, promoted_flags=self.promoted_flags,
                                       stream=stream or self.main)

    def _rerank_and_promote(self, copy, pmode):
        """Score, select, recycle and the page copies (or, with FC_PROMOTE_RIDE, only their description)."""
        ev = self.events
        if self.fused_rerank and (ev is None or "chain_begin" in ev):
            if ev is not None:
                ev["chain_begin"].record(self.main)
            self.rerank_promote(copy_stream=copy, mode=pmode)
            if ev is not None:
                ev["chain_end"].record(self.main)
            return
        if ev is not None:
            ev["rerank_begin"].record(self.main)
        self.rerank()
        if ev is not None:
            ev["rerank_end"].record(self.main)
        self.promote(copy_stream=copy, mode=pmode)
        if ev is not None:
            ev["recycle_end"].record(self.main)
            if pmode != binding.FC_PROMOTE_RIDE:
                ev["copies_end"].record(copy)

    def _attend_pair(self, first: int, second: int, first_stream=None, carries_copies=False):
        """The two attention calls of a split pass; with riding copies the first launch carries them."""
        self.attend(first, stream=first_stream)
        if self.events is not None and carries_copies and "copies_end" in self.events:
            self.events["copies_end"].record(self.main)     # the launch that carried the copies has ended
        self.attend(second)

    def step(self, t: int):
        """One pass of the hot path for decode step t (queries already set on the main stream).

        On a rerank step scoring, selection and block recycling run first; `overlap` says how the page
        copies are hidden.  "ride" (default for all but tiny workloads) needs one stream and no event:
        promotion leaves the copies to the next attention launch (FC_PROMOTE_RIDE), whose extra workgroups
        carry them beside the attention over everything already in HBM (all pages of unstable heads, the
        kept pages of stable heads); a second launch attends over the promoted pages and one merge closes
        the step.  "inline" runs the copies as a kernel of their own in line on the main stream and gives
        the resident-page attention to the second stream; True puts the copies on the second stream and
        keeps both attention calls on the main stream (the second waits, on the GPU, for the copies).
        "heads-ride" / "heads-inline" / "heads" are the same three with the split by head class instead of
        by page ("heads-inline" starts the unstable heads before the rerank); False does not split."""
        mode = self.overlap
        inline = mode in ("inline", "heads-inline")
        ride = mode in ("ride", "heads-ride") and self.promote_mode == binding.FC_PROMOTE_GATHER
        pmode = binding.FC_PROMOTE_RIDE if ride else None
        copy = self.main if inline or ride or not mode else self.copy
        rerank_now = self.cfg.is_rerank_step(t) and any(self.stable)
        RES, PRO, UNS, STA = (binding.FC_PAGES_RESIDENT, binding.FC_PAGES_PROMOTED, binding.FC_HEADS_UNSTABLE,
                              binding.FC_HEADS_STABLE)
        if self.unstable_topk:
            # the paper's variant: every head is list-driven, the unstable ones rescored at every step; a split can
            # only be by page (list entries of unstable heads are never flagged as promoted)
            if not all(self.stable):
                self.rerank_unstable()
            if rerank_now:
                self._rerank_and_promote(copy, pmode)
                if ride:
                    self._attend_pair(RES, PRO, carries_copies=True)
                    return
            self.attend()
            return
        if not rerank_now:
            self.attend()
            return
        by_head = mode in ("heads", "heads-inline", "heads-ride") and not all(self.stable)
        if mode == "heads-inline" and by_head:
            # nothing the unstable heads read is touched by the rerank: start them at once, beside it
            self.copy.wait_stream(self.main)
            self.attend(UNS, stream=self.copy)
            self._rerank_and_promote(copy, pmode)
            self.attend(STA)
            return
        self._rerank_and_promote(copy, pmode)
        if not mode:
            self.attend()
        elif by_head:
            self._attend_pair(UNS, STA, carries_copies=ride)
        else:
            self._attend_pair(RES, PRO, first_stream=self.copy if inline else None, carries_copies=ride)

    def selected(self) -> Dict[Tuple[int, int], np.ndarray]:
        pages = self.resident_pages.cpu().numpy()
        cnt = self.resident_count.cpu().numpy()
        return {(b, h): pages[b, h, :cnt[b, h]].copy() for b in range(self.cfg.batch)
                for h in range(self.cfg.num_kv_heads) if self.stable[h]}

    def close(self):
        self.torch.cuda.synchronize(self.dev)
        self.ctx.close()
