"""Seeded synthetic decode workloads.

This module only *draws inputs*: bf16 keys, values and queries, context lengths, stability flags,
per-sequence page budgets and the schedule of planted "hot" pages.  It contains none of the method's
arithmetic (no page scores, no selection, no attention, no MinMax vectors, no page layouts), so both
the HIP path and the CPU oracle may be fed from it without sharing any computation.

The inputs stand in for the long-context, long-generation serving workloads the paper evaluates
(Sec. 4.4: prompts of 10k-30k tokens, generations of up to 2000 tokens, Llama-3-8B-like 32 query / 8
KV heads, 16-token pages).  Only the shapes are taken from there; every value is drawn here.

Recipe
------
* ``K, V ~ N(0, 1)`` per element, drawn in fp32 and rounded once (nearest-even) to bf16.
* Each KV head ``h`` has a fixed direction ``d_h = 4 u_h`` with ``u_h`` uniform on the unit sphere.
  All query heads of the group use it: ``q = d_h + N(0, 0.1^2)`` per element per step, then bf16.
* Every valid key of a hot page gets ``k += 3 d_h`` (added to its bf16 value, rounded to bf16 again);
  retiring a hot page restores the saved original bits, it never subtracts.
* One child random stream per (purpose, sequence, head, step), so generation is order independent.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

SEED_BASE = 0x46C30000
DIR_NORM = 4.0
HOT_SHIFT = 3.0
Q_NOISE = 0.1


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class DecodeConfig:
    """Shape and schedule of one synthetic decode run (one attention layer)."""

    name: str
    index: int                 # which of the five benchmark configurations this derives from
    batch: int
    num_q_heads: int
    num_kv_heads: int
    ctx: Tuple[int, ...]       # context length per sequence (tokens)
    stable: Tuple[bool, ...]   # per KV head
    topk: Tuple[int, ...]      # page budget K per sequence
    steps: int
    rerank_interval: int
    hot_per_head: int          # planted hot pages per (sequence, head)
    dynamics: str              # "static" | "unstable_resample" | "drift" | "plant_nonresident"
    dynamics_pages: int = 0    # pages changed per event for drift / plant_nonresident
    shuffle_blocks: bool = False
    append_tokens: int = 0     # tokens appended to every sequence during the run (one per step), 0 = fixed context
    head_dim: int = 128
    page_size: int = 16
    seed: int = 0

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    def num_pages(self, b: int) -> int:
        return -(-self.ctx[b] // self.page_size)

    def final_pages(self, b: int) -> int:
        """Pages of sequence b once every appended token is in."""
        return -(-(self.ctx[b] + self.append_tokens) // self.page_size)

    @property
    def max_pages(self) -> int:
        return max(self.final_pages(b) for b in range(self.batch))

    @property
    def growth_pages(self) -> int:
        return max(self.final_pages(b) - self.num_pages(b) for b in range(self.batch))

    @property
    def max_topk(self) -> int:
        return max(self.topk)

    def pages_attended(self) -> int:
        """Pages one decode step attends over (all sequences, all KV heads)."""
        tot = 0
        for b in range(self.batch):
            n = self.num_pages(b)
            for h in range(self.num_kv_heads):
                tot += min(self.topk[b], n) if self.stable[h] else n
        return tot

    def is_rerank_step(self, t: int) -> bool:
        return t % self.rerank_interval == 0


def _seed(index: int, stream: int) -> int:
    return SEED_BASE + 1000 * index + stream


def make_config(index: int, *, batch: int | None = None, ctx: int | None = None,
                steps: int | None = None, name: str | None = None) -> DecodeConfig:
    """The five benchmark configurations; ``batch`` / ``ctx`` / ``steps`` shrink them for parity tests
    without changing their structure (head mix, budget fraction, dynamics)."""
    if index == 1:
        B, Hq, Hkv, T = batch or 1, 8, 2, ctx or 2048
        return DecodeConfig(name or "cfg1_tiny", 1, B, Hq, Hkv, (T,) * B, (True, False), (8,) * B,
                            steps or 4, 2, 4, "static", seed=_seed(1, 0))
    if index == 2:
        B, T = batch or 8, ctx or 32768
        n = -(-T // 16)
        K = max(1, (n * 204) // 2048)
        return DecodeConfig(name or "cfg2_llama8b_32k", 2, B, 32, 8, (T,) * B,
                            (True,) * 4 + (False,) * 4, (K,) * B, steps or 16, 4, max(1, K // 4),
                            "unstable_resample", seed=_seed(2, 0))
    if index == 3:
        B, T = batch or 4, ctx or 131072
        n = -(-T // 16)
        K = max(1, min(256, n // 32))
        return DecodeConfig(name or "cfg3_long_128k", 3, B, 32, 8, (T,) * B,
                            (True,) * 6 + (False,) * 2, (K,) * B, steps or 32, 8, max(1, K // 4),
                            "drift", 2, seed=_seed(3, 0))
    if index == 4:
        B = batch or 64
        lo, hi = (4096, 32768) if ctx is None else (max(17, ctx // 8), ctx)
        rng = np.random.default_rng(_seed(4, 1))
        lens = tuple(int(x) for x in rng.integers(lo, hi + 1, size=B))
        flags = tuple(bool(x) for x in (rng.random(8) < 0.5))
        if all(flags) or not any(flags):   # keep both kinds of head present
            flags = (True,) * 4 + (False,) * 4
        K = tuple(max(1, (-(-l // 16)) // 8) for l in lens)
        return DecodeConfig(name or "cfg4_ragged_b64", 4, B, 32, 8, lens, flags, K, steps or 8, 4,
                            0, "static", shuffle_blocks=True, seed=_seed(4, 0))
    if index == 5:
        B, T = batch or 16, ctx or 65536
        n = -(-T // 16)
        K = max(1, min(256, n // 16))
        return DecodeConfig(name or "cfg5_offload_64k", 5, B, 32, 8, (T,) * B,
                            (True,) * 5 + (False,) * 3, (K,) * B, steps or 64, 4, max(1, K // 4),
                            "plant_nonresident", min(8, max(1, K // 4)), seed=_seed(5, 0))
    raise ValueError(f"no such configuration: {index}")


def hot_per_head_for(cfg: DecodeConfig, b: int) -> int:
    """Config 4 scales its hot-page count with each sequence's own budget."""
    if cfg.index == 4:
        return max(1, cfg.topk[b] // 4)
    return cfg.hot_per_head


class Workload:
    """Master copy of one run's inputs, token-major and unpaged.

    ``k[b]`` and ``v[b]`` are uint16 (bf16 bit patterns) arrays of shape ``[Hkv, Tpad_b, D]`` where
    ``Tpad_b`` is ``ctx[b]`` rounded up to whole pages; tokens at or beyond ``ctx[b]`` hold a NaN
    pattern so that any consumer that fails to mask them is caught.
    """

    PAD_BITS = 0x7FC0  # bf16 quiet NaN

    def __init__(self, cfg: DecodeConfig):
        self.cfg = cfg
        D, P = cfg.head_dim, cfg.page_size
        self.dirs = np.empty((cfg.num_kv_heads, D), dtype=np.float32)
        for h in range(cfg.num_kv_heads):
            g = np.random.default_rng([cfg.seed, 10, h])
            u = g.standard_normal(D)
            self.dirs[h] = (DIR_NORM * u / np.linalg.norm(u)).astype(np.float32)
        self.k: List[np.ndarray] = []
        self.v: List[np.ndarray] = []
        self.hot: Dict[Tuple[int, int], List[int]] = {}
        self._pristine: Dict[Tuple[int, int, int], np.ndarray] = {}
        def draw(args):
            b, h, kb, vb, tpad = args
            g = np.random.default_rng([cfg.seed, 11, b, h])
            kb[h] = f32_to_bf16_bits(g.standard_normal((tpad, D), dtype=np.float32))
            vb[h] = f32_to_bf16_bits(g.standard_normal((tpad, D), dtype=np.float32))

        self.cur_len = list(cfg.ctx)     # grows with append()
        jobs = []
        for b in range(cfg.batch):
            tpad = cfg.final_pages(b) * P
            kb = np.empty((cfg.num_kv_heads, tpad, D), dtype=np.uint16)
            vb = np.empty((cfg.num_kv_heads, tpad, D), dtype=np.uint16)
            self.k.append(kb)
            self.v.append(vb)
            jobs += [(b, h, kb, vb, tpad) for h in range(cfg.num_kv_heads)]
        # one independent stream per (sequence, head): the order of drawing does not matter
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(draw, jobs))
        for b in range(cfg.batch):
            n = cfg.num_pages(b)
            tpad = cfg.final_pages(b) * P
            kb, vb = self.k[b], self.v[b]
            if cfg.ctx[b] < tpad:
                kb[:, cfg.ctx[b]:, :] = self.PAD_BITS
                vb[:, cfg.ctx[b]:, :] = self.PAD_BITS
            nh = hot_per_head_for(cfg, b)
            for h in range(cfg.num_kv_heads):
                g = np.random.default_rng([cfg.seed, 12, b, h])
                pages = sorted(int(x) for x in g.choice(n, size=min(nh, n), replace=False))
                self.hot[(b, h)] = []
                self._plant(b, h, pages)

    # ---- hot pages -----------------------------------------------------------------------------
    def _page_slice(self, b: int, p: int) -> slice:
        P = self.cfg.page_size
        return slice(p * P, min((p + 1) * P, self.cur_len[b]))

    def _plant(self, b: int, h: int, pages: Sequence[int]) -> None:
        for p in pages:
            if p in self.hot[(b, h)]:
                continue
            sl = self._page_slice(b, p)
            self._pristine[(b, h, p)] = self.k[b][h, sl].copy()
            base = bf16_bits_to_f32(self.k[b][h, sl])
            self.k[b][h, sl] = f32_to_bf16_bits(base + HOT_SHIFT * self.dirs[h][None, :])
            self.hot[(b, h)].append(p)

    def _retire(self, b: int, h: int, pages: Sequence[int]) -> None:
        for p in pages:
            sl = self._page_slice(b, p)
            self.k[b][h, sl] = self._pristine.pop((b, h, p))
            self.hot[(b, h)].remove(p)

    def advance(self, t: int, resident: Dict[Tuple[int, int], Sequence[int]] | None = None
                ) -> List[Tuple[int, int, List[int]]]:
        """Apply the configuration's hot-page dynamics that precede decode step ``t`` (t >= 1).

        Returns ``[(b, h, pages)]``: pages whose keys changed in the master copy and must be rewritten
        wherever a copy of them lives.  ``resident`` (pages currently selected per stable (b, h)) is
        needed only by "plant_nonresident".
        """
        cfg = self.cfg
        changed: List[Tuple[int, int, List[int]]] = []
        if t <= 0 or cfg.dynamics == "static":
            return changed
        for b in range(cfg.batch):
            n = -(-self.cur_len[b] // cfg.page_size)
            for h in range(cfg.num_kv_heads):
                g = np.random.default_rng([cfg.seed, 13, b, h, t])
                cur = self.hot[(b, h)]
                if cfg.dynamics == "unstable_resample":
                    if cfg.stable[h]:
                        continue
                    old = list(cur)
                    new = sorted(int(x) for x in g.choice(n, size=len(old), replace=False))
                    self._retire(b, h, old)
                    self._plant(b, h, new)
                    changed.append((b, h, sorted(set(old) | set(new))))
                elif cfg.dynamics in ("drift", "plant_nonresident"):
                    if not cfg.stable[h] or not cfg.is_rerank_step(t):
                        continue
                    m = min(cfg.dynamics_pages, len(cur))
                    old = list(cur[:m])                      # the oldest planted pages retire
                    banned = set(cur)
                    if cfg.dynamics == "plant_nonresident" and resident is not None:
                        banned |= set(int(x) for x in resident.get((b, h), ()))
                    cand = np.array([p for p in range(n) if p not in banned], dtype=np.int64)
                    new = sorted(int(x) for x in g.choice(cand, size=min(m, len(cand)), replace=False))
                    self._retire(b, h, old)
                    self._plant(b, h, new)
                    changed.append((b, h, sorted(set(old) | set(new))))
        return changed

    # ---- appended tokens -----------------------------------------------------------------------
    def append(self, t: int) -> Tuple[np.ndarray, np.ndarray]:
        """Draws the token every sequence appends before decode step t, stores it in the master copy
        and returns its (k, v) bit patterns, each [B, Hkv, D]."""
        cfg = self.cfg
        k = np.empty((cfg.batch, cfg.num_kv_heads, cfg.head_dim), dtype=np.uint16)
        v = np.empty_like(k)
        for b in range(cfg.batch):
            g = np.random.default_rng([cfg.seed, 16, b, t])
            k[b] = f32_to_bf16_bits(g.standard_normal((cfg.num_kv_heads, cfg.head_dim), dtype=np.float32))
            v[b] = f32_to_bf16_bits(g.standard_normal((cfg.num_kv_heads, cfg.head_dim), dtype=np.float32))
            pos = self.cur_len[b]
            assert pos < self.k[b].shape[1], "more tokens appended than the configuration announced"
            self.k[b][:, pos, :] = k[b]
            self.v[b][:, pos, :] = v[b]
            self.cur_len[b] = pos + 1
        return k, v

    # ---- queries -------------------------------------------------------------------------------
    def queries(self, t: int) -> np.ndarray:
        """bf16 bit patterns ``[B, Hq, D]`` of the step-``t`` queries."""
        cfg = self.cfg
        q = np.empty((cfg.batch, cfg.num_q_heads, cfg.head_dim), dtype=np.uint16)
        G = cfg.group
        for b in range(cfg.batch):
            g = np.random.default_rng([cfg.seed, 14, b, t])
            noise = g.standard_normal((cfg.num_q_heads, cfg.head_dim), dtype=np.float32) * np.float32(Q_NOISE)
            for hq in range(cfg.num_q_heads):
                q[b, hq] = f32_to_bf16_bits(self.dirs[hq // G] + noise[hq])
        return q

    def block_permutation(self, num_blocks: int) -> np.ndarray:
        """Order in which physical blocks 1..num_blocks are handed out (block 0 is never handed out)."""
        ids = np.arange(1, num_blocks + 1, dtype=np.int64)
        if self.cfg.shuffle_blocks:
            np.random.default_rng([self.cfg.seed, 15]).shuffle(ids)
        return ids
