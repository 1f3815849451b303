"""CPU oracle of the FlexiCache decode hot path (test infrastructure; never imported by the product).

``fc_oracle.c`` holds the arithmetic; this wrapper compiles it with gcc, marshals numpy arrays into it
and strings its routines into the decode loop of the method:

    step t:  if t mod R == 0, every stable head rescors its pages and reselects its top-K (Sec. 3.2);
             promoted / evicted sets and block recycling are booked (Sec. 3.3, 3.4);
             every head attends over its page set -- S_t for stable heads, all pages otherwise.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fc_oracle.c")
_LIB = os.path.join(_HERE, "libfc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP only parallelises the loop over independent heads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u16p, i32p, f64p, u8p = (C.POINTER(C.c_uint16), C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                 C.POINTER(C.c_uint8))
        L.fco_build_minmax.argtypes = [u16p, C.c_int, C.c_int, C.c_int, u16p]
        L.fco_page_scores.argtypes = [u16p, C.c_int, u16p, C.c_int, C.c_int, C.c_int, f64p]
        L.fco_select_topk.argtypes = [f64p, C.c_int, C.c_int, C.c_int, C.c_int, i32p]
        L.fco_select_topk.restype = C.c_int
        L.fco_recycle.argtypes = [i32p, C.c_int, i32p, C.c_int, i32p, i32p, i32p, C.POINTER(C.c_int),
                                  C.c_int, i32p]
        L.fco_recycle.restype = C.c_int
        L.fco_attention.argtypes = [u16p, u16p, u16p, C.c_int, C.c_int, C.c_int, i32p, C.c_int,
                                    C.c_double, f64p, f64p, f64p]
        L.fco_seq_scores.argtypes = [u16p, C.c_int, C.c_int, u16p, C.c_int, C.c_int, u8p, C.c_int, f64p]
        L.fco_seq_build_minmax.argtypes = [u16p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, u16p]
        L.fco_seq_attention.argtypes = [u16p, u16p, u16p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.c_int, i32p, C.c_int, i32p, C.c_double, f64p, f64p]
        L.fco_threads.restype = C.c_int
        L.fco_set_threads.argtypes = [C.c_int]
        L.fco_rco.argtypes = [i32p, i32p, C.c_int, C.c_int]
        L.fco_rco.restype = C.c_double
        L.fco_stability.argtypes = [i32p, i32p, C.c_int, C.c_int, C.c_int, C.c_int, f64p]
        L.fco_bottom_counts.argtypes = [f64p, C.c_int, C.c_int, i32p]
        L.fco_classify.argtypes = [i32p, C.c_int, C.c_int, C.c_int, u8p]
        _lib = L
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16
    return a


def threads() -> int:
    return int(lib().fco_threads())


def set_threads(n: int) -> None:
    """Threads for the whole-sequence drivers (timing only: the results do not depend on it)."""
    lib().fco_set_threads(int(n))


# ---- single-head routines -----------------------------------------------------------------------
def build_minmax(k: np.ndarray, ctx: int, P: int = 16) -> np.ndarray:
    """k: uint16 [tokens, D] -> uint16 [n_pages, 2, D] (row 0 = min, row 1 = max)."""
    k = _u16(k)
    D = k.shape[-1]
    n = -(-ctx // P)
    mm = np.empty((n, 2, D), dtype=np.uint16)
    lib().fco_build_minmax(_p(k, C.c_uint16), ctx, D, P, _p(mm, C.c_uint16))
    return mm


def page_scores(q: np.ndarray, mm: np.ndarray, mode: int = 0) -> np.ndarray:
    """q: uint16 [G, D]; mm: uint16 [n, 2, D] -> float64 [n]."""
    q, mm = _u16(q), _u16(mm)
    G, D = q.shape
    n = mm.shape[0]
    s = np.empty(n, dtype=np.float64)
    lib().fco_page_scores(_p(q, C.c_uint16), G, _p(mm, C.c_uint16), n, D, mode, _p(s, C.c_double))
    return s


def select_topk(score: np.ndarray, ctx: int, K: int, P: int = 16) -> np.ndarray:
    """Ascending page ids of the selection (length = min(K, n))."""
    score = np.ascontiguousarray(score, dtype=np.float64)
    out = np.empty(max(K, 1), dtype=np.int32)
    cnt = lib().fco_select_topk(_p(score, C.c_double), len(score), ctx, P, K, _p(out, C.c_int32))
    return out[:cnt].copy()


def recycle(old_set, new_set, table: np.ndarray, host_table: np.ndarray, free_blocks: List[int]
            ) -> Tuple[np.ndarray, List[int]]:
    """Updates ``table`` in place; returns (copies [n, 2] = (host block, GPU block), new free list)."""
    old = np.ascontiguousarray(old_set, dtype=np.int32)
    new = np.ascontiguousarray(new_set, dtype=np.int32)
    assert table.dtype == np.int32 and table.flags.c_contiguous
    host_table = np.ascontiguousarray(host_table, dtype=np.int32)
    cap = len(free_blocks) + len(old) + 1
    fb = np.zeros(cap, dtype=np.int32)
    fb[:len(free_blocks)] = free_blocks
    nf = C.c_int(len(free_blocks))
    copies = np.empty((max(len(new), 1), 2), dtype=np.int32)
    n = lib().fco_recycle(_p(old, C.c_int32), len(old), _p(new, C.c_int32), len(new),
                          _p(table, C.c_int32), _p(host_table, C.c_int32), _p(fb, C.c_int32),
                          C.byref(nf), cap, _p(copies, C.c_int32))
    if n < 0:
        raise RuntimeError("head owns too few physical blocks for its new page set")
    return copies[:n].copy(), [int(x) for x in fb[:nf.value]]


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, ctx: int, pages, scale: float, P: int = 16
              ) -> Tuple[np.ndarray, float, float]:
    """q: uint16 [D]; k, v: uint16 [tokens, D] -> (out float64 [D], lse, sum of softmax weights)."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    D = q.shape[0]
    pages = np.ascontiguousarray(pages, dtype=np.int32)
    out = np.empty(D, dtype=np.float64)
    lse, ws = C.c_double(), C.c_double()
    lib().fco_attention(_p(q, C.c_uint16), _p(k, C.c_uint16), _p(v, C.c_uint16), ctx, D, P,
                        _p(pages, C.c_int32), len(pages), scale, _p(out, C.c_double), C.byref(lse),
                        C.byref(ws))
    return out, lse.value, ws.value


# ---- offline head-stability profiling (Sec. 2.2, 2.3) -------------------------------------------
def rco(a, b, n_t: int) -> float:
    a = np.ascontiguousarray(a, dtype=np.int32)
    b = np.ascontiguousarray(b, dtype=np.int32)
    assert len(a) == len(b)
    return float(lib().fco_rco(_p(a, C.c_int32), _p(b, C.c_int32), len(a), n_t))


def stability(traces: np.ndarray, num_pages, W: int) -> np.ndarray:
    """traces: int32 [steps, heads, K]; num_pages: [steps] -> float64 [steps - W + 1, heads]."""
    traces = np.ascontiguousarray(traces, dtype=np.int32)
    steps, heads, K = traces.shape
    npg = np.ascontiguousarray(num_pages, dtype=np.int32)
    ts = np.zeros((max(steps - W + 1, 0), heads), dtype=np.float64)
    if len(ts):
        lib().fco_stability(_p(traces, C.c_int32), _p(npg, C.c_int32), steps, heads, K, W, _p(ts, C.c_double))
    return ts


def bottom_counts(ts: np.ndarray, counts: Optional[np.ndarray] = None) -> np.ndarray:
    ts = np.ascontiguousarray(ts, dtype=np.float64)
    windows, heads = ts.shape
    out = np.zeros(heads, dtype=np.int32) if counts is None else np.ascontiguousarray(counts, dtype=np.int32).copy()
    lib().fco_bottom_counts(_p(ts, C.c_double), windows, heads, _p(out, C.c_int32))
    return out


def classify(counts, num: int = 1, den: int = 4) -> np.ndarray:
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    flags = np.zeros(len(counts), dtype=np.uint8)
    lib().fco_classify(_p(counts, C.c_int32), len(counts), num, den, _p(flags, C.c_uint8))
    return flags


# ---- whole-sequence routines --------------------------------------------------------------------
def seq_build_minmax(k: np.ndarray, ctx: int, P: int = 16) -> np.ndarray:
    """k: uint16 [Hkv, tpad, D] -> uint16 [Hkv, n, 2, D]."""
    k = _u16(k)
    Hkv, tpad, D = k.shape
    n = -(-ctx // P)
    mm = np.empty((Hkv, n, 2, D), dtype=np.uint16)
    lib().fco_seq_build_minmax(_p(k, C.c_uint16), Hkv, tpad, ctx, D, P, _p(mm, C.c_uint16))
    return mm


def seq_scores(q: np.ndarray, mm: np.ndarray, stable: Sequence[bool], mode: int = 0) -> np.ndarray:
    """q: uint16 [Hq, D]; mm: uint16 [Hkv, n, 2, D] -> float64 [Hkv, n] (NaN rows for unstable heads)."""
    q, mm = _u16(q), _u16(mm)
    Hq, D = q.shape
    Hkv, n = mm.shape[0], mm.shape[1]
    st = np.ascontiguousarray(np.asarray(stable, dtype=np.uint8))
    s = np.full((Hkv, n), np.nan, dtype=np.float64)
    lib().fco_seq_scores(_p(q, C.c_uint16), Hq, Hkv, _p(mm, C.c_uint16), n, D, _p(st, C.c_uint8), mode,
                         _p(s, C.c_double))
    return s


def seq_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, ctx: int, page_lists: List[np.ndarray],
                  scale: float, P: int = 16) -> Tuple[np.ndarray, np.ndarray]:
    """q: uint16 [Hq, D]; k, v: uint16 [Hkv, tpad, D]; page_lists[h]: page ids of KV head h.
    Returns (out float64 [Hq, D], lse float64 [Hq])."""
    q, k, v = _u16(q), _u16(k), _u16(v)
    Hq, D = q.shape
    Hkv, tpad = k.shape[0], k.shape[1]
    stride = max(1, max(len(x) for x in page_lists))
    pl = np.full((Hkv, stride), -1, dtype=np.int32)
    pc = np.zeros(Hkv, dtype=np.int32)
    for h, x in enumerate(page_lists):
        pl[h, :len(x)] = x
        pc[h] = len(x)
    out = np.empty((Hq, D), dtype=np.float64)
    lse = np.empty(Hq, dtype=np.float64)
    lib().fco_seq_attention(_p(q, C.c_uint16), _p(k, C.c_uint16), _p(v, C.c_uint16), Hq, Hkv, tpad, ctx,
                            D, P, _p(pl, C.c_int32), stride, _p(pc, C.c_int32), scale,
                            _p(out, C.c_double), _p(lse, C.c_double))
    return out, lse


# ---- the decode loop of the method ---------------------------------------------------------------
class OracleDecoder:
    """State of the method for a batch of sequences: per stable (b, h) the selected set S_t, the block
    table, the free list and the running promotion counts."""

    def __init__(self, batch: int, Hq: int, Hkv: int, ctx: Sequence[int], stable: Sequence[bool],
                 topk: Sequence[int], R: int, D: int = 128, P: int = 16, scale: Optional[float] = None,
                 group_mode: int = 0, unstable_topk: bool = False):
        self.B, self.Hq, self.Hkv, self.D, self.P, self.R = batch, Hq, Hkv, D, P, R
        self.ctx = [int(c) for c in ctx]
        self.stable = [bool(s) for s in stable]
        self.topk = [int(x) for x in topk]
        self.scale = float(scale) if scale else 1.0 / float(np.sqrt(D))
        self.group_mode = group_mode
        # unstable_topk: the paper's own treatment of unstable heads (Sec. 3.1, 3.2): rescored at every
        # step, attending over their top-K pages only, everything resident.  Default: they attend over
        # all pages.
        self.unstable_topk = unstable_topk
        self.sel: Dict[Tuple[int, int], np.ndarray] = {
            (b, h): np.empty(0, dtype=np.int32) for b in range(batch) for h in range(Hkv)
            if self.stable[h] or unstable_topk}
        self.promoted_pages = 0
        self.last_scores: Dict[Tuple[int, int], np.ndarray] = {}

    def n_pages(self, b: int) -> int:
        return -(-self.ctx[b] // self.P)

    def rerank(self, b: int, q_b: np.ndarray, mm_b: np.ndarray) -> Dict[int, Tuple[np.ndarray, np.ndarray]]:
        """Rescore and reselect every stable head of sequence b.  Returns {h: (promoted, evicted)}."""
        s = seq_scores(q_b, mm_b, self.stable, self.group_mode)
        res = {}
        for h in range(self.Hkv):
            if not self.stable[h]:
                continue
            new = select_topk(s[h], self.ctx[b], self.topk[b], self.P)
            old = self.sel[(b, h)]
            promoted = np.setdiff1d(new, old).astype(np.int32)
            evicted = np.setdiff1d(old, new).astype(np.int32)
            self.sel[(b, h)] = new
            self.last_scores[(b, h)] = s[h].copy()
            self.promoted_pages += len(promoted)
            res[h] = (promoted, evicted)
        return res

    def append(self, b: int) -> Optional[int]:
        """One token joins sequence b (Sec. 2).  If it starts a new page, that page -- partially filled,
        being appended to -- joins the selection of every head that attends over a list (Sec. 3.3).
        Returns the index of the page that was started, or None."""
        pos = self.ctx[b]
        self.ctx[b] = pos + 1
        if pos % self.P != 0:
            return None
        page = pos // self.P
        for h in range(self.Hkv):
            if (b, h) in self.sel and self.stable[h]:
                self.sel[(b, h)] = np.append(self.sel[(b, h)], np.int32(page)).astype(np.int32)
        return page

    def rerank_unstable(self, b: int, q_b: np.ndarray, mm_b: np.ndarray) -> None:
        """Every-step selection of the unstable heads (only meaningful with unstable_topk)."""
        flags = [not s for s in self.stable]
        s = seq_scores(q_b, mm_b, flags, self.group_mode)
        for h in range(self.Hkv):
            if flags[h]:
                self.sel[(b, h)] = select_topk(s[h], self.ctx[b], self.topk[b], self.P)
                self.last_scores[(b, h)] = s[h].copy()

    def page_lists(self, b: int, override: Optional[Dict[Tuple[int, int], np.ndarray]] = None
                   ) -> List[np.ndarray]:
        out = []
        for h in range(self.Hkv):
            if self.stable[h] or self.unstable_topk:
                src = override if override is not None and (b, h) in override else self.sel
                out.append(np.asarray(src[(b, h)], dtype=np.int32))
            else:
                out.append(np.arange(self.n_pages(b), dtype=np.int32))
        return out

    def attend(self, b: int, q_b: np.ndarray, k_b: np.ndarray, v_b: np.ndarray,
               override: Optional[Dict[Tuple[int, int], np.ndarray]] = None):
        return seq_attention(q_b, k_b, v_b, self.ctx[b], self.page_lists(b, override), self.scale, self.P)
