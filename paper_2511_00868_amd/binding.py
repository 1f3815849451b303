"""ctypes binding of libflexicache.so: argument marshalling only, one Python function per C entry
point with the same name.  Tensors are torch tensors used as device / pinned memory; nothing is
computed here.  There is no fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libflexicache.so")

FC_OK, FC_ERR_INVALID_ARG, FC_ERR_UNSUPPORTED, FC_ERR_WORKSPACE, FC_ERR_HIP, FC_ERR_STATE = 0, -1, -2, -3, -4, -5
FC_PROMOTE_GATHER, FC_PROMOTE_MEMCPY, FC_PROMOTE_RIDE = 0, 1, 2
FC_HEADS_ALL, FC_HEADS_UNSTABLE, FC_HEADS_STABLE, FC_PAGES_RESIDENT, FC_PAGES_PROMOTED = 0, 1, 2, 3, 4

class fc_append_args(C.Structure):
    _fields_ = [("k_new", C.c_void_p), ("v_new", C.c_void_p), ("append_mask", C.c_void_p),
                ("context_lens", C.c_void_p), ("block_table", C.c_void_p), ("host_block_table", C.c_void_p),
                ("free_blocks", C.c_void_p), ("free_count", C.c_void_p), ("resident_pages", C.c_void_p),
                ("resident_count", C.c_void_p), ("minmax", C.c_void_p), ("kv_pool", C.c_void_p),
                ("num_pool_blocks", C.c_int64), ("host_pool", C.c_void_p), ("num_host_blocks", C.c_int64),
                ("stable_flag", C.c_void_p), ("batch", C.c_int32)]


class fc_stability_args(C.Structure):
    _fields_ = [("traces", C.c_void_p), ("num_pages", C.c_void_p), ("steps", C.c_int32), ("heads", C.c_int32),
                ("topk", C.c_int32), ("window", C.c_int32), ("ts_out", C.c_void_p), ("bottom_counts", C.c_void_p)]


EXPORTS = ["fc_workspace_bytes", "fc_host_scratch_bytes", "fc_create", "fc_destroy", "fc_status_string",
           "fc_last_error", "fc_write_kv_pages", "fc_build_minmax", "fc_rerank_topk", "fc_promote_pages",
           "fc_sparse_decode_attn", "fc_append_kv", "fc_offload_pages", "fc_stability_profile", "fc_classify_heads",
           "fc_check_device_state", "fc_profile_begin", "fc_profile_end", "fc_measure_stream_read",
           "fc_sparse_decode_attn_static", "fc_static_scratch_bytes", "fc_static_last_error", "fc_rerank_promote"]


class fc_config(C.Structure):
    _fields_ = [("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_size", C.c_int32), ("max_batch", C.c_int32), ("max_pages_per_seq", C.c_int32),
                ("max_topk", C.c_int32), ("softmax_scale", C.c_float), ("device", C.c_int32),
                ("attn_waves", C.c_int32), ("copy_workgroups", C.c_int32)]


class fc_rerank_args(C.Structure):
    _fields_ = [("q", C.c_void_p), ("minmax", C.c_void_p), ("context_lens", C.c_void_p),
                ("stable_flag", C.c_void_p), ("k_per_seq", C.c_void_p), ("rerank_mask", C.c_void_p),
                ("batch", C.c_int32), ("topk_pages", C.c_void_p), ("topk_count", C.c_void_p),
                ("scores_out", C.c_void_p)]


class fc_promote_args(C.Structure):
    _fields_ = [("new_pages", C.c_void_p), ("new_count", C.c_void_p), ("resident_pages", C.c_void_p),
                ("resident_count", C.c_void_p), ("block_table", C.c_void_p), ("host_block_table", C.c_void_p),
                ("free_blocks", C.c_void_p), ("free_count", C.c_void_p), ("stable_flag", C.c_void_p),
                ("rerank_mask", C.c_void_p), ("kv_pool", C.c_void_p), ("num_pool_blocks", C.c_int64),
                ("host_pool", C.c_void_p), ("num_host_blocks", C.c_int64), ("batch", C.c_int32),
                ("mode", C.c_int32), ("promoted_count", C.c_void_p), ("promoted_flags", C.c_void_p),
                ("total_promoted", C.c_void_p)]


class fc_attn_args(C.Structure):
    _fields_ = [("q", C.c_void_p), ("kv_pool", C.c_void_p), ("num_pool_blocks", C.c_int64),
                ("block_table", C.c_void_p), ("context_lens", C.c_void_p), ("stable_flag", C.c_void_p),
                ("topk_pages", C.c_void_p), ("topk_count", C.c_void_p), ("batch", C.c_int32),
                ("out", C.c_void_p), ("lse", C.c_void_p), ("head_subset", C.c_int32), ("promoted_flags", C.c_void_p)]


_lib = None


def load() -> C.CDLL:
    """Loads the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_00868_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        L.fc_workspace_bytes.argtypes = [C.POINTER(fc_config)]
        L.fc_workspace_bytes.restype = C.c_size_t
        L.fc_host_scratch_bytes.argtypes = [C.POINTER(fc_config)]
        L.fc_host_scratch_bytes.restype = C.c_size_t
        L.fc_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(fc_config), C.c_void_p, C.c_size_t,
                                C.c_void_p, C.c_size_t]
        L.fc_destroy.argtypes = [C.c_void_p]
        L.fc_status_string.argtypes = [C.c_int]
        L.fc_status_string.restype = C.c_char_p
        L.fc_last_error.argtypes = [C.c_void_p]
        L.fc_last_error.restype = C.c_char_p
        L.fc_write_kv_pages.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_int64, C.c_void_p]
        L.fc_build_minmax.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.fc_rerank_topk.argtypes = [C.c_void_p, C.POINTER(fc_rerank_args), C.c_void_p]
        L.fc_promote_pages.argtypes = [C.c_void_p, C.POINTER(fc_promote_args), C.c_void_p, C.c_void_p]
        L.fc_sparse_decode_attn.argtypes = [C.c_void_p, C.POINTER(fc_attn_args), C.c_void_p]
        L.fc_rerank_promote.argtypes = [C.c_void_p, C.POINTER(fc_rerank_args), C.POINTER(fc_promote_args), C.c_void_p, C.c_void_p]
        L.fc_append_kv.argtypes = [C.c_void_p, C.POINTER(fc_append_args), C.c_void_p]
        L.fc_offload_pages.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32,
                                       C.c_void_p]
        L.fc_stability_profile.argtypes = [C.c_void_p, C.POINTER(fc_stability_args), C.c_void_p]
        L.fc_classify_heads.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.fc_check_device_state.argtypes = [C.c_void_p, C.c_void_p]
        L.fc_profile_begin.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.fc_profile_end.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_int32)]
        L.fc_measure_stream_read.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_int32, C.c_void_p,
                                             C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.fc_sparse_decode_attn_static.argtypes = [C.POINTER(fc_config), C.POINTER(fc_attn_args), C.c_void_p]
        L.fc_static_scratch_bytes.argtypes = []
        L.fc_static_scratch_bytes.restype = C.c_size_t
        L.fc_static_last_error.argtypes = []
        L.fc_static_last_error.restype = C.c_char_p
        _lib = L
    return _lib


class FlexiCacheError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"flexicache: {text} (status {status})")
        self.status = status


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _host_u8(flags):
    arr = (C.c_uint8 * len(flags))(*[1 if f else 0 for f in flags])
    return arr


def fc_sparse_decode_attn_static(cfg: fc_config, *, q, kv_pool, num_pool_blocks: int, block_table, context_lens,
                                 stable_flag, topk_pages, topk_count, batch: int, out, lse=None, stream=None):
    """The whole-pass attention without a context or a workspace (the library's built-in scratch array)."""
    lib = load()
    flags = _host_u8(stable_flag)
    a = fc_attn_args(_ptr(q), _ptr(kv_pool), num_pool_blocks, _ptr(block_table), _ptr(context_lens),
                     C.addressof(flags), _ptr(topk_pages), _ptr(topk_count), batch, _ptr(out), _ptr(lse), FC_HEADS_ALL, None)
    st = lib.fc_sparse_decode_attn_static(C.byref(cfg), C.byref(a), None if stream is None else stream.cuda_stream)
    if st != FC_OK:
        raise FlexiCacheError(st, lib.fc_static_last_error().decode() or lib.fc_status_string(st).decode())


class Context:
    """Owns the caller-side memory an fc_ctx needs (device workspace, pinned scratch) and exposes the
    C entry points under their own names."""

    def __init__(self, *, num_q_heads: int, num_kv_heads: int, max_batch: int, max_pages_per_seq: int,
                 max_topk: int, softmax_scale: float = 0.0, device: int = 0, attn_waves: int = 0,
                 copy_workgroups: int = 0,
                 head_dim: int = 128, page_size: int = 16):
        import torch
        self.torch = torch
        self.lib = load()
        self.cfg = fc_config(num_q_heads, num_kv_heads, head_dim, page_size, max_batch, max_pages_per_seq,
                             max_topk, softmax_scale, device, attn_waves, copy_workgroups)
        ws = self.lib.fc_workspace_bytes(C.byref(self.cfg))
        hs = self.lib.fc_host_scratch_bytes(C.byref(self.cfg))
        if ws == 0 or hs == 0:
            raise FlexiCacheError(FC_ERR_INVALID_ARG, "configuration rejected")
        if not torch.cuda.is_available():
            raise RuntimeError("flexicache needs a GPU: no HIP device is visible (there is no CPU fallback)")
        self.device = torch.device("cuda", device)
        self.workspace = torch.zeros(ws, dtype=torch.uint8, device=self.device)
        self.scratch = torch.zeros(hs, dtype=torch.uint8, pin_memory=True)
        self.handle = C.c_void_p()
        st = self.lib.fc_create(C.byref(self.handle), C.byref(self.cfg), self.workspace.data_ptr(), ws,
                                self.scratch.data_ptr(), hs)
        if st != FC_OK:
            raise FlexiCacheError(st, self.lib.fc_status_string(st).decode())

    def close(self):
        if getattr(self, "handle", None) and self.handle.value:
            self.torch.cuda.synchronize(self.device)
            self.lib.fc_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != FC_OK:
            raise FlexiCacheError(st, self.lib.fc_last_error(self.handle).decode() or
                                  self.lib.fc_status_string(st).decode())

    @staticmethod
    def _stream(stream) -> Optional[int]:
        return None if stream is None else stream.cuda_stream

    # ---- entry points, same names as the C ABI ---------------------------------------------------
    def fc_write_kv_pages(self, k_src, v_src, n_pages: int, block_ids, pool, num_blocks: int, stream=None):
        self._check(self.lib.fc_write_kv_pages(self.handle, _ptr(k_src), _ptr(v_src), n_pages, _ptr(block_ids),
                                               block_ids.stride(0), _ptr(pool), num_blocks, self._stream(stream)))

    def fc_build_minmax(self, pool, num_blocks: int, block_ids, page_list, n_list: int, context_len: int,
                        minmax_seq, stream=None):
        self._check(self.lib.fc_build_minmax(self.handle, _ptr(pool), num_blocks, _ptr(block_ids),
                                             block_ids.stride(0), _ptr(page_list), n_list, context_len,
                                             _ptr(minmax_seq), self._stream(stream)))

    def fc_rerank_topk(self, *, q, minmax, context_lens, stable_flag, k_per_seq, batch: int, topk_pages,
                       topk_count, rerank_mask=None, scores_out=None, stream=None):
        flags = _host_u8(stable_flag)
        a = fc_rerank_args(_ptr(q), _ptr(minmax), _ptr(context_lens), C.addressof(flags), _ptr(k_per_seq),
                           _ptr(rerank_mask), batch, _ptr(topk_pages), _ptr(topk_count), _ptr(scores_out))
        self._check(self.lib.fc_rerank_topk(self.handle, C.byref(a), self._stream(stream)))

    def fc_promote_pages(self, *, new_pages, new_count, resident_pages, resident_count, block_table,
                         host_block_table, free_blocks, free_count, stable_flag, kv_pool, num_pool_blocks: int,
                         host_pool, num_host_blocks: int, batch: int, main_stream, side_stream,
                         mode: int = FC_PROMOTE_GATHER, rerank_mask=None, promoted_count=None, promoted_flags=None,
                         total_promoted=None):
        flags = _host_u8(stable_flag)
        a = fc_promote_args(_ptr(new_pages), _ptr(new_count), _ptr(resident_pages), _ptr(resident_count),
                            _ptr(block_table), _ptr(host_block_table), _ptr(free_blocks), _ptr(free_count),
                            C.addressof(flags), _ptr(rerank_mask), _ptr(kv_pool), num_pool_blocks, _ptr(host_pool),
                            num_host_blocks, batch, mode, _ptr(promoted_count), _ptr(promoted_flags), _ptr(total_promoted))
        self._check(self.lib.fc_promote_pages(self.handle, C.byref(a), self._stream(main_stream),
                                              self._stream(side_stream)))

    def fc_rerank_promote(self, *, q, minmax, context_lens, stable_flag, k_per_seq, batch: int, topk_pages, topk_count,
                          resident_pages, resident_count, block_table, host_block_table, free_blocks, free_count,
                          kv_pool, num_pool_blocks: int, host_pool, num_host_blocks: int, main_stream, side_stream,
                          mode: int = FC_PROMOTE_GATHER, rerank_mask=None, scores_out=None, promoted_count=None,
                          promoted_flags=None, total_promoted=None):
        flags = _host_u8(stable_flag)
        r = fc_rerank_args(_ptr(q), _ptr(minmax), _ptr(context_lens), C.addressof(flags), _ptr(k_per_seq),
                           _ptr(rerank_mask), batch, _ptr(topk_pages), _ptr(topk_count), _ptr(scores_out))
        a = fc_promote_args(_ptr(topk_pages), _ptr(topk_count), _ptr(resident_pages), _ptr(resident_count),
                            _ptr(block_table), _ptr(host_block_table), _ptr(free_blocks), _ptr(free_count),
                            C.addressof(flags), _ptr(rerank_mask), _ptr(kv_pool), num_pool_blocks, _ptr(host_pool),
                            num_host_blocks, batch, mode, _ptr(promoted_count), _ptr(promoted_flags), _ptr(total_promoted))
        self._check(self.lib.fc_rerank_promote(self.handle, C.byref(r), C.byref(a), self._stream(main_stream),
                                               self._stream(side_stream)))

    def fc_sparse_decode_attn(self, *, q, kv_pool, num_pool_blocks: int, block_table, context_lens, stable_flag,
                              topk_pages, topk_count, batch: int, out, lse=None, head_subset: int = FC_HEADS_ALL,
                              promoted_flags=None, stream=None):
        flags = _host_u8(stable_flag)
        a = fc_attn_args(_ptr(q), _ptr(kv_pool), num_pool_blocks, _ptr(block_table), _ptr(context_lens),
                         C.addressof(flags), _ptr(topk_pages), _ptr(topk_count), batch, _ptr(out), _ptr(lse), head_subset, _ptr(promoted_flags))
        self._check(self.lib.fc_sparse_decode_attn(self.handle, C.byref(a), self._stream(stream)))

    def fc_append_kv(self, *, k_new, v_new, context_lens, block_table, host_block_table, free_blocks, free_count,
                     resident_pages, resident_count, minmax, kv_pool, num_pool_blocks: int, host_pool,
                     num_host_blocks: int, stable_flag, batch: int, append_mask=None, stream=None):
        flags = _host_u8(stable_flag)
        a = fc_append_args(_ptr(k_new), _ptr(v_new), _ptr(append_mask), _ptr(context_lens), _ptr(block_table),
                           _ptr(host_block_table), _ptr(free_blocks), _ptr(free_count), _ptr(resident_pages),
                           _ptr(resident_count), _ptr(minmax), _ptr(kv_pool), num_pool_blocks, _ptr(host_pool),
                           num_host_blocks, C.addressof(flags), batch)
        self._check(self.lib.fc_append_kv(self.handle, C.byref(a), self._stream(stream)))

    def fc_offload_pages(self, kv_pool, num_pool_blocks: int, host_pool, num_host_blocks: int, pairs, n_pairs: int,
                         stream=None):
        self._check(self.lib.fc_offload_pages(self.handle, _ptr(kv_pool), num_pool_blocks, _ptr(host_pool),
                                              num_host_blocks, _ptr(pairs), n_pairs, self._stream(stream)))

    def fc_stability_profile(self, *, traces, num_pages, steps: int, heads: int, topk: int, window: int, ts_out,
                             bottom_counts, stream=None):
        a = fc_stability_args(_ptr(traces), _ptr(num_pages), steps, heads, topk, window, _ptr(ts_out),
                              _ptr(bottom_counts))
        self._check(self.lib.fc_stability_profile(self.handle, C.byref(a), self._stream(stream)))

    def fc_classify_heads(self, bottom_counts, heads: int, unstable_out, num: int = 1, den: int = 4, stream=None):
        self._check(self.lib.fc_classify_heads(self.handle, _ptr(bottom_counts), heads, num, den, _ptr(unstable_out),
                                               self._stream(stream)))

    def fc_check_device_state(self, stream=None):
        self._check(self.lib.fc_check_device_state(self.handle, self._stream(stream)))

    def fc_profile_begin(self, every_nth: int = 1, stream=None):
        self._check(self.lib.fc_profile_begin(self.handle, every_nth, self._stream(stream)))

    def fc_profile_end(self):
        """(average raw bracket ms, empty-kernel bracket ms, launches)"""
        ms, empty, n = C.c_double(), C.c_double(), C.c_int32()
        self._check(self.lib.fc_profile_end(self.handle, C.byref(ms), C.byref(empty), C.byref(n)))
        return ms.value, empty.value, n.value

    def fc_measure_stream_read(self, buf, nbytes: int, launches: int = 16, stream=None):
        """(GB/s, microseconds per launch) of a plain streaming read of the first nbytes of `buf`."""
        g, us = C.c_double(), C.c_double()
        self._check(self.lib.fc_measure_stream_read(self.handle, _ptr(buf), nbytes, launches,
                                                    self._stream(stream), C.byref(g), C.byref(us)))
        return g.value, us.value
