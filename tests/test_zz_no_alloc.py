"""The attention entry point that allocates nothing (fc_sparse_decode_attn_static) against
fc_sparse_decode_attn on the same state: two calls in a row, the second on a smaller input, plus the
refusal of a shape whose partials do not fit the built-in scratch array."""
import ctypes as C

import numpy as np
import pytest

from paper_2511_00868_amd import binding, synth
from paper_2511_00868_amd.session import DecodeSession

pytestmark = pytest.mark.gpu


def run_both(cfg_index, batch, ctx, step_count):
    """Decodes a few steps through the context-based path, then attends once more through each entry
    point from the same tables, lists and queries.  Returns (out, lse) of both."""
    import torch
    cfg = synth.make_config(cfg_index, batch=batch, ctx=ctx, steps=step_count)
    wl = synth.Workload(cfg)
    sess = DecodeSession(cfg, wl)
    try:
        for t in range(step_count):
            sess.set_queries(wl.queries(t))
            sess.step(t)
        torch.cuda.synchronize()
        sess.ctx.fc_check_device_state()
        sess.attend()                       # FC_HEADS_ALL through the context and its workspace
        torch.cuda.synchronize()
        ref_out, ref_lse = sess.out.clone(), sess.lse.clone()
        out = torch.full_like(sess.out, float("nan"))
        lse = torch.full_like(sess.lse, float("nan"))
        binding.fc_sparse_decode_attn_static(
            sess.ctx.cfg, q=sess.q, kv_pool=sess.kv_pool, num_pool_blocks=sess.num_pool_blocks,
            block_table=sess.block_table, context_lens=sess.context_lens, stable_flag=sess.stable,
            topk_pages=sess.resident_pages, topk_count=sess.resident_count, batch=cfg.batch, out=out, lse=lse,
            stream=sess.main)
        torch.cuda.synchronize()
        return ref_out.cpu().numpy(), ref_lse.cpu().numpy(), out.cpu().numpy(), lse.cpu().numpy()
    finally:
        sess.close()


def test_static_entry_point_matches_the_workspace_one_twice_in_a_row():
    # same kernels, same schedule (same wavefront count): the results are the same bits
    big = run_both(2, 4, 8192, 5)
    np.testing.assert_array_equal(big[2], big[0])
    np.testing.assert_array_equal(big[3], big[1])
    assert np.all(np.isfinite(big[2]))
    small = run_both(4, 3, 1500, 2)         # ragged contexts, partial last pages, fewer items than before
    np.testing.assert_array_equal(small[2], small[0])
    np.testing.assert_array_equal(small[3], small[1])
    assert np.all(np.isfinite(small[2]))


def test_static_entry_point_refuses_what_does_not_fit():
    import torch
    torch.cuda.init()
    lib = binding.load()
    assert lib.fc_static_scratch_bytes() == 8 << 20
    cfg = binding.fc_config(32, 8, 128, 16, 512, 64, 8, 0.0, 0, 0, 0)
    dummy = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.FlexiCacheError) as err:
        binding.fc_sparse_decode_attn_static(cfg, q=dummy, kv_pool=dummy, num_pool_blocks=2, block_table=dummy,
                                             context_lens=dummy, stable_flag=[False] * 8, topk_pages=None,
                                             topk_count=None, batch=512, out=dummy)
    assert err.value.status == binding.FC_ERR_WORKSPACE and "built-in array" in str(err.value)
    a = binding.fc_attn_args()
    assert lib.fc_sparse_decode_attn_static(C.byref(cfg), C.byref(a), None) == binding.FC_ERR_INVALID_ARG
