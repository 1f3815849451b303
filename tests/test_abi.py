"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad configurations before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2511_00868_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flexicache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    syms = declared_symbols()
    assert set(syms) == set(binding.EXPORTS)
    for s in syms:
        assert getattr(lib, s) is not None


def cfg(**kw):
    base = dict(num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16, max_batch=8, max_pages_per_seq=2048,
                max_topk=204, softmax_scale=0.0, device=0, attn_waves=0)
    base.update(kw)
    return binding.fc_config(*[base[f[0]] for f in binding.fc_config._fields_])


def test_workspace_sizes_are_positive_and_monotonic():
    lib = binding.load()
    a = lib.fc_workspace_bytes(C.byref(cfg()))
    b = lib.fc_workspace_bytes(C.byref(cfg(max_batch=16)))
    assert 0 < a < b
    assert lib.fc_host_scratch_bytes(C.byref(cfg())) >= 256 + 8 * 8 * 204 * 8


@pytest.mark.parametrize("kw", [dict(head_dim=64), dict(page_size=32), dict(num_q_heads=24), dict(num_kv_heads=0),
                                dict(num_kv_heads=65, num_q_heads=65), dict(max_topk=0), dict(max_topk=4096),
                                dict(max_batch=0), dict(softmax_scale=-1.0), dict(num_q_heads=8 * 3)])
def test_bad_configurations_are_rejected_without_a_device(kw):
    lib = binding.load()
    c = cfg(**kw)
    assert lib.fc_workspace_bytes(C.byref(c)) == 0
    h = C.c_void_p()
    buf = C.create_string_buffer(4096)
    st = lib.fc_create(C.byref(h), C.byref(c), C.addressof(buf), 4096, C.addressof(buf), 4096)
    assert st in (binding.FC_ERR_INVALID_ARG, binding.FC_ERR_UNSUPPORTED) and not h.value


def test_create_rejects_null_and_small_buffers():
    lib = binding.load()
    c = cfg()
    h = C.c_void_p()
    assert lib.fc_create(C.byref(h), C.byref(c), None, 0, None, 0) == binding.FC_ERR_INVALID_ARG
    buf = C.create_string_buffer(8192)
    base = (C.addressof(buf) + 255) & ~255
    assert lib.fc_create(C.byref(h), C.byref(c), base, 1024, base, 1024) == binding.FC_ERR_WORKSPACE
    assert lib.fc_create(C.byref(h), C.byref(c), base + 8, 1 << 40, base, 1 << 40) == binding.FC_ERR_WORKSPACE
    assert lib.fc_status_string(binding.FC_ERR_WORKSPACE).decode().startswith("workspace")


def test_struct_sizes_match_the_c_layout():
    assert C.sizeof(binding.fc_config) == 40
    assert C.sizeof(binding.fc_rerank_args) == 80
    assert C.sizeof(binding.fc_attn_args) == 104
    assert C.sizeof(binding.fc_promote_args) == 144
    assert C.sizeof(binding.fc_append_args) == 136
