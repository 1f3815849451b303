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
                max_topk=204, softmax_scale=0.0, device=0, attn_waves=0, copy_workgroups=0)
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
                                dict(max_batch=0), dict(softmax_scale=-1.0), dict(num_q_heads=8 * 3),
                                dict(copy_workgroups=-1), dict(attn_waves=-4)])
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


def test_struct_layouts_match_the_c_header(tmp_path):
    """Size and every field offset of the ctypes mirrors against what a C compiler makes of the header."""
    import subprocess
    structs = ["fc_config", "fc_rerank_args", "fc_attn_args", "fc_promote_args", "fc_append_args", "fc_stability_args"]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "flexicache.h"', 'int main(void) {']
    for name in structs:
        lines.append(f'  printf("{name} %zu\\n", sizeof({name}));')
        for f, _ in getattr(binding, name)._fields_:
            lines.append(f'  printf("{name}.{f} %zu\\n", offsetof({name}, {f}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    got = dict(l.split() for l in subprocess.check_output([str(exe)], text=True).splitlines())
    for name in structs:
        st = getattr(binding, name)
        assert int(got[name]) == C.sizeof(st), name
        for f, _ in st._fields_:
            assert int(got[f"{name}.{f}"]) == getattr(st, f).offset, f"{name}.{f}"
