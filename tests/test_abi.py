"""The C-ABI library loads, exports every call the header declares, and rejects bad
configurations on the host before anything touches a GPU.  (No GPU needed.)"""
import ctypes as C
import os
import re

import pytest

from paper_2506_15724_amd import binding as MB

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_calls():
    text = open(os.path.join(ROOT, "include", "madakv.h")).read()
    return sorted(set(re.findall(r"^int32_t\s+(madakv_\w+)\s*\(", text, flags=re.M)))


def test_header_declares_the_four_path_calls():
    names = declared_calls()
    for must in ("madakv_score", "madakv_allocate", "madakv_select_gather", "madakv_decode_attn"):
        assert must in names


def test_library_exports_every_declared_symbol():
    lib = MB.lib()
    for name in declared_calls():
        assert hasattr(lib, name), name
    assert sorted(MB.EXPORTS) == declared_calls()


def test_config_struct_matches_header_layout():
    # four-byte fields, in the header's order
    text = open(os.path.join(ROOT, "include", "madakv.h")).read()
    body = text[text.index("typedef struct {", text.index("Hyper-parameters")):text.index("} madakv_config;")]
    fields = re.findall(r"^\s*(?:int32_t|float)\s+(\w+);", body, flags=re.M)
    assert fields == [f[0] for f in MB.Config._fields_]
    assert C.sizeof(MB.Config) == 4 * len(fields)


def good(**kw):
    base = dict(n_layers=2, batch=1, n_q_heads=8, n_kv_heads=8, head_dim=128, ctx_len=1024, window=32, budget=256,
                dtype=MB.BF16, pool_k=7, mpa_mode=1, hcc_mode=1, hcc_rho=2, theta=0.9, softmax_scale=0.0,
                max_new_tokens=4, out_fp32=1, pool_mode=0, share_mode=0, select_mode=0, sink_tokens=4, cache_fp8=0, n_modalities=2, page_rows=0)
    base.update(kw)
    return MB.Config(*[base[f[0]] for f in MB.Config._fields_])


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=12, n_kv_heads=8), -2),        # heads do not divide
    (dict(head_dim=96), -2),
    (dict(window=1024), -2),                        # window must be shorter than the context
    (dict(n_q_heads=16, n_kv_heads=1), -2),         # group larger than 8
    (dict(n_q_heads=64, n_kv_heads=8, window=64), -2),   # G*W > 256
    (dict(pool_k=4), -2),
    (dict(budget=32), -3),                          # budget <= window while below the context
    (dict(budget=0), -3),
    (dict(dtype=7), -5),
    (dict(theta=0.0), -1),
    (dict(theta=1.5), -1),
    (dict(hcc_rho=0), -1),
    (dict(max_new_tokens=-1), -1),
    (dict(mpa_mode=4), -1),
    (dict(hcc_mode=3), -1),
    (dict(pool_mode=2), -1),
    (dict(n_modalities=1), -2),
    (dict(cache_fp8=1, dtype=0, head_dim=64, window=16), -5),
    (dict(cache_fp8=2), -1),
    (dict(n_modalities=5), -2),
    (dict(select_mode=1, sink_tokens=-1), -1),
    (dict(page_rows=48), -1),                      # pages are 16 .. 256 rows, powers of two
    (dict(page_rows=512), -1),
])
def test_create_rejects_bad_config_on_host(kw, status):
    h = C.c_void_p()
    rc = MB.lib().madakv_create(C.byref(good(**kw)), C.byref(h))
    assert rc == status and not h.value


def test_null_arguments():
    lib = MB.lib()
    assert lib.madakv_create(None, None) == -1
    assert lib.madakv_destroy(None) == -1
    assert lib.madakv_score(None, 0, 1, None, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.madakv_allocate(None, 0, 1, None, None, None, None) == -1
    assert lib.madakv_workspace_bytes(None, 1, None, None, None) == -1
    assert lib.madakv_compact_capacity_tokens(None, None) == -1
    assert lib.madakv_last_hip_error(None) == 0
    assert lib.madakv_decode_attn(None, 0, 1, None, None, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.madakv_decode_attn_static(None, 0, 1, None, None, None, None, None, None, None, None, None) == -1
