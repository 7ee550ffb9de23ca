"""The C-ABI boundary on a machine without a GPU: the library loads, exports every symbol the header
declares, and its host-side validation returns the documented error codes before touching HIP."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2507_10069_amd import binding as B
from paper_2507_10069_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _batch(**over):
    kw = dict(num_reqs=2, num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16, num_pages=10,
              max_pages_per_req=4, total_new_tokens=20, max_new_len=12, dtype="bf16", softmax_scale=0.1)
    kw.update(over)
    return B.make_batch(**kw)


def test_exports_match_header():
    lib = B.load()
    with open(os.path.join(ROOT, "include", "emm.h")) as f:
        header = f.read()
    declared = sorted(set(re.findall(r"\b(emm_[a-z_]+)\s*\(", header)))
    assert declared == sorted(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    from paper_2507_10069_amd import prefix_cache as PC
    with open(os.path.join(ROOT, "include", "emm_prefix_cache.h")) as f:
        header = f.read()
    declared = sorted(set(re.findall(r"\b(emm_[a-z_]+)\s*\(", header)))
    assert declared == sorted(PC.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.emm_version() >= 100
    assert B.emm_status_string(B.EMM_OK) == "ok"
    assert "workspace" in B.emm_status_string(B.EMM_ERR_WORKSPACE)


def test_struct_layout_matches_header():
    # 12 four-byte scalars then four pointers
    assert ctypes.sizeof(B.emm_batch) == 12 * 4 + 4 * ctypes.sizeof(ctypes.c_void_p)
    assert B.emm_batch.page_table.offset == 48


def test_workspace_size_and_scalar_checks():
    assert B.emm_prefill_attn_workspace_size(_batch()) > 0
    assert B.emm_prefill_attn_workspace_size(_batch(dtype="f32")) == 0
    lib = B.load()
    n = ctypes.c_size_t()
    assert lib.emm_prefill_attn_workspace_size(None, ctypes.byref(n)) == B.EMM_ERR_NULL
    assert lib.emm_prefill_attn_workspace_size(ctypes.byref(_batch()), None) == B.EMM_ERR_NULL
    bad = [dict(num_q_heads=7), dict(num_kv_heads=0), dict(softmax_scale=0.0), dict(softmax_scale=float("nan")),
           dict(softmax_scale=-1.0), dict(num_reqs=-1), dict(max_new_len=21), dict(dtype=5)]
    for over in bad:
        assert lib.emm_prefill_attn_workspace_size(ctypes.byref(_batch(**over)), ctypes.byref(n)) == \
            B.EMM_ERR_INVALID_ARG, over
    unsupported = [dict(page_size=32), dict(head_dim=64), dict(dtype="f32", head_dim=32)]
    for over in unsupported:
        assert lib.emm_prefill_attn_workspace_size(ctypes.byref(_batch(**over)), ctypes.byref(n)) == \
            B.EMM_ERR_UNSUPPORTED, over


def test_decode_entry_wants_at_most_one_new_token():
    lib = B.load()
    ok = 0x1000
    b = _batch()                     # max_new_len = 12
    b.page_table = b.prefix_lens = b.new_lens = b.cu_new_lens = ok
    assert lib.emm_decode_attn(ctypes.byref(b), ok, ok, ok, ok, None, ok, 1 << 30, None) == B.EMM_ERR_INVALID_ARG
    one = _batch(total_new_tokens=2, max_new_len=1)
    assert B.emm_prefill_attn_workspace_size(one) > 0
    assert lib.emm_decode_attn(ctypes.byref(one), ok, ok, ok, ok, None, None, 0, None) == B.EMM_ERR_NULL


@pytest.mark.parametrize("entry", ["emm_prefill_attn", "emm_cross_attn"])
def test_attention_rejects_before_launch(entry):
    lib = B.load()
    fn = getattr(lib, entry)
    ok = 0x1000                      # fake, 16-byte aligned, never dereferenced: validation fails first
    b = _batch()                     # device arrays are NULL
    assert fn(ctypes.byref(b), ok, ok, ok, ok, None, None, 0, None) == B.EMM_ERR_NULL
    b = _batch()
    b.page_table = b.prefix_lens = b.new_lens = b.cu_new_lens = ok
    need = B.emm_prefill_attn_workspace_size(b)
    assert need > 0                  # the bf16 kernels cut their last work units and merge them through it
    assert fn(ctypes.byref(b), None, ok, ok, ok, None, ok, need, None) == B.EMM_ERR_NULL
    assert fn(ctypes.byref(b), ok + 8, ok, ok, ok, None, ok, need, None) == B.EMM_ERR_INVALID_ARG
    assert fn(ctypes.byref(b), ok, ok, ok, ok, ok + 2, ok, need, None) == B.EMM_ERR_INVALID_ARG
    assert fn(ctypes.byref(b), ok, ok, ok, ok, None, None, need, None) == B.EMM_ERR_NULL
    assert fn(ctypes.byref(b), ok, ok, ok, ok, None, ok, need - 1, None) == B.EMM_ERR_WORKSPACE
    assert fn(ctypes.byref(b), ok, ok, ok, ok, None, ok + 4, need, None) == B.EMM_ERR_INVALID_ARG
    assert fn(None, ok, ok, ok, ok, None, None, 0, None) == B.EMM_ERR_NULL
    # empty batches are no-ops that never reach a launch
    assert fn(ctypes.byref(_batch(num_reqs=0, total_new_tokens=0, max_new_len=0)), None, None, None, None,
              None, None, 0, None) == B.EMM_OK
    assert fn(ctypes.byref(_batch(total_new_tokens=0, max_new_len=0)), None, None, None, None,
              None, None, 0, None) == B.EMM_OK


def test_scatter_rejects_before_launch():
    lib = B.load()
    ok = 0x1000
    b = _batch()
    b.page_table = b.prefix_lens = b.new_lens = b.cu_new_lens = ok
    assert lib.emm_kv_scatter(ctypes.byref(b), None, ok, ok, ok, None) == B.EMM_ERR_NULL
    assert lib.emm_kv_scatter(ctypes.byref(b), ok, ok, ok + 4, ok, None) == B.EMM_ERR_INVALID_ARG
    assert lib.emm_kv_scatter(ctypes.byref(_batch(page_size=8)), ok, ok, ok, ok, None) == B.EMM_ERR_UNSUPPORTED
    assert lib.emm_kv_scatter(ctypes.byref(_batch(total_new_tokens=0, max_new_len=0)), None, None, None, None,
                              None) == B.EMM_OK


def _host_batch(wl):
    return B.make_batch(num_reqs=wl.num_reqs, num_q_heads=wl.num_q_heads, num_kv_heads=wl.num_kv_heads,
                        head_dim=wl.head_dim, page_size=wl.page_size, num_pages=wl.num_pages,
                        max_pages_per_req=wl.max_pages_per_req, total_new_tokens=wl.total_new_tokens,
                        max_new_len=wl.max_new_len, dtype=wl.dtype, softmax_scale=wl.softmax_scale)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_validate_accepts_named_workloads(cfg):
    wl = W.config(cfg, 8)
    st = B.emm_validate_batch_host(_host_batch(wl), wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens,
                                   wl.kind == "causal")
    assert st == B.EMM_OK


def test_validate_rejects_broken_batches():
    wl = W.config(2, 8)
    b = _host_batch(wl)
    args = lambda **o: (o.get("pt", wl.page_table), o.get("prefix", wl.prefix_lens), o.get("new", wl.new_lens),
                        o.get("cu", wl.cu_new_lens), True)
    pt = wl.page_table.copy()
    pt[0, 0] = wl.num_pages
    assert B.emm_validate_batch_host(b, *args(pt=pt)) == B.EMM_ERR_INVALID_ARG
    pt = wl.page_table.copy()
    pt[3, 1] = -1
    assert B.emm_validate_batch_host(b, *args(pt=pt)) == B.EMM_ERR_INVALID_ARG
    # two requests writing into the same page
    pt = wl.page_table.copy()
    first_new = int(wl.prefix_lens[0]) // 16
    pt[1, first_new] = pt[0, first_new]
    assert B.emm_validate_batch_host(b, *args(pt=pt)) == B.EMM_ERR_INVALID_ARG
    cu = wl.cu_new_lens.copy()
    cu[2] += 1
    assert B.emm_validate_batch_host(b, *args(cu=cu)) == B.EMM_ERR_INVALID_ARG
    prefix = wl.prefix_lens.copy()
    prefix[0] = -3
    assert B.emm_validate_batch_host(b, *args(prefix=prefix)) == B.EMM_ERR_INVALID_ARG
    # more pages than the table has columns
    prefix = wl.prefix_lens.copy()
    prefix[0] += 16 * wl.max_pages_per_req
    assert B.emm_validate_batch_host(b, *args(prefix=prefix)) == B.EMM_ERR_INVALID_ARG
