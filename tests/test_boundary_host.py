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
    assert B.emm_prefill_attn_workspace_size(_batch(num_pages=1024, max_pages_per_req=512)) > 0
    assert B.emm_prefill_attn_workspace_size(_batch()) == 0          # contexts of at most 64 tokens: nothing to cut
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
    unsupported = [dict(page_size=8), dict(page_size=48), dict(page_size=512), dict(head_dim=64), dict(dtype="f32", head_dim=32)]
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
    b = _batch(num_pages=1024, max_pages_per_req=512)
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


def test_shared_prefix_plan_host():
    """Units found from host copies of the page tables: consecutive requests, whole shared pages that both
    requests' cached tokens fill, multiples of 32 tokens, at most 32 / G requests, never fewer keys saved."""
    def plan(pt, prefix, new, H=28, Hkv=4, min_shared=32):
        pt = np.asarray(pt, dtype=np.int32)
        b = _batch(num_reqs=pt.shape[0], num_q_heads=H, num_kv_heads=Hkv, num_pages=1000, max_pages_per_req=pt.shape[1],
                   total_new_tokens=int(sum(new)), max_new_len=max(new))
        return B.emm_shared_prefix_plan_host(b, pt, np.asarray(prefix, np.int32), np.asarray(new, np.int32), min_shared)

    base = list(range(100, 140))                                     # 40 pages = 640 tokens
    def row(n_shared, tag):
        return base[:n_shared] + [500 + 40 * tag + i for i in range(40 - n_shared)]
    # three requests share 10 pages (160 tokens), a fourth shares nothing, then two share 3 pages (48 -> 32 tokens)
    pt = [row(10, 0), row(10, 1), row(10, 2), [900 + i for i in range(40)],
          [700, 701, 702] + [600 + i for i in range(37)], [700, 701, 702] + [650 + i for i in range(37)]]
    p = plan(pt, [300, 200, 640, 640, 100, 100], [1] * 6)
    assert p["num_units"] == 2
    assert p["unit_first_req"].tolist() == [0, 4] and p["unit_num_reqs"].tolist() == [3, 2]
    assert p["unit_shared_len"].tolist() == [160, 32]
    assert p["req_unit"].tolist() == [0, 0, 0, -1, 1, 1] and p["req_shared_len"].tolist() == [160, 160, 160, 0, 32, 32]
    # tiles: units 160/32 + 32/32, own parts ceil((P + 1 - shared) / 32) = 5, 2, 16, 21, 3, 3
    assert p["planned_tiles"] == 5 + 1 + 5 + 2 + 16 + 21 + 3 + 3
    assert p["max_own_tiles"] == 21 and p["max_unit_tiles"] == 5
    # cached tokens limit the shared length: the second request has only 70 tokens in its pages -> 64
    p = plan(pt[:2], [300, 70], [1, 1])
    assert p["unit_shared_len"].tolist() == [64]
    # below the floor: no unit
    assert plan(pt[:2], [300, 70], [1, 1], min_shared=128)["num_units"] == 0
    assert plan(pt[4:], [100, 20], [1, 1])["num_units"] == 0        # 16 common tokens < 32
    # a request without a new token ends a unit; G = 7 allows 4 requests per unit
    pt8 = [row(20, i) for i in range(8)]
    p = plan(pt8, [640] * 8, [1, 1, 0, 1, 1, 1, 1, 1])
    assert p["unit_first_req"].tolist() == [0, 3] and p["unit_num_reqs"].tolist() == [2, 4]
    assert p["req_unit"].tolist() == [0, 0, -1, 1, 1, 1, 1, -1]
    # G = 4: 8 per unit; G = 32: no units possible
    assert plan(pt8, [640] * 8, [1] * 8, H=32, Hkv=8)["unit_num_reqs"].tolist() == [8]
    assert plan(pt8, [640] * 8, [1] * 8, H=32, Hkv=1)["num_units"] == 0
    # a request that shares much less is left out when it would lower the keys saved: 320 * 1 > 32 * 2
    pt3 = [row(20, 0), row(20, 1), row(2, 2)]
    p = plan(pt3, [640] * 3, [1] * 3)
    assert p["unit_num_reqs"].tolist() == [2] and p["unit_shared_len"].tolist() == [320] and p["req_unit"].tolist() == [0, 0, -1]


def test_decode_shared_argument_checks():
    lib = B.load()
    n = ctypes.c_size_t(0)
    b = _batch(num_reqs=4, total_new_tokens=4, max_new_len=1)

    def size(batch, **kw):
        sp = B.make_shared_prefix(**kw)
        return lib.emm_decode_attn_shared_workspace_size(ctypes.byref(batch), ctypes.byref(sp), ctypes.byref(n)), n.value

    plain = B.emm_prefill_attn_workspace_size(b)
    st, with_units = size(b, num_units=2)
    assert st == B.EMM_OK and with_units > plain
    assert size(b, num_units=0) == (B.EMM_OK, plain)
    st, tight = size(b, num_units=2, planned_tiles=6, max_own_tiles=1, max_unit_tiles=1)
    assert st == B.EMM_OK and 0 < tight <= with_units
    assert size(b, num_units=3)[0] == B.EMM_ERR_INVALID_ARG
    assert size(b, num_units=-1)[0] == B.EMM_ERR_INVALID_ARG
    assert size(b, num_units=1, planned_tiles=-5)[0] == B.EMM_ERR_INVALID_ARG
    assert size(b, num_units=1, max_own_tiles=-1)[0] == B.EMM_ERR_INVALID_ARG
    assert size(_batch(num_reqs=4, total_new_tokens=8, max_new_len=2), num_units=1)[0] == B.EMM_ERR_INVALID_ARG
    assert size(_batch(num_reqs=4, total_new_tokens=4, max_new_len=1, num_q_heads=34, num_kv_heads=2),
                num_units=1)[0] == B.EMM_ERR_UNSUPPORTED
    sp = B.make_shared_prefix(num_units=1)
    assert lib.emm_decode_attn_shared_workspace_size(ctypes.byref(b), ctypes.byref(sp), None) == B.EMM_ERR_NULL
    assert lib.emm_decode_attn_shared_workspace_size(ctypes.byref(b), None, ctypes.byref(n)) == B.EMM_OK   # no units, no hints
    assert n.value == plain


def test_kv_pages_argument_checks():
    lib = B.load()
    ok_ptr = ctypes.c_void_p(4096)                       # never dereferenced: n == 0 or the checks fail first
    def pack(page_bytes=16384, n=0, k=ok_ptr, staging=ok_ptr, num_pages=8, sums=None):
        return lib.emm_kv_pages_pack(k, ok_ptr, num_pages, page_bytes, ok_ptr, n, staging, sums, None)
    assert pack() == B.EMM_OK                            # nothing to move
    assert pack(page_bytes=100) == B.EMM_ERR_INVALID_ARG
    assert pack(page_bytes=0) == B.EMM_ERR_INVALID_ARG
    assert pack(page_bytes=(1 << 20) + 16) == B.EMM_ERR_INVALID_ARG
    assert pack(n=-1) == B.EMM_ERR_INVALID_ARG
    assert pack(n=1, k=None) == B.EMM_ERR_NULL
    assert pack(n=1, staging=None) == B.EMM_ERR_NULL
    assert pack(n=1, num_pages=0) == B.EMM_ERR_INVALID_ARG
    assert pack(n=1, k=ctypes.c_void_p(4100)) == B.EMM_ERR_INVALID_ARG
    assert pack(n=1, sums=ctypes.c_void_p(4098)) == B.EMM_ERR_INVALID_ARG
    assert lib.emm_kv_pages_unpack(None, ok_ptr, 1, ok_ptr, ok_ptr, 8, 16384, None, None, None, None) == B.EMM_ERR_NULL
    assert lib.emm_kv_pages_unpack(ok_ptr, ok_ptr, 0, ok_ptr, ok_ptr, 8, 16384, None, None, None, None) == B.EMM_OK


def test_decode_step_argument_checks():
    lib = B.load()
    ok_ptr = ctypes.c_void_p(4096)
    b = _batch(num_reqs=4, total_new_tokens=4, max_new_len=1)
    def step(batch=b, k_new=ok_ptr, ws=ok_ptr, ws_bytes=1 << 30, shared=None):
        return lib.emm_decode_step(ctypes.byref(batch), shared, ok_ptr, k_new, ok_ptr, ok_ptr, ok_ptr, ok_ptr, None, ws,
                                   ws_bytes, None)
    # device arrays of the batch are null here, so a call that passes the scalar checks stops at EMM_ERR_NULL
    assert step() == B.EMM_ERR_NULL
    assert step(batch=_batch(num_reqs=4, total_new_tokens=8, max_new_len=2)) == B.EMM_ERR_INVALID_ARG
    assert step(batch=_batch(num_reqs=4, total_new_tokens=4, max_new_len=1, num_q_heads=34, num_kv_heads=2)) == B.EMM_ERR_UNSUPPORTED
    assert step(batch=_batch(num_reqs=4, total_new_tokens=4, max_new_len=1, dtype="f32", head_dim=64)) == B.EMM_ERR_UNSUPPORTED
    assert step(batch=_batch(num_reqs=0, total_new_tokens=0, max_new_len=0)) == B.EMM_OK


def test_descriptors_keep_their_tensors_alive():
    """The descriptors hold raw addresses; a tensor built in the argument list must not be freed under them."""
    import gc
    import weakref

    class _Array:                                   # stands in for a device tensor
        def data_ptr(self):
            return 0x1000

    a = _Array()
    ref = weakref.ref(a)
    batch = _batch(page_table=a)
    shared = B.make_shared_prefix(0, unit_first_req=a)
    del a
    gc.collect()
    assert ref() is not None and batch._keepalive[0] is ref() and shared._keepalive[0] is ref()
    del batch, shared
    gc.collect()
    assert ref() is None
