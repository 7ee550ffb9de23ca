"""ctypes binding of the C-ABI library declared in ``include/emm.h``.

Argument marshalling only: every function has the name and the meaning of the C entry point it
calls, takes torch tensors that live on the GPU (PyTorch is used for device memory and streams,
nothing else), and raises :class:`EmmError` on a non-zero status.  There is no fallback: if
``libemm.so`` has not been built, loading fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
# EMM_LIB_PATH names another build of the same library (the host-sanitized one that tests/test_sanitized_host.py runs)
LIB_PATH = os.environ.get("EMM_LIB_PATH") or os.path.join(HERE, "libemm.so")

EMM_OK, EMM_ERR_NULL, EMM_ERR_INVALID_ARG, EMM_ERR_UNSUPPORTED, EMM_ERR_WORKSPACE, EMM_ERR_LAUNCH = range(6)
EMM_F32, EMM_BF16 = 0, 1
EMM_DECODE_STATIC_SCRATCH_BYTES = 16 << 20
EMM_PREFILL_SHARED_MIN_SAVED_KEY_TILES = 10000

EXPORTS = ["emm_kv_scatter", "emm_prefill_attn_workspace_size", "emm_prefill_attn", "emm_cross_attn", "emm_decode_attn",
           "emm_decode_attn_static", "emm_decode_attn_shared_workspace_size", "emm_decode_attn_shared", "emm_shared_prefix_plan_host",
           "emm_cross_attn_shared", "emm_decode_step", "emm_kv_pages_pack", "emm_kv_pages_unpack",
           "emm_prefill_shared_plan_host", "emm_prefill_attn_shared_workspace_size", "emm_prefill_attn_shared",
           "emm_validate_batch_host", "emm_prefill_plan_host", "emm_status_string", "emm_version"]


class EmmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (where, emm_status_string(status), status))


class emm_batch(ctypes.Structure):
    _fields_ = [("num_reqs", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32),
                ("max_pages_per_req", ctypes.c_int32), ("total_new_tokens", ctypes.c_int32),
                ("max_new_len", ctypes.c_int32), ("dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("reserved", ctypes.c_int32), ("page_table", ctypes.c_void_p), ("prefix_lens", ctypes.c_void_p),
                ("new_lens", ctypes.c_void_p), ("cu_new_lens", ctypes.c_void_p)]


class emm_prefill_plan(ctypes.Structure):
    _fields_ = [("fan", ctypes.c_int32), ("n_row_tiles", ctypes.c_int32), ("pairs_per_xcd", ctypes.c_int32),
                ("cutting", ctypes.c_int32), ("uneven", ctypes.c_int32), ("slots_per_xcd", ctypes.c_int32),
                ("grid", ctypes.c_int64), ("units", ctypes.c_int32 * 8), ("pieces", ctypes.c_int32 * 8),
                ("uneven_k", ctypes.c_int32 * 8), ("rows_only", ctypes.c_int32 * 8)]


class emm_prefill_shared_plan(ctypes.Structure):
    _fields_ = [("num_groups", ctypes.c_int32), ("rows_tiles_plain", ctypes.c_int64), ("rows_tiles_shared", ctypes.c_int64),
                ("key_tiles_plain", ctypes.c_int64), ("key_tiles_shared", ctypes.c_int64),
                ("groups", emm_batch), ("own", emm_batch), ("req_shared_len", ctypes.c_void_p),
                ("group_page_table", ctypes.c_void_p), ("group_prefix_lens", ctypes.c_void_p), ("group_new_lens", ctypes.c_void_p),
                ("group_cu_new_lens", ctypes.c_void_p), ("own_page_table", ctypes.c_void_p), ("own_prefix_lens", ctypes.c_void_p)]


class emm_shared_prefix(ctypes.Structure):
    _fields_ = [("num_units", ctypes.c_int32), ("planned_tiles", ctypes.c_int32),
                ("max_own_tiles", ctypes.c_int32), ("max_unit_tiles", ctypes.c_int32), ("unit_first_req", ctypes.c_void_p),
                ("unit_num_reqs", ctypes.c_void_p), ("unit_shared_len", ctypes.c_void_p), ("req_unit", ctypes.c_void_p),
                ("req_shared_len", ctypes.c_void_p)]


_lib = None


def load() -> ctypes.CDLL:
    """Load ``libemm.so`` (built by ``python -m paper_2507_10069_amd.build``) and declare signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build the HIP library first (python -m paper_2507_10069_amd.build, or "
            "__graft_entry__.build()).  There is no CPU fallback." % LIB_PATH)
    # The device memory and the streams handed to the library come from PyTorch, so the library must
    # bind to the HIP runtime PyTorch has loaded: import torch before dlopen-ing libemm.so.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    bp, vp, i32p = ctypes.POINTER(emm_batch), ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32)
    lib.emm_kv_scatter.restype = ctypes.c_int
    lib.emm_kv_scatter.argtypes = [bp, vp, vp, vp, vp, vp]
    lib.emm_prefill_attn_workspace_size.restype = ctypes.c_int
    lib.emm_prefill_attn_workspace_size.argtypes = [bp, ctypes.POINTER(ctypes.c_size_t)]
    for name in ("emm_prefill_attn", "emm_cross_attn", "emm_decode_attn"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [bp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.emm_decode_attn_static.restype = ctypes.c_int
    lib.emm_decode_attn_static.argtypes = [bp, vp, vp, vp, vp, vp, vp]
    lib.emm_decode_attn_shared_workspace_size.restype = ctypes.c_int
    lib.emm_decode_attn_shared_workspace_size.argtypes = [bp, ctypes.POINTER(emm_shared_prefix), ctypes.POINTER(ctypes.c_size_t)]
    lib.emm_decode_attn_shared.restype = ctypes.c_int
    lib.emm_decode_attn_shared.argtypes = [bp, ctypes.POINTER(emm_shared_prefix), vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.emm_shared_prefix_plan_host.restype = ctypes.c_int
    lib.emm_shared_prefix_plan_host.argtypes = [bp, i32p, i32p, i32p, ctypes.c_int32] + [i32p] * 5 + [ctypes.POINTER(emm_shared_prefix)]
    lib.emm_cross_attn_shared.restype = ctypes.c_int
    lib.emm_cross_attn_shared.argtypes = lib.emm_decode_attn_shared.argtypes
    lib.emm_decode_step.restype = ctypes.c_int
    lib.emm_decode_step.argtypes = [bp, ctypes.POINTER(emm_shared_prefix)] + [vp] * 8 + [ctypes.c_size_t, vp]
    lib.emm_prefill_shared_plan_host.restype = ctypes.c_int
    lib.emm_prefill_shared_plan_host.argtypes = [bp, i32p, i32p, i32p, i32p, ctypes.c_int32, ctypes.c_int64,
                                                 ctypes.POINTER(emm_prefill_shared_plan)]
    lib.emm_prefill_attn_shared_workspace_size.restype = ctypes.c_int
    lib.emm_prefill_attn_shared_workspace_size.argtypes = [bp, bp, ctypes.POINTER(ctypes.c_size_t)]
    lib.emm_prefill_attn_shared.restype = ctypes.c_int
    lib.emm_prefill_attn_shared.argtypes = [bp, bp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.emm_kv_pages_pack.restype = ctypes.c_int
    lib.emm_kv_pages_pack.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int64, vp, ctypes.c_int32, vp, vp, vp]
    lib.emm_kv_pages_unpack.restype = ctypes.c_int
    lib.emm_kv_pages_unpack.argtypes = [vp, vp, ctypes.c_int32, vp, vp, ctypes.c_int32, ctypes.c_int64, vp, vp, vp, vp]
    lib.emm_validate_batch_host.restype = ctypes.c_int
    lib.emm_validate_batch_host.argtypes = [bp, i32p, i32p, i32p, i32p, ctypes.c_int]
    lib.emm_prefill_plan_host.restype = ctypes.c_int
    lib.emm_prefill_plan_host.argtypes = [bp, i32p, ctypes.c_int, ctypes.POINTER(emm_prefill_plan)]
    lib.emm_status_string.restype = ctypes.c_char_p
    lib.emm_status_string.argtypes = [ctypes.c_int]
    lib.emm_version.restype = ctypes.c_int
    lib.emm_version.argtypes = []
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    return int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    handle = int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)
    return handle or None


def make_batch(*, num_reqs, num_q_heads, num_kv_heads, head_dim, page_size, num_pages, max_pages_per_req,
               total_new_tokens, max_new_len, dtype, softmax_scale, page_table=None, prefix_lens=None,
               new_lens=None, cu_new_lens=None) -> emm_batch:
    """Fill the descriptor; the four arrays are int32 device tensors (or None for host-only calls).

    The descriptor holds raw device addresses, so the returned object also keeps the four tensors alive: a
    tensor created in the call's argument list would otherwise be freed, and its memory handed to the next
    allocation, before the kernels that read it have run."""
    code = {"f32": EMM_F32, "bf16": EMM_BF16}.get(dtype, dtype)
    batch = emm_batch(num_reqs, num_q_heads, num_kv_heads, head_dim, page_size, num_pages, max_pages_per_req,
                      total_new_tokens, max_new_len, code, float(softmax_scale), 0,
                      _ptr(page_table), _ptr(prefix_lens), _ptr(new_lens), _ptr(cu_new_lens))
    batch._keepalive = (page_table, prefix_lens, new_lens, cu_new_lens)
    return batch


def emm_prefill_plan_host(batch: emm_batch, new_lens, with_workspace: bool = True) -> dict:
    """new_lens: host int32 array.  Returns the plan's fields, the per-XCD ones as lists of 8."""
    nl = np.ascontiguousarray(new_lens, dtype=np.int32)
    plan = emm_prefill_plan()
    st = load().emm_prefill_plan_host(ctypes.byref(batch), nl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                      int(with_workspace), ctypes.byref(plan))
    if st != EMM_OK:
        raise EmmError(st, "emm_prefill_plan_host")
    out = {k: int(getattr(plan, k)) for k in ("fan", "n_row_tiles", "pairs_per_xcd", "cutting", "uneven", "slots_per_xcd", "grid")}
    out.update({k: list(getattr(plan, k)) for k in ("units", "pieces", "uneven_k", "rows_only")})
    return out


def _check(status: int, where: str) -> None:
    if status != EMM_OK:
        raise EmmError(status, where)


def emm_status_string(status: int) -> str:
    return load().emm_status_string(int(status)).decode()


def emm_version() -> int:
    return int(load().emm_version())


def emm_kv_scatter(batch: emm_batch, k_new, v_new, k_cache, v_cache, stream=None) -> None:
    _check(load().emm_kv_scatter(ctypes.byref(batch), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                 _stream(stream)), "emm_kv_scatter")


def emm_prefill_attn_workspace_size(batch: emm_batch) -> int:
    n = ctypes.c_size_t(0)
    _check(load().emm_prefill_attn_workspace_size(ctypes.byref(batch), ctypes.byref(n)),
           "emm_prefill_attn_workspace_size")
    return int(n.value)


def _attn(name: str, batch, q, k_cache, v_cache, out, lse, workspace, stream) -> None:
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    _check(getattr(load(), name)(ctypes.byref(batch), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out),
                                 _ptr(lse), _ptr(workspace), ws_bytes, _stream(stream)), name)


def emm_prefill_attn(batch: emm_batch, q, k_cache, v_cache, out, lse=None, workspace=None, stream=None) -> None:
    _attn("emm_prefill_attn", batch, q, k_cache, v_cache, out, lse, workspace, stream)


def emm_cross_attn(batch: emm_batch, q, k_cache, v_cache, out, lse=None, workspace=None, stream=None) -> None:
    _attn("emm_cross_attn", batch, q, k_cache, v_cache, out, lse, workspace, stream)


def emm_decode_attn(batch: emm_batch, q, k_cache, v_cache, out, lse=None, workspace=None, stream=None) -> None:
    _attn("emm_decode_attn", batch, q, k_cache, v_cache, out, lse, workspace, stream)


def emm_decode_attn_static(batch: emm_batch, q, k_cache, v_cache, out, lse=None, stream=None) -> None:
    _check(load().emm_decode_attn_static(ctypes.byref(batch), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out),
                                         _ptr(lse), _stream(stream)), "emm_decode_attn_static")


def emm_decode_attn_shared_workspace_size(batch: emm_batch, shared: emm_shared_prefix) -> int:
    n = ctypes.c_size_t(0)
    _check(load().emm_decode_attn_shared_workspace_size(ctypes.byref(batch), ctypes.byref(shared), ctypes.byref(n)),
           "emm_decode_attn_shared_workspace_size")
    return int(n.value)


def make_shared_prefix(num_units: int, unit_first_req=None, unit_num_reqs=None, unit_shared_len=None, req_unit=None,
                       req_shared_len=None, planned_tiles: int = 0, max_own_tiles: int = 0,
                       max_unit_tiles: int = 0) -> emm_shared_prefix:
    """Fill the descriptor; the five arrays are int32 device tensors, which the returned object keeps alive (it
    holds their addresses only)."""
    shared = emm_shared_prefix(num_units, planned_tiles, max_own_tiles, max_unit_tiles, _ptr(unit_first_req),
                               _ptr(unit_num_reqs), _ptr(unit_shared_len), _ptr(req_unit), _ptr(req_shared_len))
    shared._keepalive = (unit_first_req, unit_num_reqs, unit_shared_len, req_unit, req_shared_len)
    return shared


def emm_decode_attn_shared(batch: emm_batch, shared: emm_shared_prefix, q, k_cache, v_cache, out, lse=None,
                           workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    _check(load().emm_decode_attn_shared(ctypes.byref(batch), ctypes.byref(shared), _ptr(q), _ptr(k_cache),
                                         _ptr(v_cache), _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes,
                                         _stream(stream)), "emm_decode_attn_shared")


def emm_cross_attn_shared(batch: emm_batch, shared: emm_shared_prefix, q, k_cache, v_cache, out, lse=None,
                          workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    _check(load().emm_cross_attn_shared(ctypes.byref(batch), ctypes.byref(shared), _ptr(q), _ptr(k_cache),
                                        _ptr(v_cache), _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes,
                                        _stream(stream)), "emm_cross_attn_shared")


def emm_decode_step(batch: emm_batch, shared: Optional[emm_shared_prefix], q, k_new, v_new, k_cache, v_cache, out, lse=None,
                    workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    _check(load().emm_decode_step(ctypes.byref(batch), ctypes.byref(shared) if shared is not None else None, _ptr(q),
                                  _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), _ptr(out), _ptr(lse),
                                  _ptr(workspace), ws_bytes, _stream(stream)), "emm_decode_step")


def emm_shared_prefix_plan_host(batch: emm_batch, page_table: np.ndarray, prefix_lens: np.ndarray,
                                new_lens: np.ndarray, min_shared_tokens: int = 32) -> dict:
    """Returns the units as host int32 arrays: unit_first_req, unit_num_reqs, unit_shared_len (length U),
    req_unit, req_shared_len (length B), and the four scalars of the descriptor."""
    i32p = ctypes.POINTER(ctypes.c_int32)
    ins = [np.ascontiguousarray(a, dtype=np.int32) for a in (page_table, prefix_lens, new_lens)]
    B_ = int(batch.num_reqs)
    outs = [np.zeros(max(B_ // 2, 1), dtype=np.int32) for _ in range(3)] + [np.zeros(max(B_, 1), dtype=np.int32) for _ in range(2)]
    sp = emm_shared_prefix()
    _check(load().emm_shared_prefix_plan_host(ctypes.byref(batch), *[a.ctypes.data_as(i32p) for a in ins],
                                              min_shared_tokens, *[a.ctypes.data_as(i32p) for a in outs],
                                              ctypes.byref(sp)), "emm_shared_prefix_plan_host")
    U = int(sp.num_units)
    return {"num_units": U, "planned_tiles": int(sp.planned_tiles), "max_own_tiles": int(sp.max_own_tiles),
            "max_unit_tiles": int(sp.max_unit_tiles), "unit_first_req": outs[0][:U], "unit_num_reqs": outs[1][:U], "unit_shared_len": outs[2][:U],
            "req_unit": outs[3][:B_], "req_shared_len": outs[4][:B_]}


def emm_prefill_shared_plan_host(batch: emm_batch, page_table: np.ndarray, prefix_lens: np.ndarray, new_lens: np.ndarray,
                                 cu_new_lens: np.ndarray, min_shared_tokens: int = 64, min_saved_key_tiles: int = -1) -> dict:
    """Returns the plan's host arrays (cut to the number of groups), its counts and the two descriptors with their
    scalar fields filled (array pointers unset).  min_saved_key_tiles: 0 keeps every group that saves a row tile,
    negative stands for the library's default threshold."""
    i32p = ctypes.POINTER(ctypes.c_int32)
    ins = [np.ascontiguousarray(a, dtype=np.int32) for a in (page_table, prefix_lens, new_lens, cu_new_lens)]
    B_, mp = int(batch.num_reqs), int(batch.max_pages_per_req)
    half = max(B_ // 2, 1)
    arr = {"req_shared_len": np.zeros(max(B_, 1), np.int32), "group_page_table": np.full((half, max(mp, 1)), -1, np.int32),
           "group_prefix_lens": np.zeros(half, np.int32), "group_new_lens": np.zeros(half, np.int32),
           "group_cu_new_lens": np.zeros(half + 1, np.int32), "own_page_table": np.full((max(B_, 1), max(mp, 1)), -1, np.int32),
           "own_prefix_lens": np.zeros(max(B_, 1), np.int32)}
    plan = emm_prefill_shared_plan()
    for k, a in arr.items():
        setattr(plan, k, a.ctypes.data)
    _check(load().emm_prefill_shared_plan_host(ctypes.byref(batch), *[a.ctypes.data_as(i32p) for a in ins], min_shared_tokens,
                                               min_saved_key_tiles, ctypes.byref(plan)), "emm_prefill_shared_plan_host")
    NG = int(plan.num_groups)
    wg, wo = max(int(plan.groups.max_pages_per_req), 1), max(int(plan.own.max_pages_per_req), 1)
    arr["group_page_table"] = arr["group_page_table"].reshape(-1)[:half * wg].reshape(half, wg)
    arr["own_page_table"] = arr["own_page_table"].reshape(-1)[:max(B_, 1) * wo].reshape(max(B_, 1), wo)
    out = {"num_groups": NG, "rows_tiles_plain": int(plan.rows_tiles_plain), "rows_tiles_shared": int(plan.rows_tiles_shared),
           "key_tiles_plain": int(plan.key_tiles_plain), "key_tiles_shared": int(plan.key_tiles_shared),
           "req_shared_len": arr["req_shared_len"][:B_], "group_page_table": arr["group_page_table"][:max(NG, 1)],
           "group_prefix_lens": arr["group_prefix_lens"][:max(NG, 1)], "group_new_lens": arr["group_new_lens"][:max(NG, 1)],
           "group_cu_new_lens": arr["group_cu_new_lens"][:max(NG, 1) + 1], "own_page_table": arr["own_page_table"][:B_],
           "own_prefix_lens": arr["own_prefix_lens"][:B_]}
    groups, own = emm_batch(), emm_batch()
    ctypes.memmove(ctypes.byref(groups), ctypes.byref(plan.groups), ctypes.sizeof(emm_batch))
    ctypes.memmove(ctypes.byref(own), ctypes.byref(plan.own), ctypes.sizeof(emm_batch))
    out["groups"], out["own"] = groups, own
    return out


def emm_prefill_attn_shared_workspace_size(groups: emm_batch, own: emm_batch) -> int:
    n = ctypes.c_size_t(0)
    _check(load().emm_prefill_attn_shared_workspace_size(ctypes.byref(groups), ctypes.byref(own), ctypes.byref(n)),
           "emm_prefill_attn_shared_workspace_size")
    return int(n.value)


def emm_prefill_attn_shared(groups: emm_batch, own: emm_batch, req_shared_len, q, k_cache, v_cache, out, lse=None,
                            workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else int(workspace.numel() * workspace.element_size())
    _check(load().emm_prefill_attn_shared(ctypes.byref(groups), ctypes.byref(own), _ptr(req_shared_len), _ptr(q), _ptr(k_cache),
                                          _ptr(v_cache), _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes, _stream(stream)),
           "emm_prefill_attn_shared")


def emm_kv_pages_pack(k_cache, v_cache, num_pages: int, page_bytes: int, page_ids, n: int, staging, checksums=None,
                      stream=None) -> None:
    _check(load().emm_kv_pages_pack(_ptr(k_cache), _ptr(v_cache), num_pages, page_bytes, _ptr(page_ids), n,
                                    _ptr(staging), _ptr(checksums), _stream(stream)), "emm_kv_pages_pack")


def emm_kv_pages_unpack(staging, page_ids, n: int, k_cache, v_cache, num_pages: int, page_bytes: int, checksums=None,
                        expected=None, mismatches=None, stream=None) -> None:
    _check(load().emm_kv_pages_unpack(_ptr(staging), _ptr(page_ids), n, _ptr(k_cache), _ptr(v_cache), num_pages,
                                      page_bytes, _ptr(checksums), _ptr(expected), _ptr(mismatches), _stream(stream)),
           "emm_kv_pages_unpack")


def emm_validate_batch_host(batch: emm_batch, page_table: np.ndarray, prefix_lens: np.ndarray,
                            new_lens: np.ndarray, cu_new_lens: np.ndarray, causal: bool) -> int:
    """Returns the status instead of raising: it is a checker."""
    i32p = ctypes.POINTER(ctypes.c_int32)
    arrs = [np.ascontiguousarray(a, dtype=np.int32) for a in (page_table, prefix_lens, new_lens, cu_new_lens)]
    return int(load().emm_validate_batch_host(ctypes.byref(batch), *[a.ctypes.data_as(i32p) for a in arrs],
                                              1 if causal else 0))


# ---------------------------------------------------------------------------------------------
# Moving a host workload (paper_2507_10069_amd.workloads.Workload) to the device.
# ---------------------------------------------------------------------------------------------
class DeviceWorkload:
    """Device copies of a workload's tensors plus the filled descriptor."""

    def __init__(self, wl, device="cuda:0"):
        import torch
        self.wl = wl
        self.device = torch.device(device)

        def dev(a):
            if a is None:
                return None
            if a.dtype == np.uint16:
                return torch.from_numpy(a.view(np.int16)).to(self.device).view(torch.bfloat16)
            return torch.from_numpy(a).to(self.device)

        self.page_table = dev(wl.page_table)
        self.prefix_lens = dev(wl.prefix_lens)
        self.new_lens = dev(wl.new_lens)
        self.cu_new_lens = dev(wl.cu_new_lens)
        self.q = dev(wl.q)
        self.k_new = dev(wl.k_new)
        self.v_new = dev(wl.v_new)
        self.k_cache = dev(wl.k_cache)
        self.v_cache = dev(wl.v_cache)
        self.out = torch.empty_like(self.q)
        self.lse = torch.empty((wl.total_new_tokens, wl.num_q_heads), dtype=torch.float32, device=self.device)
        self.batch = make_batch(num_reqs=wl.num_reqs, num_q_heads=wl.num_q_heads, num_kv_heads=wl.num_kv_heads,
                                head_dim=wl.head_dim, page_size=wl.page_size, num_pages=wl.num_pages,
                                max_pages_per_req=wl.max_pages_per_req, total_new_tokens=wl.total_new_tokens,
                                max_new_len=wl.max_new_len, dtype=wl.dtype, softmax_scale=wl.softmax_scale,
                                page_table=self.page_table, prefix_lens=self.prefix_lens,
                                new_lens=self.new_lens, cu_new_lens=self.cu_new_lens)
        ws = emm_prefill_attn_workspace_size(self.batch)
        self.workspace = torch.empty(max(ws, 16), dtype=torch.uint8, device=self.device) if ws else None

    def scatter(self, stream=None) -> None:
        if self.wl.kind == "causal":
            emm_kv_scatter(self.batch, self.k_new, self.v_new, self.k_cache, self.v_cache, stream)

    def attention(self, stream=None) -> None:
        fn = emm_prefill_attn if self.wl.kind == "causal" else emm_cross_attn
        fn(self.batch, self.q, self.k_cache, self.v_cache, self.out, self.lse, self.workspace, stream)

    def plan_shared(self, min_shared_tokens: int = 32, use_hint: bool = True) -> dict:
        """Find the shared-prefix units of a decode batch (host) and move them to the device."""
        import torch
        wl = self.wl
        plan = emm_shared_prefix_plan_host(self.batch, wl.page_table, wl.prefix_lens, wl.new_lens, min_shared_tokens)
        self.shared_arrays = {k: torch.from_numpy(np.ascontiguousarray(v if len(v) else np.zeros(1, np.int32))).to(self.device)
                              for k, v in plan.items() if isinstance(v, np.ndarray)}
        scalars = {k: plan[k] for k in ("planned_tiles", "max_own_tiles", "max_unit_tiles")} if use_hint else {}
        self.shared = make_shared_prefix(plan["num_units"], **scalars, **self.shared_arrays)
        ws = emm_decode_attn_shared_workspace_size(self.batch, self.shared)
        self.shared_workspace = torch.empty(max(ws, 16), dtype=torch.uint8, device=self.device)
        self.shared_plan = plan
        return plan

    def plan_prefill_shared(self, min_shared_tokens: int = 64, min_saved_key_tiles: int = -1) -> dict:
        """Find the sharing groups of a prefill batch (host), move what the two passes need to the device and finish
        the two descriptors."""
        import torch
        wl = self.wl
        plan = emm_prefill_shared_plan_host(self.batch, wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens, min_shared_tokens,
                                            min_saved_key_tiles)
        dev = {k: torch.from_numpy(np.ascontiguousarray(v)).to(self.device) for k, v in plan.items() if isinstance(v, np.ndarray)}
        groups, own = plan["groups"], plan["own"]
        groups.page_table, groups.prefix_lens = _ptr(dev["group_page_table"]), _ptr(dev["group_prefix_lens"])
        groups.new_lens, groups.cu_new_lens = _ptr(dev["group_new_lens"]), _ptr(dev["group_cu_new_lens"])
        own.page_table, own.prefix_lens = _ptr(dev["own_page_table"]), _ptr(dev["own_prefix_lens"])
        own.new_lens, own.cu_new_lens = _ptr(self.new_lens), _ptr(self.cu_new_lens)
        self.prefill_shared = {"plan": plan, "dev": dev, "groups": groups, "own": own}
        ws = emm_prefill_attn_shared_workspace_size(groups, own)
        self.prefill_shared["workspace"] = torch.empty(max(ws, 256), dtype=torch.uint8, device=self.device)
        return plan

    def attention_prefill_shared(self, stream=None) -> None:
        ps = self.prefill_shared
        emm_prefill_attn_shared(ps["groups"], ps["own"], ps["dev"]["req_shared_len"], self.q, self.k_cache, self.v_cache,
                                self.out, self.lse, ps["workspace"], stream)

    def decode_step(self, shared: bool = False, stream=None) -> None:
        """Scatter + decode attention in one call (emm_decode_step), with the planned units or without."""
        emm_decode_step(self.batch, self.shared if shared else None, self.q, self.k_new, self.v_new, self.k_cache,
                        self.v_cache, self.out, self.lse, self.shared_workspace if shared else self.workspace, stream)

    def attention_shared(self, stream=None) -> None:
        fn = emm_decode_attn_shared if self.wl.kind == "causal" else emm_cross_attn_shared
        fn(self.batch, self.shared, self.q, self.k_cache, self.v_cache, self.out, self.lse,
                               self.shared_workspace, stream)

    def step(self, stream=None) -> None:
        """One pass of the hot path: scatter the new K/V, then attention."""
        self.scatter(stream)
        self.attention(stream)

    @staticmethod
    def to_numpy_bits(t) -> np.ndarray:
        """Device tensor -> host numpy array in the workload's storage form."""
        import torch
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()
