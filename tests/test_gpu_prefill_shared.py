"""GPU parity of prefill with shared prefixes (Section 3.3: requests of a batch that hold the same cached pages):
emm_prefill_attn_shared, through the C ABI, against the fp64 CPU oracle, which knows nothing of sharing: it attends
every request over its own page table.  Same bars as the plain prefill path; the merge of the two parts rounds the
outputs once more to bf16, which the bars have room for."""
import ctypes

import numpy as np
import pytest
import torch

from helpers import as_f64
from paper_2507_10069_amd import binding as B
from paper_2507_10069_amd import workloads as W
from test_gpu_parity import _compare, _plant_key, _sample_tokens

pytestmark = pytest.mark.gpu


def _run_shared(wl, min_shared_tokens=64):
    dw = B.DeviceWorkload(wl)
    plan = dw.plan_prefill_shared(min_shared_tokens, min_saved_key_tiles=0)        # every group that saves a row tile
    dw.out.zero_()
    dw.lse.zero_()
    dw.scatter()
    dw.attention_prefill_shared()
    torch.cuda.synchronize()
    return dw, plan


def _case(prefix, new, group, shared, H=28, Hkv=4, ps=16, seed=31):
    return W.build_workload("case", "causal", "bf16", seed, num_q_heads=H, num_kv_heads=Hkv, head_dim=128, page_size=ps,
                            prefix_lens=prefix, new_lens=new, share_group=group, shared_len=shared)


@pytest.mark.parametrize("name", W.PREFILL_SHARED_CONFIGS)
def test_named_workloads_elementwise(name):
    print("case %s shrink 8" % name, flush=True)
    wl = W.prefill_shared_config(name, 8)
    dw, plan = _run_shared(wl)
    assert plan["num_groups"] > 0
    print("   groups %d, row tiles %d -> %d, errors (max, mean, lse):" % (plan["num_groups"], plan["rows_tiles_plain"],
                                                                          plan["rows_tiles_shared"]), _compare(wl, dw), flush=True)


@pytest.mark.parametrize("name", W.PREFILL_SHARED_CONFIGS)
def test_named_workloads_full_size_sampled(name):
    print("case %s full size" % name, flush=True)
    wl = W.prefill_shared_config(name, 1)
    dw, plan = _run_shared(wl)
    assert plan["num_groups"] > 0
    tokens = _sample_tokens(wl, 24, seed=5)
    print("   errors (max, mean, lse):", _compare(wl, dw, tokens), flush=True)
    # and the plain path on the same batch: two routes to the same numbers
    shared_out = as_f64(B.DeviceWorkload.to_numpy_bits(dw.out))
    shared_lse = dw.lse.cpu().numpy()
    dw.out.zero_()
    dw.attention()
    torch.cuda.synchronize()
    plain_out = as_f64(B.DeviceWorkload.to_numpy_bits(dw.out))
    assert np.abs(shared_out - plain_out).max() <= 2e-2
    assert np.abs(shared_lse - dw.lse.cpu().numpy()).max() <= 8e-3


MIXED = [
    # members and requests on their own, a request without new tokens, one whose own cached part is empty, groups of
    # different shared lengths, a group of two
    ("mixed_28_4", 28, 4, [1100, 1056, 1056, 1200, 300, 0, 2048, 2048, 2048 + 7, 640, 640],
     [4, 6, 3, 5, 40, 9, 8, 8, 1, 0, 5], [0, 0, 0, 0, 1, 2, 3, 3, 3, 4, 4], [1056] * 4 + [0, 0] + [2048] * 3 + [640] * 2),
    # one query head per KV head: 256 tokens fill a tile
    ("mha_8_8", 8, 8, [512 + 16 * i for i in range(6)], [30, 17, 64, 1, 90, 12], [0] * 6, [512] * 6),
    # a group whose packed rows span several tiles with a ragged tail: 5 x 50 tokens x 4 heads = 1000 rows
    ("several_tiles_32_8", 32, 8, [1280 + 3 * i for i in range(5)], [50] * 5, [0] * 5, [1280] * 5),
    # a long shared part with very few rows: cut along the keys in both passes
    ("long_shared_few_rows", 28, 4, [8192 + 100, 8192 + 900, 8192], [2, 3, 1], [0] * 3, [8192] * 3),
    # shared part exactly one key tile
    ("one_tile_shared", 28, 4, [64, 64 + 50, 64 + 500], [10, 10, 10], [0] * 3, [64] * 3),
]


@pytest.mark.parametrize("name,H,Hkv,prefix,new,group,shared", MIXED)
def test_mixed_batches_elementwise(name, H, Hkv, prefix, new, group, shared):
    print("case %s" % name, flush=True)
    wl = _case(prefix, new, group, shared, H=H, Hkv=Hkv)
    dw, plan = _run_shared(wl)
    assert plan["num_groups"] > 0
    print("   groups %d, shared lengths %s, errors (max, mean, lse):" % (plan["num_groups"], plan["req_shared_len"].tolist()),
          _compare(wl, dw), flush=True)


@pytest.mark.parametrize("ps", [32, 64, 128, 256])
def test_page_sizes(ps):
    print("case page size %d" % ps, flush=True)
    wl = _case([1536 + 40, 1536, 1536 + 300, 200], [7, 2, 11, 30], [0, 0, 0, 1], [1536] * 3 + [0], ps=ps, seed=40 + ps)
    dw, plan = _run_shared(wl)
    assert plan["num_groups"] == 1
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)


@pytest.mark.parametrize("seed", range(8))
def test_random_batches_elementwise(seed):
    """Random groups, lengths, head counts and page sizes; requests outside any group and requests without new tokens
    mixed in; a member whose cached part ends inside the group's shared pages."""
    rng = np.random.default_rng(1000 + seed)
    ps = int(rng.choice([16, 32, 64]))
    H, Hkv = [(28, 4), (32, 8), (8, 8), (16, 2), (4, 1)][seed % 5]
    n = int(rng.integers(3, 11))
    group = sorted(int(g) for g in rng.integers(0, max(2, n // 2), size=n))
    shared_of = {g: int(rng.integers(1, 24)) * 64 for g in set(group)}
    shared = [shared_of[g] for g in group]
    prefix = [s_ + int(rng.integers(0, 150)) for s_ in shared]
    new = [int(rng.integers(1, 30)) for _ in range(n)]
    if n > 4:
        new[int(rng.integers(0, n))] = 0
        k = int(rng.integers(0, n))
        prefix[k] = int(rng.integers(shared[k] // 2, shared[k] + 1))
    print("case seed %d: ps %d, heads %d/%d, groups %s, shared %s, prefix %s, new %s" % (seed, ps, H, Hkv, group, shared, prefix, new), flush=True)
    wl = _case(prefix, new, group, shared, H=H, Hkv=Hkv, ps=ps, seed=2000 + seed)
    dw, plan = _run_shared(wl)
    print("   groups %d, shared lengths %s, errors (max, mean, lse):" % (plan["num_groups"], plan["req_shared_len"].tolist()),
          _compare(wl, dw), flush=True)


def test_a_batch_without_groups_equals_the_plain_path_bitwise():
    wl = _case([700, 64, 0], [20, 3, 45], None, None)
    dw, plan = _run_shared(wl)
    assert plan["num_groups"] == 0
    out = B.DeviceWorkload.to_numpy_bits(dw.out).copy()
    lse = dw.lse.cpu().numpy().copy()
    dw.out.zero_()
    dw.attention()
    torch.cuda.synchronize()
    assert out.tobytes() == B.DeviceWorkload.to_numpy_bits(dw.out).tobytes()
    assert lse.tobytes() == dw.lse.cpu().numpy().tobytes()
    _compare(wl, dw)


@pytest.mark.parametrize("where", ["shared", "own"])
def test_one_part_far_above_the_other(where):
    """A key whose score towers over all others sits in the shared part, or in a request's own part: the merge then
    gives the other part a weight that rounds to nothing."""
    print("case planted in %s part" % where, flush=True)
    wl = _case([2048 + 300] * 4, [6, 6, 6, 6], [0] * 4, [2048] * 4, seed=77)
    pos = 1000 if where == "shared" else 2048 + 150
    for r in range(4 if where == "shared" else 2):
        _plant_key(wl, r, pos, 6.0)
        if where == "shared":
            break                                            # one physical page: planting it once plants it for all
    dw, plan = _run_shared(wl)
    assert plan["num_groups"] == 1
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)


def test_without_lse_and_repeated_calls_are_deterministic():
    wl = W.prefill_shared_config("prefill_shared_image_b32", 8)
    dw, plan = _run_shared(wl)
    first = B.DeviceWorkload.to_numpy_bits(dw.out).copy()
    ps = dw.prefill_shared
    dw.out.zero_()
    ps["workspace"].fill_(0xA5)                              # what an earlier call left behind must not matter
    B.emm_prefill_attn_shared(ps["groups"], ps["own"], ps["dev"]["req_shared_len"], dw.q, dw.k_cache, dw.v_cache, dw.out, None,
                              ps["workspace"])
    torch.cuda.synchronize()
    assert first.tobytes() == B.DeviceWorkload.to_numpy_bits(dw.out).tobytes()


def test_the_three_steps_can_be_captured_in_a_hip_graph_and_replayed():
    """emm_prefill_attn_shared only launches kernels on the given stream, so the step (scatter, then the grouped
    attention) can be captured in a HIP graph; every replay, with eager work between the replays, reproduces the
    eager result bit for bit."""
    print("case graph capture", flush=True)
    bits = B.DeviceWorkload.to_numpy_bits
    wl = _case([2048 + 90, 2048, 2048 + 700, 300, 1024, 1024 + 33], [6, 9, 2, 40, 11, 7], [0, 0, 0, 1, 2, 2], [2048] * 3 + [0] + [1024] * 2,
               seed=91)
    eager, plan = _run_shared(wl)
    assert plan["num_groups"] == 2
    want_out, want_lse, want_k = bits(eager.out).tobytes(), eager.lse.cpu().numpy().tobytes(), bits(eager.k_cache).tobytes()
    dw = B.DeviceWorkload(wl)
    dw.plan_prefill_shared(min_saved_key_tiles=0)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        dw.scatter()
        dw.attention_prefill_shared()                    # warm up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            dw.scatter()
            dw.attention_prefill_shared()
    for replay in range(3):
        dw.out.zero_()                                   # eager work and a synchronisation between the replays
        dw.lse.zero_()
        dw.prefill_shared["workspace"].fill_(0x5A)       # stale workspace contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert bits(dw.out).tobytes() == want_out, replay
        assert dw.lse.cpu().numpy().tobytes() == want_lse, replay
        assert bits(dw.k_cache).tobytes() == want_k, replay
    _compare(wl, dw)


def test_error_codes():
    wl = W.prefill_shared_config("prefill_shared_video_b8_n12", 16)
    dw = B.DeviceWorkload(wl)
    dw.plan_prefill_shared(min_saved_key_tiles=0)
    dw.scatter()
    ps = dw.prefill_shared
    lib = B.load()
    need = B.emm_prefill_attn_shared_workspace_size(ps["groups"], ps["own"])
    args = (ctypes.byref(ps["groups"]), ctypes.byref(ps["own"]), B._ptr(ps["dev"]["req_shared_len"]), B._ptr(dw.q), B._ptr(dw.k_cache),
            B._ptr(dw.v_cache), B._ptr(dw.out), B._ptr(dw.lse))
    assert lib.emm_prefill_attn_shared(*args, B._ptr(ps["workspace"]), need - 1, None) == B.EMM_ERR_WORKSPACE
    assert lib.emm_prefill_attn_shared(*args, None, need, None) == B.EMM_ERR_NULL
    assert lib.emm_prefill_attn_shared(*args, B._ptr(ps["workspace"]) + 16, need, None) == B.EMM_ERR_INVALID_ARG
    no_len = args[:2] + (None,) + args[3:]
    assert lib.emm_prefill_attn_shared(*no_len, B._ptr(ps["workspace"]), need, None) == B.EMM_ERR_NULL
    assert lib.emm_prefill_attn_shared(*args, B._ptr(ps["workspace"]), need, None) == B.EMM_OK
    torch.cuda.synchronize()
    _compare(wl, dw)
