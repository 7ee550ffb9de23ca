"""emm_decode_attn_static (the decode step for callers that cannot allocate: piece records in the library's own
fixed device array) against emm_decode_attn with a caller's workspace, through the C ABI: same output bits and
same lse bits on two calls in a row, the second on a smaller batch (which finds the first call's records still in
the array), and both within the oracle's bars.  Collected last: the other GPU tests do not depend on it."""
import numpy as np
import pytest
import torch

import oracle
from helpers import as_f64, err_stats
from paper_2507_10069_amd import binding as B
from paper_2507_10069_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_MAX_ABS, BF16_MEAN_ABS, LSE_ABS = 2e-2, 2e-3, 4e-3


def _run_both(wl):
    bits = B.DeviceWorkload.to_numpy_bits
    dw = B.DeviceWorkload(wl)
    dw.scatter()
    need = B.emm_prefill_attn_workspace_size(dw.batch)
    assert 0 < need <= B.EMM_DECODE_STATIC_SCRATCH_BYTES
    # the existing entry point, with a workspace the caller allocated
    dw.out.zero_()
    dw.lse.zero_()
    B.emm_decode_attn(dw.batch, dw.q, dw.k_cache, dw.v_cache, dw.out, dw.lse, dw.workspace)
    torch.cuda.synchronize()
    want_out, want_lse = bits(dw.out).copy(), dw.lse.cpu().numpy().copy()
    # the allocation-free one: no workspace argument at all
    dw.out.zero_()
    dw.lse.zero_()
    B.emm_decode_attn_static(dw.batch, dw.q, dw.k_cache, dw.v_cache, dw.out, dw.lse)
    torch.cuda.synchronize()
    got_out, got_lse = bits(dw.out), dw.lse.cpu().numpy()
    assert got_out.tobytes() == want_out.tobytes(), "outputs differ from emm_decode_attn's"
    assert got_lse.tobytes() == want_lse.tobytes(), "lse differs from emm_decode_attn's"
    # and against the oracle, to the bars of the other parity tests
    _, _, out_ref, lse_ref = oracle.run_workload(wl)
    mx, mean = err_stats(as_f64(got_out), out_ref)
    assert mx <= BF16_MAX_ABS and mean <= BF16_MEAN_ABS, (mx, mean)
    finite = np.isfinite(lse_ref)
    assert float(np.abs(got_lse.astype(np.float64)[finite] - lse_ref[finite]).max()) <= LSE_ABS
    return mx, mean


def test_static_scratch_decode_twice_second_smaller():
    print("case no-alloc decode: 6 requests, up to 20000 tokens, several pieces each", flush=True)
    big = W.build_workload("noalloc_big", "causal", "bf16", 3100, num_q_heads=28, num_kv_heads=4, head_dim=128,
                           page_size=16, prefix_lens=[20000, 18431, 3, 7000, 0, 9000], new_lens=[1, 1, 1, 1, 1, 1])
    print("   errors (max, mean):", _run_both(big), flush=True)
    print("case no-alloc decode: 2 requests, shorter contexts, same array", flush=True)
    small = W.build_workload("noalloc_small", "causal", "bf16", 3101, num_q_heads=28, num_kv_heads=4, head_dim=128,
                             page_size=16, prefix_lens=[2500, 640], new_lens=[1, 1])
    print("   errors (max, mean):", _run_both(small), flush=True)


def test_static_scratch_refuses_what_does_not_fit():
    """A batch whose piece records exceed the fixed array is refused before any launch; so is a batch that is
    not a decode step."""
    print("case no-alloc decode: refusals", flush=True)
    too_big = B.make_batch(num_reqs=256, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16, num_pages=4096,
                           max_pages_per_req=4096, total_new_tokens=256, max_new_len=1, dtype="bf16",
                           softmax_scale=0.088)
    assert B.emm_prefill_attn_workspace_size(too_big) > B.EMM_DECODE_STATIC_SCRATCH_BYTES
    st = B.load().emm_decode_attn_static(too_big, None, None, None, None, None, None)
    assert st == B.EMM_ERR_WORKSPACE
    prefill = B.make_batch(num_reqs=1, num_q_heads=28, num_kv_heads=4, head_dim=128, page_size=16, num_pages=64,
                           max_pages_per_req=64, total_new_tokens=5, max_new_len=5, dtype="bf16", softmax_scale=0.088)
    assert B.load().emm_decode_attn_static(prefill, None, None, None, None, None, None) == B.EMM_ERR_INVALID_ARG
