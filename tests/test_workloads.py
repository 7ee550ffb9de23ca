"""The seeded input generators: determinism, bf16 rounding, and the structure the named workloads state."""
import numpy as np
import torch

from paper_2507_10069_amd import workloads as W


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 37,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40], np.float32)])
    ours = W.to_bf16_bits(x)
    theirs = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(ours, theirs)
    back = W.bf16_bits_to_f32(ours)
    np.testing.assert_array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_same_seed_same_bytes():
    a, b = W.config(2, 8), W.config(2, 8)
    for f in ("page_table", "prefix_lens", "new_lens", "q", "k_new", "v_new", "k_cache", "v_cache"):
        assert getattr(a, f).tobytes() == getattr(b, f).tobytes()


def test_config1_shape():
    wl = W.config(1)
    assert (wl.dtype, wl.num_reqs, wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size) == \
        ("f32", 1, 4, 1, 64, 16)
    assert wl.num_pages == 64 and wl.prefix_lens.tolist() == [256] and wl.new_lens.tolist() == [64]
    row = wl.page_table[0]
    assert len(set(row.tolist())) == 20 and row.min() >= 0 and row.max() < 64
    assert abs(wl.softmax_scale - 0.125) < 1e-15
    assert wl.attention_flops() == 4 * 64 * 4 * (64 * 256 + 64 * 65 // 2)


def test_config2_sharing():
    wl = W.config(2)
    assert wl.prefix_lens.tolist() == [1056] * 8 and (wl.new_lens >= 128).all() and (wl.new_lens <= 512).all()
    for grp in ((0, 1, 2, 3), (4, 5, 6, 7)):
        for r in grp[1:]:
            np.testing.assert_array_equal(wl.page_table[r, :66], wl.page_table[grp[0], :66])
    assert len(set(wl.page_table[0, :66]) & set(wl.page_table[4, :66])) == 0
    # pages that receive new tokens are private
    own = [set(wl.page_table[r, 66:66 + -(-int(wl.new_lens[r]) // 16)].tolist()) for r in range(8)]
    for a in range(8):
        for b in range(a + 1, 8):
            assert not (own[a] & own[b])


def test_config3_outliers_and_flops():
    wl = W.config(3)
    assert wl.prefix_lens.tolist() == [16384, 16384] and wl.new_lens.tolist() == [2048, 2048]
    assert wl.attention_flops() == 4 * 128 * 28 * 2 * (2048 * 16384 + 2048 * 2049 // 2)
    k = W.bf16_bits_to_f32(wl.k_new)
    frac_big = float((np.abs(k) > 5.0).mean())
    assert 0.004 < frac_big < 0.008          # P(|8 z| > 5) ~ 0.53 of the 1% outliers
    v = W.bf16_bits_to_f32(wl.v_new)
    assert float((np.abs(v) > 5.0).mean()) < 1e-5


def test_config4_mix():
    wl = W.config(4)
    text_only = wl.prefix_lens == 0
    assert wl.num_reqs == 32 and wl.num_q_heads == 32 and wl.num_kv_heads == 8
    # cache-hit fraction 0 on a multimodal request also gives prefix 0, so at least the 16 text-only ones
    assert text_only.sum() >= 16
    used = wl.page_table[wl.page_table >= 0]
    assert len(used) == len(set(used.tolist()))            # all pages private
    assert (wl.prefix_lens % 16 != 0).any()                # unaligned cached prefixes occur


def test_config5_cross_pairs():
    wl = W.config(5)
    assert wl.kind == "cross" and wl.k_new is None and wl.prefix_lens.tolist() == [6404] * 16
    assert wl.max_pages_per_req == 401
    for r in range(0, 16, 2):
        np.testing.assert_array_equal(wl.page_table[r], wl.page_table[r + 1])
    # the last page holds 4 valid tokens and 12 sentinel slots
    last = wl.k_cache[wl.page_table[0, 400]]
    assert (last[:, 4:, :] == W.SENTINEL_BF16_BITS).all() and not (last[:, :4, :] == W.SENTINEL_BF16_BITS).all()


def test_distinct_kv_bytes_count_shared_pages_once():
    plain = W.decode_config("decode_video_b8", 16)
    assert plain.kv_distinct_read_bytes() == plain.kv_read_bytes()
    shared = W.decode_config("decode_shared_video_b8", 16)          # 8 requests, 1024 shared + 128 own tokens + the new one
    per_token = 2 * shared.num_kv_heads * shared.head_dim * shared.elt_bytes
    assert shared.kv_read_bytes() == 8 * (1024 + 128 + 1) * per_token
    assert shared.kv_distinct_read_bytes() == (1024 + 8 * (128 + 1)) * per_token
