"""Pins for the KV page migration reference (oracle/kv_migrate_model.py): the published Adler-32 example,
the checksum's definition evaluated the slow way on small inputs, and exactness of the round trip against
direct numpy indexing (Appendix B.5: the copy has zero error)."""
from __future__ import annotations

import numpy as np

from oracle import kv_migrate_model as M


def _pools(rng, num_pages, hkv, d):
    shape = (num_pages, hkv, 16, d)
    return (rng.integers(0, 1 << 16, shape, dtype=np.uint16), rng.integers(0, 1 << 16, shape, dtype=np.uint16))


def test_checksum_is_adler32():
    # the example everyone quotes: Adler-32("Wikipedia") = 0x11E60398
    k = np.frombuffer(b"Wiki", dtype=np.uint8).reshape(1, 4)
    v = np.frombuffer(b"pedia", dtype=np.uint8).reshape(1, 5)
    _, sums = M.pack(k, v, [0])
    assert int(sums[0]) == 0x11E60398
    # RFC 1950: A = 1 + sum of bytes, B = sum of the successive values of A, both mod 65521
    rng = np.random.default_rng(3)
    kc, vc = _pools(rng, 3, 2, 8)
    staging, sums = M.pack(kc, vc, [2, 0])
    for row, s in zip(staging, sums):
        a, b = 1, 0
        for byte in row.tolist():
            a = (a + byte) % 65521
            b = (b + a) % 65521
        assert int(s) == (b << 16 | a)


def test_checksum_of_a_large_page_with_high_bytes():
    """A staging page of 2 MiB (the largest the library admits: 1 MiB per pool) whose bytes are all large: the
    position-weighted sum passes 2^32 many times over.  Closed form in exact integers: for n bytes d_i at positions
    i = 0 .. n-1, A = 1 + sum d_i and B = n + sum (n - i) d_i, both mod 65521 (RFC 1950 written as sums)."""
    n_half = 1 << 20
    rng = np.random.default_rng(5)
    for fill in ("ff", "random_high", "ff_head"):
        if fill == "ff":
            data = np.full(2 * n_half, 0xFF, np.uint8)
        elif fill == "random_high":
            data = rng.integers(200, 256, 2 * n_half, dtype=np.uint8)
        else:
            data = np.zeros(2 * n_half, np.uint8)
            data[:4096] = 0xFF
        k = data[:n_half].reshape(1, n_half)
        v = data[n_half:].reshape(1, n_half)
        _, sums = M.pack(k, v, [0])
        n = 2 * n_half
        d = data.astype(object)                              # Python integers: no overflow anywhere
        a = (1 + int(d.sum())) % 65521
        weights = np.arange(n, 0, -1).astype(object)
        b = (n + int((weights * d).sum())) % 65521
        assert int(sums[0]) == (b << 16 | a), fill


def test_round_trip_is_exact_and_touches_nothing_else():
    rng = np.random.default_rng(4)
    kc, vc = _pools(rng, 12, 4, 128)
    ids = [7, 0, 11, 3]
    staging, sums = M.pack(kc, vc, ids)
    assert staging.shape == (4, 2 * 4 * 16 * 128 * 2)
    for row, p in zip(staging, ids):                         # K bytes of the page, then its V bytes
        assert row[:16384].tobytes() == kc[p].tobytes() and row[16384:].tobytes() == vc[p].tobytes()
    kd, vd = _pools(rng, 9, 4, 128)                          # a destination pool with other contents
    dest = [5, 8, 1, 2]
    k2, v2, sums2 = M.unpack(staging, dest, kd, vd)
    assert (sums2 == sums).all()
    for src, dst in zip(ids, dest):
        assert (k2[dst] == kc[src]).all() and (v2[dst] == vc[src]).all()
    untouched = [p for p in range(9) if p not in dest]
    assert (k2[untouched] == kd[untouched]).all() and (v2[untouched] == vd[untouched]).all()
    # a flipped bit in transit changes the checksum of that page only
    bad = staging.copy()
    bad[2, 777] ^= 0x10
    _, _, sums3 = M.unpack(bad, dest, kd, vd)
    assert (sums3 != sums).tolist() == [False, False, True, False]
    assert M.pack(kc, vc, [])[0].shape == (0, 32768)
