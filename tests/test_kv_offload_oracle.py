"""Pins of the KV offload oracle (CPU only): it is an index map, so the pins are its invariants
and a token-by-token brute force."""
import numpy as np
import pytest

from oracle import kv_offload_oracle as KO


def pools(seed, n_layers=2, n_pages=11, h=3, page=4, dh=5):
    rng = np.random.default_rng(seed)
    shape = (n_layers, n_pages, h, page, dh)
    return rng.integers(0, 60000, shape).astype(np.uint16), rng.integers(0, 60000, shape).astype(np.uint16)


def test_pack_holds_every_cached_token_where_the_definition_says():
    k, v = pools(1)
    row = np.array([7, 2, 9, 0])
    n = 14                                   # 3.5 pages -> 4 pages
    p = KO.pack(k, v, row, n)
    assert p.shape == (2, 2, 4, 3, 4, 5)
    for l in range(2):
        for t in range(n):
            for head in range(3):
                assert np.array_equal(p[l, 0, t // 4, head, t % 4], k[l, row[t // 4], head, t % 4])
                assert np.array_equal(p[l, 1, t // 4, head, t % 4], v[l, row[t // 4], head, t % 4])


def test_round_trip_into_other_pages_moves_the_request_and_nothing_else():
    k, v = pools(2)
    k0, v0 = k.copy(), v.copy()
    old, new = np.array([3, 5, 1]), np.array([8, 0, 10])
    p = KO.pack(k, v, old, 9)
    k[:, old] = 0xFFFF                     # the freed pages are reused by someone else
    v[:, old] = 0xFFFF
    KO.unpack(p, k, v, new)
    for j in range(3):
        assert np.array_equal(k[:, new[j]], k0[:, old[j]]) and np.array_equal(v[:, new[j]], v0[:, old[j]])
    untouched = [pg for pg in range(11) if pg not in old and pg not in new]
    assert np.array_equal(k[:, untouched], k0[:, untouched]) and np.array_equal(v[:, untouched], v0[:, untouched])


def test_page_count_and_empty_request():
    assert [KO.n_pages_of(n, 16) for n in (0, 1, 16, 17, 2048)] == [0, 1, 1, 2, 128]
    k, v = pools(3)
    assert KO.pack(k, v, np.array([1, 2]), 0).size == 0


def test_memory_check_is_inclusive():
    assert KO.memory_available(70, 30, 100) and not KO.memory_available(70, 31, 100)
