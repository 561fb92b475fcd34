"""Host-only tests of the paged multimodal-token cache: the oracle's index map
and the library's block manager (created without a device pool)."""
import ctypes
import os

import numpy as np
import pytest

from oracle import epd_oracle as O
from paper_2501_05460_amd import binding as B

pytestmark = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="library not built")


def test_oracle_paged_layout_round_trip_and_isolation():
    rng = np.random.default_rng(0)
    bt, dim, n_blocks = 16, 5, 12
    tokens = rng.standard_normal((3 * bt, dim))
    ids = [7, 2, 9]
    pool = np.full((n_blocks, bt, dim), -5.0)
    O.paged_scatter(pool, tokens, ids, bt)
    # block b of the request is a contiguous copy of its 16 tokens
    for j, b in enumerate(ids):
        np.testing.assert_array_equal(pool[b], tokens[j * bt:(j + 1) * bt])
    for b in set(range(n_blocks)) - set(ids):
        assert np.all(pool[b] == -5.0)
    np.testing.assert_array_equal(O.paged_gather(pool, ids, 3 * bt), tokens)
    # token 37 = block 2 of the list, slot 5
    assert np.array_equal(pool[ids[37 // bt], 37 % bt], tokens[37])


def _mgr(n_blocks=10, bt=16):
    h = ctypes.c_void_p()
    assert B.lib().epd_mm_cache_create(n_blocks, bt, 0, 1, ctypes.byref(h)) == B.EPD_OK   # token_dim 0: no pool
    return h


def _alloc(h, n_tokens, cap=64):
    ids = (ctypes.c_int32 * cap)()
    n = ctypes.c_int32(-1)
    s = B.lib().epd_mm_alloc(h, n_tokens, ids, cap, ctypes.byref(n))
    return s, [ids[i] for i in range(max(n.value, 0))]


def test_block_manager_alloc_free_reuse():
    L = B.lib()
    h = _mgr(10, 16)
    assert L.epd_mm_cache_free_blocks(h) == 10
    s, a = _alloc(h, 256 // 16 * 16 // 4)          # 64 tokens -> 4 blocks
    assert s == B.EPD_OK and len(a) == 4 and len(set(a)) == 4
    s, b = _alloc(h, 17)                           # 17 tokens -> 2 blocks (ceil)
    assert s == B.EPD_OK and len(b) == 2 and not (set(a) & set(b))
    assert L.epd_mm_cache_free_blocks(h) == 4
    s, c = _alloc(h, 5 * 16)                       # 5 blocks wanted, 4 free: nothing is taken
    assert s == B.EPD_ERR_NOMEM and c == [] and L.epd_mm_cache_free_blocks(h) == 4
    assert b"not enough" in L.epd_mm_last_error(h)
    s, z = _alloc(h, 0)
    assert s == B.EPD_OK and z == []
    # free validation: unallocated, out of range, duplicate -> nothing freed
    free = [i for i in range(10) if i not in a + b]
    for bad in ([free[0]], [10], [-1], [a[0], a[0]]):
        assert L.epd_mm_free(h, B._i32(bad), len(bad)) == B.EPD_ERR_INVALID_ARG
        assert L.epd_mm_cache_free_blocks(h) == 4
    assert L.epd_mm_free(h, B._i32(a), len(a)) == B.EPD_OK
    assert L.epd_mm_cache_free_blocks(h) == 8
    assert L.epd_mm_free(h, B._i32(a[:1]), 1) == B.EPD_ERR_INVALID_ARG   # double free
    s, d = _alloc(h, 8 * 16)
    assert s == B.EPD_OK and sorted(d) == sorted(set(range(10)) - set(b))
    L.epd_mm_cache_destroy(h)


def test_block_manager_argument_checks():
    L = B.lib()
    h = ctypes.c_void_p()
    assert L.epd_mm_cache_create(0, 16, 8, 1, ctypes.byref(h)) == B.EPD_ERR_INVALID_ARG
    assert L.epd_mm_cache_create(4, 16, 8, 7, ctypes.byref(h)) == B.EPD_ERR_INVALID_ARG
    assert L.epd_mm_cache_create(4, 1, 3, 1, ctypes.byref(h)) == B.EPD_ERR_UNSUPPORTED    # 6-byte blocks
    assert L.epd_mm_cache_create(4, 16, 8, 1, None) == B.EPD_ERR_INVALID_ARG
    m = _mgr(4, 16)
    n = ctypes.c_int32()
    ids = (ctypes.c_int32 * 1)()
    assert L.epd_mm_alloc(m, 64, ids, 1, ctypes.byref(n)) == B.EPD_ERR_INVALID_ARG      # list too short
    assert L.epd_mm_alloc(m, -1, ids, 1, ctypes.byref(n)) == B.EPD_ERR_INVALID_ARG
    assert L.epd_mm_cache_free_blocks(m) == 4
    assert L.epd_mm_cache_free_blocks(None) == -1
    L.epd_mm_cache_destroy(m)
    L.epd_mm_cache_destroy(None)
