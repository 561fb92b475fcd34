"""Property tests (hypothesis) of the host-side logic and of the oracle's index and format functions: random
request partitions against the partition predicate written out, random allocate / free sequences against a
model of the block manager, pixel shuffle as a bijection for any even grid, and the MXFP8 conversion's
invariants.  No GPU."""
import ctypes
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import epd_oracle as O
from paper_2501_05460_amd import binding as B

needs_lib = pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="library not built")


@needs_lib
@settings(max_examples=300, deadline=None)
@given(st.lists(st.integers(min_value=-3, max_value=40), min_size=1, max_size=12), st.integers(min_value=-1, max_value=40))
def test_offset_check_is_the_partition_predicate(offsets, n_tiles):
    """offsets[0] == 0, non-decreasing, offsets[-1] == n_tiles, n_tiles >= 0 (Section 3.2.2: a request is a
    contiguous run of slices; empty requests are legal)."""
    n_req = len(offsets) - 1
    valid = (n_tiles >= 0 and offsets[0] == 0 and offsets[-1] == n_tiles
             and all(a <= b for a, b in zip(offsets, offsets[1:])))
    s = B.check_offsets(offsets, n_req, n_tiles)
    assert (s == B.EPD_OK) == valid
    if not valid:
        assert s in (B.EPD_ERR_OFFSETS, B.EPD_ERR_INVALID_ARG)


@needs_lib
@settings(max_examples=100, deadline=None)
@given(st.integers(min_value=1, max_value=24),
       st.lists(st.tuples(st.booleans(), st.integers(min_value=0, max_value=200)), min_size=1, max_size=40))
def test_block_manager_against_a_model(n_blocks, ops):
    """Any sequence of allocations (by token count) and frees (of a whole earlier allocation): an allocation takes
    ceil(tokens / 16) distinct free blocks or nothing, a free returns exactly its blocks, the free count is
    conserved (Section 3.2.1: blocks are pre-allocated per request and released when the tokens have moved)."""
    L = B.lib()
    h = ctypes.c_void_p()
    assert L.epd_mm_cache_create(n_blocks, 16, 0, 1, ctypes.byref(h)) == B.EPD_OK
    try:
        free, held = set(range(n_blocks)), []
        for is_alloc, n in ops:
            if is_alloc or not held:
                want = -(-n // 16)
                ids = (ctypes.c_int32 * 64)()
                got = ctypes.c_int32(-1)
                s = L.epd_mm_alloc(h, n, ids, 64, ctypes.byref(got))
                if want <= len(free):
                    assert s == B.EPD_OK and got.value == want
                    blocks = [ids[i] for i in range(want)]
                    assert len(set(blocks)) == want and set(blocks) <= free
                    free -= set(blocks)
                    if blocks:
                        held.append(blocks)
                else:
                    assert s == B.EPD_ERR_NOMEM
            else:
                blocks = held.pop(n % len(held))
                arr = (ctypes.c_int32 * len(blocks))(*blocks)
                assert L.epd_mm_free(h, arr, len(blocks)) == B.EPD_OK
                assert L.epd_mm_free(h, arr, len(blocks)) != B.EPD_OK      # a second free of the same blocks is refused
                free |= set(blocks)
            assert L.epd_mm_cache_free_blocks(h) == len(free)
    finally:
        L.epd_mm_cache_destroy(h)


@settings(max_examples=60, deadline=None)
@given(st.integers(min_value=1, max_value=8), st.integers(min_value=1, max_value=6))
def test_pixel_shuffle_is_a_bijection_for_any_even_grid(half_g, D):
    g = 2 * half_g
    x = np.arange(g * g * D).reshape(g * g, D)
    y = O.pixel_shuffle_half(x, g)
    assert y.shape == (g * g // 4, 4 * D)
    assert np.array_equal(np.sort(y.ravel()), x.ravel())          # every (token, channel) exactly once
    for m in range(y.shape[0]):                                    # and where the definition puts it
        Y, X = divmod(m, g // 2)
        for dy in range(2):
            for dx in range(2):
                assert np.array_equal(y[m, (dy * 2 + dx) * D:(dy * 2 + dx + 1) * D], x[(2 * Y + dy) * g + 2 * X + dx])


finite = st.floats(min_value=-1e6, max_value=1e6, allow_nan=False, allow_infinity=False, width=32)


@settings(max_examples=200, deadline=None)
@given(st.lists(finite, min_size=32, max_size=32), st.integers(min_value=-20, max_value=20))
def test_mx_conversion_invariants(block, k):
    v = np.array(block, np.float64)
    codes, byte = O.mx_quantize(v)
    back = O.mx_dequantize(codes, byte)
    # converting again changes nothing (unless rounding carried the block's largest value into the next binade,
    # which moves the scale); a power of two moves the scale byte and nothing else
    c2, b2 = O.mx_quantize(back)
    if int(b2[0]) == int(byte[0]):
        assert np.array_equal(c2, codes)
    else:
        assert int(b2[0]) == int(byte[0]) + 1
    amax = np.abs(v).max()
    if amax > 0 and 0 < int(byte[0]) + k < 255:
        ck, bk = O.mx_quantize(np.ldexp(v, k))
        assert np.array_equal(ck, codes) and int(bk[0]) == int(byte[0]) + k
    # signs survive, magnitudes grow by at most half a spacing (a sixteenth), and the error is bounded by the format:
    # half a spacing of the element's binade, or the eighth a saturated element loses
    assert np.all(np.sign(back) * np.sign(v) >= 0)
    assert np.abs(back).max() <= amax * (1 + 1 / 16)
    if amax > 0:
        X = 2.0 ** (int(byte[0]) - 127)
        binade = np.maximum(np.floor(np.log2(np.maximum(np.abs(v) / X, 2.0 ** -30))), -6)
        bound = np.where(np.abs(v) / X > 448, np.abs(v) / 8, 2.0 ** (binade - 4) * X)
        assert np.all(np.abs(back - v) <= bound * (1 + 1e-12))
    else:
        assert not (codes & 0x7F).any() and byte[0] == 0     # zeros (a negative zero keeps its sign bit)
