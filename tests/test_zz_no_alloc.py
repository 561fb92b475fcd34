"""The block transfer that allocates nothing (its id lists sit in a static device array of the library)
against the ordinary one: same bits in the destination pool, on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from paper_2501_05460_amd import binding as B

pytestmark = pytest.mark.gpu

BT, DIM = 16, 96


def _pools(n_src, n_dst, seed):
    src = B.MMCache(n_src, BT, DIM, True)
    a, b = B.MMCache(n_dst, BT, DIM, True), B.MMCache(n_dst, BT, DIM, True)
    g = torch.Generator(device="cuda").manual_seed(seed)
    bits = torch.randint(-32768, 32767, (n_src, BT, DIM), dtype=torch.int16, device="cuda", generator=g)
    src.pool_tensor().view(torch.int16).copy_(bits)
    for c in (a, b):
        c.pool_tensor().view(torch.int16).fill_(-21555)
    return src, a, b


def test_noalloc_transfer_matches_the_ordinary_transfer_twice_in_a_row():
    src, a, b = _pools(300, 260, 7)
    src_ids = src.alloc(300 * BT)
    a_ids, b_ids = a.alloc(260 * BT), b.alloc(260 * BT)
    assert a_ids == b_ids
    rng = np.random.default_rng(5)
    # first call: 200 blocks in a scattered order; second call: 37 other blocks onto partly the same places
    for n, seed in ((200, 1), (37, 2)):
        pick_s = [src_ids[i] for i in rng.permutation(300)[:n]]
        pick_d = [a_ids[i] for i in rng.permutation(260)[:n]]
        src.transfer_to(pick_s, a, pick_d)
        src.transfer_to(pick_s, b, pick_d, noalloc=True)
        torch.cuda.synchronize()
        pa, pb = a.pool_tensor().view(torch.int16), b.pool_tensor().view(torch.int16)
        assert torch.equal(pa, pb), n
        # and both hold the source blocks (checked without the library: plain tensor indexing)
        want = src.pool_tensor().view(torch.int16)[torch.tensor(pick_s, device="cuda")]
        assert torch.equal(pb[torch.tensor(pick_d, device="cuda")], want), n
    untouched = b.pool_tensor().view(torch.int16) == -21555
    assert bool(untouched.any())          # blocks no call named still hold the fill value
    for c in (src, a, b):
        c.close()


def test_noalloc_transfer_rejects_what_it_cannot_hold_and_bad_ids():
    src, a, b = _pools(8, 8, 9)
    s_ids, b_ids = src.alloc(8 * BT), b.alloc(4 * BT)
    big = [0] * (65536 + 1)
    with pytest.raises(B.EpdError) as e:
        src.transfer_to(big, b, big, noalloc=True)
    assert e.value.status == B.EPD_ERR_UNSUPPORTED and "65536" in str(e.value)
    with pytest.raises(B.EpdError) as e:
        src.transfer_to(s_ids[:2], b, [b_ids[0], 7], noalloc=True)     # block 7 of b is not allocated
    assert e.value.status == B.EPD_ERR_OFFSETS
    src.transfer_to([], b, [], noalloc=True)                           # empty: no-op
    torch.cuda.synchronize()
    assert bool((b.pool_tensor().view(torch.int16) == -21555).all())
    for c in (src, a, b):
        c.close()
