"""Paged multimodal-token cache on the GPU: the paged encode writes exactly the
bits of the contiguous encode into the request's blocks, leaves every other
block alone, and the encode-to-prefill block transfer moves them unchanged."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import epd_oracle as O
from paper_2501_05460_amd import binding as B
from gpu_util import make_encoder, rel_err, tol

pytestmark = pytest.mark.gpu

BT = 16   # tokens per block, the paper's setting


def desc_for(dtype, tail="shuffle_mlp"):
    common = dict(dtype=dtype, tile_size=224, patch=14, hidden=128, heads=2, mlp=256, layers=1,
                  norm=wl.NORM_LAYERNORM, qk_norm=wl.QKNORM_NONE, act=wl.ACT_GELU_ERF, eps=1e-6,
                  max_tiles_per_call=2)     # 5 slices -> 3 micro-batches
    if tail == "resampler_class_token":   # 64 learned queries per slice (4 blocks), class token in the trunk
        return wl.ModelDesc(final_norm=1, pixel_shuffle=0, proj_kind=wl.PROJ_RESAMPLER, proj_prenorm=0, proj_mid=64,
                            proj_out=96, proj_heads=2, class_token=1, **common)
    return wl.ModelDesc(final_norm=0, pixel_shuffle=1, proj_kind=wl.PROJ_MLP, proj_prenorm=1, proj_mid=128,
                        proj_out=96, **common)


def bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy()


@pytest.mark.parametrize("tail", ["shuffle_mlp", "resampler_class_token"])
@pytest.mark.parametrize("dtype", [wl.DT_BF16, wl.DT_FP32], ids=["bf16", "fp32"])
def test_paged_encode_transfer_and_release(dtype, tail):
    desc = desc_for(dtype, tail)
    w = wl.gen_weights(desc, 41, std=0.06)
    tiles_np = wl.gen_tiles(desc, 41, 5)
    tiles = torch.from_numpy(tiles_np).cuda()
    offsets = [0, 2, 2, 5]                       # requests of 2, 0 and 3 slices
    enc = make_encoder(desc, w)
    n_out = enc.tokens_per_tile                  # 64 tokens per slice = 4 blocks
    full = enc.encode(tiles, offsets)
    torch.cuda.synchronize()

    bf = dtype == wl.DT_BF16
    e_cache = B.MMCache(40, BT, desc.out_dim, bf)    # encode worker's cache
    p_cache = B.MMCache(32, BT, desc.out_dim, bf)    # stand-in for the prefill worker's cache
    hole = e_cache.alloc(3 * BT)                     # make the request tables non-contiguous
    tables = [e_cache.alloc((offsets[r + 1] - offsets[r]) * n_out) for r in range(3)]
    e_cache.free(hole)
    tables[2] = tables[2][::-1]                      # any order of blocks is legal
    assert [len(t) for t in tables] == [8, 0, 12]
    B.encode_paged(enc, tiles, offsets, e_cache, tables)
    torch.cuda.synchronize()
    for r in (0, 2):
        got = e_cache.gather(tables[r])
        torch.cuda.synchronize()
        want = full[offsets[r] * n_out:offsets[r + 1] * n_out]
        assert np.array_equal(bits(got), bits(want)), r
        # the CPU oracle's index map says the same: block j of the list holds tokens 16j .. 16j+15
        pool = np.zeros((40, BT, desc.out_dim), np.float32)
        O.paged_scatter(pool, want.float().cpu().numpy(), tables[r], BT)
        for j, b in enumerate(tables[r]):
            blk = e_cache.gather([b])
            torch.cuda.synchronize()
            assert np.array_equal(blk.float().cpu().numpy(), pool[b]), (r, j)

    # the tokens themselves are right (oracle parity through the paged path)
    want0 = O.encode(tiles_np[:2], [0, 2], w, desc)
    assert rel_err(e_cache.gather(tables[0]).float().cpu().numpy(), want0) < tol(desc)

    # encode -> prefill migration of request 2, then release of the source blocks
    dst_ids = p_cache.alloc(len(tables[2]) * BT)
    e_cache.transfer_to(tables[2], p_cache, dst_ids)
    torch.cuda.synchronize()
    moved = p_cache.gather(dst_ids)
    torch.cuda.synchronize()
    assert np.array_equal(bits(moved), bits(full[offsets[2] * n_out:offsets[3] * n_out]))
    free_before = e_cache.free_blocks
    e_cache.free(tables[2])
    assert e_cache.free_blocks == free_before + 12
    # request 0 is still intact in the encode worker's cache
    assert np.array_equal(bits(e_cache.gather(tables[0])), bits(full[:2 * n_out]))
    for c in (e_cache, p_cache):
        c.close()
    enc.close()


@pytest.mark.parametrize("dtype", [wl.DT_BF16, wl.DT_FP32], ids=["bf16", "fp32"])
def test_raw_pool_holds_the_oracle_index_map(dtype):
    """The layout check without any copy kernel of the library: the pool is read as a plain tensor view of
    its device pointer.  Every block a table names holds the 16 tokens the oracle's index map puts there
    (the bits of the contiguous encode), every other block still holds the fill value."""
    desc = desc_for(dtype)
    w = wl.gen_weights(desc, 43, std=0.06)
    tiles = torch.from_numpy(wl.gen_tiles(desc, 43, 5)).cuda()
    offsets = [0, 2, 2, 5]
    enc = make_encoder(desc, w)
    n_out = enc.tokens_per_tile
    full = enc.encode(tiles, offsets)
    torch.cuda.synchronize()
    cache = B.MMCache(40, BT, desc.out_dim, dtype == wl.DT_BF16)
    pool = cache.pool_tensor()
    assert tuple(pool.shape) == (40, BT, desc.out_dim)
    pool.fill_(-7.0)
    hole = cache.alloc(5 * BT)
    tables = [cache.alloc((offsets[r + 1] - offsets[r]) * n_out) for r in range(3)]
    cache.free(hole)
    tables[0] = tables[0][::-1]
    B.encode_paged(enc, tiles, offsets, cache, tables)
    torch.cuda.synchronize()
    want = np.full((40, BT, desc.out_dim), -7.0, np.float32)
    for r in range(3):
        O.paged_scatter(want, full[offsets[r] * n_out:offsets[r + 1] * n_out].float().cpu().numpy(), tables[r], BT)
    assert np.array_equal(pool.float().cpu().numpy(), want)
    del pool
    cache.close()
    enc.close()


def test_paged_encode_leaves_other_blocks_untouched_and_rejects_bad_tables():
    desc = desc_for(wl.DT_BF16)
    w = wl.gen_weights(desc, 42, std=0.06)
    tiles = torch.from_numpy(wl.gen_tiles(desc, 42, 3)).cuda()
    enc = make_encoder(desc, w)
    n_out = enc.tokens_per_tile
    cache = B.MMCache(20, BT, desc.out_dim, True)
    mine = cache.alloc(3 * n_out)                 # 12 blocks
    rest = cache.alloc(cache.free_blocks * BT)    # the other 8, allocated so they can be read back
    before = bits(cache.gather(rest)).copy()
    torch.cuda.synchronize()
    B.encode_paged(enc, tiles, [0, 3], cache, [mine])
    torch.cuda.synchronize()
    assert np.array_equal(bits(cache.gather(rest)), before)
    # error paths: nothing is enqueued
    snap = bits(cache.gather(mine)).copy()
    with pytest.raises(B.EpdError) as e:
        B.encode_paged(enc, tiles, [0, 3], cache, [mine[:-1]])          # table too short
    assert e.value.status == B.EPD_ERR_OFFSETS
    cache.free(rest[:1])
    with pytest.raises(B.EpdError) as e:
        B.encode_paged(enc, tiles, [0, 3], cache, [mine[:-1] + rest[:1]])   # unallocated block
    assert e.value.status == B.EPD_ERR_OFFSETS
    with pytest.raises(B.EpdError) as e:
        B.encode_paged(enc, tiles, [0, 3], cache, [mine[:-1] + mine[:1]])   # one block listed twice
    assert e.value.status == B.EPD_ERR_OFFSETS and "second time" in str(e.value)
    other = B.MMCache(20, BT, desc.out_dim + 8, True)
    with pytest.raises(B.EpdError) as e:
        B.encode_paged(enc, tiles, [0, 3], other, [other.alloc(3 * n_out)])  # wrong token width
    assert e.value.status == B.EPD_ERR_SHAPE
    odd = B.MMCache(64, 48, desc.out_dim, True)
    with pytest.raises(B.EpdError) as e:
        B.encode_paged(enc, tiles, [0, 3], odd, [odd.alloc(3 * n_out)])      # 64 % 48 != 0
    assert e.value.status == B.EPD_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert np.array_equal(bits(cache.gather(mine)), snap)
    for c in (cache, other, odd):
        c.close()
    enc.close()
