"""Projection on the prefill side (Section 3.2.2): encode workers cache the
pre-projection tokens of their shard, the blocks travel to the prefill
worker's cache, and one call there puts the shards in slice order, projects
and merges them.  Checked against the oracle's trunk_tile / project_merge and
against the fused encode."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import epd_oracle as O
from paper_2501_05460_amd import binding as B
from gpu_util import make_encoder, rel_err, tol

pytestmark = pytest.mark.gpu

BT = 16


def desc_for(dtype, variant):
    common = dict(dtype=dtype, tile_size=224, patch=14, hidden=128, heads=2, mlp=256, layers=2,
                  norm=wl.NORM_LAYERNORM, qk_norm=wl.QKNORM_NONE, act=wl.ACT_GELU_ERF, eps=1e-6,
                  max_tiles_per_call=2)
    if variant == "resampler":   # 16 learned queries per slice: one cache block of projected tokens
        return wl.ModelDesc(final_norm=1, pixel_shuffle=0, proj_kind=wl.PROJ_RESAMPLER, proj_prenorm=0, proj_mid=16,
                            proj_out=96, proj_heads=2, **common)
    if variant == "class_token_shuffle_mlp":   # the class token never reaches the cache: 256 patch tokens per slice
        return wl.ModelDesc(final_norm=0, pixel_shuffle=1, proj_kind=wl.PROJ_MLP, proj_prenorm=1, proj_mid=128,
                            proj_out=96, class_token=1, **common)
    if variant == "shuffle_mlp":      # InternViT-like tail: pixel shuffle, LayerNorm, MLP
        return wl.ModelDesc(final_norm=0, pixel_shuffle=1, proj_kind=wl.PROJ_MLP, proj_prenorm=1, proj_mid=128,
                            proj_out=96, **common)
    return wl.ModelDesc(final_norm=1, pixel_shuffle=0, proj_kind=wl.PROJ_LINEAR, proj_prenorm=0, proj_mid=0,
                        proj_out=96, **common)  # SigLIP-like tail: post norm, one Linear


def bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy()


@pytest.mark.parametrize("variant", ["shuffle_mlp", "postnorm_linear", "class_token_shuffle_mlp", "resampler"])
@pytest.mark.parametrize("dtype", [wl.DT_BF16, wl.DT_FP32], ids=["bf16", "fp32"])
def test_shards_cached_transferred_projected_and_merged(dtype, variant):
    desc = desc_for(dtype, variant)
    bf = dtype == wl.DT_BF16
    w = wl.gen_weights(desc, 57, std=0.06)
    n_tiles = 5
    tiles_np = wl.gen_tiles(desc, 57, n_tiles)
    tiles = torch.from_numpy(tiles_np).cuda()
    enc = make_encoder(desc, w)
    N = desc.n_patches                              # 256 patches per slice = 16 blocks
    fused = enc.encode(tiles, [0, n_tiles])
    torch.cuda.synchronize()

    # two encode workers, each with its own cache, take slices [0, 3) and [3, 5)
    shards = [(0, 3), (3, 5)]
    e_caches = [B.MMCache(64, BT, desc.hidden, bf) for _ in shards]
    p_cache = B.MMCache(96, BT, desc.hidden, bf)
    e_caches[0].free(e_caches[0].alloc(2 * BT)[:1])  # shift the allocation pattern a little
    bystander = p_cache.alloc(3 * BT)
    before = bits(p_cache.gather(bystander))
    p_table = []
    for (b, e), cache in zip(shards, e_caches):
        ids = cache.alloc((e - b) * N)[::-1]
        B.encode_trunk_paged(enc, tiles, b, e, cache, ids)
        torch.cuda.synchronize()
        # pre-projection tokens against the oracle, slice by slice
        got = cache.gather(ids).float().cpu().numpy()
        want = np.concatenate([O.trunk_tile(tiles_np[t], w, desc) for t in range(b, e)])
        assert got.shape == want.shape
        assert rel_err(got, want) < tol(desc), (b, e)
        dst = p_cache.alloc((e - b) * N)
        cache.transfer_to(ids, p_cache, dst)
        cache.free(ids)
        p_table += dst
    torch.cuda.synchronize()
    assert np.array_equal(bits(p_cache.gather(bystander)), before)

    merged = B.project_merge(enc, p_cache, p_table, n_tiles)
    torch.cuda.synchronize()
    assert merged.shape == fused.shape
    want = O.encode(tiles_np, [0, n_tiles], w, desc)
    assert rel_err(merged.float().cpu().numpy(), want) < tol(desc)
    # the oracle's own split agrees with its fused definition
    pre = [np.concatenate([O.trunk_tile(tiles_np[t], w, desc) for t in range(b, e)]) for b, e in shards]
    assert np.allclose(O.project_merge(pre, w, desc), want, rtol=0, atol=1e-12)
    if not bf or variant == "postnorm_linear":
        # fp32: the cache round trip is exact.  bf16 with a bare Linear projector: the fused path
        # rounds the same fp32 rows to bf16 once, the split path rounds, widens and rounds again.
        assert np.array_equal(bits(merged), bits(fused))
    else:
        assert rel_err(merged.float().cpu().numpy(), fused.float().cpu().numpy()) < 1e-2

    # slices listed in another order come out in that order
    perm = [3, 0, 4]
    table = [b for t in perm for b in p_table[t * (N // BT):(t + 1) * (N // BT)]]
    sub = B.project_merge(enc, p_cache, table, len(perm))
    torch.cuda.synchronize()
    n_out = enc.tokens_per_tile
    for i, t in enumerate(perm):
        assert np.array_equal(bits(sub[i * n_out:(i + 1) * n_out]), bits(merged[t * n_out:(t + 1) * n_out]))
    for c in e_caches + [p_cache]:
        c.close()
    enc.close()


def test_argument_errors_are_reported_not_launched():
    desc = desc_for(wl.DT_BF16, "shuffle_mlp")
    w = wl.gen_weights(desc, 3, std=0.06)
    enc = make_encoder(desc, w)
    tiles = torch.from_numpy(wl.gen_tiles(desc, 3, 2)).cuda()
    N = desc.n_patches
    wrong_width = B.MMCache(64, BT, desc.out_dim, True)
    ids = wrong_width.alloc(2 * N)
    with pytest.raises(B.EpdError) as ei:
        B.encode_trunk_paged(enc, tiles, 0, 2, wrong_width, ids)
    assert ei.value.status == B.EPD_ERR_SHAPE
    cache = B.MMCache(64, BT, desc.hidden, True)
    ids = cache.alloc(2 * N)
    cache.free(ids[-1:])
    with pytest.raises(B.EpdError) as ei:                      # last block no longer allocated
        B.encode_trunk_paged(enc, tiles, 0, 2, cache, ids)
    assert ei.value.status == B.EPD_ERR_OFFSETS
    with pytest.raises(B.EpdError) as ei:
        B.project_merge(enc, cache, ids, 2)
    assert ei.value.status == B.EPD_ERR_OFFSETS
    with pytest.raises(B.EpdError) as ei:                      # range outside the batch
        B.encode_trunk_paged(enc, tiles, 1, 3, cache, ids)
    assert ei.value.status == B.EPD_ERR_OFFSETS
    odd = B.MMCache(64, 48, desc.hidden, True)                 # 256 patches are not a multiple of 48
    ids48 = odd.alloc(2 * N)
    with pytest.raises(B.EpdError) as ei:
        B.encode_trunk_paged(enc, tiles, 0, 2, odd, ids48)
    assert ei.value.status == B.EPD_ERR_UNSUPPORTED
    B.encode_trunk_paged(enc, tiles, 1, 1, cache, [])          # empty range: nothing to do
    assert B.project_merge(enc, cache, [], 0).shape[0] == 0
    for c in (wrong_width, cache, odd):
        c.close()
    enc.close()
