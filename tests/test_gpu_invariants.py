"""Properties of the HIP path that hold at any size: slices are encoded
independently (Section 3.2.2), so permuting slices permutes row blocks, one
slice's pixels touch no other slice's rows, any grouping into calls, shards or
micro-batches gives the same bits, and runs repeat bit for bit."""
import numpy as np
import pytest
import torch

import workloads as wl
from paper_2501_05460_amd import binding as B
from gpu_util import make_encoder

pytestmark = pytest.mark.gpu


def desc_for(dtype, **kw):
    base = dict(dtype=dtype, tile_size=224, patch=14, hidden=192, heads=3, mlp=384, layers=2,
                norm=wl.NORM_LAYERNORM, qk_norm=wl.QKNORM_NONE, act=wl.ACT_GELU_ERF, final_norm=0,
                pixel_shuffle=1, proj_kind=wl.PROJ_MLP, proj_prenorm=1, proj_mid=256, proj_out=128,
                eps=1e-6, max_tiles_per_call=8)
    base.update(kw)
    return wl.ModelDesc(**base)


def bits(t: torch.Tensor) -> np.ndarray:
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).cpu().numpy()


@pytest.fixture(scope="module", params=[wl.DT_BF16, wl.DT_FP32], ids=["bf16", "fp32"])
def setup(request):
    desc = desc_for(request.param)
    w = wl.gen_weights(desc, 31, std=0.06)
    tiles = torch.from_numpy(wl.gen_tiles(desc, 31, 7)).cuda()
    enc = make_encoder(desc, w)
    full = enc.encode(tiles, [0, 7])
    torch.cuda.synchronize()
    yield desc, w, tiles, enc, full
    enc.close()


def test_runs_repeat_bit_for_bit(setup):
    desc, w, tiles, enc, full = setup
    again = enc.encode(tiles, [0, 3, 3, 7])      # request structure does not change the rows
    torch.cuda.synchronize()
    assert np.array_equal(bits(again), bits(full))


def test_permuting_slices_permutes_row_blocks(setup):
    desc, w, tiles, enc, full = setup
    perm = [4, 0, 6, 2, 1, 5, 3]
    out = enc.encode(tiles[perm].contiguous(), [0, 7])
    torch.cuda.synchronize()
    n = enc.tokens_per_tile
    a, b = bits(out), bits(full)
    for i, src in enumerate(perm):
        assert np.array_equal(a[i * n:(i + 1) * n], b[src * n:(src + 1) * n])


def test_one_slice_does_not_leak_into_another(setup):
    desc, w, tiles, enc, full = setup
    t2 = tiles.clone()
    t2[3] = t2[3] * 0.5 + 0.1
    out = enc.encode(t2, [0, 7])
    torch.cuda.synchronize()
    n = enc.tokens_per_tile
    a, b = bits(out), bits(full)
    for t in range(7):
        same = np.array_equal(a[t * n:(t + 1) * n], b[t * n:(t + 1) * n])
        assert same == (t != 3), t
    alone = enc.encode(tiles[5:6].contiguous(), [0, 1])
    torch.cuda.synchronize()
    assert np.array_equal(bits(alone), b[5 * n:6 * n])


def test_shards_write_only_their_rows_and_union_equals_one_call(setup):
    desc, w, tiles, enc, full = setup
    offsets = [0, 3, 3, 7]                       # requests of 3, 0 and 4 slices
    n = enc.tokens_per_tile
    out = enc.alloc_out(7)
    sentinel = 12345.0
    out.fill_(sentinel)
    covered = np.zeros(7, int)
    for s in range(4):
        for r in range(3):
            cnt = offsets[r + 1] - offsets[r]
            b, e = wl.shard_range(cnt, s, 4)
            before = bits(out).copy()
            enc.encode_range(tiles, offsets[r] + b, offsets[r] + e, out)
            torch.cuda.synchronize()
            changed = np.any(bits(out) != before, axis=1).reshape(7, n).any(axis=1)
            assert set(np.nonzero(changed)[0]) <= set(range(offsets[r] + b, offsets[r] + e))
            covered[offsets[r] + b:offsets[r] + e] += 1
    assert np.all(covered == 1)
    assert np.array_equal(bits(out), bits(full))


def test_micro_batch_size_does_not_change_the_bits(setup):
    desc, w, tiles, enc, full = setup
    for mb in (1, 2, 3):
        enc2 = make_encoder(desc.replace(max_tiles_per_call=mb), w)
        out = enc2.encode(tiles, [0, 7])
        torch.cuda.synchronize()
        assert np.array_equal(bits(out), bits(full)), mb
        enc2.close()


def test_a_call_captured_in_a_hip_graph_replays_the_eager_bits(setup):
    """A call allocates nothing, copies nothing from the host and clears no memory with the runtime's fill, so
    after one eager call on the context (kernel attributes are set at a kernel's first launch) its launch
    sequence can be recorded into a HIP graph (a serving loop's way to issue the ~10 launches per layer of a
    one-slice share, Section 3.2.2).  Every replay, with eager calls on the same context and a cleared
    output between the replays, gives the bits of the eager call."""
    desc, w, tiles, enc, full = setup
    out = enc.alloc_out(7)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        enc.encode(tiles, [0, 7], out)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            enc.encode(tiles, [0, 7], out)
    torch.cuda.synchronize()
    n = enc.tokens_per_tile
    for rep in range(3):
        out.fill_(3.0)
        part = enc.encode(tiles[rep:rep + 2].contiguous(), [0, 2])     # eager work on the same workspace
        torch.cuda.synchronize()
        assert np.array_equal(bits(part), bits(full[rep * n:(rep + 2) * n])), rep
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(bits(out), bits(full)), rep


def test_empty_batch_and_error_paths_leave_the_cache_untouched(setup):
    desc, w, tiles, enc, full = setup
    out = enc.alloc_out(7)
    out.fill_(7.0)
    before = bits(out).copy()
    lib = B.lib()
    import ctypes
    off0 = (ctypes.c_int32 * 1)(0)
    assert lib.epd_encode(enc._h, None, 0, off0, 0, None, None) == B.EPD_OK      # empty batch: no-op
    bad = (ctypes.c_int32 * 2)(0, 6)
    st = torch.cuda.current_stream().cuda_stream
    assert lib.epd_encode(enc._h, tiles.data_ptr(), 7, bad, 1, out.data_ptr(), st) == B.EPD_ERR_OFFSETS
    assert b"tile_offsets" in lib.epd_last_error(enc._h)
    assert lib.epd_encode_range(enc._h, tiles.data_ptr(), 7, 5, 9, out.data_ptr(), st) == B.EPD_ERR_OFFSETS
    assert lib.epd_encode_range(enc._h, tiles.data_ptr(), 7, 4, 2, out.data_ptr(), st) == B.EPD_ERR_OFFSETS
    assert lib.epd_encode_range(enc._h, tiles.data_ptr(), 7, 2, 2, out.data_ptr(), st) == B.EPD_OK  # empty shard
    assert lib.epd_encode_range(enc._h, tiles.data_ptr() + 4, 7, 0, 1, out.data_ptr(), st) == B.EPD_ERR_INVALID_ARG
    assert lib.epd_encode_range(enc._h, None, 7, 0, 1, out.data_ptr(), st) == B.EPD_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert np.array_equal(bits(out), before)


def test_a_slice_alone_has_the_bits_it_has_inside_a_large_batch():
    """The GEMM picks its tile width by how many tiles the launch has (narrow tiles when half of the
    chip would idle), the persistent form for long tile sequences: all forms order their sums alike, so
    a slice encoded alone (4 tiles per product) carries the bits it has inside a 70-slice batch."""
    desc = desc_for(wl.DT_BF16, hidden=512, heads=8, mlp=1024, layers=2, max_tiles_per_call=72, proj_out=256)
    w = wl.gen_weights(desc, 37, std=0.05)
    tiles = torch.from_numpy(wl.gen_tiles(desc, 37, 70)).cuda()
    enc = make_encoder(desc, w)
    full = enc.encode(tiles, [0, 70])
    torch.cuda.synchronize()
    n = enc.tokens_per_tile
    for t in (0, 5, 69):
        alone = enc.encode(tiles[t:t + 1], [0, 1])
        torch.cuda.synchronize()
        assert np.array_equal(bits(alone), bits(full[t * n:(t + 1) * n])), t
    few = enc.encode(tiles[3:7], [0, 4])
    torch.cuda.synchronize()
    assert np.array_equal(bits(few), bits(full[3 * n:7 * n]))
    enc.close()


def test_a_slice_of_nan_pixels_poisons_neither_its_neighbours_nor_later_calls():
    """Class-token shape: 65 tokens in 72 rows, so the last key block of every slice reaches into the next
    slice's rows and values (masked keys, weight exactly zero).  A slice full of NaN must leave the other
    slices of its batch bit-identical, and a smaller clean batch encoded afterwards on the same context (its
    workspace still holding the NaN rows) must give the bits a fresh context gives."""
    desc = desc_for(wl.DT_BF16, tile_size=112, class_token=1)
    w = wl.gen_weights(desc, 61, std=0.08)
    tiles = torch.from_numpy(wl.gen_tiles(desc, 61, 4)).cuda()
    enc = make_encoder(desc, w)
    n = enc.tokens_per_tile
    clean = enc.encode(tiles, [0, 4]).clone()
    bad = tiles.clone()
    bad[2] = float("nan")
    out = enc.encode(bad, [0, 4]).clone()
    torch.cuda.synchronize()
    assert bool(torch.isnan(out[2 * n:3 * n].float()).any())
    for t in (0, 1, 3):
        assert np.array_equal(bits(out[t * n:(t + 1) * n]), bits(clean[t * n:(t + 1) * n])), t
    # a later, smaller call: slices 0 and 1 land where they were, the NaN rows of slice 2 stay behind them
    later = enc.encode(tiles[:2], [0, 2]).clone()
    fresh_enc = make_encoder(desc, w)
    fresh = fresh_enc.encode(tiles[:2], [0, 2])
    torch.cuda.synchronize()
    assert np.array_equal(bits(later), bits(fresh))
    assert np.array_equal(bits(later), bits(clean[:2 * n]))
    fresh_enc.close()
    enc.close()
