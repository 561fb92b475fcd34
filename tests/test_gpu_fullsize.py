"""Parity at the full sizes of the named configurations, in the launch
configuration bench.py times: the whole batch runs on the GPU, the oracle
encodes a fixed sample of slices at full depth, and the sampled row blocks
are compared element by element."""
import time

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import epd_oracle as O
from paper_2501_05460_amd import binding as B
from gpu_util import rel_err, rel_l2, tol

pytestmark = pytest.mark.gpu


def build(wk, desc=None):
    desc = desc or wk.desc
    bf = desc.dtype == wl.DT_BF16
    dev = [B.to_device(wl.gen_weight(desc, wk.weight_seed, i), bf) for i in range(len(wl.weight_specs(desc)))]
    enc = B.Encoder(desc, dev)
    del dev
    S = desc.tile_size
    tiles = torch.empty((wk.n_tiles, 3, S, S), dtype=torch.float32, device="cuda")
    for t in range(wk.n_tiles):
        tiles[t] = torch.from_numpy(wl.gen_tile(desc, wk.input_seed, t))
    return enc, tiles


def check_sample(wk, enc, out, sample, desc=None):
    desc = desc or wk.desc
    w = wl.gen_weights(desc, wk.weight_seed)
    n = enc.tokens_per_tile
    worst = 0.0
    for t in sample:
        t0 = time.time()
        want = O.encode_tile(wl.gen_tile(desc, wk.input_seed, t), w, desc)
        got = out[t * n:(t + 1) * n].float().cpu().numpy()
        e = rel_err(got, want)
        print(f"{wk.name} slice {t}: max_rel_err={e:.3e} rel_l2={rel_l2(got, want):.3e} oracle {time.time() - t0:.1f}s",
              flush=True)
        worst = max(worst, e)
    assert worst < tol(desc)


def test_c2_siglip_shape_10_slices():
    wk = wl.workload("c2")
    enc, tiles = build(wk)
    out = enc.encode(tiles, list(wk.tile_offsets))
    torch.cuda.synchronize()
    assert tuple(out.shape) == (10 * 1024, 3584)
    check_sample(wk, enc, out, wk.oracle_sample_tiles)
    enc.close()


def test_c2_paged_encode_and_shares_carry_the_bits_of_the_whole_call():
    """At this size the library cuts some products by rows (whole rounds of 256-wide tiles plus one round of
    narrower ones): the paged output, whose rows go through the block table on both sides of the cut, and the
    shares of 3 + 7 slices, whose products are cut elsewhere or not at all, must carry the same bits."""
    wk = wl.workload("c2")
    enc, tiles = build(wk)
    n = enc.tokens_per_tile
    whole = enc.encode(tiles, list(wk.tile_offsets)).clone()
    parts = torch.empty_like(whole)
    enc.encode(tiles[:3], [0, 3], parts[:3 * n])
    enc.encode(tiles[3:], [0, 7], parts[3 * n:])
    torch.cuda.synchronize()
    assert torch.equal(whole.view(torch.int16), parts.view(torch.int16))
    n_blocks = 10 * n // 16
    cache = B.MMCache(n_blocks + 7, 16, wk.desc.out_dim, True)
    hole = cache.alloc(5 * 16)
    table = cache.alloc(10 * n)[::-1]            # scattered, descending
    cache.free(hole)
    B.encode_paged(enc, tiles, list(wk.tile_offsets), cache, [table])
    torch.cuda.synchronize()
    got = cache.gather(table)
    torch.cuda.synchronize()
    assert torch.equal(whole.view(torch.int16), got.view(torch.int16))
    cache.close()
    enc.close()


def test_c3_internvit300m_shape_104_slices():
    wk = wl.workload("c3")
    enc, tiles = build(wk)
    out = enc.encode(tiles, list(wk.tile_offsets))
    torch.cuda.synchronize()
    assert tuple(out.shape) == (104 * 256, 4096)
    assert bool(torch.isfinite(out.float()).all())
    check_sample(wk, enc, out, wk.oracle_sample_tiles)
    enc.close()


def test_c3_with_mx_fp8_104_slices():
    """The MXFP8 option at the full C3 size, in the configuration `bench.py --mx-fp8` times: the last slice of the batch
    against the oracle that converts at the same places (the option's own bound, two independent draws of the
    format's noise at this depth) and against the exact oracle (no noisier than the format itself), and the whole
    batch again for the same bits."""
    wk = wl.workload("c3")
    desc = wk.desc.replace(mx_fp8=1)
    enc, tiles = build(wk, desc)
    out = enc.encode(tiles, list(wk.tile_offsets)).clone()
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all())
    again = enc.encode(tiles, list(wk.tile_offsets))
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), again.view(torch.int16))
    t = wk.n_tiles - 1
    n = enc.tokens_per_tile
    w = wl.gen_weights(desc, wk.weight_seed)
    tile = wl.gen_tile(desc, wk.input_seed, t)
    want = O.encode_tile(tile, w, desc)
    exact = O.encode_tile(tile, w, wk.desc)
    got = out[t * n:(t + 1) * n].float().cpu().numpy()
    e, e_exact, fmt = rel_err(got, want), rel_err(got, exact), rel_err(want, exact)
    print(f"c3 + mx_fp8 slice {t}: vs converting oracle {e:.3e} (l2 {rel_l2(got, want):.3e}), vs exact oracle {e_exact:.3e} "
          f"(l2 {rel_l2(got, exact):.3e}), converting oracle vs exact {fmt:.3e} (l2 {rel_l2(want, exact):.3e})", flush=True)
    assert e < 1e-1
    assert e_exact < 1.5 * fmt + 2e-2
    enc.close()


def test_c5_mixed_batch_sharded_equals_one_call_and_oracle():
    wk = wl.workload("c5")
    enc, tiles = build(wk)
    off = list(wk.tile_offsets)
    n = enc.tokens_per_tile
    full = enc.encode(tiles, off)
    torch.cuda.synchronize()
    assert full.shape[0] == wk.n_tiles * n
    # 4 shards per request, each its own call, rows landing at their final place
    out = enc.alloc_out(wk.n_tiles)
    out.fill_(-3.0)
    for s in range(4):
        for r in range(wk.n_requests):
            b, e = wl.shard_range(off[r + 1] - off[r], s, 4)
            enc.encode_range(tiles, off[r] + b, off[r] + e, out)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), full.view(torch.int16))
    del out
    # first / last slice of the first and the last request, and the first slice of each of the four
    # shards of the largest request (the last slice of the batch lies in the partial last micro-batch)
    assert len(wk.oracle_sample_tiles) == 8 and wk.oracle_sample_tiles[-1] == wk.n_tiles - 1
    check_sample(wk, enc, full, wk.oracle_sample_tiles)
    enc.close()


@pytest.fixture(scope="module")
def c4_sample_rows():
    """The 6B-shaped batch of 40 slices encoded once; the row blocks of the oracle's sample slices on the host."""
    wk = wl.workload("c4")
    enc, tiles = build(wk)
    out = enc.encode(tiles, list(wk.tile_offsets))
    torch.cuda.synchronize()
    assert tuple(out.shape) == (40 * 256, 5120)
    assert bool(torch.isfinite(out.float()).all())
    n = enc.tokens_per_tile
    rows = {t: out[t * n:(t + 1) * n].float().cpu().numpy() for t in wk.oracle_sample_tiles}
    enc.close()
    del out, tiles
    torch.cuda.empty_cache()
    return wk, rows


@pytest.mark.parametrize("which", [0, 1, 2], ids=["first", "middle", "last"])
def test_c4_internvit6b_shape_40_slices(c4_sample_rows, which):
    """First, middle and last slice of the batch against the oracle (about 25 s of CPU time each, hence one
    test per slice); the last slice sits behind the largest buffer offsets of any workload here."""
    wk, rows = c4_sample_rows
    t = wk.oracle_sample_tiles[which]
    assert wk.oracle_sample_tiles == (0, 20, 39)
    t0 = time.time()
    want = O.encode_tile(wl.gen_tile(wk.desc, wk.input_seed, t), wl.gen_weights(wk.desc, wk.weight_seed), wk.desc)
    e = rel_err(rows[t], want)
    print(f"{wk.name} slice {t}: max_rel_err={e:.3e} rel_l2={rel_l2(rows[t], want):.3e} oracle {time.time() - t0:.1f}s", flush=True)
    assert e < tol(wk.desc)


def test_c7_internvit300m_shape_with_class_token_and_layer_scale():
    """1025 tokens per slice in rows padded to 1032: every GEMM has a ragged last tile, the last key
    block of every slice reaches into the next slice and is masked from its second key on."""
    wk = wl.workload("c7")
    enc, tiles = build(wk)
    out = enc.encode(tiles, list(wk.tile_offsets))
    torch.cuda.synchronize()
    assert tuple(out.shape) == (104 * 256, 4096)
    assert bool(torch.isfinite(out.float()).all())
    check_sample(wk, enc, out, wk.oracle_sample_tiles)
    again = enc.encode(tiles, list(wk.tile_offsets))
    torch.cuda.synchronize()
    assert torch.equal(again.view(torch.int16), out.view(torch.int16))
    enc.close()


def test_c8_siglip_shape_with_resampler_10_slices():
    wk = wl.workload("c8")
    enc, tiles = build(wk)
    out = enc.encode(tiles, list(wk.tile_offsets))
    torch.cuda.synchronize()
    assert tuple(out.shape) == (10 * 64, 3584)
    check_sample(wk, enc, out, wk.oracle_sample_tiles)
    enc.close()


def test_siglip_shape_at_378_pixels_729_patches_per_slice():
    """The C2 encoder at 378-pixel slices: a 27 x 27 patch grid, 729 tokens per slice in rows padded to
    736, the last key block masked from key 729 on; more slices than a micro-batch holds."""
    desc = wl.workload("c2").desc.replace(tile_size=378, max_tiles_per_call=4)
    wk = wl.Workload("siglip_378", desc, 1012, 1012, (0, 6), ((6,),), (0, 5))
    enc, tiles = build(wk)
    out = enc.encode(tiles, [0, 6])
    torch.cuda.synchronize()
    assert tuple(out.shape) == (6 * 729, 3584)
    check_sample(wk, enc, out, wk.oracle_sample_tiles)
    enc.close()


def test_c6_video_requests_batched_equals_one_request_per_call_and_oracle():
    """Video workload: 16 requests of 8 to 64 frames, one slice per frame.  Encoding every request in
    its own call (maximum encode batch size 1) gives the bits of the one batched call."""
    wk = wl.workload("c6")
    enc, tiles = build(wk)
    off = list(wk.tile_offsets)
    n = enc.tokens_per_tile
    full = enc.encode(tiles, off)
    torch.cuda.synchronize()
    assert full.shape == (480 * 1024, 3584)
    out = enc.alloc_out(wk.n_tiles)
    out.fill_(-3.0)
    for r in range(wk.n_requests):
        enc.encode(tiles[off[r]:off[r + 1]], [0, off[r + 1] - off[r]], out[off[r] * n:off[r + 1] * n])
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), full.view(torch.int16))
    check_sample(wk, enc, full, wk.oracle_sample_tiles)
    enc.close()


@pytest.mark.parametrize("name,reps", [("c2", 300), ("c3", 30)])
def test_full_size_runs_repeat_bit_for_bit(name, reps):
    """The same batch encoded again and again gives the same bits at the full GEMM shapes, where every
    compute unit holds a tile and the chip is at its power limit: a data hazard in a kernel (a register
    rewritten while a store still reads it, a missing wait) shows up here as an occasional run that differs
    in whole slices, never in the small cases."""
    wk = wl.workload(name)
    enc, tiles = build(wk)
    off = list(wk.tile_offsets)
    ref = enc.encode(tiles, off).clone()
    torch.cuda.synchronize()
    differing = 0
    for _ in range(reps):
        out = enc.encode(tiles, off)
        torch.cuda.synchronize()
        differing += int(not torch.equal(out.view(torch.int16), ref.view(torch.int16)))
    assert differing == 0, f"{differing} of {reps} runs differ from the first"
    # One worker's share of the first request, alone: other kernels altogether (64 x 64 tiles fed through an LDS ring,
    # both projections of the input in one launch), whose hand-over rests on counted waits.  Every repeat carries the
    # bits the same slices have inside the whole batch.
    n = enc.tokens_per_tile
    for k in (1, 2, 3):
        differing = 0
        for _ in range(60):
            out = enc.encode(tiles[:k], [0, k])
            torch.cuda.synchronize()
            differing += int(not torch.equal(out.view(torch.int16), ref[:k * n].view(torch.int16)))
        assert differing == 0, f"{k} slices alone: {differing} of 60 runs differ from their rows of the whole batch"
    enc.close()
