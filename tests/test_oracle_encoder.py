"""Pins for the whole-encoder oracle: an independent composition of PyTorch
CPU library ops (conv2d patch embedding, layer_norm / rms_norm,
scaled_dot_product_attention, gelu, linear, pixel_unshuffle), special cases
with closed forms, and the invariants that follow from slices being encoded
independently (Section 3.2.2)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as wl
from oracle import epd_oracle as O


def small_desc(**kw):
    base = dict(dtype=wl.DT_FP32, tile_size=56, patch=14, hidden=32, heads=2, mlp=64, layers=2,
                norm=wl.NORM_LAYERNORM, qk_norm=wl.QKNORM_NONE, act=wl.ACT_GELU_ERF, final_norm=0,
                pixel_shuffle=0, proj_kind=wl.PROJ_LINEAR, proj_prenorm=0, proj_mid=0, proj_out=24,
                eps=1e-6, max_tiles_per_call=8)
    base.update(kw)
    return wl.ModelDesc(**base)


VARIANTS = {
    "ln_linear": dict(),
    "tanh_mlp": dict(act=wl.ACT_GELU_TANH, proj_kind=wl.PROJ_MLP, proj_mid=40),
    "shuffle_ln_mlp": dict(pixel_shuffle=1, proj_prenorm=1, proj_kind=wl.PROJ_MLP, proj_mid=48),
    "rms_qkfull": dict(norm=wl.NORM_RMSNORM, qk_norm=wl.QKNORM_FULL, pixel_shuffle=1,
                       proj_prenorm=1, proj_kind=wl.PROJ_MLP, proj_mid=48),
    "rms_qkhead_final": dict(norm=wl.NORM_RMSNORM, qk_norm=wl.QKNORM_PER_HEAD, final_norm=1),
    "ln_final": dict(final_norm=1, heads=4),
    "layer_scale": dict(layer_scale=1, pixel_shuffle=1, proj_prenorm=1, proj_kind=wl.PROJ_MLP, proj_mid=48),
    "class_token": dict(class_token=1, final_norm=1),
    "resampler": dict(final_norm=1, proj_kind=wl.PROJ_RESAMPLER, proj_mid=5, proj_heads=3, act=wl.ACT_GELU_TANH),
    "resampler_class_token": dict(class_token=1, proj_kind=wl.PROJ_RESAMPLER, proj_mid=7, proj_heads=2),
    "class_token_shuffle_scale": dict(class_token=1, layer_scale=1, pixel_shuffle=1, proj_prenorm=1,
                                      proj_kind=wl.PROJ_MLP, proj_mid=48),
}


def torch_second_opinion(tile, w, desc):
    """Same encoder from PyTorch CPU library ops, float64."""
    t = {k: torch.from_numpy(np.asarray(v, np.float64)) for k, v in w.items()}
    D, H, p = desc.hidden, desc.heads, desc.patch
    g = desc.tile_size // p
    img = torch.from_numpy(np.asarray(tile, np.float64))[None]            # [1,3,S,S]
    x = F.conv2d(img, t["pe_w"].reshape(D, 3, p, p), t["pe_b"], stride=p)  # [1,D,g,g]
    x = x.flatten(2).transpose(1, 2)[0]                                    # [N,D]
    if desc.class_token:
        # attention does not care where a token sits in the sequence: here the class token goes LAST
        # (with its own position row, row 0 of the table) and is cut off at the end
        x = torch.cat([x + t["pos"][1:], (t["cls"] + t["pos"][0])[None]], dim=0)
    else:
        x = x + t["pos"]

    def norm(x, prefix, kind):
        if kind == wl.NORM_LAYERNORM:
            return F.layer_norm(x, (x.shape[-1],), t[prefix + "_g"], t[prefix + "_b"], desc.eps)
        return F.rms_norm(x, (x.shape[-1],), t[prefix + "_g"], desc.eps)

    for l in range(desc.layers):
        pre = f"l{l}_"
        u = norm(x, pre + "n1", desc.norm)
        q, k, v = F.linear(u, t[pre + "qkv_w"], t[pre + "qkv_b"]).chunk(3, dim=-1)
        if desc.qk_norm == wl.QKNORM_FULL:
            q = F.rms_norm(q, (D,), t[pre + "qn_g"], desc.eps)
            k = F.rms_norm(k, (D,), t[pre + "kn_g"], desc.eps)
        hd = D // H
        q, k, v = (a.reshape(-1, H, hd).transpose(0, 1) for a in (q, k, v))  # [H,N,hd]
        if desc.qk_norm == wl.QKNORM_PER_HEAD:
            q = F.rms_norm(q, (hd,), t[pre + "qn_g"], desc.eps)
            k = F.rms_norm(k, (hd,), t[pre + "kn_g"], desc.eps)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None])[0]    # [H,N,hd]
        o = o.transpose(0, 1).reshape(-1, D)
        ls1 = t[pre + "ls1"] if desc.layer_scale else 1.0
        ls2 = t[pre + "ls2"] if desc.layer_scale else 1.0
        x = torch.addcmul(x, F.linear(o, t[pre + "o_w"], t[pre + "o_b"]), torch.as_tensor(ls1, dtype=x.dtype).expand(D))
        u = norm(x, pre + "n2", desc.norm)
        hmid = F.gelu(F.linear(u, t[pre + "fc1_w"], t[pre + "fc1_b"]),
                      approximate="tanh" if desc.act == wl.ACT_GELU_TANH else "none")
        x = torch.addcmul(x, F.linear(hmid, t[pre + "fc2_w"], t[pre + "fc2_b"]), torch.as_tensor(ls2, dtype=x.dtype).expand(D))
    if desc.final_norm:
        x = norm(x, "fn", desc.norm)
    if desc.class_token:
        x = x[:-1]
    if desc.pixel_shuffle:
        # pixel_unshuffle emits channel c*4 + dy*2 + dx; the encoder's order is (dy*2+dx)*D + c
        y = F.pixel_unshuffle(x.T.reshape(1, D, g, g), 2)                    # [1, 4D, g/2, g/2]
        y = y.reshape(D, 4, -1).permute(2, 1, 0).reshape(-1, 4 * D)
        x = y
    if desc.proj_prenorm:
        x = F.layer_norm(x, (x.shape[-1],), t["pn_g"], t["pn_b"], desc.eps)
    if desc.proj_kind == wl.PROJ_RESAMPLER:
        # the library's multi-head attention module does the in-projections, head split, softmax and out-projection
        E = desc.proj_out
        mha = torch.nn.MultiheadAttention(E, desc.proj_heads, bias=True, batch_first=False, dtype=torch.float64)
        with torch.no_grad():
            mha.in_proj_weight.copy_(t["r_in_w"]); mha.in_proj_bias.copy_(t["r_in_b"])
            mha.out_proj.weight.copy_(t["r_out_w"]); mha.out_proj.bias.copy_(t["r_out_b"])
            kv = F.layer_norm(x @ t["r_kv_w"].T, (E,), t["r_lnkv_g"], t["r_lnkv_b"], desc.eps)
            q = F.layer_norm(t["r_query"], (E,), t["r_lnq_g"], t["r_lnq_b"], desc.eps)
            o = mha(q[:, None], (kv + t["r_pos"])[:, None], kv[:, None], need_weights=False)[0][:, 0]
            x = F.layer_norm(o, (E,), t["r_lnp_g"], t["r_lnp_b"], desc.eps) @ t["r_proj_w"].T
        return x.numpy()
    if desc.proj_kind == wl.PROJ_LINEAR:
        x = F.linear(x, t["pa_w"], t["pa_b"])
    else:
        x = F.linear(F.gelu(F.linear(x, t["pa_w"], t["pa_b"])), t["pb_w"], t["pb_b"])
    return x.numpy()


@pytest.mark.parametrize("variant", sorted(VARIANTS))
def test_encoder_vs_torch_cpu_library_ops(variant):
    desc = small_desc(**VARIANTS[variant])
    # std 0.3 and sharper q/k so that every branch matters numerically
    w = wl.gen_weights(desc, 7, std=0.3)
    tile = wl.gen_tile(desc, 7, 0)
    got = O.encode_tile(tile, w, desc)
    want = torch_second_opinion(tile, w, desc)
    assert got.shape == (desc.tokens_per_tile, desc.out_dim)
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-10)


def test_c1_shape_vs_torch_cpu_library_ops():
    w_ = wl.workload("c1")
    desc = w_.desc
    w = wl.gen_weights(desc, w_.weight_seed)
    tile = wl.gen_tile(desc, w_.input_seed, 0)
    got = O.encode_tile(tile, w, desc)
    assert got.shape == (256, 512)
    np.testing.assert_allclose(got, torch_second_opinion(tile, w, desc), rtol=1e-9, atol=1e-11)


def test_second_opinion_is_sensitive_to_each_part():
    """Guards against a vacuous pin: breaking any single part of the weights
    moves the output by far more than the comparison tolerance."""
    desc = small_desc(**VARIANTS["rms_qkfull"])
    w = wl.gen_weights(desc, 7, std=0.3)
    tile = wl.gen_tile(desc, 7, 0)
    base = O.encode_tile(tile, w, desc)
    for name in w:
        w2 = dict(w)
        # non-constant bump: a constant shift of the last bias is removed by the projector's LayerNorm
        w2[name] = w[name] + 0.05 * np.cos(np.arange(w[name].size)).reshape(w[name].shape)
        assert np.abs(O.encode_tile(tile, w2, desc) - base).max() > 1e-6, name


def test_zero_layers_linear_projector_is_affine_in_pixels():
    desc = small_desc(layers=0)
    w = wl.gen_weights(desc, 11, std=0.2)
    tile = wl.gen_tile(desc, 11, 0)
    got = O.encode_tile(tile, w, desc)
    # brute force: out[n] = pa_w (pe_w a_n + pe_b + pos_n) + pa_b with a_n gathered by hand
    g, p = desc.grid, desc.patch
    for n in (0, 5, g * g - 1):
        y, x = divmod(n, g)
        a = np.array([tile[c, p * y + dy, p * x + dx] for c in range(3) for dy in range(p) for dx in range(p)],
                     dtype=np.float64)
        e = w["pe_w"].astype(np.float64) @ a + w["pe_b"] + w["pos"][n]
        want = w["pa_w"].astype(np.float64) @ e + w["pa_b"]
        np.testing.assert_allclose(got[n], want, rtol=1e-11, atol=1e-12)


def test_zero_output_projections_make_layers_the_identity():
    desc = small_desc()
    w = wl.gen_weights(desc, 12, std=0.2)
    for l in range(desc.layers):
        for nm in ("o_w", "o_b", "fc2_w", "fc2_b"):
            w[f"l{l}_{nm}"] = np.zeros_like(w[f"l{l}_{nm}"])
    tile = wl.gen_tile(desc, 12, 0)
    emb = O.embed_tile(tile, w, desc)
    np.testing.assert_array_equal(O.encode_tile(tile, w, desc), O.linear(emb, w["pa_w"], w["pa_b"]))


def test_tiles_are_independent_and_permutation_permutes_rows():
    desc = small_desc(**VARIANTS["shuffle_ln_mlp"])
    w = wl.gen_weights(desc, 3, std=0.2)
    tiles = wl.gen_tiles(desc, 3, 5)
    n_out = desc.tokens_per_tile
    full = O.encode(tiles, [0, 2, 2, 5], w, desc)
    assert full.shape == (5 * n_out, desc.out_dim)
    perm = [3, 0, 4, 2, 1]
    permuted = O.encode(tiles[perm], [0, 5], w, desc)
    for i, src in enumerate(perm):
        np.testing.assert_array_equal(permuted[i * n_out:(i + 1) * n_out], full[src * n_out:(src + 1) * n_out])
    # a tile alone equals the tile in the batch
    np.testing.assert_array_equal(O.encode(tiles[2:3], [0, 1], w, desc), full[2 * n_out:3 * n_out])
    # changing one tile's pixels changes no other tile's tokens
    tiles2 = tiles.copy(); tiles2[1] += 0.25
    full2 = O.encode(tiles2, [0, 2, 2, 5], w, desc)
    for t in range(5):
        same = np.array_equal(full2[t * n_out:(t + 1) * n_out], full[t * n_out:(t + 1) * n_out])
        assert same == (t != 1)


def test_shards_write_final_rows_and_union_equals_unsharded():
    desc = small_desc()
    w = wl.gen_weights(desc, 4, std=0.2)
    offsets = [0, 3, 3, 9, 10]                      # requests of 3, 0, 6, 1 tiles
    tiles = wl.gen_tiles(desc, 4, offsets[-1])
    n_out = desc.tokens_per_tile
    full = O.encode(tiles, offsets, w, desc)
    sentinel = -777.0
    out = np.full_like(full, sentinel)
    covered = np.zeros(offsets[-1], dtype=int)
    for s in range(4):
        for r in range(len(offsets) - 1):
            n = offsets[r + 1] - offsets[r]
            b, e = wl.shard_range(n, s, 4)
            before = out.copy()
            O.encode_range(tiles, offsets[-1], offsets[r] + b, offsets[r] + e, w, desc, out)
            covered[offsets[r] + b:offsets[r] + e] += 1
            touched = np.any(out != before, axis=1).reshape(-1, n_out).any(axis=1)
            assert set(np.nonzero(touched)[0]) <= set(range(offsets[r] + b, offsets[r] + e))
    assert np.all(covered == 1)
    np.testing.assert_array_equal(out, full)


def test_shard_range_is_a_balanced_partition():
    for n in range(0, 40):
        pieces = [wl.shard_range(n, s, 4) for s in range(4)]
        assert pieces[0][0] == 0 and pieces[-1][1] == n
        assert all(pieces[i][1] == pieces[i + 1][0] for i in range(3))
        sizes = [e - b for b, e in pieces]
        assert max(sizes) - min(sizes) <= 1


def test_workload_shapes_match_the_paper_tables():
    # 13 slices per 4K image for the InternVL-style encoders, 10 for the MiniCPM-V style (Table 3)
    c3 = wl.workload("c3")
    assert c3.n_tiles == 104 and c3.n_requests == 8 and all(t == (13,) for t in c3.image_tiles)
    assert wl.workload("c2").n_tiles == 10
    c5 = wl.workload("c5")
    assert c5.n_requests == 32
    assert all(1 <= len(t) <= 10 and all(1 <= v <= 9 for v in t) for t in c5.image_tiles)
    assert c5.tile_offsets[-1] == sum(sum(t) for t in c5.image_tiles)
    for name, tokens, dim in (("c1", 256, 512), ("c2", 1024, 3584), ("c3", 256, 4096), ("c4", 256, 5120)):
        d = wl.workload(name).desc
        assert (d.tokens_per_tile, d.out_dim) == (tokens, dim)
    assert abs(wl.flops_per_tile(c3.desc) / 1e9 - 740.0) < 1.0


def test_bf16_grid_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -0.3, 1e-3], np.float32)
    r = wl.to_bf16_grid(x)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, want)
    assert r[1] == 1.0 and r[2] == np.float32(1.0 + 2 ** -6)        # ties go to even
    bits = wl.bf16_bits(r)
    back = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(back, r)


@pytest.mark.parametrize("final_norm", [0, 1])
def test_trunk_is_the_encoder_with_an_identity_projector(final_norm):
    """With no shuffle, no projector norm and a Linear projector whose weight is
    the identity, the multimodal tokens are the pre-projection tokens; the
    library-op composition of that encoder pins trunk_tile on its own."""
    desc = small_desc(final_norm=final_norm, proj_out=32)
    w = wl.gen_weights(desc, 21, std=0.08)
    w["pa_w"] = np.eye(32)
    w["pa_b"] = np.zeros(32)
    tile = wl.gen_tiles(desc, 21, 1)[0]
    ref = torch_second_opinion(tile, w, desc)
    got = O.trunk_tile(tile, w, desc)
    assert got.shape == (16, 32)
    assert np.abs(got - ref).max() < 1e-10 * max(1.0, np.abs(ref).max())


def test_project_merge_of_shards_in_slice_order_is_the_encode():
    """Section 3.2.2: shards of pre-projection tokens, put in slice order, projected and merged,
    are the request's multimodal tokens; a wrong shard order is not."""
    desc = small_desc(**VARIANTS["shuffle_ln_mlp"])
    w = wl.gen_weights(desc, 22, std=0.08)
    tiles = wl.gen_tiles(desc, 22, 5)
    ref = np.concatenate([torch_second_opinion(t, w, desc) for t in tiles])
    pre = [O.trunk_tile(t, w, desc) for t in tiles]
    shards = [np.concatenate(pre[0:2]), np.concatenate(pre[2:3]), np.concatenate(pre[3:5])]
    got = O.project_merge(shards, w, desc)
    assert got.shape == (5 * O.tokens_per_tile(desc), desc.proj_out)
    assert np.abs(got - ref).max() < 1e-10 * np.abs(ref).max()
    swapped = O.project_merge([shards[2], shards[1], shards[0]], w, desc)
    assert np.abs(swapped - ref).max() > 1e-3 * np.abs(ref).max()
    n = O.tokens_per_tile(desc)
    assert np.allclose(swapped[:2 * n], ref[3 * n:5 * n], rtol=0, atol=1e-12)


def test_layer_scale_of_ones_changes_nothing_and_of_zeros_removes_the_layers():
    plain = small_desc(final_norm=1)
    scaled = small_desc(final_norm=1, layer_scale=1)
    w = wl.gen_weights(scaled, 23, std=0.08)
    tile = wl.gen_tiles(scaled, 23, 1)[0]
    got = O.encode_tile(tile, w, scaled)
    w_plain = {k: v for k, v in w.items() if not k.endswith(("ls1", "ls2"))}
    base = O.encode_tile(tile, w_plain, plain)
    assert np.abs(got - base).max() > 1e-3 * np.abs(base).max()          # the factors are in use
    for k in w:
        if k.endswith(("ls1", "ls2")):
            w[k] = np.ones_like(w[k])
    assert np.array_equal(O.encode_tile(tile, w, scaled), base)
    for k in w:
        if k.endswith(("ls1", "ls2")):
            w[k] = np.zeros_like(w[k])
    no_layers = O.encode_tile(tile, w_plain, small_desc(final_norm=1, layers=0))
    assert np.allclose(O.encode_tile(tile, w, scaled), no_layers, rtol=0, atol=1e-13)


def test_layer_scale_acts_per_channel_on_the_branch_not_on_the_stream():
    """x + ls * f(x): doubling one channel of ls2 of the last layer moves exactly that channel of
    the pre-projection tokens, by exactly the branch value."""
    desc = small_desc(layer_scale=1)
    w = wl.gen_weights(desc, 24, std=0.08)
    tile = wl.gen_tiles(desc, 24, 1)[0]
    a = O.trunk_tile(tile, w, desc)
    w2 = dict(w)
    ls = np.array(w["l1_ls2"], np.float64).copy()
    ls[5] *= 2.0
    w2["l1_ls2"] = ls
    b = O.trunk_tile(tile, w2, desc)
    diff = b - a
    assert np.abs(np.delete(diff, 5, axis=1)).max() == 0.0
    w3 = dict(w)
    z = np.array(w["l1_ls2"], np.float64).copy()
    z[5] = 0.0
    w3["l1_ls2"] = z
    branch5 = (a - O.trunk_tile(tile, w3, desc))[:, 5]                   # ls2[5] * mlp(x)[:, 5]
    assert np.allclose(diff[:, 5], branch5, rtol=1e-12, atol=1e-14)


def test_class_token_without_layers_only_shifts_the_position_rows():
    """No layers: the class token cannot reach any patch, so token n is the affine map of patch n with
    position row n + 1 (row 0 belongs to the class token), and the class token's own row is not emitted."""
    desc = small_desc(layers=0, class_token=1)
    w = wl.gen_weights(desc, 13, std=0.2)
    tile = wl.gen_tile(desc, 13, 0)
    got = O.encode_tile(tile, w, desc)
    g, p = desc.grid, desc.patch
    assert got.shape == (g * g, desc.out_dim)
    for n in (0, 1, g, g * g - 1):
        y, x = divmod(n, g)
        a = np.array([tile[c, p * y + dy, p * x + dx] for c in range(3) for dy in range(p) for dx in range(p)],
                     dtype=np.float64)
        e = w["pe_w"].astype(np.float64) @ a + w["pe_b"] + w["pos"][n + 1]
        np.testing.assert_allclose(got[n], w["pa_w"].astype(np.float64) @ e + w["pa_b"], rtol=1e-11, atol=1e-12)


def test_class_token_is_one_more_key_for_every_patch():
    """One layer, brute force for one patch query: its attention runs over the g*g patch keys AND the class
    token's key; leaving that key out (or the class vector, or its position row) changes the result."""
    desc = small_desc(layers=1, class_token=1, heads=1)
    w = wl.gen_weights(desc, 17, std=0.3)
    tile = wl.gen_tile(desc, 17, 0)
    trace = {}
    O.trunk_tile(tile, w, desc, trace)
    x0 = trace["embed"]
    assert x0.shape == (desc.n_patches + 1, desc.hidden)
    np.testing.assert_allclose(x0[0], w["cls"].astype(np.float64) + w["pos"][0], rtol=0, atol=1e-15)
    D = desc.hidden
    u = O.layer_norm(x0, w["l0_n1_g"], w["l0_n1_b"], desc.eps)
    qkv = u @ w["l0_qkv_w"].astype(np.float64).T + w["l0_qkv_b"]
    q, k, v = qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:]
    n = 5                                                    # sequence row of patch 4
    logits = np.array([sum(q[n, d] * k[j, d] for d in range(D)) for j in range(x0.shape[0])]) / np.sqrt(D)
    pr = np.exp(logits - logits.max()); pr /= pr.sum()
    o = sum(pr[j] * v[j] for j in range(x0.shape[0]))
    x1 = x0[n] + w["l0_o_w"].astype(np.float64) @ o + w["l0_o_b"]
    u2 = O.layer_norm(x1[None], w["l0_n2_g"], w["l0_n2_b"], desc.eps)[0]
    h = O.gelu_erf(w["l0_fc1_w"].astype(np.float64) @ u2 + w["l0_fc1_b"])
    x2 = x1 + w["l0_fc2_w"].astype(np.float64) @ h + w["l0_fc2_b"]
    np.testing.assert_allclose(trace["layer0"][n], x2, rtol=1e-10, atol=1e-12)
    assert pr[0] > 1e-4      # the class key carries weight, so dropping it would show


def test_resampler_one_query_one_head_by_hand():
    """One learned query, one head: the output token is LayerNorm_post(out_w (sum_j p_j v_j) + out_b) Wp^T with
    p = softmax over the N patch keys of q . k_j / sqrt(E), keys built from LayerNorm_kv(x Wkv^T) + pos and
    values without pos, all written as explicit loops."""
    desc = small_desc(layers=0, proj_kind=wl.PROJ_RESAMPLER, proj_mid=1, proj_heads=1, proj_out=8)
    w = {k: v.astype(np.float64) for k, v in wl.gen_weights(desc, 19, std=0.4).items()}
    tile = wl.gen_tile(desc, 19, 0)
    x = O.trunk_tile(tile, w, desc)
    got = O.project(x, w, desc)
    assert got.shape == (1, 8)
    N, E = x.shape[0], 8

    def ln(v, g, b):
        mu = sum(v) / len(v)
        var = sum((a - mu) ** 2 for a in v) / len(v)
        return np.array([(a - mu) / np.sqrt(var + desc.eps) for a in v]) * g + b

    kv = np.array([ln([sum(w["r_kv_w"][e, d] * x[j, d] for d in range(desc.hidden)) for e in range(E)],
                      w["r_lnkv_g"], w["r_lnkv_b"]) for j in range(N)])
    q = ln(list(w["r_query"][0]), w["r_lnq_g"], w["r_lnq_b"])
    Wq, Wk, Wv = w["r_in_w"][:E], w["r_in_w"][E:2 * E], w["r_in_w"][2 * E:]
    bq, bk, bv = w["r_in_b"][:E], w["r_in_b"][E:2 * E], w["r_in_b"][2 * E:]
    qp = Wq @ q + bq
    logits = np.array([qp @ (Wk @ (kv[j] + w["r_pos"][j]) + bk) for j in range(N)]) / np.sqrt(E)
    pr = np.exp(logits - logits.max()); pr /= pr.sum()
    o = sum(pr[j] * (Wv @ kv[j] + bv) for j in range(N))
    o = w["r_out_w"] @ o + w["r_out_b"]
    want = w["r_proj_w"] @ ln(list(o), w["r_lnp_g"], w["r_lnp_b"])
    np.testing.assert_allclose(got[0], want, rtol=1e-10, atol=1e-12)
    assert pr.max() < 0.9 and pr.max() > 1.5 / N     # neither uniform nor one-hot: the key side matters


def test_resampler_emits_one_token_per_query_for_any_patch_count():
    for tile_size in (56, 84):
        desc = small_desc(tile_size=tile_size, proj_kind=wl.PROJ_RESAMPLER, proj_mid=6, proj_heads=2)
        w = wl.gen_weights(desc, 23, std=0.2)
        out = O.encode([wl.gen_tile(desc, 23, t) for t in range(2)], [0, 2], w, desc)
        assert out.shape == (2 * 6, desc.proj_out) and O.tokens_per_tile(desc) == desc.tokens_per_tile == 6


def test_resampler_does_not_care_about_patch_order_when_the_position_rows_move_along():
    """Cross attention sums over the keys: feeding the patch tokens in another order, with the rows of the
    key position table permuted the same way, gives the same tokens; permuting only one of the two does not."""
    desc = small_desc(layers=0, proj_kind=wl.PROJ_RESAMPLER, proj_mid=4, proj_heads=2)
    w = {k: v.astype(np.float64) for k, v in wl.gen_weights(desc, 29, std=0.4).items()}
    x = O.trunk_tile(wl.gen_tile(desc, 29, 0), w, desc)
    base = O.project(x, w, desc)
    perm = np.random.default_rng(0).permutation(x.shape[0])
    w2 = dict(w)
    w2["r_pos"] = w["r_pos"][perm]
    np.testing.assert_allclose(O.project(x[perm], w2, desc), base, rtol=1e-11, atol=1e-13)
    assert np.abs(O.project(x[perm], w, desc) - base).max() > 1e-3


def test_resampler_with_zero_value_projection_returns_the_bias_path_only():
    """Zero value in-projection weights: every query's attention output is the value bias b_v whatever the
    patches hold, so the tokens equal LayerNorm_post(out_w b_v + out_b) proj_w^T for every query and slice."""
    desc = small_desc(layers=1, proj_kind=wl.PROJ_RESAMPLER, proj_mid=3, proj_heads=2)
    w = {k: v.astype(np.float64) for k, v in wl.gen_weights(desc, 31, std=0.3).items()}
    E = desc.proj_out
    w["r_in_w"] = w["r_in_w"].copy()
    w["r_in_w"][2 * E:] = 0.0
    got = O.encode_tile(wl.gen_tile(desc, 31, 0), w, desc)
    o = w["r_out_w"] @ w["r_in_b"][2 * E:] + w["r_out_b"]
    want = w["r_proj_w"] @ O.layer_norm(o[None], w["r_lnp_g"], w["r_lnp_b"], desc.eps)[0]
    for q in range(3):
        np.testing.assert_allclose(got[q], want, rtol=1e-10, atol=1e-12)
