"""The pre-norms folded into the products (bf16 mode): row statistics, the residual epilogue that emits them,
and the product that applies them, each against the CPU oracle's steps; and the whole encoder with and without
the fold."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import epd_oracle as O
from paper_2501_05460_amd import binding as B
from bf16_model import snap_bf16
from gpu_util import make_encoder, rel_err, to_host, tol

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bf16_grid(rng, shape, scale=1.0):
    return wl.to_bf16_grid((rng.standard_normal(shape) * scale).astype(np.float32))


def _combine(pairs, dim):
    """Mean and biased variance of every row from its (mean, squared-deviation) pairs, in float64."""
    pairs = pairs.astype(np.float64)
    n_part = pairs.shape[1]
    cnt = np.array([min(128, dim - 128 * g) for g in range(n_part)], np.float64)
    mu = (pairs[:, :, 0] * cnt).sum(1) / dim
    m2 = (pairs[:, :, 1] + cnt * (pairs[:, :, 0] - mu[:, None]) ** 2).sum(1)
    return mu, m2 / dim


@pytest.mark.parametrize("dim", [1024, 1152, 200, 3200])
def test_row_statistics_vs_numpy_including_rows_far_from_zero(dim):
    """Rows with a mean of 1000 standard deviations: a variance taken from sums of squares would lose every
    digit there; the pairs (per 128 columns: mean, squared deviations from that mean) keep it to rounding."""
    rng = np.random.default_rng(dim)
    x = rng.standard_normal((37, dim)).astype(np.float32)
    x[3] += 1000.0
    x[4] = x[4] * 0.05 - 250.0                    # 5000 standard deviations from zero
    x[5] = 7.25                                    # constant row: variance exactly 0
    xb, stats = B.op_row_stats(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(xb.float().cpu().numpy(), snap_bf16(x))
    pairs = stats.cpu().numpy()
    assert not np.isnan(pairs).any()
    for g in range(pairs.shape[1]):
        blk = x[:, 128 * g:128 * (g + 1)].astype(np.float64)
        np.testing.assert_allclose(pairs[:, g, 0], blk.mean(1), rtol=2e-6, atol=1e-6)
        want_m2 = ((blk - blk.mean(1, keepdims=True)) ** 2).sum(1)
        np.testing.assert_allclose(pairs[:, g, 1], want_m2, rtol=2e-4, atol=1e-9 * blk.shape[1])
    mu, var = _combine(pairs, dim)
    np.testing.assert_allclose(mu, x.astype(np.float64).mean(1), rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(var, x.astype(np.float64).var(1), rtol=3e-4, atol=1e-12)
    assert var[5] == 0.0


@pytest.mark.parametrize("M,N,K", [(512, 1024, 256), (256, 1152, 384), (768, 128, 512)])
def test_residual_epilogue_emits_the_rows_and_their_statistics_in_every_tile_shape(M, N, K):
    rng = np.random.default_rng(M + N + K)
    a = B.to_device(_bf16_grid(rng, (M, K)), True)
    w = B.to_device(_bf16_grid(rng, (N, K), 0.05), True)
    bias = torch.from_numpy(rng.standard_normal(N).astype(np.float32)).cuda()
    r0 = rng.standard_normal((M, N)).astype(np.float32)
    r0[5] += 500.0
    plain = B.op_gemm_bf16_form(a, w, bias, 3, 0, torch.from_numpy(r0).cuda())
    torch.cuda.synchronize()
    forms = [0, 1, 2] + ([3] if K % 256 == 0 else []) + ([6, 7, 8] if N % 256 == 0 else [])
    ref = None
    for form in forms:
        r = torch.from_numpy(r0).cuda()
        xb, stats = B.op_gemm_residual_stats(a, w, bias, r, form)
        torch.cuda.synchronize()
        assert torch.equal(r.view(torch.int32), plain.view(torch.int32)), form     # emitting changes no bit of R
        assert np.array_equal(xb.float().cpu().numpy(), snap_bf16(r.cpu().numpy())), form
        if ref is None:
            ref = stats.clone()
            mu, var = _combine(stats.cpu().numpy(), N)
            x = r.cpu().numpy().astype(np.float64)
            np.testing.assert_allclose(mu, x.mean(1), rtol=1e-6, atol=1e-6)
            np.testing.assert_allclose(var, x.var(1), rtol=3e-4)
        else:
            assert torch.equal(stats.view(torch.int32), ref.view(torch.int32)), form   # same bits in every shape


@pytest.mark.parametrize("kind", ["layernorm", "rmsnorm"])
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_folded_norm_product_vs_oracle(kind, epi):
    """act(norm(x) W^T + b): the product runs on bf16(x) against gain-scaled weights and takes mean and rstd
    in its epilogue.  Rows with a mean of a few standard deviations and with a large scale are in the batch.
    Every tile shape gives the same bits."""
    M, N, D = 512, 512, 1024
    rng = np.random.default_rng(11 + epi)
    x = rng.standard_normal((M, D)).astype(np.float32)
    x[7] += 4.0
    x[8] *= 300.0
    x[9] = x[9] * 0.01 + 0.02
    gamma = (1.0 + 0.1 * rng.standard_normal(D)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(D)).astype(np.float32) if kind == "layernorm" else None
    w = _bf16_grid(rng, (N, D), 0.03)
    bias = rng.standard_normal(N).astype(np.float32)
    eps = 1e-6
    u = O.layer_norm(x, gamma, beta, eps) if beta is not None else O.rms_norm(x, gamma, eps)
    want = O.linear(u, w, bias)
    want = O.gelu_erf(want) if epi == 1 else O.gelu_tanh(want) if epi == 2 else want
    dev = lambda a: torch.from_numpy(a).cuda()
    ref = None
    for form in (0, 1, 2, 3, 6, 7, 8, 9):
        c = B.op_norm_gemm_bf16(dev(x), dev(gamma), dev(beta) if beta is not None else None, B.to_device(w, True),
                                dev(bias), eps, epi, form)
        torch.cuda.synchronize()
        if ref is None:
            ref = c.clone()
            got = c.float().cpu().numpy()
            e = rel_err(got, want)
            print(f"{kind} epi {epi}: max_rel_err {e:.3e}")
            assert e < 6e-3
        else:
            assert torch.equal(c.view(torch.int16), ref.view(torch.int16)), form


def _encode_in_subprocess(mode: str, path: str):
    """How the pre-norms run is chosen when a context is created (EPD_NORM_MODE): run the same small encode in
    a process of its own with the variable set, and hand the tokens back through a file."""
    code = f"""
import sys, numpy as np, torch
sys.path.insert(0, {ROOT!r}); sys.path.insert(0, {os.path.join(ROOT, 'tests')!r})
import workloads as wl
from gpu_util import make_encoder
desc = wl.ModelDesc(dtype=wl.DT_BF16, tile_size=224, patch=14, hidden=192, heads=3, mlp=384, layers=3, norm=wl.NORM_LAYERNORM,
                    qk_norm=wl.QKNORM_NONE, act=wl.ACT_GELU_ERF, final_norm=0, pixel_shuffle=1, proj_kind=wl.PROJ_MLP,
                    proj_prenorm=1, proj_mid=256, proj_out=128, eps=1e-6, max_tiles_per_call=8)
w = wl.gen_weights(desc, 77, std=0.06)
enc = make_encoder(desc, w)
out = enc.encode(torch.from_numpy(wl.gen_tiles(desc, 77, 3)).cuda(), [0, 3])
torch.cuda.synchronize()
np.save({path!r}, out.float().cpu().numpy())
"""
    env = dict(os.environ)
    env["EPD_NORM_MODE"] = mode
    subprocess.run([sys.executable, "-c", code], check=True, env=env, timeout=300)
    return np.load(path)


def test_the_three_forms_of_the_pre_norms_agree_with_the_oracle_and_each_other(tmp_path):
    out = {m: _encode_in_subprocess(m, str(tmp_path / f"{m}.npy")) for m in ("classic", "copy", "fold")}
    desc = wl.ModelDesc(dtype=wl.DT_BF16, tile_size=224, patch=14, hidden=192, heads=3, mlp=384, layers=3, norm=wl.NORM_LAYERNORM,
                        qk_norm=wl.QKNORM_NONE, act=wl.ACT_GELU_ERF, final_norm=0, pixel_shuffle=1, proj_kind=wl.PROJ_MLP,
                        proj_prenorm=1, proj_mid=256, proj_out=128, eps=1e-6, max_tiles_per_call=8)
    w = wl.gen_weights(desc, 77, std=0.06)
    want = O.encode(wl.gen_tiles(desc, 77, 3), [0, 3], w, desc)
    for m, got in out.items():
        e = rel_err(got, want)
        print(f"{m}: max_rel_err {e:.3e}")
        assert e < tol(desc), m
    for a, b in (("classic", "copy"), ("classic", "fold"), ("copy", "fold")):
        assert not np.array_equal(out[a], out[b]), (a, b)          # three different arithmetic paths did run
        assert rel_err(out[a], out[b]) < 1e-2, (a, b)
