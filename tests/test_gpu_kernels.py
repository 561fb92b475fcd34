"""Kernel-level parity on the GPU: MFMA lane layout, the bf16 GEMM and the
tile-local flash attention against the CPU oracle's steps."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import epd_oracle as O
from paper_2501_05460_amd import binding as B
from gpu_util import rel_err

pytestmark = pytest.mark.gpu


def _bf16_grid(rng, shape, scale=1.0):
    return wl.to_bf16_grid((rng.standard_normal(shape) * scale).astype(np.float32))


def test_mfma_lane_layout():
    rng = np.random.default_rng(0)
    a = _bf16_grid(rng, (32, 16))
    b = _bf16_grid(rng, (16, 32))
    d = B.op_mfma_probe(B.to_device(a, True), B.to_device(b, True))
    torch.cuda.synchronize()
    want = a.astype(np.float64) @ b.astype(np.float64)
    np.testing.assert_allclose(d.cpu().numpy(), want, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("M,N,K", [(256, 128, 128), (512, 256, 256), (768, 384, 384), (256, 1152, 1152), (2560, 640, 640),
                                   (1024, 4352, 1152), (2048, 1024, 4096)])
def test_gemm_bf16_vs_oracle_linear(M, N, K):
    rng = np.random.default_rng(M + N + K)
    a = _bf16_grid(rng, (M, K))
    w = _bf16_grid(rng, (N, K), 0.05)
    bias = rng.standard_normal(N).astype(np.float32)
    c, _ = B.op_gemm_bf16(B.to_device(a, True), B.to_device(w, True), torch.from_numpy(bias).cuda())
    torch.cuda.synchronize()
    want = O.linear(a, w, bias)
    # fp32 accumulation, one bf16 rounding of the result: 2^-9 relative per element
    got = c.float().cpu().numpy()
    assert rel_err(got, want) < 6e-3
    np.testing.assert_allclose(got, want, rtol=2 ** -7, atol=2 ** -7 * np.abs(want).max() * 0.05)


def _scaled_q(q, hd):
    """The attention kernel takes its logits in the log2 domain straight from q . k: q carries the factor
    log2(e) / sqrt(hd) (the library folds it into the q projection).  Returns that q on the bf16 grid, and the
    q the oracle has to be given so that its logits q . k / sqrt(hd) are the same numbers."""
    c = math.log2(math.e) / math.sqrt(hd)
    qs = torch.from_numpy(np.asarray(q * c, np.float32)).bfloat16().float().numpy()
    return qs, qs.astype(np.float64) / c


def _attention_case(n_slices, n_tok, heads, hd, hd_pad, qk_scale, seed):
    rng = np.random.default_rng(seed)
    M = n_slices * n_tok
    D = heads * hd
    q = _bf16_grid(rng, (M, D), qk_scale)
    k = _bf16_grid(rng, (M, D), qk_scale)
    v = _bf16_grid(rng, (M, D))
    Dq = heads * hd_pad

    def pad_heads(x):
        out = np.zeros((M, Dq), np.float32)
        for h in range(heads):
            out[:, h * hd_pad:h * hd_pad + hd] = x[:, h * hd:(h + 1) * hd]
        return out

    q_dev, q = _scaled_q(q, hd)
    qk = np.concatenate([pad_heads(q_dev), pad_heads(k)], axis=1)          # [M, 2*Dq]
    vt = pad_heads(v).reshape(n_slices, n_tok, heads, hd_pad).transpose(0, 2, 3, 1).copy()
    qk_d = B.to_device(qk, True)
    o = B.op_attention_bf16(qk_d, qk_d[:, Dq:], B.to_device(vt, True), n_slices, n_tok, heads, hd_pad, 2 * Dq)
    torch.cuda.synchronize()
    got = o.float().cpu().numpy().reshape(M, heads, hd_pad)
    assert np.all(got[:, :, hd:] == 0.0)
    got = got[:, :, :hd].reshape(M, D)
    want = np.concatenate([O.attention(q[s * n_tok:(s + 1) * n_tok], k[s * n_tok:(s + 1) * n_tok],
                                       v[s * n_tok:(s + 1) * n_tok], heads) for s in range(n_slices)])
    return got, want


@pytest.mark.parametrize("n_slices,n_tok,heads,hd,hd_pad", [
    (1, 64, 1, 64, 64), (2, 256, 3, 64, 64), (3, 1024, 2, 64, 64), (2, 1024, 2, 72, 96),
    (2, 1024, 2, 128, 128), (1, 192, 2, 32, 64), (2, 1024, 2, 72, 72), (1, 128, 3, 72, 72),
    (1, 256, 2, 80, 96)])
@pytest.mark.parametrize("qk_scale", [0.25, 1.0])
def test_attention_bf16_vs_oracle(n_slices, n_tok, heads, hd, hd_pad, qk_scale):
    # N(0,1) q/k give logits with std ~ 1..3 after scaling by 1/sqrt(hd) * hd^0.5:
    # sharp softmax rows, so a wrong key set or a cross-slice leak is visible
    got, want = _attention_case(n_slices, n_tok, heads, hd, hd_pad, qk_scale, seed=n_tok + hd)
    assert rel_err(got, want) < 1.5e-2


@pytest.mark.parametrize("n_tok,n_keys,heads,hd,hd_pad", [
    (128, 65, 2, 64, 64), (320, 257, 1, 64, 64), (1088, 1025, 2, 64, 64), (64, 1, 1, 64, 64),
    (128, 96, 2, 72, 72), (256, 197, 2, 128, 128), (192, 129, 1, 80, 96)])
def test_attention_bf16_ignores_rows_past_n_keys(n_tok, n_keys, heads, hd, hd_pad):
    """A slice owns n_tok rows but only n_keys of them are tokens (class token + patches, padded to the
    key block): the real queries see exactly the real keys, whatever the padding rows hold (here: large
    values that would take all the softmax weight if they leaked in)."""
    rng = np.random.default_rng(n_tok + n_keys + hd)
    n_slices = 2
    M = n_slices * n_tok
    D, Dq = heads * hd, heads * hd_pad
    q = _bf16_grid(rng, (M, D), 0.5)
    k = _bf16_grid(rng, (M, D), 0.5)
    v = _bf16_grid(rng, (M, D))
    real = (np.arange(M) % n_tok) < n_keys
    k[~real] *= 16.0
    v[~real] = 100.0

    def pad_heads(x):
        out = np.zeros((M, Dq), np.float32)
        for h in range(heads):
            out[:, h * hd_pad:h * hd_pad + hd] = x[:, h * hd:(h + 1) * hd]
        return out

    q_dev, q = _scaled_q(q, hd)
    qk = np.concatenate([pad_heads(q_dev), pad_heads(k)], axis=1)
    vt = pad_heads(v).reshape(n_slices, n_tok, heads, hd_pad).transpose(0, 2, 3, 1).copy()
    qk_d = B.to_device(qk, True)
    o = B.op_attention_bf16(qk_d, qk_d[:, Dq:], B.to_device(vt, True), n_slices, n_tok, heads, hd_pad,
                            2 * Dq, n_keys=n_keys)
    torch.cuda.synchronize()
    got = o.float().cpu().numpy().reshape(M, heads, hd_pad)[:, :, :hd].reshape(M, D)
    assert np.isfinite(got).all()
    for s in range(n_slices):
        r = slice(s * n_tok, s * n_tok + n_keys)
        want = O.attention(q[r], k[r], v[r], heads)
        assert rel_err(got[r], want) < 1.5e-2, s


def _attention_run(q, k, v, n_slices, n_tok, heads, hd):
    """q, k, v [M, heads * hd] on the bf16 grid -> kernel output and oracle output, both [M, heads * hd]."""
    M, D = q.shape
    q_dev, q = _scaled_q(q, hd)
    qk = np.concatenate([q_dev, k], axis=1).astype(np.float32)
    vt = v.reshape(n_slices, n_tok, heads, hd).transpose(0, 2, 3, 1).copy().astype(np.float32)
    qk_d = B.to_device(qk, True)
    o = B.op_attention_bf16(qk_d, qk_d[:, D:], B.to_device(vt, True), n_slices, n_tok, heads, hd, 2 * D)
    torch.cuda.synchronize()
    got = o.float().cpu().numpy().reshape(M, D)
    want = np.concatenate([O.attention(q[s * n_tok:(s + 1) * n_tok], k[s * n_tok:(s + 1) * n_tok],
                                       v[s * n_tok:(s + 1) * n_tok], heads) for s in range(n_slices)])
    return got, want


def _snap_bf16(x):
    return torch.from_numpy(np.asarray(x, np.float32)).bfloat16().float().numpy()


@pytest.mark.parametrize("hd", [64, 72, 128])
@pytest.mark.parametrize("kind", ["all_low", "rising", "falling", "wide"])
def test_attention_bf16_extreme_logits(kind, hd):
    """Logits far from zero and running maxima that move by large steps: the kernel shifts the logits
    by a reference value that follows the running maximum lazily, and every move rescales what has
    been accumulated.  all_low: every logit is -128 (closed form: the mean of V); rising: the
    maximum grows by ~11 (log2 units) per 32 keys, so the reference moves at every step; falling:
    the first key dominates and the later weights underflow; wide: random logits with std ~ 9."""
    n_slices, n_tok, heads = 2, 1024, 2
    M, D = n_slices * n_tok, heads * hd
    rng = np.random.default_rng(7 + hd)
    v = _bf16_grid(rng, (M, D))
    pos = (np.arange(M) % n_tok).astype(np.float32)[:, None]
    if kind == "all_low":
        q = np.full((M, D), 4.0, np.float32) * math.sqrt(64.0 / hd)
        k = -q
    elif kind in ("rising", "falling"):
        q = np.ones((M, D), np.float32)
        ramp = pos / n_tok if kind == "rising" else 1.0 - pos / n_tok
        k = np.broadcast_to(ramp * 32.0 * math.sqrt(64.0 / hd), (M, D)).copy()
    else:
        q = _bf16_grid(rng, (M, D), 3.0)
        k = _bf16_grid(rng, (M, D), 3.0)
    q, k = _snap_bf16(q), _snap_bf16(k)
    got, want = _attention_run(q, k, v, n_slices, n_tok, heads, hd)
    assert np.isfinite(got).all()
    assert rel_err(got, want) < 1.5e-2
    if kind == "all_low":
        mean_v = np.concatenate([np.broadcast_to(v[s * n_tok:(s + 1) * n_tok].mean(axis=0), (n_tok, D))
                                 for s in range(n_slices)])
        assert np.abs(got - mean_v).max() < 1e-2 * np.abs(v).max()


@pytest.mark.parametrize("epi,abs_err", [(1, 2.7e-4), (2, 2e-6)])
def test_gemm_gelu_epilogues_vs_oracle(epi, abs_err):
    """The activation inside the product's epilogue, element by element: pre-activations spread over
    +-5; the erf form is a fitted logistic with |error| <= 2.7e-4 against x Phi(x), the tanh form is
    exact up to fp32 rounding; on top of either comes one bf16 rounding of the output (at most 2^-8 relative)."""
    rng = np.random.default_rng(90 + epi)
    M, N, K = 640, 256, 256
    a = _bf16_grid(rng, (M, K), 1.0)
    w = _bf16_grid(rng, (N, K), 0.1)
    bias = (rng.standard_normal(N) * 0.5).astype(np.float32)
    out = B.op_gemm_bf16_form(B.to_device(a, True), B.to_device(w, True), torch.from_numpy(bias).cuda(), epi, 0)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    pre = O.linear(a, w, bias)
    assert np.abs(pre).max() > 4.0 and (np.abs(pre) < 0.5).mean() > 0.1    # both tails and the middle are sampled
    want = O.gelu_erf(pre) if epi == 1 else O.gelu_tanh(pre)
    # fp32 accumulation of K = 256 products adds ~1e-6 to the pre-activation: far below either term
    bound = abs_err + 1e-5 + 2.0 ** -8 * np.abs(want)   # half a bf16 step is 2^-8 relative at the bottom of a binade
    excess = np.abs(got - want) - bound
    assert excess.max() <= 0.0, (float(excess.max()), float(pre.flat[excess.argmax()]))


@pytest.mark.parametrize("M,N,K", [(256, 256, 128), (1000, 512, 256), (2304, 1024, 1024), (77, 256, 384)])
@pytest.mark.parametrize("epi", [0, 1, 2, 3])
def test_gemm_forms_agree_bit_for_bit(M, N, K, epi):
    """The plain loop, the pipelined loop (weights straight into LDS, fragments one k-step ahead) and
    the persistent kernel order every sum the same way: identical bits, ragged M included; the
    256x128, 128x128 and 64x64 tiles too."""
    rng = np.random.default_rng(M + N + K + epi)
    A = B.to_device(_bf16_grid(rng, (M, K), 0.5), True)
    W = B.to_device(_bf16_grid(rng, (N, K), 0.05), True)
    bias = torch.from_numpy(rng.standard_normal(N).astype(np.float32) * 0.1).cuda()
    r0 = torch.from_numpy(rng.standard_normal((M, N)).astype(np.float32)).cuda()

    def run(form):
        R = r0.clone() if epi == 3 else None
        out = B.op_gemm_bf16_form(A, W, bias, epi, form, R)
        torch.cuda.synchronize()
        return out.view(torch.int16 if epi != 3 else torch.int32).cpu().numpy()

    ref = run(6)
    forms = [0, 1, 2, 7, 8, 11] + ([3] if K % 256 == 0 else []) + ([9] if epi != 3 else [10])
    for form in forms:
        assert np.array_equal(run(form), ref), form
    if epi == 0:   # and the value itself, against the oracle
        want = O.linear(A.float().cpu().numpy(), W.float().cpu().numpy(), bias.cpu().numpy())
        got = B.op_gemm_bf16_form(A, W, bias, 0, 0).float().cpu().numpy()
        assert rel_err(got, want) < 6e-3


@pytest.mark.parametrize("M,N,K", [(256, 384, 128), (1000, 1152, 256), (2900, 1152, 1152), (77, 384, 384), (10240, 1152, 128)])
def test_gemm_192_wide_tiles_agree_bit_for_bit(M, N, K):
    """The residual product on 256 x 192 tiles (widths that are whole multiples of 192 and not of 256) leaves the
    bits of the other tile shapes: whole and ragged M, one tile and several per workgroup, and a launch with more
    tiles than CUs (the persistent walk takes a second tile)."""
    rng = np.random.default_rng(M + N + K)
    A = B.to_device(_bf16_grid(rng, (M, K), 0.5), True)
    W = B.to_device(_bf16_grid(rng, (N, K), 0.05), True)
    bias = torch.from_numpy(rng.standard_normal(N).astype(np.float32) * 0.1).cuda()
    r0 = torch.from_numpy(rng.standard_normal((M, N)).astype(np.float32)).cuda()

    def run(form):
        R = r0.clone()
        B.op_gemm_bf16_form(A, W, bias, 3, form, R)
        torch.cuda.synchronize()
        return R.view(torch.int32).cpu().numpy()

    ref = run(1)
    assert np.array_equal(run(12), ref)
    assert np.array_equal(run(2), ref)
    assert np.array_equal(run(0), ref)          # whichever form the library picks for this shape
    want = r0.cpu().numpy().astype(np.float64) + O.linear(A.float().cpu().numpy(), W.float().cpu().numpy(), bias.cpu().numpy())
    assert rel_err(ref.view(np.float32), want) < 1e-4


def test_measurement_probes_run_and_report_sane_figures():
    """The probes behind `bench.py --roof` (no part of the encode path): the register-resident MFMA loop stays below the
    nominal bf16 peak and above a fifth of it, the streaming copy below the nominal HBM rate, and a SIMD that runs a
    wave of MFMAs and a wave of exp + fma pairs together takes longer than either alone and less than both in turn
    (the partial overlap the attention kernel's floor is derived from)."""
    t = B.op_mfma_peak(True, iters=500, reps=2)
    assert 500.0 < t < 2600.0, t
    g = B.op_copy_peak(1 << 28, reps=2)
    assert 1000.0 < g < 8000.0, g
    m, v, both = B.op_coissue(1, 1000, 1250, 2), B.op_coissue(2, 1000, 1250, 2), B.op_coissue(3, 1000, 1250, 2)
    assert m > 0 and v > 0 and max(m, v) * 0.98 <= both <= (m + v) * 1.02, (m, v, both)
