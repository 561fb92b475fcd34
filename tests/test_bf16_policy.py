"""Host-side checks of the bf16 mode's arithmetic choices (no GPU): the error the rounding policy
alone costs on the sharpened resampler case, and the bound of the fitted GELU of the bf16 epilogues."""
import os
import re

import numpy as np
import torch

import workloads as wl
from oracle import epd_oracle as O
from bf16_model import encoder_policy_error, resampler_policy_error, snap_bf16

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_snap_bf16_is_round_to_nearest_even():
    rng = np.random.default_rng(3)
    a = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 4096),
                        np.float32([0.0, 1.0, 1.00390625, 1.01171875, -3.0e38, 65280.0, 65408.0])])
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(snap_bf16(a), want)


def resampler_case(seed, sharpen):
    desc = wl.ModelDesc(dtype=wl.DT_BF16, tile_size=448, patch=14, hidden=128, heads=2, mlp=304, layers=1,
                        norm=wl.NORM_LAYERNORM, qk_norm=wl.QKNORM_NONE, act=wl.ACT_GELU_ERF, final_norm=1,
                        pixel_shuffle=0, proj_kind=wl.PROJ_RESAMPLER, proj_prenorm=0, proj_mid=64, proj_out=256,
                        eps=1e-6, max_tiles_per_call=2, proj_heads=2)
    w = wl.gen_weights(desc, seed, std=0.08, scale={"r_in_w": sharpen})
    return desc, w, wl.gen_tiles(desc, seed, 2)


def test_sharpened_resampler_sits_at_the_bf16_tolerance_by_construction():
    """The GPU stress test of the resampler (1024 keys per query) sharpens the in-projections by 1.25, not
    1.5.  Reason, shown here without any kernel: with in-projections x 1.5 the roundings of the bf16 mode
    alone (bf16 operands of every product, bf16 softmax weights, exact arithmetic otherwise, exact trunk)
    cost 1.1e-2 .. 1.4e-2 of the 2e-2 tolerance, and the rounding of q, k and the weights alone, which no
    bf16 attention kernel avoids, 0.5e-2 .. 1.1e-2; what a kernel adds on top (fp32 accumulation order,
    the bf16 trunk) then decides between pass and fail.  At x 1.25 the policy costs about half the
    tolerance."""
    for seed in (25, 26):
        desc, w, tiles = resampler_case(seed, 1.5)
        full = resampler_policy_error(desc, w, tiles)
        least = resampler_policy_error(desc, w, tiles, only_qkp=True)
        print(f"seed {seed} x1.5: policy {full:.3e}, q/k/weights only {least:.3e}")
        assert 0.9e-2 < full < 2e-2, (seed, full)
        assert 4e-3 < least <= full * 1.2, (seed, least)
        desc, w, tiles = resampler_case(seed, 1.25)
        mild = resampler_policy_error(desc, w, tiles)
        print(f"seed {seed} x1.25: policy {mild:.3e}")
        assert mild < 1.3e-2 and mild < full * 1.05, (seed, mild)


def test_a_bf16_residual_stream_triples_what_the_rounding_policy_costs():
    """The residual stream stays fp32 between kernels.  A bf16 stream would halve the bytes the residual epilogues
    and the pre-norms move, and is allowed if it keeps the 2e-2 bound at the deepest encoder; decided by what the
    roundings alone cost (no kernel involved), one slice of the full-size workloads, fp32 stream against bf16
    stream, max |model - oracle| / max |oracle|:
        SigLIP-shaped, 27 layers         4.2e-3  ->  1.26e-2
        InternViT-300M-shaped, 24 layers 3.7e-3  ->  1.15e-2
        InternViT-6B-shaped, 45 layers   4.1e-3  ->  1.53e-2
    With what the kernels add on top (fp32 summation order, the fitted GELU: the 24-layer shape measures 5.5e-3
    against its 3.7e-3) the 45-layer shape would sit at the bound, so the stream is fp32.  Here the same
    comparison on an encoder small enough for the CPU suite: the bf16 stream at least doubles the error, and the
    error of the fp32 stream does not grow with depth the way the bf16 one does."""
    def case(layers):
        desc = wl.ModelDesc(dtype=wl.DT_BF16, tile_size=112, patch=14, hidden=128, heads=2, mlp=512, layers=layers,
                            norm=wl.NORM_LAYERNORM, qk_norm=wl.QKNORM_NONE, act=wl.ACT_GELU_ERF, final_norm=0,
                            pixel_shuffle=0, proj_kind=wl.PROJ_LINEAR, proj_prenorm=0, proj_mid=0, proj_out=128,
                            eps=1e-6, max_tiles_per_call=1)
        w = wl.gen_weights(desc, 77)
        tile = wl.gen_tile(desc, 77, 0)
        return encoder_policy_error(tile, w, desc, False), encoder_policy_error(tile, w, desc, True)
    f6, b6 = case(6)
    f24, b24 = case(24)
    print(f"6 layers: fp32 stream {f6:.3e}, bf16 stream {b6:.3e}; 24 layers: {f24:.3e}, {b24:.3e}")
    assert b6 > 2.0 * f6 and b24 > 2.0 * f24
    assert b24 > 1.5 * b6          # a rounding per residual add: grows like the square root of the depth
    assert f24 < 2e-2 / 3 and b24 < 2e-2


def _gelu_fast_coefficients(name):
    src = open(os.path.join(ROOT, "paper_2501_05460_amd", "csrc", "common.h")).read()
    body = src[src.index(f"float {name}(float x)"):]
    m = re.search(r"fmaf\(x \* x, (-?[0-9.e+-]+)f, (-?[0-9.e+-]+)f\)", body)
    return float(m.group(1)), float(m.group(2))


def test_fitted_gelu_of_the_bf16_epilogues_stays_within_its_stated_bound():
    """The bf16 epilogues evaluate GELU as x / (1 + exp2(x (b x^2 + a))) with the two coefficients in
    csrc/common.h (read from the source here).  Evaluated in float64 on a dense grid, the erf form stays
    within 2.71e-4 of x Phi(x) and the tanh form reproduces the tanh formula to rounding."""
    x = np.linspace(-12.0, 12.0, 480001)
    b, a = _gelu_fast_coefficients("gelu_erf_fast")
    got = x / (1.0 + np.exp2(x * (b * x * x + a)))
    err = np.abs(got - O.gelu_erf(x))
    print(f"fitted erf-form GELU: max |error| = {err.max():.3e} at x = {x[err.argmax()]:.3f}")
    assert err.max() <= 2.72e-4
    assert err[np.abs(x) > 6.0].max() < 1e-6            # the tails follow x and 0
    b, a = _gelu_fast_coefficients("gelu_tanh_fast")
    got = x / (1.0 + np.exp2(x * (b * x * x + a)))
    assert np.abs(got - O.gelu_tanh(x)).max() < 2e-7      # same function, coefficients folded in fp32
