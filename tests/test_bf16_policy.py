"""Host-side checks of the bf16 mode's arithmetic choices (no GPU): the error the rounding policy
alone costs on the sharpened resampler case, and the bound of the fitted GELU of the bf16 epilogues."""
import os
import re

import numpy as np
import torch

import workloads as wl
from oracle import epd_oracle as O
from bf16_model import resampler_policy_error, snap_bf16

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
