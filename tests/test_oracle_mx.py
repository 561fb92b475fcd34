"""Pins of the oracle's MXFP8 functions (OCP 8-bit floating point specification, E4M3; OCP Microscaling
Formats specification v1.0, section 6.3 conversion).  Nothing here touches the HIP path."""
import itertools

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import epd_oracle as O

ALL_CODES = np.arange(256, dtype=np.uint8)


def _finite_table():
    v = O.e4m3_decode(ALL_CODES)
    keep = ~np.isnan(v)
    return ALL_CODES[keep], v[keep]


def test_e4m3_decode_equals_the_library_float8_type_on_all_256_codes():
    lib = torch.from_numpy(ALL_CODES.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = O.e4m3_decode(ALL_CODES)
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    assert np.isnan(mine).sum() == 2                       # s.1111.111 only: the format has no infinities
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], mine[ok])


def test_e4m3_landmarks_of_the_format():
    # largest finite 448 = 0x7E, smallest normal 2^-6 = 0x08, smallest subnormal 2^-9 = 0x01, one = 0x38
    assert O.e4m3_decode(0x7E) == 448.0 and O.e4m3_decode(0xFE) == -448.0
    assert O.e4m3_decode(0x08) == 2.0 ** -6
    assert O.e4m3_decode(0x01) == 2.0 ** -9
    assert O.e4m3_decode(0x38) == 1.0
    assert O.e4m3_encode(np.array([448.0, 2.0 ** -6, 2.0 ** -9, 1.0, -1.0, 0.0])).tolist() == [0x7E, 0x08, 0x01, 0x38, 0xB8, 0x00]


def test_e4m3_round_is_the_nearest_code_value_by_brute_force_ties_to_even_mantissa():
    codes, vals = _finite_table()
    rng = np.random.default_rng(7)
    x = rng.normal(size=4000) * np.exp(rng.uniform(-9, 6.2, size=4000))
    pos = np.sort(vals[vals >= 0])
    mid = (pos[:-1] + pos[1:]) / 2                        # every tie of the format
    x = np.concatenate([x, mid, -mid, pos, -pos, [500.0, -1e6, 464.0, 463.9, 2.0 ** -10, 2.0 ** -10 * 1.01, 0.0]])
    got = O.e4m3_round(x)
    for xi, gi in zip(x, got):
        d = np.abs(vals - np.clip(xi, -448, 448))
        best = d.min()
        cand = codes[d == best]
        cand_vals = np.unique(O.e4m3_decode(cand))
        if len(cand_vals) == 1 or (len(cand_vals) == 2 and cand_vals[0] == -cand_vals[1]):   # unique (or +-0)
            assert abs(gi) == abs(cand_vals[-1]) and (gi == 0 or np.sign(gi) == np.sign(xi))
        else:                                             # a tie: the even mantissa wins
            even = np.unique(np.abs(O.e4m3_decode(np.array([c for c in cand if (c & 1) == 0]))))   # +0 and -0 are one value
            assert len(even) == 1 and abs(gi) == even[0]


def test_e4m3_hand_worked_roundings():
    # spacing 1/8 in [1, 2): 1.0625 ties between 1.0 (mantissa 000) and 1.125 (001) -> 1.0;
    # 1.1875 ties between 1.125 (001) and 1.25 (010) -> 1.25; 1.07 -> 1.125
    assert O.e4m3_round(np.array([1.0625, 1.1875, 1.07, -1.0625])).tolist() == [1.0, 1.25, 1.125, -1.0]
    # saturation, and subnormals: multiples of 2^-9, half of the smallest ties to zero (even)
    assert O.e4m3_round(np.array([1000.0, 449.0, -1e9])).tolist() == [448.0, 448.0, -448.0]
    assert O.e4m3_round(np.array([2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -9 * 2.6])).tolist() == [0.0, 2 * 2.0 ** -9, 3 * 2.0 ** -9]


def test_e4m3_round_and_encode_agree_with_the_library_conversion_in_range():
    rng = np.random.default_rng(11)
    x = (rng.normal(size=200000) * np.exp(rng.uniform(-12, 6, size=200000))).astype(np.float32)
    x = np.clip(x, -448, 448)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn)
    assert np.array_equal(lib.to(torch.float64).numpy(), O.e4m3_round(x.astype(np.float64)))
    assert np.array_equal(lib.view(torch.uint8).numpy(), O.e4m3_encode(x.astype(np.float64)))


def test_encode_decode_round_trip_and_idempotence():
    codes, vals = _finite_table()
    back = O.e4m3_encode(vals)
    assert np.array_equal(O.e4m3_decode(back), vals)
    assert np.array_equal(back[vals != 0], codes[vals != 0])
    x = np.random.default_rng(3).normal(size=1000) * 50
    assert np.array_equal(O.e4m3_round(O.e4m3_round(x)), O.e4m3_round(x))


def test_mx_hand_worked_blocks():
    # largest magnitude 1.0: floor(log2) = 0, shared exponent -8, byte 119, 1.0 / 2^-8 = 256 is an E4M3 value
    b = np.zeros(32); b[0] = 1.0; b[1] = -0.5; b[2] = 2.0 ** -8 * 1.5
    codes, byte = O.mx_quantize(b)
    assert byte.tolist() == [119]
    assert O.e4m3_decode(codes[:3]).tolist() == [256.0, -128.0, 1.5]
    assert np.array_equal(O.mx_dequantize(codes, byte), b)
    # largest magnitude 3.0: floor(log2 3) = 1 -> byte 120, 3 / 2^-7 = 384 = 1.5 * 2^8
    b = np.zeros(32); b[5] = 3.0
    codes, byte = O.mx_quantize(b)
    assert byte.tolist() == [120] and O.e4m3_decode(codes[5]) == 384.0
    # largest magnitude 0.9: floor(log2) = -1 -> byte 118, 0.9 * 2^9 = 460.8 saturates to 448 -> reads back 0.875
    b = np.zeros(32); b[31] = -0.9
    codes, byte = O.mx_quantize(b)
    assert byte.tolist() == [118] and O.mx_dequantize(codes, byte)[31] == -0.875
    # a block of zeros: byte 0, codes 0
    codes, byte = O.mx_quantize(np.zeros(64))
    assert byte.tolist() == [0, 0] and not codes.any()


def test_mx_blocks_are_32_consecutive_elements_of_the_last_axis_and_independent():
    rng = np.random.default_rng(5)
    x = rng.normal(size=(3, 128))
    codes, byte = O.mx_quantize(x)
    assert codes.shape == (3, 128) and byte.shape == (3, 4)
    for r, j in itertools.product(range(3), range(4)):
        c1, b1 = O.mx_quantize(x[r, 32 * j:32 * j + 32])
        assert np.array_equal(c1, codes[r, 32 * j:32 * j + 32]) and b1[0] == byte[r, j]
    y = x.copy(); y[1, 40] = 1000.0                        # only block (1, 1) may change
    c2, b2 = O.mx_quantize(y)
    same = np.ones((3, 4), bool); same[1, 1] = False
    assert np.array_equal(b2[same], byte[same])
    assert np.array_equal(c2.reshape(3, 4, 32)[same], codes.reshape(3, 4, 32)[same])
    assert b2[1, 1] == 127 + 9 - 8                         # floor(log2 1000) = 9


def test_mx_power_of_two_invariance_and_error_bound():
    rng = np.random.default_rng(9)
    x = rng.normal(size=(50, 64)) * np.exp(rng.uniform(-3, 3, size=(50, 1)))
    c0, b0 = O.mx_quantize(x)
    for k in (-7, 3, 20):
        c, b = O.mx_quantize(np.ldexp(x, k))
        assert np.array_equal(c, c0) and np.array_equal(b.astype(int), b0.astype(int) + k)
    # error per element: half a spacing of the top binade (2^-4 of 2^floor(log2 amax)) unless it was
    # saturated, where it is below 2^-2 of it (512 -> 448)
    err = np.abs(O.mx_values(x) - x).reshape(50, 2, 32)
    top = 2.0 ** np.floor(np.log2(np.abs(x).reshape(50, 2, 32).max(axis=-1, keepdims=True)))
    sat = np.abs(x).reshape(50, 2, 32) > 448.0 / 256.0 * top
    assert (err[~sat] <= top.repeat(32, -1)[~sat] / 16 + 1e-300).all()
    assert (err[sat] <= top.repeat(32, -1)[sat] / 4).all()


def test_mx_linear_triple_loop_over_codes_and_block_scales():
    rng = np.random.default_rng(13)
    for (M, N, K) in ((3, 4, 64), (2, 5, 96), (4, 3, 50)):   # 50: zero padded to 64
        x, W, b = rng.normal(size=(M, K)), rng.normal(size=(N, K)) * 0.02, rng.normal(size=N)
        Kp = -(-K // 32) * 32
        xp, Wp = np.zeros((M, Kp)), np.zeros((N, Kp))
        xp[:, :K], Wp[:, :K] = x, W
        cx, bx = O.mx_quantize(xp)
        cw, bw = O.mx_quantize(Wp)
        table = O.e4m3_decode(ALL_CODES)
        want = np.zeros((M, N))
        for m in range(M):
            for n in range(N):
                acc = 0.0
                for j in range(Kp // 32):
                    s = 0.0
                    for k in range(32 * j, 32 * j + 32):
                        s += table[cx[m, k]] * table[cw[n, k]]
                    acc += s * 2.0 ** (int(bx[m, j]) - 127) * 2.0 ** (int(bw[n, j]) - 127)
                want[m, n] = acc + b[n]
        got = O.mx_linear(x, W, b)
        assert np.allclose(got, want, rtol=1e-13, atol=1e-15)
        # and it is a coarse version of the exact product, not something else
        exact = O.linear(x, W, b)
        assert 1e-4 < np.abs(got - exact).max() / np.abs(exact).max() < 0.1


def test_mx_linear_is_exact_on_operands_the_format_holds():
    rng = np.random.default_rng(17)
    x = rng.integers(-8, 9, size=(5, 64)).astype(np.float64) * 0.25      # 4-bit significands
    W = rng.integers(-4, 5, size=(6, 64)).astype(np.float64) * 2.0 ** -5
    assert np.array_equal(O.mx_linear(x, W, None), O.linear(x, W, None))


def _tiny_desc(**kw):
    return wl.DESC_C1.replace(layers=2, **kw)


def test_encoder_layer_with_mx_fp8_quantises_exactly_the_four_products_it_names():
    """Composition check: the layer with the option equals the layer written out with explicit conversions
    (block scales from log2 here; the element rounding itself is pinned against the library's float8 type in the
    tests above -- going through it here would round float64 -> float32 -> float8, and that double rounding moves
    an element that sits within 2^-24 of a tie), and each of the four conversions matters."""
    desc = _tiny_desc(mx_fp8=1)
    w = wl.gen_weights(desc, 4242)
    rng = np.random.default_rng(1)
    x = rng.normal(size=(desc.n_patches, desc.hidden))

    def lib_mx(a):
        a = np.asarray(a, np.float64)
        K = a.shape[-1]
        blk = a.reshape(-1, K // 32, 32)
        amax = np.abs(blk).max(-1, keepdims=True)
        X = 2.0 ** (np.floor(np.log2(np.where(amax > 0, amax, 1.0))) - 8)
        q = O.e4m3_round(blk / X)
        return (q * X).reshape(a.shape)

    def layer(xx, l, which):
        p = f"l{l}_"
        q = lambda a, name: lib_mx(a) if name in which else np.asarray(a, np.float64)
        u = O.layer_norm(xx, w[p + "n1_g"], w[p + "n1_b"], desc.eps)
        qkv = q(u, "qkv") @ q(w[p + "qkv_w"], "qkv").T + w[p + "qkv_b"]
        D = desc.hidden
        o = O.attention(qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:], desc.heads)
        xx = xx + q(o, "o") @ q(w[p + "o_w"], "o").T + w[p + "o_b"]
        u = O.layer_norm(xx, w[p + "n2_g"], w[p + "n2_b"], desc.eps)
        h = O.gelu_erf(q(u, "fc1") @ q(w[p + "fc1_w"], "fc1").T + w[p + "fc1_b"])
        return xx + q(h, "fc2") @ q(w[p + "fc2_w"], "fc2").T + w[p + "fc2_b"]

    got = O.encoder_layer(x, w, desc, 0)
    want = layer(x, 0, {"qkv", "o", "fc1", "fc2"})
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    plain = O.encoder_layer(x, w, desc.replace(mx_fp8=0), 0)
    assert np.allclose(plain, layer(x, 0, set()), rtol=1e-12, atol=1e-12)
    for drop in ("qkv", "o", "fc1", "fc2"):                # leaving any one conversion out is visible
        other = layer(x, 0, {"qkv", "o", "fc1", "fc2"} - {drop})
        assert np.abs(other - got).max() > 1e-6
    # the option is a perturbation of the plain layer, not a different function
    assert 1e-6 < np.abs(got - plain).max() / np.abs(plain).max() < 5e-2


def test_out_projection_stays_unconverted_for_head_dims_the_kernels_pad():
    """Head dim 48 (padded to 64 in the packed layout): blocks of 32 along the padded index are not blocks of 32
    along the hidden dimension, so the reading leaves that product alone; head dim 64 converts it."""
    import unittest.mock as mock
    rng = np.random.default_rng(2)
    for heads, calls in ((4, 3), (3, 4)):       # hidden 192: head dims 48 and 64
        desc = _tiny_desc(mx_fp8=1, heads=heads)
        w = wl.gen_weights(desc, 4243)
        x = rng.normal(size=(desc.n_patches, desc.hidden))
        with mock.patch.object(O, "mx_linear", side_effect=O.mx_linear) as spy:
            got = O.encoder_layer(x, w, desc, 0)
        assert spy.call_count == calls
        assert np.isfinite(got).all()
