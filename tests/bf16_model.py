"""Test-side model of the bf16 mode's rounding points (not the oracle, not the product).

The HIP path keeps activations between kernels in bf16 (operands of every matrix product, the softmax
weights in front of the second attention product) and everything else in fp32.  The functions here take
the oracle's float64 steps and snap exactly those values to the bf16 grid, with exact arithmetic in
between: what comes out is the error the precision policy alone costs, whatever kernel implements it.
Tests use it to tell a kernel defect from a case that sits at the tolerance by construction."""
import numpy as np

from oracle import epd_oracle as O


def snap_bf16(a) -> np.ndarray:
    """Round to the nearest bf16 value (ties to even), returned as float64."""
    a = np.ascontiguousarray(a, np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).astype(np.float64).reshape(a.shape)


def resampler_bf16_policy(x, w, desc, only_qkp: bool = False) -> np.ndarray:
    """oracle.resampler with the bf16 mode's roundings.  only_qkp: snap nothing but the in-projected
    queries, keys and the softmax weights (the least any bf16 attention kernel rounds)."""
    s = (lambda a: np.asarray(a, np.float64)) if only_qkp else snap_bf16
    E, H = desc.proj_out, desc.proj_heads
    hd = E // H
    kvraw = s(O.linear(s(x), w["r_kv_w"], None))
    ln = O.layer_norm(kvraw, w["r_lnkv_g"], w["r_lnkv_b"], desc.eps)
    vin, kin = s(ln), s(ln + np.asarray(w["r_pos"], np.float64))
    q = s(O.layer_norm(np.asarray(w["r_query"], np.float64), w["r_lnq_g"], w["r_lnq_b"], desc.eps))
    in_w, in_b = np.asarray(w["r_in_w"], np.float64), np.asarray(w["r_in_b"], np.float64)
    qp = snap_bf16(O.linear(q, in_w[:E], in_b[:E]))
    kp = snap_bf16(O.linear(kin, in_w[E:2 * E], in_b[E:2 * E]))
    vp = s(O.linear(vin, in_w[2 * E:], in_b[2 * E:]))
    out = np.empty((qp.shape[0], E))
    for h in range(H):
        sl = slice(h * hd, (h + 1) * hd)
        logits = qp[:, sl] @ kp[:, sl].T / np.sqrt(float(hd))
        e = snap_bf16(np.exp(logits - logits.max(axis=-1, keepdims=True)))
        out[:, sl] = (e / e.sum(axis=-1, keepdims=True)) @ vp[:, sl]   # the sum runs over the rounded weights
    o2 = s(O.linear(s(out), w["r_out_w"], w["r_out_b"]))
    o3 = s(O.layer_norm(o2, w["r_lnp_g"], w["r_lnp_b"], desc.eps))
    return s(O.linear(o3, w["r_proj_w"], None))


def resampler_policy_error(desc, w, tiles, only_qkp: bool = False) -> float:
    """max |model - oracle| / max |oracle| over the given slices, the trunk taken exact."""
    num = den = 0.0
    for t in tiles:
        x = O.trunk_tile(t, w, desc)
        ref = O.resampler(x, w, desc)
        got = resampler_bf16_policy(x, w, desc, only_qkp)
        num, den = max(num, float(np.abs(got - ref).max())), max(den, float(np.abs(ref).max()))
    return num / den
