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


def encoder_policy_error(tile, w, desc, stream_bf16: bool) -> float:
    """max |model - oracle| / max |oracle| for one slice, the layers taken with the bf16 mode's roundings (bf16
    operands of every product: norm outputs, q, k, v, softmax weights, attention output, MLP activations; exact
    arithmetic in between; embedding and projector exact).  stream_bf16: the residual stream is snapped to bf16
    after every residual add as well, which is what a bf16 stream would store; False is the fp32 stream."""
    keep = snap_bf16 if stream_bf16 else (lambda a: np.asarray(a, np.float64))
    D, H = desc.hidden, desc.heads
    hd = D // H
    x = keep(O.embed_tile(tile, w, desc))
    for l in range(desc.layers):
        p = f"l{l}_"
        u = snap_bf16(O._norm(x, w, p + "n1", desc.norm, desc.eps))
        qkv = O.linear(u, w[p + "qkv_w"], w[p + "qkv_b"])
        q, k, v = snap_bf16(qkv[:, :D]), snap_bf16(qkv[:, D:2 * D]), snap_bf16(qkv[:, 2 * D:])
        o = np.empty_like(q)
        for h in range(H):
            sl = slice(h * hd, (h + 1) * hd)
            logits = q[:, sl] @ k[:, sl].T / np.sqrt(float(hd))
            e = snap_bf16(np.exp(logits - logits.max(axis=-1, keepdims=True)))
            o[:, sl] = (e / e.sum(axis=-1, keepdims=True)) @ v[:, sl]
        x = keep(x + O.linear(snap_bf16(o), w[p + "o_w"], w[p + "o_b"]))
        u = snap_bf16(O._norm(x, w, p + "n2", desc.norm, desc.eps))
        hmid = snap_bf16(O._act(O.linear(u, w[p + "fc1_w"], w[p + "fc1_b"]), desc.act))
        x = keep(x + O.linear(hmid, w[p + "fc2_w"], w[p + "fc2_b"]))
    if desc.final_norm:
        x = O._norm(x, w, "fn", desc.norm, desc.eps)
    got, ref = O.project(x, w, desc), O.encode_tile(tile, w, desc)
    return float(np.abs(got - ref).max() / np.abs(ref).max())
