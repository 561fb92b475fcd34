"""CPU oracle for the EPD encode stage  --  TEST INFRASTRUCTURE ONLY.

What it is: the plain definition of what the encode stage E computes
(Section 3.1: multimodal tokens v = E(i_m)) for a vision-transformer encoder
fed with image slices, one slice at a time, in float64 numpy.  Slices of a
request are encoded independently of each other and merged in slice order
(Section 3.2.2, intra-request parallelism); a shard of a request is therefore
just a range of slices whose rows land at their final place in the request's
token buffer.

The paper treats E as a given model and prints none of its internals, so each
step below is the textbook definition (patch embedding, LayerNorm / RMSNorm,
softmax attention, GELU, space-to-depth pixel shuffle, linear / MLP
projector); where the workload description leaves a choice open the reading
taken is written next to the step.

Rules this file keeps:
  * float64 everywhere; numpy `@` is the only library primitive used for a
    contraction, `scipy.special.erf` for the error function;
  * no blocking, fusion or reordering beyond the definitions;
  * shares no code with the HIP path and imports nothing from it;
  * may be imported only by tests/, by __graft_entry__.smoke() and by
    bench.py's cpu_baseline leg.

Pins (tests/test_oracle_*.py): brute-force loops for the contractions and
attention on tiny shapes, closed forms for the norms and softmax, tabulated
values of the normal CDF for GELU, index arithmetic for patchify and pixel
shuffle, an affine special case (zero layers), an identity special case (zero
output projections), a composition of PyTorch CPU library ops for the whole
tiny encoder (class token placed last there, the library's multi-head
attention module for the resampler), explicit loops for one resampler query
and for one patch query next to a class token, and the independence /
permutation / shard invariants.
The MXFP8 option (`desc.mx_fp8`) follows the OCP Microscaling Formats (MX)
specification v1.0 and the OCP 8-bit floating point specification (E4M3); its
pins (tests/test_oracle_mx.py): the library's own float8 decode and conversion,
brute-force nearest-value search over the 256 codes, hand-worked blocks,
power-of-two invariance, a triple loop over codes and block scales.
Parity unpinned: fidelity to the *trained* SigLIP / InternViT checkpoints (no
weights or reference activations exist here; the target does not need them).
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional, Sequence

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64

# integer codes of the model description (same values as the C header)
NORM_LAYERNORM, NORM_RMSNORM = 0, 1
QKNORM_NONE, QKNORM_FULL, QKNORM_PER_HEAD = 0, 1, 2
ACT_GELU_ERF, ACT_GELU_TANH = 0, 1
PROJ_LINEAR, PROJ_MLP, PROJ_RESAMPLER = 0, 1, 2


# ---------------------------------------------------------------- steps ----

def patchify(tile: np.ndarray, p: int) -> np.ndarray:
    """[3, S, S] -> [N, 3*p*p].  Grid cell (y, x) becomes row n = y*g + x; the
    patch vector is ordered (channel, dy, dx), the order of a convolution
    weight [D, 3, p, p] flattened over its last three axes."""
    C, S, S2 = tile.shape
    assert S == S2 and S % p == 0
    g = S // p
    t = np.asarray(tile, dtype=F64).reshape(C, g, p, g, p)   # c, y, dy, x, dx
    return t.transpose(1, 3, 0, 2, 4).reshape(g * g, C * p * p)


def linear(x: np.ndarray, W: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    """y = x W^T + b with W stored [out, in]."""
    y = np.asarray(x, F64) @ np.asarray(W, F64).T
    if b is not None:
        y = y + np.asarray(b, F64)
    return y


def layer_norm(x, gamma, beta, eps):
    """(x - mean) / sqrt(biased variance + eps) * gamma + beta over the last axis."""
    x = np.asarray(x, F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, F64) + np.asarray(beta, F64)


def rms_norm(x, gamma, eps):
    """x / sqrt(mean(x^2) + eps) * gamma over the last axis (no shift)."""
    x = np.asarray(x, F64)
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gamma, F64)


def gelu_erf(x):
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_tanh(x):
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def softmax_rows(s):
    s = np.asarray(s, F64)
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention(q, k, v, heads: int):
    """Non-causal softmax attention inside one slice.  q: [Nq, D], k, v: [Nk, D]
    (Nq = Nk in the encoder layers); head h owns columns h*hd .. (h+1)*hd-1;
    logits are scaled by 1/sqrt(hd)."""
    q, k, v = (np.asarray(a, F64) for a in (q, k, v))
    N, D = q.shape
    hd = D // heads
    out = np.empty((N, D), F64)
    for h in range(heads):
        sl = slice(h * hd, (h + 1) * hd)
        P = softmax_rows((q[:, sl] @ k[:, sl].T) / np.sqrt(float(hd)))
        out[:, sl] = P @ v[:, sl]
    return out


def pixel_shuffle_half(x, g: int):
    """Space-to-depth with block 2 on a g x g token grid: [g*g, D] -> [g*g/4, 4D].
    Output token m = Y*(g/2) + X, channel (dy*2 + dx)*D + c, is input token
    (2Y+dy)*g + (2X+dx), channel c."""
    x = np.asarray(x)
    N, D = x.shape
    assert N == g * g and g % 2 == 0
    h = g // 2
    t = x.reshape(h, 2, h, 2, D)            # Y, dy, X, dx, c
    return t.transpose(0, 2, 1, 3, 4).reshape(h * h, 4 * D)


# ------------------------------------------------------------- MXFP8 option ----
# Checkpoint-fidelity option `mx_fp8` (narrower than the FP16 the paper serves in, Appendix
# "Implementation Details": an option, never the headline precision).  The operands of the q/k/v,
# out-projection, FC1 and FC2 products of every layer are quantised to the MXFP8 format of the OCP Microscaling
# Formats specification v1.0: along the contraction dimension, blocks of 32 consecutive elements
# share one power-of-two scale (E8M0: an 8-bit biased exponent, X = 2^(byte - 127)) and each element
# is an OCP FP8 E4M3 number (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; subnormals;
# largest finite value 448; no infinities).  Conversion (section 6.3 of that specification):
#   shared exponent = floor(log2(max |v_i|)) - 8      (8 = exponent of the largest E4M3 binade)
#   element_i       = E4M3 value nearest to v_i / X, ties to the even mantissa, saturated to +-448
# Readings: a block of zeros takes the scale byte 0 (the specification leaves it open); the scale
# byte is clamped to 0 .. 254 (255 is the format's NaN); inputs are finite.

MX_BLOCK = 32
E4M3_MAX = 448.0
_E4M3_EMAX = 8          # 448 = 1.75 * 2^8
_E4M3_EMIN = -6         # smallest normal 2^-6; subnormals are multiples of 2^-9
_E8M0_BIAS = 127


def e4m3_decode(code) -> np.ndarray:
    """Value of an E4M3 byte: (-1)^s * 2^(e - 7) * (1 + m / 8) for e > 0, (-1)^s * 2^-6 * (m / 8)
    for e = 0; s.1111.111 is NaN."""
    c = np.asarray(code).astype(np.int64)
    s, e, m = (c >> 7) & 1, (c >> 3) & 15, c & 7
    mag = np.where(e > 0, np.ldexp(1.0 + m / 8.0, e - 7), np.ldexp(m / 8.0, _E4M3_EMIN))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return np.where(s == 1, -mag, mag).astype(F64)


def e4m3_round(x) -> np.ndarray:
    """Nearest E4M3 value, ties to the even mantissa, saturating at +-448."""
    x = np.asarray(x, F64)
    a = np.abs(x)
    _, e = np.frexp(a)                               # a = f * 2^e with f in [0.5, 1)
    binade = np.maximum(e - 1, _E4M3_EMIN)           # exponent of the value's binade, subnormals share 2^-6's
    quantum = np.ldexp(1.0, binade - 3)              # spacing of E4M3 values in that binade (3 mantissa bits)
    r = np.minimum(np.rint(a / quantum) * quantum, E4M3_MAX)   # rint rounds halves to even
    return np.copysign(r, x)


def e4m3_encode(x) -> np.ndarray:
    """Byte of e4m3_round(x) (the sign bit of a negative zero is kept)."""
    v = e4m3_round(x)
    a = np.abs(v)
    _, e = np.frexp(a)
    normal = a >= np.ldexp(1.0, _E4M3_EMIN)
    ebits = np.where(normal, e - 1 + 7, 0)
    mbits = np.where(normal, np.rint(np.ldexp(a, -(e - 1)) * 8.0) - 8, np.rint(np.ldexp(a, -_E4M3_EMIN) * 8.0))
    sign = np.signbit(v).astype(np.int64)
    return ((sign << 7) | (ebits.astype(np.int64) << 3) | mbits.astype(np.int64)).astype(np.uint8)


def mx_quantize(x):
    """MXFP8 conversion of the rows of x along its last axis (length a multiple of 32).
    Returns (codes uint8 of x's shape, scale bytes uint8 [..., K / 32])."""
    x = np.asarray(x, F64)
    K = x.shape[-1]
    assert K % MX_BLOCK == 0
    blocks = x.reshape(x.shape[:-1] + (K // MX_BLOCK, MX_BLOCK))
    amax = np.abs(blocks).max(axis=-1)
    _, e = np.frexp(amax)                            # floor(log2(amax)) = e - 1 for amax > 0
    byte = np.where(amax > 0, np.clip(e - 1 - _E4M3_EMAX + _E8M0_BIAS, 0, 254), 0)
    scaled = blocks / np.ldexp(1.0, byte - _E8M0_BIAS)[..., None]
    return e4m3_encode(scaled).reshape(x.shape), byte.astype(np.uint8)


def mx_dequantize(codes, scale_bytes) -> np.ndarray:
    """Values an MXFP8 tensor stands for: element value times its block's 2^(byte - 127)."""
    codes = np.asarray(codes)
    K = codes.shape[-1]
    v = e4m3_decode(codes).reshape(codes.shape[:-1] + (K // MX_BLOCK, MX_BLOCK))
    return (v * np.ldexp(1.0, np.asarray(scale_bytes).astype(np.int64) - _E8M0_BIAS)[..., None]).reshape(codes.shape)


def mx_values(x) -> np.ndarray:
    """x as an MXFP8 product sees it: converted and read back."""
    return mx_dequantize(*mx_quantize(x))


def mx_linear(x, W, b) -> np.ndarray:
    """y = Q(x) Q(W)^T + b: both operands converted to MXFP8 along the contraction dimension (zero
    padded to a multiple of 32; zeros change neither a block's scale nor the sum), exact product."""
    x, W = np.asarray(x, F64), np.asarray(W, F64)
    pad = (-x.shape[-1]) % MX_BLOCK
    if pad:
        x = np.concatenate([x, np.zeros(x.shape[:-1] + (pad,), F64)], axis=-1)
        W = np.concatenate([W, np.zeros(W.shape[:-1] + (pad,), F64)], axis=-1)
    return linear(mx_values(x), mx_values(W), b)


# -------------------------------------------------------------- encoder ----

def _norm(x, w: Dict[str, np.ndarray], prefix: str, kind: int, eps: float):
    if kind == NORM_LAYERNORM:
        return layer_norm(x, w[prefix + "_g"], w[prefix + "_b"], eps)
    return rms_norm(x, w[prefix + "_g"], eps)


def _act(x, kind: int):
    return gelu_erf(x) if kind == ACT_GELU_ERF else gelu_tanh(x)


def encoder_layer(x, w, desc, l: int):
    """One pre-norm transformer layer on the [N, D] tokens of one slice.  With `desc.mx_fp8` the four
    weight products of the layer (q/k/v, out-projection, FC1, FC2) take MXFP8 operands; the two attention
    products do not.  Reading: the out-projection's operand is converted only when the head dim is one the
    kernels store without padding (64, 72, 96, 128: every encoder the paper evaluates); for any other head dim
    the packed layout pads each head, blocks of 32 along it would not be the blocks of 32 along the hidden
    dimension this definition converts, and the out-projection stays unconverted on both sides."""
    D, H = desc.hidden, desc.heads
    p = f"l{l}_"
    big = mx_linear if getattr(desc, "mx_fp8", 0) else linear
    big_o = big if (D // H) in (64, 72, 96, 128) else linear
    u = _norm(x, w, p + "n1", desc.norm, desc.eps)
    qkv = big(u, w[p + "qkv_w"], w[p + "qkv_b"])         # rows of W: q block, k block, v block
    q, k, v = qkv[:, :D], qkv[:, D:2 * D], qkv[:, 2 * D:]
    if desc.qk_norm == QKNORM_FULL:
        # reading: RMSNorm of q and of k over all heads together, after the
        # bias, before the head split and the 1/sqrt(hd) scale
        q = rms_norm(q, w[p + "qn_g"], desc.eps)
        k = rms_norm(k, w[p + "kn_g"], desc.eps)
    elif desc.qk_norm == QKNORM_PER_HEAD:
        hd = D // H
        q = rms_norm(q.reshape(-1, H, hd), w[p + "qn_g"], desc.eps).reshape(-1, D)
        k = rms_norm(k.reshape(-1, H, hd), w[p + "kn_g"], desc.eps).reshape(-1, D)
    o = attention(q, k, v, H)
    branch = big_o(o, w[p + "o_w"], w[p + "o_b"])
    if getattr(desc, "layer_scale", 0):
        branch = branch * np.asarray(w[p + "ls1"], F64)     # per-channel layer scale
    x = x + branch
    u = _norm(x, w, p + "n2", desc.norm, desc.eps)
    hmid = _act(big(u, w[p + "fc1_w"], w[p + "fc1_b"]), desc.act)
    branch = big(hmid, w[p + "fc2_w"], w[p + "fc2_b"])
    if getattr(desc, "layer_scale", 0):
        branch = branch * np.asarray(w[p + "ls2"], F64)
    x = x + branch
    return x


def embed_tile(tile, w, desc):
    """Patch embedding + learned position embedding.  With a class token the
    sequence is [cls, patch 0, patch 1, ...]: the learned vector `cls` is put in
    front of the embedded patches and the position table has one more row,
    row 0 for the class token (the usual ViT input; Section 3.1 takes the
    encoder as given)."""
    a = patchify(tile, desc.patch)
    x = linear(a, w["pe_w"], w["pe_b"])
    if getattr(desc, "class_token", 0):
        x = np.concatenate([np.asarray(w["cls"], F64).reshape(1, -1), x], axis=0)
    return x + np.asarray(w["pos"], F64)


def resampler(x, w, desc):
    """Cross-attention projector of the MiniCPM-V family (one of the three models
    of Section 4): `proj_mid` learned queries read the N patch tokens of a slice,
    so a slice yields that many tokens whatever its patch count.
        kv  = LayerNorm_kv(x Wkv^T)                      x: [N, hidden] -> [N, E], no bias
        q   = LayerNorm_q(query)                         [Q, E], the same for every slice
        o   = MHA(q, kv + pos, kv)                       keys carry the position table, values do not;
                                                         in-projections Wq, Wk, Wv = row blocks of in_w
                                                         [3E, E] with bias in_b, `proj_heads` heads,
                                                         logits / sqrt(E / heads), then out_w, out_b
        out = LayerNorm_post(o) Wp^T                     [Q, E], no bias
    reading: the position table `r_pos [N, E]` is a weight tensor (the checkpoints
    compute a 2-D sin-cos table of that shape; its values do not matter here)."""
    E = desc.proj_out
    kv = layer_norm(linear(x, w["r_kv_w"], None), w["r_lnkv_g"], w["r_lnkv_b"], desc.eps)
    q = layer_norm(np.asarray(w["r_query"], F64), w["r_lnq_g"], w["r_lnq_b"], desc.eps)
    in_w, in_b = np.asarray(w["r_in_w"], F64), np.asarray(w["r_in_b"], F64)
    qp = linear(q, in_w[:E], in_b[:E])
    kp = linear(kv + np.asarray(w["r_pos"], F64), in_w[E:2 * E], in_b[E:2 * E])
    vp = linear(kv, in_w[2 * E:], in_b[2 * E:])
    o = linear(attention(qp, kp, vp, desc.proj_heads), w["r_out_w"], w["r_out_b"])
    return linear(layer_norm(o, w["r_lnp_g"], w["r_lnp_b"], desc.eps), w["r_proj_w"], None)


def project(x, w, desc):
    """Optional pixel shuffle, optional LayerNorm, then Linear,
    Linear-GELU(erf)-Linear, or the cross-attention resampler."""
    if desc.proj_kind == PROJ_RESAMPLER:
        return resampler(x, w, desc)
    if desc.pixel_shuffle:
        x = pixel_shuffle_half(x, desc.tile_size // desc.patch)
    if desc.proj_prenorm:
        x = layer_norm(x, w["pn_g"], w["pn_b"], desc.eps)
    if desc.proj_kind == PROJ_LINEAR:
        return linear(x, w["pa_w"], w["pa_b"])
    hmid = gelu_erf(linear(x, w["pa_w"], w["pa_b"]))
    return linear(hmid, w["pb_w"], w["pb_b"])


def trunk_tile(tile, w, desc, trace: Optional[dict] = None):
    """Pre-projection tokens of one slice, [N, hidden] (N patches): the encoder
    up to and including its last norm, before pixel shuffle and projector (the
    part an encode worker runs when projection happens on the prefill side,
    Section 3.2.2).  The traced streams keep the class token's row, if any."""
    x = embed_tile(tile, w, desc)
    if trace is not None:
        trace["embed"] = x.copy()
    for l in range(desc.layers):
        x = encoder_layer(x, w, desc, l)
        if trace is not None:
            trace[f"layer{l}"] = x.copy()
    if desc.final_norm:
        x = _norm(x, w, "fn", desc.norm, desc.eps)
    if getattr(desc, "class_token", 0):
        # reading: the class token takes part in every attention layer and is dropped
        # after the last norm; pixel shuffle and projector see the patch tokens only
        x = x[1:]
    return x


def encode_tile(tile, w, desc, trace: Optional[dict] = None):
    """Tokens of one slice: [tokens_per_tile, out_dim], float64."""
    return project(trunk_tile(tile, w, desc, trace), w, desc)


def project_merge(shards: Sequence[np.ndarray], w, desc) -> np.ndarray:
    """Prefill side of intra-request parallelism (Section 3.2.2): `shards` are
    the pre-projection tokens the encode workers sent, each [slices_i * N,
    hidden], listed in slice order.  They are put one after the other, every
    slice is projected on its own, and the results are stacked in slice order."""
    N = (desc.tile_size // desc.patch) ** 2
    rows = np.concatenate([np.asarray(s, F64) for s in shards], axis=0)
    assert rows.shape[0] % N == 0
    return np.concatenate([project(rows[t * N:(t + 1) * N], w, desc) for t in range(rows.shape[0] // N)], axis=0)


def tokens_per_tile(desc) -> int:
    if desc.proj_kind == PROJ_RESAMPLER:
        return desc.proj_mid            # one token per learned query
    n = (desc.tile_size // desc.patch) ** 2
    return n // 4 if desc.pixel_shuffle else n


def encode_range(tiles, n_tiles_total: int, tile_begin: int, tile_end: int, w, desc,
                 out: np.ndarray) -> np.ndarray:
    """Encode slices [tile_begin, tile_end) of a packed batch and write their
    tokens to rows [tile_begin*N_out, tile_end*N_out) of `out`; other rows are
    left alone (one encode worker's share of the batch)."""
    assert 0 <= tile_begin <= tile_end <= n_tiles_total
    n_out = tokens_per_tile(desc)
    for t in range(tile_begin, tile_end):
        out[t * n_out:(t + 1) * n_out, :] = encode_tile(tiles[t], w, desc)
    return out


def encode(tiles, tile_offsets: Sequence[int], w, desc) -> np.ndarray:
    """Whole batch.  tile_offsets[r] .. tile_offsets[r+1] are request r's
    slices; request r's token buffer is the contiguous row block
    out[tile_offsets[r]*N_out : tile_offsets[r+1]*N_out]."""
    off = list(tile_offsets)
    assert off[0] == 0 and all(a <= b for a, b in zip(off, off[1:]))
    n_tiles = off[-1]
    assert len(tiles) == n_tiles
    out = np.zeros((n_tiles * tokens_per_tile(desc), desc.proj_out), F64)
    return encode_range(tiles, n_tiles, 0, n_tiles, w, desc, out)


def encode_sample(tile_list: Iterable[np.ndarray], w, desc) -> np.ndarray:
    """Tokens of the given slices stacked in the given order (used when only a
    sample of a large batch is affordable on the CPU)."""
    return np.concatenate([encode_tile(t, w, desc) for t in tile_list], axis=0)


# ---------------------------------------------------------- paged MM cache ----
# Section 3.2.1: the tokens of a finished encode wait in the encode worker's
# multimodal cache, whose blocks a block manager pre-allocated for the request;
# the paper's setting is blocks of 16 tokens (Appendix "Hyper-parameters in EPD
# system").  The layout is a pure index map, written here one token at a time.

def paged_scatter(pool: np.ndarray, tokens: np.ndarray, block_ids: Sequence[int], block_tokens: int) -> np.ndarray:
    """Token i of a request goes to block block_ids[i // block_tokens], slot
    i % block_tokens.  pool: [n_blocks, block_tokens, dim]; other blocks are
    left alone."""
    n = tokens.shape[0]
    assert len(block_ids) * block_tokens >= n
    for i in range(n):
        pool[block_ids[i // block_tokens], i % block_tokens, :] = tokens[i]
    return pool


def paged_gather(pool: np.ndarray, block_ids: Sequence[int], n_tokens: int) -> np.ndarray:
    """Inverse view: the request's tokens in order, read through its block list."""
    bt = pool.shape[1]
    out = np.empty((n_tokens, pool.shape[2]), pool.dtype)
    for i in range(n_tokens):
        out[i] = pool[block_ids[i // bt], i % bt]
    return out
