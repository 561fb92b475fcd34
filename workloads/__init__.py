"""Seeded synthetic workloads for the EPD encode stage.

This module is the only thing the CPU oracle and the HIP path have in common.
It holds NO arithmetic of the method: it names the encoder shapes, lists the
weight tensors in the order the C boundary expects them, and draws pixels,
weights and request structure from a seed.  Every value it produces is an
*input* of the encoder.

Workload shapes follow the paper's own workloads: 448x448 image slices, 13
slices for a 4K image under InternVL-style tiling and up to 10 under
MiniCPM-V-style slicing (Table 3, "#Patch" column), 1..10 images per request
(Section 4.1, Table 3), encode batch of 8 single-image requests in the offline
runs (Appendix "Throughput Comparison for Offline and Heterogeneous scenario").
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

DT_FP32 = 0
DT_BF16 = 1

NORM_LAYERNORM = 0
NORM_RMSNORM = 1

QKNORM_NONE = 0
QKNORM_FULL = 1      # RMSNorm of q and of k over the full hidden dim
QKNORM_PER_HEAD = 2  # RMSNorm of q and of k inside each head

ACT_GELU_ERF = 0
ACT_GELU_TANH = 1

PROJ_LINEAR = 0
PROJ_MLP = 1
PROJ_RESAMPLER = 2   # proj_mid learned queries cross-attend to the patch tokens (proj_heads heads)


@dataclass(frozen=True)
class ModelDesc:
    """Mirror of the C struct `epd_model_desc` (same field order)."""
    dtype: int
    tile_size: int
    patch: int
    hidden: int
    heads: int
    mlp: int
    layers: int
    norm: int
    qk_norm: int
    act: int
    final_norm: int
    pixel_shuffle: int
    proj_kind: int
    proj_prenorm: int
    proj_mid: int
    proj_out: int
    eps: float
    max_tiles_per_call: int
    layer_scale: int = 0
    class_token: int = 0
    proj_heads: int = 0
    mx_fp8: int = 0      # 1: MXFP8 operands for the q/k/v, FC1 and FC2 products (bf16 mode only)

    # ---- shape bookkeeping only (counts, no arithmetic on data) ----
    @property
    def grid(self) -> int:
        return self.tile_size // self.patch

    @property
    def n_patches(self) -> int:
        return self.grid * self.grid

    @property
    def seq_len(self) -> int:
        """Tokens per slice inside the encoder: the patches plus the class token."""
        return self.n_patches + self.class_token

    @property
    def patch_dim(self) -> int:
        return 3 * self.patch * self.patch

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    @property
    def tokens_per_tile(self) -> int:
        if self.proj_kind == PROJ_RESAMPLER:
            return self.proj_mid
        return self.n_patches // 4 if self.pixel_shuffle else self.n_patches

    @property
    def proj_in(self) -> int:
        return self.hidden * 4 if self.pixel_shuffle else self.hidden

    @property
    def out_dim(self) -> int:
        return self.proj_out

    def replace(self, **kw) -> "ModelDesc":
        return dataclasses.replace(self, **kw)


@dataclass(frozen=True)
class Workload:
    name: str
    desc: ModelDesc
    weight_seed: int
    input_seed: int
    tile_offsets: Tuple[int, ...]        # [n_requests + 1], tiles per request prefix sum
    image_tiles: Tuple[Tuple[int, ...], ...]  # per request: tiles of each image
    oracle_sample_tiles: Tuple[int, ...]  # tiles the oracle encodes for full-size parity

    @property
    def n_tiles(self) -> int:
        return self.tile_offsets[-1]

    @property
    def n_requests(self) -> int:
        return len(self.tile_offsets) - 1


def _desc(**kw) -> ModelDesc:
    base = dict(dtype=DT_BF16, tile_size=448, patch=14, norm=NORM_LAYERNORM,
                qk_norm=QKNORM_NONE, act=ACT_GELU_ERF, final_norm=0,
                pixel_shuffle=0, proj_kind=PROJ_MLP, proj_prenorm=0,
                proj_mid=0, proj_out=0, eps=1e-6, max_tiles_per_call=0)
    base.update(kw)
    return ModelDesc(**base)


DESC_C1 = _desc(dtype=DT_FP32, tile_size=224, hidden=192, heads=3, mlp=768, layers=4,
                proj_kind=PROJ_LINEAR, proj_out=512, max_tiles_per_call=4)
DESC_C2 = _desc(hidden=1152, heads=16, mlp=4304, layers=27, act=ACT_GELU_TANH,
                proj_mid=3584, proj_out=3584, max_tiles_per_call=128)
DESC_C3 = _desc(hidden=1024, heads=16, mlp=4096, layers=24, pixel_shuffle=1,
                proj_prenorm=1, proj_mid=4096, proj_out=4096, max_tiles_per_call=104)
DESC_C4 = _desc(hidden=3200, heads=25, mlp=12800, layers=45, norm=NORM_RMSNORM,
                qk_norm=QKNORM_FULL, pixel_shuffle=1, proj_prenorm=1,
                proj_mid=5120, proj_out=5120, max_tiles_per_call=40)


def _video_structure(seed: int, per_length: int = 4) -> Tuple[int, ...]:
    """Frames per request: `per_length` requests of each of 8, 16, 32 and 64 frames, in a seeded order."""
    frames = np.repeat(np.array([8, 16, 32, 64]), per_length)
    np.random.default_rng([seed, 0]).shuffle(frames)
    return tuple(int(f) for f in frames)


def _prefix(counts) -> Tuple[int, ...]:
    off = [0]
    for c in counts:
        off.append(off[-1] + int(c))
    return tuple(off)


def _mixed_structure(seed: int, n_requests: int = 32):
    """Request structure of the mixed batch: images per request uniform in
    1..10, tiles per image uniform in 1..9.  Draw order: all image counts
    first, then the tile counts request-major."""
    rng = np.random.default_rng([seed, 0])
    n_images = rng.integers(1, 11, size=n_requests)
    image_tiles = []
    for r in range(n_requests):
        image_tiles.append(tuple(int(v) for v in rng.integers(1, 10, size=int(n_images[r]))))
    return tuple(image_tiles)


def workload(name: str) -> Workload:
    """The named configurations."""
    if name == "c1":
        return Workload("c1_tiny_fp32", DESC_C1, 1001, 1001, (0, 1), ((1,),), (0,))
    if name == "c2":
        return Workload("c2_siglip_so400m_10tiles", DESC_C2, 1002, 1002, (0, 10), ((10,),), (0, 9))
    if name == "c3":
        img = tuple((13,) for _ in range(8))
        return Workload("c3_internvit300m_8x13tiles", DESC_C3, 1003, 1003,
                        _prefix([13] * 8), img, (0, 12, 103))
    if name == "c4":
        # oracle sample: first, middle and last slice (the last one sits behind the largest buffer offsets)
        return Workload("c4_internvit6b_40tiles", DESC_C4, 1004, 1004, (0, 40), ((40,),), (0, 20, 39))
    if name == "c5":
        image_tiles = _mixed_structure(1005)
        off = _prefix([sum(t) for t in image_tiles])
        n_req = len(image_tiles)
        sizes = [off[r + 1] - off[r] for r in range(n_req)]
        big = int(np.argmax(sizes))
        sample = {off[0], off[1] - 1, off[n_req - 1], off[n_req] - 1}
        for s in range(4):
            b, e = shard_range(sizes[big], s, 4)
            if e > b:
                sample.add(off[big] + b)
        desc = DESC_C2.replace(max_tiles_per_call=128)
        return Workload("c5_mixed_siglip_32req", desc, 1002, 1005, off, image_tiles,
                        tuple(sorted(sample)))
    if name == "c6":
        # Video requests (Section 4.2, the table of latency versus number of frames): 8, 16, 32 or 64
        # sampled frames per request, every frame one 448x448 slice of a SigLIP-shaped encoder.
        frames = _video_structure(1006)
        off = _prefix(frames)
        desc = DESC_C2.replace(max_tiles_per_call=128)
        return Workload("c6_video_siglip_16req", desc, 1002, 1006, off, tuple((1,) * f for f in frames),
                        (0, off[len(frames) // 2], off[-1] - 1))
    if name == "c7":
        # The C3 batch through the encoder shape of the InternViT-300M checkpoints themselves: class token
        # (1025 tokens per slice) and layer scale on both residual branches.
        img = tuple((13,) for _ in range(8))
        desc = DESC_C3.replace(class_token=1, layer_scale=1)
        return Workload("c7_internvit300m_cls_ls_8x13tiles", desc, 1007, 1003, _prefix([13] * 8), img, (0, 51, 103))
    if name == "c8":
        # The C2 batch through the MiniCPM-V-shaped encoder: SigLIP trunk with its post norm, then the
        # resampler (64 learned queries, width 3584, 28 heads of 128) in place of the MLP projector:
        # 64 tokens per slice.
        desc = DESC_C2.replace(final_norm=1, proj_kind=PROJ_RESAMPLER, proj_mid=64, proj_out=3584, proj_heads=28)
        return Workload("c8_siglip_resampler_10tiles", desc, 1008, 1002, (0, 10), ((10,),), (0, 9))
    raise KeyError(name)


ALL_WORKLOADS = ("c1", "c2", "c3", "c4", "c5", "c6", "c7", "c8")


def shard_range(n_tiles: int, shard: int, n_shards: int) -> Tuple[int, int]:
    """Balanced contiguous split of a request's tiles across encode workers
    (Section 3.2.2: a request's slices are divided among workers and later
    merged in order).  Index bookkeeping only."""
    return (shard * n_tiles) // n_shards, ((shard + 1) * n_tiles) // n_shards


# --------------------------------------------------------------------------
# weight tensor list: the fixed order of `epd_weights.tensors`
# --------------------------------------------------------------------------

def weight_specs(desc: ModelDesc) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) in boundary order.  kind: 'w' matrix/bias/pos-emb,
    'g' norm gain, 'b' norm shift, 's' layer-scale vector."""
    D, F, N = desc.hidden, desc.mlp, desc.n_patches
    specs: List[Tuple[str, Tuple[int, ...], str]] = []

    def norm(prefix: str, dim: int, kind: int):
        specs.append((prefix + "_g", (dim,), "g"))
        if kind == NORM_LAYERNORM:
            specs.append((prefix + "_b", (dim,), "b"))

    specs.append(("pe_w", (D, desc.patch_dim), "w"))
    specs.append(("pe_b", (D,), "w"))
    specs.append(("pos", (N + desc.class_token, D), "w"))
    if desc.class_token:
        specs.append(("cls", (D,), "w"))
    for l in range(desc.layers):
        p = f"l{l}_"
        norm(p + "n1", D, desc.norm)
        specs.append((p + "qkv_w", (3 * D, D), "w"))
        specs.append((p + "qkv_b", (3 * D,), "w"))
        if desc.qk_norm == QKNORM_FULL:
            specs.append((p + "qn_g", (D,), "g"))
            specs.append((p + "kn_g", (D,), "g"))
        elif desc.qk_norm == QKNORM_PER_HEAD:
            specs.append((p + "qn_g", (desc.head_dim,), "g"))
            specs.append((p + "kn_g", (desc.head_dim,), "g"))
        specs.append((p + "o_w", (D, D), "w"))
        specs.append((p + "o_b", (D,), "w"))
        if desc.layer_scale:
            specs.append((p + "ls1", (D,), "s"))
        norm(p + "n2", D, desc.norm)
        specs.append((p + "fc1_w", (F, D), "w"))
        specs.append((p + "fc1_b", (F,), "w"))
        specs.append((p + "fc2_w", (D, F), "w"))
        specs.append((p + "fc2_b", (D,), "w"))
        if desc.layer_scale:
            specs.append((p + "ls2", (D,), "s"))
    if desc.final_norm:
        norm("fn", D, desc.norm)
    if desc.proj_prenorm:
        norm("pn", desc.proj_in, NORM_LAYERNORM)
    if desc.proj_kind == PROJ_RESAMPLER:
        E, Q = desc.proj_out, desc.proj_mid
        specs.append(("r_kv_w", (E, D), "w"))
        specs.append(("r_query", (Q, E), "w"))
        specs.append(("r_pos", (N, E), "w"))
        norm("r_lnq", E, NORM_LAYERNORM)
        norm("r_lnkv", E, NORM_LAYERNORM)
        specs.append(("r_in_w", (3 * E, E), "w"))
        specs.append(("r_in_b", (3 * E,), "w"))
        specs.append(("r_out_w", (E, E), "w"))
        specs.append(("r_out_b", (E,), "w"))
        norm("r_lnp", E, NORM_LAYERNORM)
        specs.append(("r_proj_w", (E, E), "w"))
    elif desc.proj_kind == PROJ_LINEAR:
        specs.append(("pa_w", (desc.proj_out, desc.proj_in), "w"))
        specs.append(("pa_b", (desc.proj_out,), "w"))
    else:
        specs.append(("pa_w", (desc.proj_mid, desc.proj_in), "w"))
        specs.append(("pa_b", (desc.proj_mid,), "w"))
        specs.append(("pb_w", (desc.proj_out, desc.proj_mid), "w"))
        specs.append(("pb_b", (desc.proj_out,), "w"))
    return specs


def n_params(desc: ModelDesc) -> int:
    return sum(int(np.prod(s)) for _, s, _ in weight_specs(desc))


def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Return fp32 values that are exactly representable in bfloat16
    (round-to-nearest-even on the upper 16 bits).  Used to *define* the bf16
    random-init weights; both sides then read the same numbers."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    u = (u + r) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of fp32 values already on the bf16 grid (for upload)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def gen_weight(desc: ModelDesc, seed: int, index: int, std: float = 0.02,
               scale: Dict[str, float] | None = None) -> np.ndarray:
    """Tensor `index` of weight_specs(desc), drawn from its own stream so any
    tensor can be regenerated alone.  Matrices, biases and the position
    embedding are N(0, std); norm gains are 1 + N(0, std) (a gain of ~0.02
    would shrink every branch to nothing and hide mistakes); norm shifts are
    N(0, std).  For bf16 models the values are snapped to the bf16 grid."""
    name, shape, kind = weight_specs(desc)[index]
    rng = np.random.default_rng([seed, 1, index])
    w = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    if kind == "g":
        w = w + np.float32(1.0)
    if kind == "s":   # layer scale: spread over 0.1 .. 1, so a missing or misplaced factor shows
        w = np.float32(0.1) + np.float32(0.9) * rng.random(size=shape, dtype=np.float32)
    if scale:
        for key, s in scale.items():
            if name.endswith(key):
                w = w * np.float32(s)
    if desc.dtype == DT_BF16:
        w = to_bf16_grid(w)
    return w


def gen_weights(desc: ModelDesc, seed: int, std: float = 0.02,
                scale: Dict[str, float] | None = None) -> Dict[str, np.ndarray]:
    return {name: gen_weight(desc, seed, i, std, scale)
            for i, (name, _, _) in enumerate(weight_specs(desc))}


def gen_tile(desc: ModelDesc, seed: int, tile_index: int) -> np.ndarray:
    """One [3, S, S] fp32 tile, pixels uniform in [-1, 1); each tile has its
    own stream so a sample of a large batch can be drawn without the rest."""
    rng = np.random.default_rng([seed, 2, tile_index])
    S = desc.tile_size
    return rng.random(size=(3, S, S), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)


def gen_tiles(desc: ModelDesc, seed: int, n_tiles: int, first: int = 0) -> np.ndarray:
    S = desc.tile_size
    out = np.empty((n_tiles, 3, S, S), dtype=np.float32)
    for t in range(n_tiles):
        out[t] = gen_tile(desc, seed, first + t)
    return out


# --------------------------------------------------------------------------
# algorithmic work (for throughput reporting; counts, not data arithmetic)
# --------------------------------------------------------------------------

def flops_per_tile(desc: ModelDesc) -> int:
    """Multiply-add = 2 flops; dense contractions only, no padding."""
    N, D, F, L = desc.seq_len, desc.hidden, desc.mlp, desc.layers
    f = 2 * desc.n_patches * desc.patch_dim * D
    f += L * (2 * N * D * 3 * D + 2 * N * D * D + 4 * N * D * F + 4 * N * N * D)
    No, Pi = desc.tokens_per_tile, desc.proj_in
    if desc.proj_kind == PROJ_RESAMPLER:
        E, Np = desc.proj_out, desc.n_patches
        f += 2 * Np * D * E + 4 * Np * E * E + 4 * No * Np * E + 4 * No * E * E   # kv, k/v in-proj, attention, out + proj
    elif desc.proj_kind == PROJ_LINEAR:
        f += 2 * No * Pi * desc.proj_out
    else:
        f += 2 * No * Pi * desc.proj_mid + 2 * No * desc.proj_mid * desc.proj_out
    return f
