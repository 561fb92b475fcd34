"""ctypes binding of libepd_encode.so: argument marshalling only.

Every step of the encode path runs in the library's HIP kernels; PyTorch is
used here for device memory and the current HIP stream, nothing else.  There
is no CPU fallback: if the library is not built, importing a symbol raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# EPD_LIB_PATH: another build of the library (the host-sanitizer build of build.py --sanitize, an A/B build)
LIB_PATH = os.environ.get("EPD_LIB_PATH") or os.path.join(_HERE, "libepd_encode.so")

EPD_OK = 0
EPD_ERR_INVALID_ARG = -1
EPD_ERR_SHAPE = -2
EPD_ERR_OFFSETS = -3
EPD_ERR_UNSUPPORTED = -4
EPD_ERR_NOMEM = -5
EPD_ERR_HIP = -6

PROF_FAMILIES = ("embed", "norm", "gemm_qkv", "attention", "qk_norm", "proj_input",
                 "gemm_out", "gemm_fc1", "gemm_fc2", "gemm_proj")

EXPORTS = (
    "epd_weight_count", "epd_check_desc", "epd_check_offsets", "epd_create", "epd_encode",
    "epd_encode_range", "epd_tokens_per_tile", "epd_out_dim", "epd_last_error", "epd_destroy",
    "epd_debug_read_stream", "epd_op_gemm_bf16", "epd_op_gemm_bf16_form", "epd_op_attention_bf16", "epd_op_mfma_probe",
    "epd_profile_enable", "epd_profile_read", "epd_op_mfma_peak", "epd_op_copy_peak", "epd_op_coissue",
    "epd_op_row_stats", "epd_op_gemm_residual_stats", "epd_op_norm_gemm_bf16",
    "epd_op_mx_rows", "epd_op_mx_gemm", "epd_op_mx_mfma_probe", "epd_op_attention_mx",
    "epd_mm_cache_create", "epd_mm_cache_destroy", "epd_mm_cache_free_blocks", "epd_mm_cache_base",
    "epd_mm_last_error", "epd_mm_alloc", "epd_mm_free", "epd_encode_paged", "epd_mm_transfer", "epd_mm_transfer_noalloc", "epd_mm_gather",
    "epd_encode_trunk_paged", "epd_project_merge",
)


class ModelDescC(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "dtype", "tile_size", "patch", "hidden", "heads", "mlp", "layers", "norm", "qk_norm", "act",
        "final_norm", "pixel_shuffle", "proj_kind", "proj_prenorm", "proj_mid", "proj_out")] + [
        ("eps", ctypes.c_float), ("max_tiles_per_call", ctypes.c_int32), ("layer_scale", ctypes.c_int32),
        ("class_token", ctypes.c_int32), ("proj_heads", ctypes.c_int32), ("mx_fp8", ctypes.c_int32)]


class WeightsC(ctypes.Structure):
    _fields_ = [("tensors", ctypes.POINTER(ctypes.c_void_p)), ("n_tensors", ctypes.c_int32)]


class EpdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"epd status {status}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2501_05460_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.epd_weight_count.argtypes = [ctypes.POINTER(ModelDescC)]
        L.epd_weight_count.restype = i32
        L.epd_check_desc.argtypes = [ctypes.POINTER(ModelDescC), ctypes.c_char_p, i32]
        L.epd_check_desc.restype = i32
        L.epd_check_offsets.argtypes = [ctypes.POINTER(i32), i32, i32]
        L.epd_check_offsets.restype = i32
        L.epd_create.argtypes = [ctypes.POINTER(ModelDescC), ctypes.POINTER(WeightsC), vp, ctypes.POINTER(vp)]
        L.epd_create.restype = i32
        L.epd_encode.argtypes = [vp, vp, i32, ctypes.POINTER(i32), i32, vp, vp]
        L.epd_encode.restype = i32
        L.epd_encode_range.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        L.epd_encode_range.restype = i32
        L.epd_tokens_per_tile.argtypes = [vp]
        L.epd_tokens_per_tile.restype = i64
        L.epd_out_dim.argtypes = [vp]
        L.epd_out_dim.restype = i64
        L.epd_last_error.argtypes = [vp]
        L.epd_last_error.restype = ctypes.c_char_p
        L.epd_destroy.argtypes = [vp]
        L.epd_destroy.restype = None
        L.epd_debug_read_stream.argtypes = [vp, vp, i64, i64]
        L.epd_debug_read_stream.restype = i32
        L.epd_op_gemm_bf16.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_float), vp]
        L.epd_op_gemm_bf16.restype = i32
        L.epd_op_gemm_bf16_form.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]
        L.epd_op_gemm_bf16_form.restype = i32
        L.epd_op_attention_bf16.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]
        L.epd_op_attention_bf16.restype = i32
        L.epd_op_mfma_probe.argtypes = [vp, vp, vp, vp]
        L.epd_op_mfma_probe.restype = i32
        L.epd_profile_enable.argtypes = [vp, i32]
        L.epd_profile_enable.restype = i32
        L.epd_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        L.epd_profile_read.restype = i32
        L.epd_op_mfma_peak.argtypes = [vp, i32, i32, vp, ctypes.POINTER(ctypes.c_float), vp]
        L.epd_op_mfma_peak.restype = i32
        L.epd_op_copy_peak.argtypes = [vp, vp, i64, i32, ctypes.POINTER(ctypes.c_float), vp]
        L.epd_op_copy_peak.restype = i32
        L.epd_op_coissue.argtypes = [vp, i32, i32, i32, i32, vp, ctypes.POINTER(ctypes.c_float), vp]
        L.epd_op_coissue.restype = i32
        L.epd_op_row_stats.argtypes = [vp, i64, i32, vp, vp, vp]
        L.epd_op_row_stats.restype = i32
        L.epd_op_gemm_residual_stats.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]
        L.epd_op_gemm_residual_stats.restype = i32
        L.epd_op_norm_gemm_bf16.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, ctypes.c_float, i32, i32, vp]
        L.epd_op_norm_gemm_bf16.restype = i32
        L.epd_op_mx_rows.argtypes = [vp, i32, i64, i32, i32, vp, vp, ctypes.c_float, vp, vp, vp]
        L.epd_op_mx_rows.restype = i32
        L.epd_op_mx_gemm.argtypes = [i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, i32, i32, i32, vp]
        L.epd_op_mx_gemm.restype = i32
        L.epd_op_attention_mx.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]
        L.epd_op_attention_mx.restype = i32
        L.epd_op_mx_mfma_probe.argtypes = [vp, vp, vp, vp, vp, vp]
        L.epd_op_mx_mfma_probe.restype = i32
        L.epd_mm_cache_create.argtypes = [i32, i32, i32, i32, ctypes.POINTER(vp)]
        L.epd_mm_cache_create.restype = i32
        L.epd_mm_cache_destroy.argtypes = [vp]
        L.epd_mm_cache_destroy.restype = None
        L.epd_mm_cache_free_blocks.argtypes = [vp]
        L.epd_mm_cache_free_blocks.restype = i32
        L.epd_mm_cache_base.argtypes = [vp]
        L.epd_mm_cache_base.restype = vp
        L.epd_mm_last_error.argtypes = [vp]
        L.epd_mm_last_error.restype = ctypes.c_char_p
        L.epd_mm_alloc.argtypes = [vp, i64, ctypes.POINTER(i32), i32, ctypes.POINTER(i32)]
        L.epd_mm_alloc.restype = i32
        L.epd_mm_free.argtypes = [vp, ctypes.POINTER(i32), i32]
        L.epd_mm_free.restype = i32
        L.epd_encode_paged.argtypes = [vp, vp, i32, ctypes.POINTER(i32), i32, vp, ctypes.POINTER(i32),
                                       ctypes.POINTER(i32), vp]
        L.epd_encode_paged.restype = i32
        L.epd_mm_transfer.argtypes = [vp, ctypes.POINTER(i32), vp, ctypes.POINTER(i32), i32, vp]
        L.epd_mm_transfer.restype = i32
        L.epd_mm_transfer_noalloc.argtypes = [vp, ctypes.POINTER(i32), vp, ctypes.POINTER(i32), i32, vp]
        L.epd_mm_transfer_noalloc.restype = i32
        L.epd_mm_gather.argtypes = [vp, ctypes.POINTER(i32), i32, vp, vp]
        L.epd_mm_gather.restype = i32
        L.epd_encode_trunk_paged.argtypes = [vp, vp, i32, i32, i32, vp, ctypes.POINTER(i32), vp]
        L.epd_encode_trunk_paged.restype = i32
        L.epd_project_merge.argtypes = [vp, vp, ctypes.POINTER(i32), i32, vp, vp]
        L.epd_project_merge.restype = i32
        _lib = L
    return _lib


def desc_to_c(desc) -> ModelDescC:
    d = ModelDescC()
    for name, _ in ModelDescC._fields_:
        setattr(d, name, getattr(desc, name))
    return d


def check_desc(desc) -> (int, str):
    buf = ctypes.create_string_buffer(512)
    s = lib().epd_check_desc(ctypes.byref(desc_to_c(desc)), buf, 512)
    return s, buf.value.decode()


def weight_count(desc) -> int:
    return lib().epd_weight_count(ctypes.byref(desc_to_c(desc)))


def check_offsets(offsets: Optional[Sequence[int]], n_requests: int, n_tiles: int) -> int:
    if offsets is None:
        return lib().epd_check_offsets(None, n_requests, n_tiles)
    arr = (ctypes.c_int32 * len(offsets))(*offsets)
    return lib().epd_check_offsets(arr, n_requests, n_tiles)


def _stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def to_device(arr: np.ndarray, bf16: bool, device="cuda") -> torch.Tensor:
    """Upload one fp32 host array; for bf16 the values must already lie on the
    bf16 grid and their upper 16 bits are shipped as they are."""
    a = np.ascontiguousarray(arr, dtype=np.float32)
    if not bf16:
        return torch.from_numpy(a).to(device)
    bits = (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    return torch.from_numpy(bits.view(np.int16)).to(device).view(torch.bfloat16)


class Encoder:
    """One encode worker: a library context plus the current device."""

    def __init__(self, desc, device_weights: List[torch.Tensor]):
        L = lib()
        if not torch.cuda.is_available():
            raise RuntimeError("the encode library needs a GPU; there is no CPU path")
        self.desc = desc
        self.bf16 = desc.dtype == 1
        want = torch.bfloat16 if self.bf16 else torch.float32
        for i, t in enumerate(device_weights):
            if not (t.is_cuda and t.is_contiguous() and t.dtype == want):
                raise ValueError(f"weight tensor {i} must be a contiguous {want} CUDA tensor")
        ptrs = (ctypes.c_void_p * len(device_weights))(*[t.data_ptr() for t in device_weights])
        w = WeightsC(ctypes.cast(ptrs, ctypes.POINTER(ctypes.c_void_p)), len(device_weights))
        handle = ctypes.c_void_p()
        s = L.epd_create(ctypes.byref(desc_to_c(desc)), ctypes.byref(w), _stream_ptr(), ctypes.byref(handle))
        if s != EPD_OK:
            raise EpdError(s, L.epd_last_error(None).decode())
        self._h = handle
        self.tokens_per_tile = int(L.epd_tokens_per_tile(handle))
        self.out_dim = int(L.epd_out_dim(handle))
        self.out_dtype = want

    def close(self):
        if getattr(self, "_h", None):
            lib().epd_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _raise(self, s: int):
        raise EpdError(s, lib().epd_last_error(self._h).decode())

    def alloc_out(self, n_tiles: int) -> torch.Tensor:
        return torch.empty((n_tiles * self.tokens_per_tile, self.out_dim), dtype=self.out_dtype, device="cuda")

    def encode(self, tiles: torch.Tensor, tile_offsets: Sequence[int], out: Optional[torch.Tensor] = None):
        n_tiles = int(tiles.shape[0]) if tiles is not None else 0
        if out is None:
            out = self.alloc_out(n_tiles)
        off = (ctypes.c_int32 * len(tile_offsets))(*tile_offsets)
        s = lib().epd_encode(self._h, tiles.data_ptr() if n_tiles else None, n_tiles, off,
                             len(tile_offsets) - 1, out.data_ptr() if n_tiles else None, _stream_ptr())
        if s != EPD_OK:
            self._raise(s)
        return out

    def encode_range(self, tiles: torch.Tensor, tile_begin: int, tile_end: int, out: torch.Tensor):
        s = lib().epd_encode_range(self._h, tiles.data_ptr(), int(tiles.shape[0]), tile_begin, tile_end,
                                   out.data_ptr(), _stream_ptr())
        if s != EPD_OK:
            self._raise(s)
        return out

    def read_stream(self, rows: int) -> np.ndarray:
        buf = np.empty((rows, self.desc.hidden), np.float32)
        s = lib().epd_debug_read_stream(self._h, buf.ctypes.data, rows, buf.nbytes)
        if s != EPD_OK:
            self._raise(s)
        return buf

    def profile_enable(self, on: bool = True):
        s = lib().epd_profile_enable(self._h, 1 if on else 0)
        if s != EPD_OK:
            self._raise(s)

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        ms = (ctypes.c_float * len(PROF_FAMILIES))()
        n = (ctypes.c_int32 * len(PROF_FAMILIES))()
        s = lib().epd_profile_read(self._h, ms, n)
        if s != EPD_OK:
            self._raise(s)
        return {name: {"ms": float(ms[i]), "launches": int(n[i])} for i, name in enumerate(PROF_FAMILIES)}


def _i32(values: Sequence[int]):
    return (ctypes.c_int32 * len(values))(*values)


class MMCache:
    """One paged multimodal-token cache (device pool + block manager)."""

    def __init__(self, n_blocks: int, block_tokens: int, token_dim: int, bf16: bool):
        h = ctypes.c_void_p()
        s = lib().epd_mm_cache_create(n_blocks, block_tokens, token_dim, 1 if bf16 else 0, ctypes.byref(h))
        if s != EPD_OK:
            raise EpdError(s, lib().epd_mm_last_error(None).decode())
        self._h = h
        self.n_blocks, self.block_tokens, self.token_dim, self.bf16 = n_blocks, block_tokens, token_dim, bf16

    def close(self):
        if getattr(self, "_h", None):
            lib().epd_mm_cache_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _raise(self, s):
        raise EpdError(s, lib().epd_mm_last_error(self._h).decode())

    @property
    def free_blocks(self) -> int:
        return lib().epd_mm_cache_free_blocks(self._h)

    def pool_tensor(self) -> torch.Tensor:
        """The device pool itself as a tensor [n_blocks, block_tokens, token_dim] (a view of the library's
        memory, no copy): valid until close()."""
        base = lib().epd_mm_cache_base(self._h)
        shape = (self.n_blocks, self.block_tokens, self.token_dim)

        class _Raw:   # bf16 has no typestr: the pool is exposed as 16-bit integers and viewed as bf16
            __cuda_array_interface__ = {"shape": shape, "typestr": "<i2" if self.bf16 else "<f4",
                                        "data": (int(base), False), "version": 2}
        t = torch.as_tensor(_Raw(), device="cuda")
        return t.view(torch.bfloat16) if self.bf16 else t

    def alloc(self, n_tokens: int) -> List[int]:
        cap = (n_tokens + self.block_tokens - 1) // self.block_tokens
        ids = (ctypes.c_int32 * max(cap, 1))()
        n = ctypes.c_int32()
        s = lib().epd_mm_alloc(self._h, n_tokens, ids, cap, ctypes.byref(n))
        if s != EPD_OK:
            self._raise(s)
        return [ids[i] for i in range(n.value)]

    def free(self, ids: Sequence[int]):
        s = lib().epd_mm_free(self._h, _i32(ids), len(ids))
        if s != EPD_OK:
            self._raise(s)

    def gather(self, ids: Sequence[int]) -> torch.Tensor:
        dtype = torch.bfloat16 if self.bf16 else torch.float32
        out = torch.empty((len(ids) * self.block_tokens, self.token_dim), dtype=dtype, device="cuda")
        s = lib().epd_mm_gather(self._h, _i32(ids), len(ids), out.data_ptr(), _stream_ptr())
        if s != EPD_OK:
            self._raise(s)
        return out

    def transfer_to(self, src_ids: Sequence[int], dst: "MMCache", dst_ids: Sequence[int], noalloc: bool = False):
        """noalloc: the entry point that keeps its id lists in the library's static device array."""
        fn = lib().epd_mm_transfer_noalloc if noalloc else lib().epd_mm_transfer
        s = fn(self._h, _i32(src_ids), dst._h, _i32(dst_ids), len(src_ids), _stream_ptr())
        if s != EPD_OK:
            dst._raise(s)


def encode_paged(enc: "Encoder", tiles: torch.Tensor, tile_offsets: Sequence[int], cache: MMCache,
                 block_tables: Sequence[Sequence[int]]):
    """block_tables[r] = block ids of request r in token order."""
    flat, offs = [], [0]
    for t in block_tables:
        flat.extend(t)
        offs.append(len(flat))
    s = lib().epd_encode_paged(enc._h, tiles.data_ptr(), int(tiles.shape[0]), _i32(tile_offsets),
                               len(tile_offsets) - 1, cache._h, _i32(flat or [0]), _i32(offs), _stream_ptr())
    if s != EPD_OK:
        enc._raise(s)


def encode_trunk_paged(enc: "Encoder", tiles: torch.Tensor, tile_begin: int, tile_end: int, cache: MMCache,
                       block_table: Sequence[int]):
    """Slices [tile_begin, tile_end) -> pre-projection tokens in `cache`, blocks in slice order."""
    s = lib().epd_encode_trunk_paged(enc._h, tiles.data_ptr(), int(tiles.shape[0]), tile_begin, tile_end,
                                     cache._h, _i32(block_table or [0]), _stream_ptr())
    if s != EPD_OK:
        enc._raise(s)


def project_merge(enc: "Encoder", cache: MMCache, block_table: Sequence[int], n_tiles: int,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Pre-projection tokens listed by `block_table` (slice order) -> merged multimodal tokens."""
    if out is None:
        out = enc.alloc_out(n_tiles)
    s = lib().epd_project_merge(enc._h, cache._h, _i32(block_table or [0]), n_tiles, out.data_ptr(), _stream_ptr())
    if s != EPD_OK:
        enc._raise(s)
    return out


def op_gemm_bf16(A: torch.Tensor, W: torch.Tensor, bias: Optional[torch.Tensor], iters: int = 1):
    """C = A W^T (+ bias) with the library's MFMA GEMM; returns (C, ms per launch)."""
    M, K = A.shape
    N = W.shape[0]
    C = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    ms = ctypes.c_float()
    s = lib().epd_op_gemm_bf16(A.data_ptr(), W.data_ptr(), bias.data_ptr() if bias is not None else None,
                               C.data_ptr(), M, N, K, iters, ctypes.byref(ms), _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, lib().epd_last_error(None).decode())
    return C, ms.value


def op_gemm_bf16_form(A: torch.Tensor, W: torch.Tensor, bias: torch.Tensor, epi: int, form: int,
                      R: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One GEMM launch in the given form; returns C (bf16) or, for epi 3, the updated R (fp32, in place).

    The output buffer carries guard rows behind row M; a call that writes any of them raises."""
    M, K = A.shape
    N = W.shape[0]
    guard = 12345.0
    Cg = torch.full((M + 64, N), guard, dtype=torch.bfloat16, device=A.device) if epi != 3 else None
    Rg = None
    if epi == 3:
        Rg = torch.full((M + 64, N), guard, dtype=torch.float32, device=A.device)
        Rg[:M] = R
    s = lib().epd_op_gemm_bf16_form(A.contiguous().data_ptr(), W.data_ptr(), bias.data_ptr(),
                                    Cg.data_ptr() if Cg is not None else None,
                                    Rg.data_ptr() if Rg is not None else None, M, N, K, epi, form, _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, lib().epd_last_error(None).decode())
    tail = Cg[M:] if epi != 3 else Rg[M:]
    if not bool((tail == guard).all()):
        raise RuntimeError("GEMM form %d wrote rows past M=%d" % (form, M))
    if epi != 3:
        return Cg[:M]
    R.copy_(Rg[:M])
    return R


def op_attention_bf16(q: torch.Tensor, k: torch.Tensor, vt: torch.Tensor, n_slices: int, n_tokens: int,
                      heads: int, hd_pad: int, ld_qk: int, n_keys: Optional[int] = None) -> torch.Tensor:
    """q must carry the logit scale log2(e) / sqrt(hd): the kernel's weights are 2^(q . k)."""
    o = torch.empty((n_slices * n_tokens, heads * hd_pad), dtype=torch.bfloat16, device=q.device)
    s = lib().epd_op_attention_bf16(q.data_ptr(), k.data_ptr(), vt.data_ptr(), o.data_ptr(), n_slices,
                                    n_tokens, n_tokens if n_keys is None else n_keys, heads, hd_pad, ld_qk,
                                    _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, lib().epd_last_error(None).decode())
    return o


def op_mfma_probe(A: torch.Tensor, B: torch.Tensor) -> torch.Tensor:
    D = torch.empty((32, 32), dtype=torch.float32, device=A.device)
    s = lib().epd_op_mfma_probe(A.data_ptr(), B.data_ptr(), D.data_ptr(), _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, "mfma probe failed")
    return D


def op_mfma_peak(random_operands: bool, iters: int = 2000, reps: int = 5) -> float:
    """Dense bf16 TFLOP/s of a register-resident MFMA loop on every CU (random or constant operands)."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(2 * cus * 256, dtype=torch.float32, device="cuda")
    ops = None
    if random_operands:
        g = torch.Generator(device="cuda").manual_seed(1)
        ops = torch.randn(8192, device="cuda", generator=g).to(torch.bfloat16)
    out = ctypes.c_float()
    s = lib().epd_op_mfma_peak(ops.data_ptr() if ops is not None else None, iters, reps, sink.data_ptr(),
                               ctypes.byref(out), _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, "mfma peak probe failed")
    return out.value


def op_coissue(which: int, iters_mfma: int = 4000, iters_valu: int = 5000, reps: int = 5) -> float:
    """ms per launch of the issue-port probe: which = 1 matrix waves alone, 2 vector waves alone, 3 both."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(cus * 512, dtype=torch.float32, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(1)
    ops = torch.randn(4096, device="cuda", generator=g).to(torch.bfloat16)
    out = ctypes.c_float()
    s = lib().epd_op_coissue(ops.data_ptr(), iters_mfma, iters_valu, which, reps, sink.data_ptr(), ctypes.byref(out),
                             _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, "co-issue probe failed")
    return out.value


def op_copy_peak(n_bytes: int = 1 << 30, reps: int = 5) -> float:
    """Read + write GB/s of a plain streaming copy of n_bytes."""
    src = torch.ones(n_bytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    out = ctypes.c_float()
    s = lib().epd_op_copy_peak(src.data_ptr(), dst.data_ptr(), n_bytes, reps, ctypes.byref(out), _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, "copy peak probe failed")
    return out.value


def op_row_stats(x: torch.Tensor):
    """(bf16 copy, statistics pairs [rows, ceil(dim / 128), 2]) of the rows of x [rows, dim] fp32."""
    rows, dim = x.shape
    xb = torch.empty((rows, dim), dtype=torch.bfloat16, device=x.device)
    stats = torch.full((rows, (dim + 127) // 128, 2), float("nan"), dtype=torch.float32, device=x.device)
    s = lib().epd_op_row_stats(x.data_ptr(), rows, dim, xb.data_ptr(), stats.data_ptr(), _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, "row stats failed")
    return xb, stats


def op_gemm_residual_stats(A: torch.Tensor, W: torch.Tensor, bias: torch.Tensor, R: torch.Tensor, form: int):
    """R += A W^T + bias in place (fp32) in the given form; returns (bf16 copy of the new R, its statistics pairs)."""
    M, K = A.shape
    N = W.shape[0]
    Rp = torch.zeros(M * N + 256, dtype=torch.float32, device=A.device)
    Rp[:M * N] = R.reshape(-1)
    xb = torch.empty((M, N), dtype=torch.bfloat16, device=A.device)
    stats = torch.full((M, N // 128, 2), float("nan"), dtype=torch.float32, device=A.device)
    s = lib().epd_op_gemm_residual_stats(A.data_ptr(), W.data_ptr(), bias.data_ptr(), Rp.data_ptr(), xb.data_ptr(),
                                         stats.data_ptr(), M, N, K, form, _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, lib().epd_last_error(None).decode())
    R.copy_(Rp[:M * N].view(M, N))
    return xb, stats


def op_norm_gemm_bf16(x: torch.Tensor, gamma: torch.Tensor, beta: Optional[torch.Tensor], W: torch.Tensor,
                      bias: torch.Tensor, eps: float, epi: int, form: int) -> torch.Tensor:
    """act(norm(x) W^T + bias) with the norm folded into the product (beta None: RMSNorm)."""
    M, D = x.shape
    N = W.shape[0]
    C = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    s = lib().epd_op_norm_gemm_bf16(x.data_ptr(), gamma.data_ptr(), beta.data_ptr() if beta is not None else None,
                                    W.data_ptr(), bias.data_ptr(), C.data_ptr(), M, N, D, eps, epi, form, _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, lib().epd_last_error(None).decode())
    return C


def op_mx_rows(x: torch.Tensor, kind: int = 2, gamma: Optional[torch.Tensor] = None, beta: Optional[torch.Tensor] = None,
               eps: float = 0.0):
    """MXFP8 conversion of the rows of x [rows, dim] (fp32 or bf16), optionally behind a LayerNorm (kind 0) or an
    RMSNorm (kind 1).  Returns (codes uint8 [rows, dim], scale words int32 [dim / 128, rows])."""
    rows, dim = x.shape
    codes = torch.full((rows, dim), 0xAA, dtype=torch.uint8, device=x.device)
    scales = torch.full((dim // 128, rows), -1, dtype=torch.int32, device=x.device)
    s = lib().epd_op_mx_rows(x.contiguous().data_ptr(), 1 if x.dtype == torch.bfloat16 else 0, rows, dim, kind,
                             gamma.data_ptr() if gamma is not None else None, beta.data_ptr() if beta is not None else None,
                             eps, codes.data_ptr(), scales.data_ptr(), _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, lib().epd_last_error(None).decode())
    return codes, scales


def op_mx_gemm(epi: int, A: torch.Tensor, SA: torch.Tensor, W: torch.Tensor, SW: torch.Tensor, bias: torch.Tensor,
               cscale: Optional[torch.Tensor] = None, R: Optional[torch.Tensor] = None, n_tok: int = 0, heads: int = 0,
               hd_pad: int = 0):
    """Product of MXFP8 operands (codes uint8 [M, K] / [N, K], scale words int32 [K / 128, M] / [K / 128, N]).
    epi 0: bf16 [M, N]; 5: bf16 [M / n_tok, heads, hd_pad, n_tok]; 1 / 2: (codes [M, N], scale words [N / 128, M])
    of the activated output; 3: R (fp32, in place) += product."""
    M, K = A.shape
    N = W.shape[0]
    C = Cq = SC = None
    if epi in (0, 5):
        C = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=A.device)
    elif epi in (1, 2):
        Cq = torch.full((M, N), 0xAA, dtype=torch.uint8, device=A.device)
        SC = torch.full((N // 128, M), -1, dtype=torch.int32, device=A.device)
    ptr = lambda t: t.data_ptr() if t is not None else None
    s = lib().epd_op_mx_gemm(epi, A.data_ptr(), SA.data_ptr(), W.data_ptr(), SW.data_ptr(), bias.data_ptr(), ptr(cscale),
                             M, N, K, ptr(C), ptr(R), ptr(Cq), ptr(SC), n_tok, heads, hd_pad, _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, lib().epd_last_error(None).decode())
    if epi == 0:
        return C
    if epi == 5:
        return C.view(M // n_tok, heads, hd_pad, n_tok)
    if epi == 3:
        return R
    return Cq, SC


def op_mx_mfma_probe(a: torch.Tensor, b: torch.Tensor, sa: torch.Tensor, sb: torch.Tensor) -> torch.Tensor:
    """One 32x32x64 scaled FP8 MFMA on raw registers: a, b int32 [64, 8], sa, sb int32 [64] -> fp32 [64, 16]."""
    d = torch.empty((64, 16), dtype=torch.float32, device=a.device)
    s = lib().epd_op_mx_mfma_probe(a.data_ptr(), b.data_ptr(), sa.data_ptr(), sb.data_ptr(), d.data_ptr(), _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, "mx mfma probe failed")
    return d


def op_attention_mx(q: torch.Tensor, k: torch.Tensor, vt: torch.Tensor, n_slices: int, n_tokens: int, heads: int,
                    hd_pad: int, ld_qk: int, n_keys: Optional[int] = None):
    """op_attention_bf16 with the output as MXFP8: (codes uint8 [rows, heads * hd_pad], scale words int32 [cols / 128, rows])."""
    rows, cols = n_slices * n_tokens, heads * hd_pad
    codes = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device=q.device)
    scales = torch.full((cols // 128, rows), -1, dtype=torch.int32, device=q.device)
    s = lib().epd_op_attention_mx(q.data_ptr(), k.data_ptr(), vt.data_ptr(), codes.data_ptr(), scales.data_ptr(), n_slices,
                                  n_tokens, n_tokens if n_keys is None else n_keys, heads, hd_pad, ld_qk, _stream_ptr())
    if s != EPD_OK:
        raise EpdError(s, lib().epd_last_error(None).decode())
    return codes, scales
