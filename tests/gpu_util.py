"""Helpers shared by the GPU parity tests (marshalling and error norms only)."""
import numpy as np
import torch

import workloads as wl
from paper_2501_05460_amd import binding as B

TOL_BF16 = 2e-2   # max |gpu - oracle| / max |oracle|, bf16 mode
TOL_FP32 = 1e-4   # same norm, fp32 mode


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Largest absolute deviation relative to the largest reference magnitude
    of the compared buffer (element-wise relative error is unbounded at
    near-zero outputs)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.abs(got - ref).max() / np.abs(ref).max())


def rel_l2(got, ref) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(got - ref) / np.linalg.norm(ref))


def device_weights(desc, weights):
    bf = desc.dtype == wl.DT_BF16
    return [B.to_device(weights[name], bf) for name, _, _ in wl.weight_specs(desc)]


def make_encoder(desc, weights):
    return B.Encoder(desc, device_weights(desc, weights))


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


def tol(desc) -> float:
    return TOL_BF16 if desc.dtype == wl.DT_BF16 else TOL_FP32
