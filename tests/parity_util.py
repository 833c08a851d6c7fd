"""Shared helpers of the GPU parity tests: upload seeded inputs, run the fp64 checker, compare.

Error metric (used for every floating-point output): for each output vector x (one H'[u,c,i,:] or one
z[u,c,:]) the error is max|x_gpu - x_ref| / max|x_ref|; the reported figure is the maximum over vectors.
Vectors whose reference is exactly zero (empty segments) must be exactly zero on the GPU.
Tolerances: 1e-5 for fp32 storage; 2e-2 for bf16 storage with fp32 accumulation.

Second figure, element by element (`elem_rel_err`): |x_gpu - x_ref| / max(|x_ref|, floor) with floor = the root mean
square of the reference vector the element belongs to, so that the small components of a vector are bounded one by one
and not only through its largest one, while components that cancel to nearly nothing do not divide by nearly nothing.
Its bound is the vector tolerance times 2.5, the ratio of the largest component to the root mean square in a vector
of 64 to 128 roughly Gaussian components: the two figures then ask the same of the largest component and the second
asks it of every other one too.
"""
from __future__ import annotations

import numpy as np

import oracle
from workloads.configs import Workload, stored_values

TOL = {"f32": 1e-5, "bf16": 2e-2}
ELEM_TOL = {"f32": 2.5e-5, "bf16": 5e-2}


def to_device(arr: np.ndarray):
    """Storage array (float32, uint16 bf16 bits, int32) -> device tensor of the matching torch dtype."""
    import torch
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def to_host_f64(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float64).cpu().numpy()


class DeviceWorkload:
    def __init__(self, wl: Workload):
        self.wl = wl
        self.spec = wl.spec
        for name in ("q", "k", "v", "t0", "wq", "wk", "wv"):
            setattr(self, name, to_device(getattr(wl, name)))
        self.lens = to_device(wl.lens.astype(np.int32))


def oracle_batch(wl: Workload, gamma=None):
    """Checker outputs for a (small) workload: (H' f64, cnt int32, z f64)."""
    s = wl.spec
    g = s.gamma if gamma is None else gamma
    return oracle.laser_forward(wl.f64("q"), wl.f64("k"), wl.f64("v"), wl.f64("t0"), wl.f64("wq"), wl.f64("wk"),
                                wl.f64("wv"), wl.lens, s.w, g)


def oracle_pair(wl: Workload, row: int, c: int, gamma=None):
    """Checker outputs of one (user row, candidate): (H' [S,d], z [d])."""
    s = wl.spec
    g = s.gamma if gamma is None else gamma
    Hp = oracle.sta_pair(wl.f64("q", row)[c], wl.f64("k", row), wl.f64("v", row), int(wl.lens[row]), s.w, g)
    cnt = oracle.segment_counts(wl.lens[row:row + 1], s.L, s.w)[0]
    z = oracle.gsta_pair(Hp, wl.f64("t0", row)[c], wl.f64("wq"), wl.f64("wk"), wl.f64("wv"), cnt > 0)
    return Hp, z


def vec_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Maximum over vectors (last axis) of max|got - ref| / max|ref|; exact-zero references must match exactly."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite value in GPU output"
    num = np.abs(got - ref).max(axis=-1)
    den = np.abs(ref).max(axis=-1)
    zero = den == 0
    assert (num[zero] == 0).all(), "a vector that must be exactly zero is not"
    den = np.where(zero, 1.0, den)
    return float((num / den).max()) if num.size else 0.0


def elem_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Maximum over elements of |got - ref| / max(|ref|, rms of the element's reference vector (last axis))."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    floor = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    den = np.maximum(np.abs(ref), floor)
    zero = den == 0                      # whole vector exactly zero: must match exactly (checked by vec_rel_err too)
    assert (got[np.broadcast_to(zero, got.shape)] == 0).all(), "an element that must be exactly zero is not"
    return float((np.abs(got - ref) / np.where(zero, 1.0, den)).max())


def round_like(x: np.ndarray, dtype: str) -> np.ndarray:
    """fp64 reference values as they read after storage in `dtype` (used when a stored H' feeds GSTA)."""
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    from workloads.bf16 import round_to_bf16
    return round_to_bf16(x.astype(np.float32)).astype(np.float64)
