"""The five benchmark workloads, as seeded synthetic inputs.

Shapes follow the paper's setting (one long behaviour history per user, thousands
of items, up to ~10K for lifelong histories; a small candidate set per request;
Sec. 3.1 and Sec. 4.1) in the many-candidates-per-user serving regime. Every
array is produced per user from its own seed so that a single user can be
regenerated without building the whole batch.

Nothing here computes scores, gates, segment sums or attention.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import numpy as np

from .bf16 import f32_to_bf16_bits, bf16_bits_to_f32

TAIL_SCALE = 16.0  # padding rows (j >= len[u]) hold finite but large values


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    dtype: str            # "f32" | "bf16"  (storage type of q,k,v,t0,weights)
    U: int                # users
    C: int                # candidates per user
    L: int                # maximum history length
    d: int                # value / embedding dim
    d_q: int              # query / key dim
    w: int                # segment length
    M: int                # GSTA layers
    lens_kind: str        # "full" | "uniform" | "loguniform"
    lens_lo: int = 0
    lens_hi: int = 0
    aligned_frac: float = 0.0   # fraction of history items whose key is aligned to a candidate
    aligned_cos: float = 0.8
    seed: int = 0

    @property
    def S(self) -> int:
        return -(-self.L // self.w)

    @property
    def gamma(self) -> float:
        return math.sqrt(self.d_q)

    @property
    def pairs(self) -> int:
        return self.U * self.C

    def replace(self, **kw) -> "WorkloadSpec":
        return dataclasses.replace(self, **kw)


CONFIGS: Dict[str, WorkloadSpec] = {
    "cfg1_tiny_f32": WorkloadSpec("cfg1_tiny_f32", "f32", U=1, C=16, L=1024, d=64, d_q=64, w=64, M=1,
                                  lens_kind="full", seed=1001),
    "cfg2_bf16": WorkloadSpec("cfg2_bf16", "bf16", U=64, C=64, L=2048, d=64, d_q=64, w=128, M=1,
                              lens_kind="uniform", lens_lo=512, lens_hi=2048, seed=1002),
    "cfg3_high_fanout": WorkloadSpec("cfg3_high_fanout", "bf16", U=32, C=256, L=4096, d=128, d_q=128, w=128, M=1,
                                     lens_kind="full", aligned_frac=0.05, seed=1003),
    "cfg4_low_fanout": WorkloadSpec("cfg4_low_fanout", "bf16", U=4096, C=1, L=4096, d=64, d_q=64, w=256, M=1,
                                    lens_kind="loguniform", lens_lo=64, lens_hi=4096, seed=1004),
    "cfg5_lifelong": WorkloadSpec("cfg5_lifelong", "bf16", U=16, C=128, L=10000, d=128, d_q=128, w=256, M=2,
                                  lens_kind="full", seed=1005),
}


def _rng(*key) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(list(key))))


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values -> storage array (float32, or uint16 bfloat16 bit patterns)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return x if dtype == "f32" else f32_to_bf16_bits(x)


def stored_values(a: np.ndarray) -> np.ndarray:
    """Exact float32 values held by a storage array."""
    return bf16_bits_to_f32(a) if a.dtype == np.uint16 else np.asarray(a, dtype=np.float32)


def make_lens(spec: WorkloadSpec) -> np.ndarray:
    """Valid history length of every user, int32 [U]."""
    r = _rng(spec.seed, 2)
    if spec.lens_kind == "full":
        return np.full(spec.U, spec.L, dtype=np.int32)
    if spec.lens_kind == "uniform":
        return r.integers(spec.lens_lo, spec.lens_hi + 1, size=spec.U).astype(np.int32)
    if spec.lens_kind == "loguniform":
        x = r.uniform(math.log(spec.lens_lo), math.log(spec.lens_hi + 1), size=spec.U)
        return np.clip(np.floor(np.exp(x)), spec.lens_lo, spec.lens_hi).astype(np.int32)
    raise ValueError(spec.lens_kind)


def make_weights(spec: WorkloadSpec) -> Dict[str, np.ndarray]:
    """GSTA projection matrices, [M,d,d] each, entries N(0, sigma=1/sqrt(d)), y = x @ W."""
    r = _rng(spec.seed, 3)
    sd = 1.0 / math.sqrt(spec.d)
    out = {}
    for name in ("wq", "wk", "wv"):
        out[name] = _store(r.standard_normal((spec.M, spec.d, spec.d), dtype=np.float32) * np.float32(sd), spec.dtype)
    return out


def make_user(spec: WorkloadSpec, u: int, length: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Inputs of one user: q [C,d_q], k [L,d_q], v [L,d], t0 [C,d] as storage arrays."""
    r = _rng(spec.seed, 1, int(u))
    q = r.standard_normal((spec.C, spec.d_q), dtype=np.float32) * np.float32(1.0 / math.sqrt(spec.d_q))
    k = r.standard_normal((spec.L, spec.d_q), dtype=np.float32) * np.float32(1.0 / math.sqrt(spec.d_q))
    v = r.standard_normal((spec.L, spec.d), dtype=np.float32) * np.float32(1.0 / math.sqrt(spec.d))
    if spec.d_q == spec.d:
        t0 = q.copy()          # the workloads list only "queries": the target vector is the same values
    else:
        t0 = r.standard_normal((spec.C, spec.d), dtype=np.float32) * np.float32(1.0 / math.sqrt(spec.d))
    if spec.aligned_frac > 0.0:
        n = int(round(spec.aligned_frac * spec.L))
        pos = r.choice(spec.L, size=n, replace=False)
        cand = r.integers(0, spec.C, size=n)
        qh = q[cand].astype(np.float64)
        qh /= np.linalg.norm(qh, axis=1, keepdims=True)
        kj = k[pos].astype(np.float64)
        nk = np.linalg.norm(kj, axis=1, keepdims=True)
        orth = kj - (kj * qh).sum(1, keepdims=True) * qh
        orth /= np.linalg.norm(orth, axis=1, keepdims=True)
        c = spec.aligned_cos
        k[pos] = (nk * (c * qh + math.sqrt(1.0 - c * c) * orth)).astype(np.float32)
    if length is not None and length < spec.L:
        k[length:] *= np.float32(TAIL_SCALE)
        v[length:] *= np.float32(TAIL_SCALE)
    return {"q": _store(q, spec.dtype), "k": _store(k, spec.dtype), "v": _store(v, spec.dtype),
            "t0": _store(t0, spec.dtype)}


@dataclass
class Workload:
    spec: WorkloadSpec
    users: np.ndarray         # which user indices of the spec these rows are
    lens: np.ndarray          # int32 [n]
    q: np.ndarray             # [n,C,d_q] storage
    k: np.ndarray             # [n,L,d_q] storage
    v: np.ndarray             # [n,L,d]   storage
    t0: np.ndarray            # [n,C,d]   storage
    wq: np.ndarray            # [M,d,d]   storage
    wk: np.ndarray
    wv: np.ndarray

    def f64(self, name: str, u: Optional[int] = None) -> np.ndarray:
        """Exact stored values as float64 (optionally only row u of a per-user array)."""
        a = getattr(self, name)
        if u is not None:
            a = a[u]
        return stored_values(a).astype(np.float64)


def make_workload(spec: WorkloadSpec, users: Optional[Sequence[int]] = None) -> Workload:
    """Build the batch (or only the listed users of it) on the host."""
    all_lens = make_lens(spec)
    idx = np.arange(spec.U) if users is None else np.asarray(list(users), dtype=np.int64)
    n = len(idx)
    sdt = np.float32 if spec.dtype == "f32" else np.uint16
    q = np.empty((n, spec.C, spec.d_q), sdt)
    k = np.empty((n, spec.L, spec.d_q), sdt)
    v = np.empty((n, spec.L, spec.d), sdt)
    t0 = np.empty((n, spec.C, spec.d), sdt)
    for i, u in enumerate(idx):
        one = make_user(spec, int(u), int(all_lens[u]))
        q[i], k[i], v[i], t0[i] = one["q"], one["k"], one["v"], one["t0"]
    wts = make_weights(spec)
    return Workload(spec, idx, all_lens[idx].copy(), q, k, v, t0, wts["wq"], wts["wk"], wts["wv"])
