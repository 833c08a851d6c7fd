"""Work accounting for the STA + GSTA path.

Two separate things live here:

1. The paper's own analytic cost model (Sec. 3.6), which counts ONE operation per
   multiply-accumulate: C_proj, C_attn, C_ffn, C_STA, C_GSTA, C_LASER, C_SA, C_TA.
   It is reproduced so that the repo's accounting can be checked against the
   numbers the paper prints (Sec. 3.6.2 worked example, Table 2 FLOPs column,
   Table 4 relative FLOPs).

2. The algorithmic flops (2 per multiply-accumulate) and bytes of the kernels in
   this repo, per batch, used for roofline arithmetic by the benchmark.
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------- paper model (1 op per MAC)


def c_proj(L, d, d_q):
    """K and V projections of the whole history (Sec. 3.6.1, C_proj)."""
    return L * d * d + L * d * d_q


def c_attn(L, d, d_q):
    """Score dot products plus gated aggregation (Sec. 3.6.1, C_attn)."""
    return L * d_q + L * d


def c_ffn(L, d, w, r):
    """FFN on the compressed sequence only (Sec. 3.6.1, C_ffn)."""
    return (L / w) * (2 * r * d * d)


def c_sta(L, d, d_q, w, r):
    """C_STA ~ L d (d + d_q) + (L / w) 2 r d^2 (Sec. 3.6.1)."""
    return L * d * (d + d_q) + (L / w) * (2 * r * d * d)


def c_gsta(L, d, w, M):
    """C_GSTA ~ M L' (2 d^2 + 2 d) (Sec. 3.6.1)."""
    return M * (L / w) * (2 * d * d + 2 * d)


def c_laser(L, d, d_q, w, r, M):
    """C_LASER ~ L d^2 (1 + d_q / d + (2 r + 2 M) / w) (Sec. 3.6.1)."""
    return L * d * d * (1.0 + d_q / d + (2 * r + 2 * M) / w)


def c_self_attention(L, d):
    """C_SA ~ 4 L d^2 + 2 L^2 d (Sec. 3.6.2)."""
    return 4 * L * d * d + 2 * L * L * d


def c_target_attention(L, d):
    """C_TA ~ 2 L d^2 + 2 L d (Sec. 3.6.2)."""
    return 2 * L * d * d + 2 * L * d


# ---------------------------------------------------------------- this repo's kernels (2 flops per MAC)

_ESIZE = {"f32": 4, "bf16": 2}


def sta_flops(lens, C, d_q, d):
    """Score + aggregation over valid items only: 2 * len * (d_q + d) per (user, candidate)."""
    return 2.0 * float(np.sum(np.asarray(lens, dtype=np.float64))) * C * (d_q + d)


def sta_bytes(lens, U, C, L, d_q, d, w, dtype):
    """HBM bytes one STA launch must move: valid K and V rows once, Q once, lens, H' written once."""
    e = _ESIZE[dtype]
    S = -(-L // w)
    n = float(np.sum(np.asarray(lens, dtype=np.float64)))
    return n * (d_q + d) * e + U * C * d_q * e + U * 4 + U * C * S * d * e


def gsta_flops(lens, C, d, w, M):
    """Re-associated order: per layer 3 d^2 (q', W_k q', pooled * W_v) + 2 S_valid d MACs per pair."""
    sv = np.ceil(np.asarray(lens, dtype=np.float64) / w)
    return 2.0 * M * float(np.sum(3.0 * d * d + 2.0 * sv * d)) * C


def gsta_bytes(lens, U, C, L, d, w, M, dtype):
    """H' rows of valid segments read once, t0 read, weights read once, z written (fp32)."""
    e = _ESIZE[dtype]
    sv = float(np.sum(np.ceil(np.asarray(lens, dtype=np.float64) / w)))
    return sv * C * d * e + U * C * d * e + 3 * M * d * d * e + U * 4 + U * C * d * 4


def path_bytes(lens, U, C, L, d_q, d, w, M, dtype, seg_out_written=True):
    """HBM bytes one pass of the whole path (STA then GSTA) must move: valid K and V rows, Q, t0, the GSTA weights and
    lens read once; H' written once when it is returned; z written (fp32). H' is not counted as read: the method
    does not need it back from memory (GSTA could consume it where it is produced), so a second pass over it is
    overhead of an implementation, not work of the algorithm."""
    e = _ESIZE[dtype]
    S = -(-L // w)
    n = float(np.sum(np.asarray(lens, dtype=np.float64)))
    b = n * (d_q + d) * e + U * C * (d_q + d) * e + 3 * M * d * d * e + U * 4 + U * C * d * 4
    return b + (U * C * S * d * e if seg_out_written else 0)


def path_flops(lens, C, d_q, d, w, M):
    """STA over valid items plus GSTA in the re-associated order."""
    return sta_flops(lens, C, d_q, d) + gsta_flops(lens, C, d, w, M)
