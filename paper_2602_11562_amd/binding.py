"""Thin ctypes binding over liblaser.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/laser.h).
Tensors are PyTorch device tensors used purely as owners of HBM allocations; the
current torch stream is handed to the library. There is no fallback: if the
shared library is missing or an entry point reports an error, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblaser.so")

LASER_F32, LASER_BF16 = 0, 1
STA_AUTO, STA_GENERIC, STA_MFMA, STA_STREAM, STA_MFMA_CACHED = 0, 1, 2, 3, 4
GSTA_AUTO, GSTA_GENERIC, GSTA_TILED, GSTA_SPLIT, GSTA_ONE = 0, 1, 2, 3, 4
FFN_AUTO, FFN_GENERIC, FFN_MFMA = 0, 1, 2
PROJECT_AUTO, PROJECT_GENERIC, PROJECT_MFMA = 0, 1, 2

EXPORTS = [
    "laser_sta_forward", "laser_sta_forward_variant", "laser_sta_forward_heads", "laser_sta_forward_softmax", "laser_sta_forward_ragged",
    "laser_gsta_forward_ragged", "laser_forward_ragged", "laser_multires_forward_ragged",
    "laser_segment_ffn_forward_ragged", "laser_gsta_forward", "laser_gsta_forward_variant",
    "laser_forward", "laser_forward_fused", "laser_forward_fused_work_bytes", "laser_multires_forward", "laser_forward_multires", "laser_gsta_forward_multires",
    "laser_sta_kernel_name",
    "laser_gsta_kernel_name", "laser_segment_ffn_forward", "laser_segment_ffn_forward_variant", "laser_ffn_gsta_forward", "laser_ffn_gsta_forward_multires",
    "laser_gsta_kernel_name_layers", "laser_project_q_forward", "laser_project_q_forward_variant",
    "laser_project_kv_forward", "laser_project_kv_forward_variant", "laser_fold_query_weights",
    "laser_project_heads_forward", "laser_sta_folded_forward", "laser_sta_backward", "laser_sta_backward_bf16", "laser_sta_backward_static", "laser_sta_backward_work_bytes", "laser_gsta_backward",
    "laser_gsta_backward_work_bytes",
    "laser_status_string", "laser_version",
]


class LaserError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (status {code})")


_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen liblaser.so (built by paper_2602_11562_amd.build) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_11562_amd.build` "
                          "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ip, i32, f32 = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.laser_sta_forward.argtypes = [vp, vp, vp, ip, i32, i32, i32, i32, i32, i32, f32, i32, vp, ip, vp]
    lib.laser_sta_forward_variant.argtypes = lib.laser_sta_forward.argtypes + [i32]
    lib.laser_sta_forward_heads.argtypes = [vp, vp, vp, ip, i32, i32, i32, i32, i32, i32, f32, i32, i32, vp, ip, vp, i32]
    lib.laser_sta_forward_heads.restype = i32
    lib.laser_sta_forward_softmax.argtypes = lib.laser_sta_forward_heads.argtypes
    lib.laser_sta_forward_softmax.restype = i32
    lib.laser_gsta_forward.argtypes = [vp, vp, vp, vp, vp, ip, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.laser_gsta_forward_variant.argtypes = lib.laser_gsta_forward.argtypes + [i32]
    lib.laser_forward.argtypes = [vp, vp, vp, vp, vp, vp, vp, ip, i32, i32, i32, i32, i32, i32, f32, i32, i32,
                                  vp, ip, vp, vp]
    lib.laser_forward_fused.argtypes = [vp, vp, vp, vp, vp, vp, vp, ip, i32, i32, i32, i32, i32, i32, f32, i32,
                                        ip, vp, vp, ctypes.c_size_t, vp]
    lib.laser_forward_fused.restype = i32
    lib.laser_forward_fused_work_bytes.argtypes = [i32, i32, i32, i32, i32, i32, i32]
    lib.laser_forward_fused_work_bytes.restype = ctypes.c_size_t
    for name in ("laser_sta_forward", "laser_sta_forward_variant", "laser_gsta_forward",
                 "laser_gsta_forward_variant", "laser_forward", "laser_version"):
        getattr(lib, name).restype = i32
    lib.laser_multires_forward.argtypes = [vp, ip, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.laser_multires_forward.restype = i32
    lib.laser_forward_multires.argtypes = lib.laser_forward.argtypes[:-1] + [i32, vp, vp, vp]
    lib.laser_forward_multires.restype = i32
    lib.laser_gsta_forward_multires.argtypes = lib.laser_gsta_forward.argtypes[:-1] + [i32, vp, vp, vp]
    lib.laser_gsta_forward_multires.restype = i32
    fp = ctypes.c_void_p
    lib.laser_segment_ffn_forward.argtypes = [vp, ip, vp, fp, vp, fp, fp, fp, i32, i32, i32, i32, i32, i32, f32, i32,
                                              vp, vp]
    lib.laser_segment_ffn_forward.restype = i32
    lib.laser_segment_ffn_forward_variant.argtypes = lib.laser_segment_ffn_forward.argtypes + [i32]
    lib.laser_segment_ffn_forward_variant.restype = i32
    lib.laser_ffn_gsta_forward.argtypes = [vp, vp, vp, vp, vp, ip, vp, fp, vp, fp, fp, fp, i32, i32, i32, i32, i32, i32,
                                           i32, f32, i32, vp, vp, vp]
    lib.laser_ffn_gsta_forward.restype = i32
    lib.laser_ffn_gsta_forward_multires.argtypes = lib.laser_ffn_gsta_forward.argtypes[:-1] + [i32, vp, vp, vp]
    lib.laser_ffn_gsta_forward_multires.restype = i32
    lib.laser_project_q_forward.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp]
    lib.laser_project_q_forward_variant.argtypes = lib.laser_project_q_forward.argtypes + [i32]
    lib.laser_project_kv_forward.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.laser_project_kv_forward_variant.argtypes = lib.laser_project_kv_forward.argtypes + [i32]
    for name in ("laser_project_q_forward", "laser_project_q_forward_variant", "laser_project_kv_forward",
                 "laser_project_kv_forward_variant"):
        getattr(lib, name).restype = i32
    lib.laser_fold_query_weights.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp]
    lib.laser_project_heads_forward.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, i32]
    lib.laser_sta_folded_forward.argtypes = [vp, vp, vp, vp, ip, i32, i32, i32, i32, i32, i32, f32, i32, i32,
                                             vp, vp, vp, ip, vp]
    for name in ("laser_fold_query_weights", "laser_project_heads_forward", "laser_sta_folded_forward"):
        getattr(lib, name).restype = i32
    lib.laser_sta_forward_ragged.argtypes = [vp, vp, vp, ip, ip, i32, i32, i32, i32, i32, i32, i32, f32, i32, vp, ip, vp]
    lib.laser_gsta_forward_ragged.argtypes = [vp, vp, vp, vp, vp, ip, ip, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.laser_forward_ragged.argtypes = [vp, vp, vp, vp, vp, vp, vp, ip, ip, i32, i32, i32, i32, i32, i32, i32, f32,
                                         i32, i32, vp, ip, vp, vp]
    lib.laser_multires_forward_ragged.argtypes = [vp, ip, ip, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.laser_segment_ffn_forward_ragged.argtypes = [vp, ip, ip, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32,
                                                     i32, f32, i32, vp, vp]
    for name in ("laser_sta_forward_ragged", "laser_gsta_forward_ragged", "laser_forward_ragged",
                 "laser_multires_forward_ragged", "laser_segment_ffn_forward_ragged"):
        getattr(lib, name).restype = i32
    lib.laser_sta_backward_work_bytes.argtypes = [i32, i32, i32, i32, i32]
    lib.laser_sta_backward_work_bytes.restype = ctypes.c_size_t
    lib.laser_sta_backward.argtypes = [vp, vp, vp, ip, vp, i32, i32, i32, i32, i32, i32, f32, i32, vp, vp, vp, vp,
                                       ctypes.c_size_t, vp]
    lib.laser_sta_backward.restype = i32
    lib.laser_sta_backward_bf16.argtypes = [vp, vp, vp, ip, vp, i32, i32, i32, i32, i32, i32, f32, vp, vp, vp, vp,
                                            ctypes.c_size_t, vp]
    lib.laser_sta_backward_bf16.restype = i32
    lib.laser_sta_backward_static.argtypes = [vp, vp, vp, ip, vp, i32, i32, i32, i32, i32, i32, f32, i32, vp, vp, vp, vp]
    lib.laser_sta_backward_static.restype = i32
    lib.laser_gsta_backward_work_bytes.argtypes = [i32, i32, i32, i32]
    lib.laser_gsta_backward_work_bytes.restype = ctypes.c_size_t
    lib.laser_gsta_backward.argtypes = [vp, vp, vp, vp, vp, ip, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp,
                                        vp, ctypes.c_size_t, vp]
    lib.laser_gsta_backward.restype = i32
    lib.laser_sta_kernel_name.argtypes = [i32, i32, i32, i32, i32]
    lib.laser_sta_kernel_name.restype = ctypes.c_char_p
    lib.laser_gsta_kernel_name.argtypes = [i32, i32, i32, i32]
    lib.laser_gsta_kernel_name.restype = ctypes.c_char_p
    lib.laser_gsta_kernel_name_layers.argtypes = [i32, i32, i32, i32, i32]
    lib.laser_gsta_kernel_name_layers.restype = ctypes.c_char_p
    lib.laser_status_string.argtypes = [i32]
    lib.laser_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load_library().laser_status_string(int(code)).decode()


def laser_version() -> int:
    return int(load_library().laser_version())


def laser_sta_kernel_name(C: int, d_q: int, d: int, w: int, dt: int) -> str:
    return load_library().laser_sta_kernel_name(C, d_q, d, w, dt).decode()


def laser_gsta_kernel_name(C: int, S: int, d: int, dt: int, M: int = 1) -> str:
    return load_library().laser_gsta_kernel_name_layers(C, S, d, M, dt).decode()


# ----------------------------------------------------------------------------- tensor marshalling
def _torch():
    import torch
    return torch


def _dt(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return LASER_F32
    if t.dtype == torch.bfloat16:
        return LASER_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t, name: str, dtype=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _check(code: int, where: str) -> None:
    if code != 0:
        raise LaserError(code, where)


def laser_sta_forward(q, k, v, lens, w: int, gamma: float, seg_out=None, seg_cnt=None, stream=None,
                      variant: int = STA_AUTO, want_cnt: bool = True, heads: int = 1, softmax: bool = False):
    """q [U,C,d_q], k [U,L,d_q], v [U,L,d], lens int32 [U] or None -> (H' [U,C,S,d], cnt [U,S] or None).
    heads > 1 calls laser_sta_forward_heads (head h owns the h-th run of columns of q, k, v and H'); softmax=True
    calls laser_sta_forward_softmax (softmax over a segment's valid items instead of sigmoid gates)."""
    torch = _torch()
    U, C, d_q = q.shape
    L, d = v.shape[1], v.shape[2]
    if k.shape != (U, L, d_q) or v.shape[0] != U:
        raise ValueError("q, k, v shapes disagree")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise TypeError("q, k, v must share a dtype")
    S = -(-L // w)
    if seg_out is None:
        seg_out = torch.empty((U, C, S, d), dtype=q.dtype, device=q.device)
    elif tuple(seg_out.shape) != (U, C, S, d) or seg_out.dtype != q.dtype:
        raise ValueError("seg_out must be [U,C,S,d] in the input dtype")
    if seg_cnt is None and want_cnt:
        seg_cnt = torch.empty((U, S), dtype=torch.int32, device=q.device)
    if lens is not None and tuple(lens.shape) != (U,):
        raise ValueError("lens must be [U]")
    if softmax or int(heads) != 1:
        fn = load_library().laser_sta_forward_softmax if softmax else load_library().laser_sta_forward_heads
        code = fn(
            _ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(lens, "lens", torch.int32), U, C, L, d_q, d, int(w),
            float(gamma), int(heads), _dt(q), _ptr(seg_out, "seg_out"), _ptr(seg_cnt, "seg_cnt", torch.int32),
            _stream(stream), int(variant))
        _check(code, "laser_sta_forward_softmax" if softmax else "laser_sta_forward_heads")
        return seg_out, seg_cnt
    code = load_library().laser_sta_forward_variant(
        _ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(lens, "lens", torch.int32), U, C, L, d_q, d, int(w),
        float(gamma), _dt(q), _ptr(seg_out, "seg_out"), _ptr(seg_cnt, "seg_cnt", torch.int32), _stream(stream),
        int(variant))
    _check(code, "laser_sta_forward")
    return seg_out, seg_cnt


def laser_gsta_forward(seg, t0, wq, wk, wv, lens, L: int, w: int, z_out=None, stream=None,
                       variant: int = GSTA_AUTO):
    """seg [U,C,S,d], t0 [U,C,d], w* [M,d,d], lens int32 [U] or None -> z [U,C,d] fp32."""
    torch = _torch()
    U, C, S, d = seg.shape
    M = wq.shape[0]
    if S != -(-L // w):
        raise ValueError("seg.shape[2] must be ceil(L / w)")
    if tuple(t0.shape) != (U, C, d) or any(tuple(x.shape) != (M, d, d) for x in (wq, wk, wv)):
        raise ValueError("t0 / weight shapes disagree with seg")
    if any(x.dtype != seg.dtype for x in (t0, wq, wk, wv)):
        raise TypeError("seg, t0 and the weights must share a dtype")
    if z_out is None:
        z_out = torch.empty((U, C, d), dtype=torch.float32, device=seg.device)
    code = load_library().laser_gsta_forward_variant(
        _ptr(seg, "seg"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"), _ptr(wv, "wv"),
        _ptr(lens, "lens", torch.int32), U, C, int(L), d, int(w), M, _dt(seg), _ptr(z_out, "z_out", torch.float32),
        _stream(stream), int(variant))
    _check(code, "laser_gsta_forward")
    return z_out


def laser_segment_ffn_forward(seg, lens, w1, b1, w2, b2, ln_g, ln_b, L: int, w: int, eps: float = 1e-5, seg_out=None,
                              stream=None, variant: int = FFN_AUTO):
    """seg [U,C,S,d] -> LN(FFN(seg) + seg) [U,C,S,d] (same dtype); w1 [d,d_ff], w2 [d_ff,d] in seg's dtype, the rest fp32.
    seg_out may be seg itself."""
    torch = _torch()
    U, C, S, d = seg.shape
    d_ff = w1.shape[1]
    if S != -(-L // w):
        raise ValueError("seg.shape[2] must be ceil(L / w)")
    if tuple(w1.shape) != (d, d_ff) or tuple(w2.shape) != (d_ff, d):
        raise ValueError("w1 must be [d, d_ff] and w2 [d_ff, d]")
    if tuple(b1.shape) != (d_ff,) or any(tuple(x.shape) != (d,) for x in (b2, ln_g, ln_b)):
        raise ValueError("b1 must be [d_ff]; b2, ln_g, ln_b must be [d]")
    if w1.dtype != seg.dtype or w2.dtype != seg.dtype:
        raise TypeError("w1 and w2 must have the dtype of seg")
    if seg_out is None:
        seg_out = torch.empty_like(seg)
    code = load_library().laser_segment_ffn_forward_variant(
        _ptr(seg, "seg"), _ptr(lens, "lens", torch.int32), _ptr(w1, "w1"), _ptr(b1, "b1", torch.float32),
        _ptr(w2, "w2"), _ptr(b2, "b2", torch.float32), _ptr(ln_g, "ln_g", torch.float32),
        _ptr(ln_b, "ln_b", torch.float32), U, C, int(L), d, d_ff, int(w), float(eps), _dt(seg),
        _ptr(seg_out, "seg_out", seg.dtype), _stream(stream), int(variant))
    _check(code, "laser_segment_ffn_forward")
    return seg_out


def laser_project_q_forward(t, w_q, q_out=None, stream=None, variant: int = PROJECT_AUTO):
    """Q = t W_q: t [U,C,d_in], w_q [d_in,d_q] (same dtype) -> [U,C,d_q]."""
    torch = _torch()
    U, C, d_in = t.shape
    if w_q.dim() != 2 or w_q.shape[0] != d_in:
        raise ValueError("w_q must be [d_in, d_q]")
    if w_q.dtype != t.dtype:
        raise TypeError("w_q must have the dtype of t")
    d_q = w_q.shape[1]
    if q_out is None:
        q_out = torch.empty((U, C, d_q), dtype=t.dtype, device=t.device)
    elif tuple(q_out.shape) != (U, C, d_q):
        raise ValueError("q_out must be [U, C, d_q]")
    code = load_library().laser_project_q_forward_variant(
        _ptr(t, "t"), _ptr(w_q, "w_q"), U, C, d_in, d_q, _dt(t), _ptr(q_out, "q_out", t.dtype), _stream(stream),
        int(variant))
    _check(code, "laser_project_q_forward")
    return q_out


def laser_project_kv_forward(h, w_k, w_v, k_out=None, v_out=None, stream=None, variant: int = PROJECT_AUTO):
    """K = H W_k, V = H W_v from one pass over h [U,L,d_in]: w_k [d_in,d_q], w_v [d_in,d] -> ([U,L,d_q], [U,L,d])."""
    torch = _torch()
    U, L, d_in = h.shape
    if w_k.dim() != 2 or w_v.dim() != 2 or w_k.shape[0] != d_in or w_v.shape[0] != d_in:
        raise ValueError("w_k must be [d_in, d_q] and w_v [d_in, d]")
    if w_k.dtype != h.dtype or w_v.dtype != h.dtype:
        raise TypeError("w_k and w_v must have the dtype of h")
    d_q, d = w_k.shape[1], w_v.shape[1]
    if k_out is None:
        k_out = torch.empty((U, L, d_q), dtype=h.dtype, device=h.device)
    elif tuple(k_out.shape) != (U, L, d_q):
        raise ValueError("k_out must be [U, L, d_q]")
    if v_out is None:
        v_out = torch.empty((U, L, d), dtype=h.dtype, device=h.device)
    elif tuple(v_out.shape) != (U, L, d):
        raise ValueError("v_out must be [U, L, d]")
    code = load_library().laser_project_kv_forward_variant(
        _ptr(h, "h"), _ptr(w_k, "w_k"), _ptr(w_v, "w_v"), U, L, d_in, d_q, d, _dt(h), _ptr(k_out, "k_out", h.dtype),
        _ptr(v_out, "v_out", h.dtype), _stream(stream), int(variant))
    _check(code, "laser_project_kv_forward")
    return k_out, v_out


def laser_forward_ragged(q, k, v, t0, wq, wk, wv, lens, cand_off, c_max: int, w: int, gamma: float, seg_out=None,
                         seg_cnt=None, z_out=None, stream=None, want_cnt: bool = True, stage: str = "both"):
    """Packed pairs: q [P,d_q], t0 [P,d] with cand_off int32 [U+1] (device) -> (H' [P,S,d], cnt [U,S], z [P,d] fp32).
    stage = "sta" runs STA only (t0 and the weights may be None, z is None), "gsta" runs GSTA only on seg_out."""
    torch = _torch()
    U, L = k.shape[0], k.shape[1]
    P = q.shape[0] if q is not None else seg_out.shape[0]
    d = v.shape[2]
    S = -(-L // w)
    if tuple(cand_off.shape) != (U + 1,):
        raise ValueError("cand_off must be [U + 1]")
    dev, tdt = k.device, k.dtype
    if seg_out is None:
        seg_out = torch.empty((P, S, d), dtype=tdt, device=dev)
    if seg_cnt is None and want_cnt and stage != "gsta":
        seg_cnt = torch.empty((U, S), dtype=torch.int32, device=dev)
    if z_out is None and stage != "sta":
        z_out = torch.empty((P, d), dtype=torch.float32, device=dev)
    lib = load_library()
    common = (_ptr(lens, "lens", torch.int32), _ptr(cand_off, "cand_off", torch.int32), U, int(c_max), P, L)
    if stage == "sta":
        code = lib.laser_sta_forward_ragged(_ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), *common, q.shape[1], d, int(w),
                                            float(gamma), _dt(k), _ptr(seg_out, "seg_out", tdt),
                                            _ptr(seg_cnt, "seg_cnt", torch.int32), _stream(stream))
    elif stage == "gsta":
        code = lib.laser_gsta_forward_ragged(_ptr(seg_out, "seg_out"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"),
                                             _ptr(wv, "wv"), *common, d, int(w), wq.shape[0], _dt(k),
                                             _ptr(z_out, "z_out", torch.float32), _stream(stream))
    else:
        code = lib.laser_forward_ragged(_ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(t0, "t0"), _ptr(wq, "wq"),
                                        _ptr(wk, "wk"), _ptr(wv, "wv"), *common, q.shape[1], d, int(w), float(gamma),
                                        wq.shape[0], _dt(k), _ptr(seg_out, "seg_out", tdt),
                                        _ptr(seg_cnt, "seg_cnt", torch.int32), _ptr(z_out, "z_out", torch.float32),
                                        _stream(stream))
    _check(code, "laser_forward_ragged")
    return seg_out, seg_cnt, z_out


def laser_sta_backward(q, k, v, lens, dseg, w: int, gamma: float, dq_out=None, dk_out=None, dv_out=None, work=None,
                       stream=None, grads_bf16: bool = False):
    """Gradients of STA: dseg = dL/dH' [U,C,S,d] (dtype of q) -> (dq [U,C,d_q], dk [U,L,d_q], dv [U,L,d]) in fp32;
    with grads_bf16 (bf16 inputs) dk and dv come back in bf16 (laser_sta_backward_bf16)."""
    torch = _torch()
    U, C, d_q = q.shape
    L, d = v.shape[1], v.shape[2]
    S = -(-L // w)
    if tuple(k.shape) != (U, L, d_q) or tuple(v.shape) != (U, L, d) or tuple(dseg.shape) != (U, C, S, d):
        raise ValueError("q, k, v, dseg shapes disagree")
    if any(x.dtype != q.dtype for x in (k, v, dseg)):
        raise TypeError("q, k, v and dseg must share a dtype")
    f32 = dict(dtype=torch.float32, device=q.device)
    dq_out = torch.empty((U, C, d_q), **f32) if dq_out is None else dq_out
    gkw = dict(dtype=torch.bfloat16, device=q.device) if grads_bf16 else f32
    dk_out = torch.empty((U, L, d_q), **gkw) if dk_out is None else dk_out
    dv_out = torch.empty((U, L, d), **gkw) if dv_out is None else dv_out
    lib = load_library()
    need = lib.laser_sta_backward_work_bytes(U, C, L, d_q, int(w))
    if work is None:
        work = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    if grads_bf16:
        if q.dtype != torch.bfloat16:
            raise TypeError("grads_bf16 needs bf16 inputs")
        code = lib.laser_sta_backward_bf16(_ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(lens, "lens", torch.int32),
                                           _ptr(dseg, "dseg"), U, C, L, d_q, d, int(w), float(gamma),
                                           _ptr(dq_out, "dq_out", torch.float32),
                                           _ptr(dk_out, "dk_out", torch.bfloat16),
                                           _ptr(dv_out, "dv_out", torch.bfloat16), _ptr(work, "work"),
                                           work.numel() * work.element_size(), _stream(stream))
        _check(code, "laser_sta_backward_bf16")
        return dq_out, dk_out, dv_out
    code = lib.laser_sta_backward(_ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(lens, "lens", torch.int32),
                                  _ptr(dseg, "dseg"), U, C, L, d_q, d, int(w), float(gamma), _dt(q),
                                  _ptr(dq_out, "dq_out", torch.float32), _ptr(dk_out, "dk_out", torch.float32),
                                  _ptr(dv_out, "dv_out", torch.float32), _ptr(work, "work"),
                                  work.numel() * work.element_size(), _stream(stream))
    _check(code, "laser_sta_backward")
    return dq_out, dk_out, dv_out


STATIC_SCRATCH_BYTES = 8 << 20     # LASER_STATIC_SCRATCH_BYTES of include/laser.h


def laser_sta_backward_static(q, k, v, lens, dseg, w: int, gamma: float, dq_out, dk_out, dv_out, stream=None):
    """laser_sta_backward with the library's own fixed scratch: the call allocates nothing, so the three outputs
    [U,C,d_q], [U,L,d_q], [U,L,d] (fp32) are the caller's."""
    torch = _torch()
    U, C, d_q = q.shape
    L, d = v.shape[1], v.shape[2]
    S = -(-L // w)
    if tuple(k.shape) != (U, L, d_q) or tuple(v.shape) != (U, L, d) or tuple(dseg.shape) != (U, C, S, d):
        raise ValueError("q, k, v, dseg shapes disagree")
    if tuple(dq_out.shape) != (U, C, d_q) or tuple(dk_out.shape) != (U, L, d_q) or tuple(dv_out.shape) != (U, L, d):
        raise ValueError("output shapes disagree with the inputs")
    if any(x.dtype != q.dtype for x in (k, v, dseg)):
        raise TypeError("q, k, v and dseg must share a dtype")
    code = load_library().laser_sta_backward_static(
        _ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(lens, "lens", torch.int32), _ptr(dseg, "dseg"), U, C, L, d_q, d,
        int(w), float(gamma), _dt(q), _ptr(dq_out, "dq_out", torch.float32), _ptr(dk_out, "dk_out", torch.float32),
        _ptr(dv_out, "dv_out", torch.float32), _stream(stream))
    _check(code, "laser_sta_backward_static")
    return dq_out, dk_out, dv_out


def laser_gsta_backward(seg, t0, wq, wk, wv, lens, dz, L: int, w: int, work=None, stream=None):
    """Gradients of GSTA from dz [U,C,d] fp32: (dseg [U,C,S,d] in seg's dtype, dt0 [U,C,d], dwq, dwk, dwv [M,d,d] fp32)."""
    torch = _torch()
    U, C, S, d = seg.shape
    M = wq.shape[0]
    if S != -(-L // w) or tuple(dz.shape) != (U, C, d) or tuple(t0.shape) != (U, C, d):
        raise ValueError("seg, t0, dz shapes disagree")
    f32 = dict(dtype=torch.float32, device=seg.device)
    dseg = torch.empty_like(seg)
    dt0 = torch.empty((U, C, d), **f32)
    dwq, dwk, dwv = (torch.empty((M, d, d), **f32) for _ in range(3))
    lib = load_library()
    need = lib.laser_gsta_backward_work_bytes(U, C, d, M)
    if work is None:
        work = torch.empty(max(need, 16), dtype=torch.uint8, device=seg.device)
    code = lib.laser_gsta_backward(_ptr(seg, "seg"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"), _ptr(wv, "wv"),
                                   _ptr(lens, "lens", torch.int32), _ptr(dz, "dz", torch.float32), U, C, int(L), d,
                                   int(w), M, _dt(seg), _ptr(dseg, "dseg"), _ptr(dt0, "dt0"), _ptr(dwq, "dwq"),
                                   _ptr(dwk, "dwk"), _ptr(dwv, "dwv"), _ptr(work, "work"),
                                   work.numel() * work.element_size(), _stream(stream))
    _check(code, "laser_gsta_backward")
    return dseg, dt0, dwq, dwk, dwv


def laser_multires_forward_ragged(seg, lens, cand_off, c_max: int, L: int, w: int, r: int, stream=None):
    """Packed pairs: seg [P,S,d] with cand_off [U+1] -> (pool [P,d], recent [P,r,d] or None)."""
    torch = _torch()
    P, S, d = seg.shape
    U = cand_off.shape[0] - 1
    pool = torch.empty((P, d), dtype=seg.dtype, device=seg.device)
    recent = torch.empty((P, r, d), dtype=seg.dtype, device=seg.device) if r > 0 else None
    code = load_library().laser_multires_forward_ragged(
        _ptr(seg, "seg"), _ptr(lens, "lens", torch.int32), _ptr(cand_off, "cand_off", torch.int32), U, int(c_max), P,
        int(L), d, int(w), int(r), _dt(seg), _ptr(pool, "pool"), _ptr(recent, "recent"), _stream(stream))
    _check(code, "laser_multires_forward_ragged")
    return pool, recent


def laser_segment_ffn_forward_ragged(seg, lens, cand_off, c_max: int, w1, b1, w2, b2, ln_g, ln_b, L: int, w: int,
                                     eps: float = 1e-5, seg_out=None, stream=None):
    """Packed pairs: seg [P,S,d] with cand_off [U+1] -> LN(FFN(seg) + seg) [P,S,d]; seg_out may be seg."""
    torch = _torch()
    P, S, d = seg.shape
    U = cand_off.shape[0] - 1
    if seg_out is None:
        seg_out = torch.empty_like(seg)
    code = load_library().laser_segment_ffn_forward_ragged(
        _ptr(seg, "seg"), _ptr(lens, "lens", torch.int32), _ptr(cand_off, "cand_off", torch.int32), _ptr(w1, "w1"),
        _ptr(b1, "b1", torch.float32), _ptr(w2, "w2"), _ptr(b2, "b2", torch.float32), _ptr(ln_g, "ln_g", torch.float32),
        _ptr(ln_b, "ln_b", torch.float32), U, int(c_max), P, int(L), d, w1.shape[1], int(w), float(eps), _dt(seg),
        _ptr(seg_out, "seg_out", seg.dtype), _stream(stream))
    _check(code, "laser_segment_ffn_forward_ragged")
    return seg_out


def laser_fold_query_weights(w_q, w_k, heads: int = 1, a_out=None, stream=None):
    """A = [W_q,h W_k,h^T for every head] : w_q, w_k [d_in, d_q] -> [d_in, heads * d_in] (same dtype)."""
    torch = _torch()
    d_in, d_q = w_q.shape
    if tuple(w_k.shape) != (d_in, d_q) or w_k.dtype != w_q.dtype:
        raise ValueError("w_q and w_k must both be [d_in, d_q] in one dtype")
    if a_out is None:
        a_out = torch.empty((d_in, heads * d_in), dtype=w_q.dtype, device=w_q.device)
    code = load_library().laser_fold_query_weights(_ptr(w_q, "w_q"), _ptr(w_k, "w_k"), d_in, d_q, int(heads), _dt(w_q),
                                                   _ptr(a_out, "a_out", w_q.dtype), _stream(stream))
    _check(code, "laser_fold_query_weights")
    return a_out


def laser_project_heads_forward(x, w_v, y=None, stream=None, variant: int = PROJECT_AUTO):
    """x [P, heads, S, d_in], w_v [d_in, d] -> y [P, S, d]: head h's columns of w_v applied to x[:, h]."""
    torch = _torch()
    P, heads, S, d_in = x.shape
    if w_v.dim() != 2 or w_v.shape[0] != d_in or w_v.dtype != x.dtype:
        raise ValueError("w_v must be [d_in, d] in the dtype of x")
    d = w_v.shape[1]
    if y is None:
        y = torch.empty((P, S, d), dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != (P, S, d):
        raise ValueError("y must be [P, S, d]")
    code = load_library().laser_project_heads_forward(_ptr(x, "x"), _ptr(w_v, "w_v"), P, S, d_in, d, heads, _dt(x),
                                                      _ptr(y, "y", x.dtype), _stream(stream), int(variant))
    _check(code, "laser_project_heads_forward")
    return y


def laser_sta_folded_forward(t, h, a_fold, w_v, lens, w: int, gamma: float, heads: int = 1, qf_work=None, g_work=None,
                             seg_out=None, seg_cnt=None, stream=None, want_cnt: bool = True):
    """Raw embeddings t [U,C,d_in], h [U,L,d_in] -> (H' [U,C,S,d], cnt [U,S] or None) without forming K and V.
    a_fold comes from laser_fold_query_weights. Pass your own work buffers (qf_work [U,C*heads,d_in],
    g_work [U,C*heads,S,d_in]) to reuse them across calls; otherwise they are allocated here, by torch."""
    torch = _torch()
    U, C, d_in = t.shape
    L = h.shape[1]
    d = w_v.shape[1]
    S = -(-L // w)
    if tuple(h.shape) != (U, L, d_in) or tuple(a_fold.shape) != (d_in, heads * d_in) or w_v.shape[0] != d_in:
        raise ValueError("t, h, a_fold, w_v shapes disagree")
    if any(x.dtype != t.dtype for x in (h, a_fold, w_v)):
        raise TypeError("t, h, a_fold and w_v must share a dtype")
    if qf_work is None:
        qf_work = torch.empty((U, C * heads, d_in), dtype=t.dtype, device=t.device)
    if g_work is None:
        g_work = torch.empty((U, C * heads, S, d_in), dtype=t.dtype, device=t.device)
    if seg_out is None:
        seg_out = torch.empty((U, C, S, d), dtype=t.dtype, device=t.device)
    if seg_cnt is None and want_cnt:
        seg_cnt = torch.empty((U, S), dtype=torch.int32, device=t.device)
    if tuple(qf_work.shape) != (U, C * heads, d_in) or tuple(g_work.shape) != (U, C * heads, S, d_in) or \
            tuple(seg_out.shape) != (U, C, S, d):
        raise ValueError("work / output buffer shapes disagree")
    code = load_library().laser_sta_folded_forward(
        _ptr(t, "t"), _ptr(h, "h"), _ptr(a_fold, "a_fold"), _ptr(w_v, "w_v"), _ptr(lens, "lens", torch.int32), U, C, L,
        d_in, d, int(w), float(gamma), int(heads), _dt(t), _ptr(qf_work, "qf_work", t.dtype),
        _ptr(g_work, "g_work", t.dtype), _ptr(seg_out, "seg_out", t.dtype), _ptr(seg_cnt, "seg_cnt", torch.int32),
        _stream(stream))
    _check(code, "laser_sta_folded_forward")
    return seg_out, seg_cnt


def laser_forward_multires(q, k, v, t0, wq, wk, wv, lens, w: int, gamma: float, r: int, seg_out=None, seg_cnt=None,
                           z_out=None, pool_out=None, recent_out=None, stream=None):
    """The whole path with all three views. Returns (H', cnt, z fp32, pool [U,C,d], recent [U,C,r,d] or None)."""
    torch = _torch()
    U, C, d_q = q.shape
    L, d = v.shape[1], v.shape[2]
    M = wq.shape[0]
    S = -(-L // w)
    if any(x.dtype != q.dtype for x in (k, v, t0, wq, wk, wv)):
        raise TypeError("all inputs must share a dtype")
    if seg_out is None:
        seg_out = torch.empty((U, C, S, d), dtype=q.dtype, device=q.device)
    if seg_cnt is None:
        seg_cnt = torch.empty((U, S), dtype=torch.int32, device=q.device)
    if z_out is None:
        z_out = torch.empty((U, C, d), dtype=torch.float32, device=q.device)
    if pool_out is None:
        pool_out = torch.empty((U, C, d), dtype=q.dtype, device=q.device)
    if recent_out is None and r > 0:
        recent_out = torch.empty((U, C, r, d), dtype=q.dtype, device=q.device)
    for name, x in (("seg_out", seg_out), ("pool_out", pool_out), ("recent_out", recent_out)):
        if x is not None and x.dtype != q.dtype:
            raise TypeError(f"{name} must have the dtype of the inputs")
    code = load_library().laser_forward_multires(
        _ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"), _ptr(wv, "wv"),
        _ptr(lens, "lens", torch.int32), U, C, L, d_q, d, int(w), float(gamma), M, _dt(q), _ptr(seg_out, "seg_out"),
        _ptr(seg_cnt, "seg_cnt", torch.int32), _ptr(z_out, "z_out", torch.float32), int(r),
        _ptr(pool_out, "pool_out"), _ptr(recent_out, "recent_out"), _stream(stream))
    _check(code, "laser_forward_multires")
    return seg_out, seg_cnt, z_out, pool_out, recent_out


def laser_gsta_forward_multires(seg, t0, wq, wk, wv, lens, L: int, w: int, r: int, z_out=None, pool_out=None,
                                recent_out=None, stream=None):
    """GSTA and the two other views from a stored H' [U,C,S,d]. Returns (z fp32 [U,C,d], pool [U,C,d], recent
    [U,C,r,d] or None)."""
    torch = _torch()
    U, C, S, d = seg.shape
    M = wq.shape[0]
    if S != -(-L // w):
        raise ValueError("seg.shape[2] must be ceil(L / w)")
    if any(x.dtype != seg.dtype for x in (t0, wq, wk, wv)):
        raise TypeError("all inputs must share a dtype")
    if z_out is None:
        z_out = torch.empty((U, C, d), dtype=torch.float32, device=seg.device)
    if pool_out is None:
        pool_out = torch.empty((U, C, d), dtype=seg.dtype, device=seg.device)
    if recent_out is None and r > 0:
        recent_out = torch.empty((U, C, r, d), dtype=seg.dtype, device=seg.device)
    for name, x in (("pool_out", pool_out), ("recent_out", recent_out)):
        if x is not None and x.dtype != seg.dtype:
            raise TypeError(f"{name} must have the dtype of seg")
    code = load_library().laser_gsta_forward_multires(
        _ptr(seg, "seg"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"), _ptr(wv, "wv"),
        _ptr(lens, "lens", torch.int32), U, C, int(L), d, int(w), M, _dt(seg), _ptr(z_out, "z_out", torch.float32),
        int(r), _ptr(pool_out, "pool_out"), _ptr(recent_out, "recent_out"), _stream(stream))
    _check(code, "laser_gsta_forward_multires")
    return z_out, pool_out, recent_out


def laser_ffn_gsta_forward(seg, t0, wq, wk, wv, lens, w1, b1, w2, b2, ln_g, ln_b, L: int, w: int, eps: float = 1e-5,
                           seg_out=None, z_out=None, stream=None, want_seg: bool = True, r: Optional[int] = None,
                           pool_out=None, recent_out=None):
    """seg [U,C,S,d] -> (s = LN(FFN(seg) + seg) [U,C,S,d] or None, z = GSTA(t0; s) [U,C,d] fp32). want_seg=False
    passes a null seg_out (s is not written); seg_out may be seg itself. With r (an int >= 0) the call is
    laser_ffn_gsta_forward_multires and returns (s or None, z, pool [U,C,d], recent [U,C,r,d] or None)."""
    torch = _torch()
    U, C, S, d = seg.shape
    d_ff = w1.shape[1]
    M = wq.shape[0]
    if S != -(-L // w):
        raise ValueError("seg.shape[2] must be ceil(L / w)")
    if tuple(w1.shape) != (d, d_ff) or tuple(w2.shape) != (d_ff, d):
        raise ValueError("w1 must be [d, d_ff] and w2 [d_ff, d]")
    if tuple(b1.shape) != (d_ff,) or any(tuple(x.shape) != (d,) for x in (b2, ln_g, ln_b)):
        raise ValueError("b1 must be [d_ff]; b2, ln_g, ln_b must be [d]")
    if tuple(t0.shape) != (U, C, d) or any(tuple(x.shape) != (M, d, d) for x in (wq, wk, wv)):
        raise ValueError("t0 / weight shapes disagree with seg")
    if any(x.dtype != seg.dtype for x in (t0, wq, wk, wv, w1, w2)):
        raise TypeError("seg, t0 and the weight matrices must share a dtype")
    if seg_out is None and want_seg:
        seg_out = torch.empty_like(seg)
    if z_out is None:
        z_out = torch.empty((U, C, d), dtype=torch.float32, device=seg.device)
    if r is not None:
        if pool_out is None:
            pool_out = torch.empty((U, C, d), dtype=seg.dtype, device=seg.device)
        if recent_out is None and r > 0:
            recent_out = torch.empty((U, C, r, d), dtype=seg.dtype, device=seg.device)
        code = load_library().laser_ffn_gsta_forward_multires(
            _ptr(seg, "seg"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"), _ptr(wv, "wv"),
            _ptr(lens, "lens", torch.int32), _ptr(w1, "w1"), _ptr(b1, "b1", torch.float32), _ptr(w2, "w2"),
            _ptr(b2, "b2", torch.float32), _ptr(ln_g, "ln_g", torch.float32), _ptr(ln_b, "ln_b", torch.float32), U, C,
            int(L), d, d_ff, int(w), M, float(eps), _dt(seg), _ptr(seg_out, "seg_out", seg.dtype),
            _ptr(z_out, "z_out", torch.float32), int(r), _ptr(pool_out, "pool_out", seg.dtype),
            _ptr(recent_out, "recent_out", seg.dtype), _stream(stream))
        _check(code, "laser_ffn_gsta_forward_multires")
        return seg_out, z_out, pool_out, recent_out
    code = load_library().laser_ffn_gsta_forward(
        _ptr(seg, "seg"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"), _ptr(wv, "wv"),
        _ptr(lens, "lens", torch.int32), _ptr(w1, "w1"), _ptr(b1, "b1", torch.float32), _ptr(w2, "w2"),
        _ptr(b2, "b2", torch.float32), _ptr(ln_g, "ln_g", torch.float32), _ptr(ln_b, "ln_b", torch.float32), U, C,
        int(L), d, d_ff, int(w), M, float(eps), _dt(seg), _ptr(seg_out, "seg_out", seg.dtype),
        _ptr(z_out, "z_out", torch.float32), _stream(stream))
    _check(code, "laser_ffn_gsta_forward")
    return seg_out, z_out


def laser_multires_forward(seg, lens, L: int, w: int, r: int, pool_out=None, recent_out=None, stream=None,
                           want_pool: bool = True):
    """seg [U,C,S,d], lens int32 [U] or None -> (pool [U,C,d] or None, recent [U,C,r,d] or None), dtype of seg."""
    torch = _torch()
    U, C, S, d = seg.shape
    if S != -(-L // w):
        raise ValueError("seg.shape[2] must be ceil(L / w)")
    if pool_out is None and want_pool:
        pool_out = torch.empty((U, C, d), dtype=seg.dtype, device=seg.device)
    if recent_out is None and r > 0:
        recent_out = torch.empty((U, C, r, d), dtype=seg.dtype, device=seg.device)
    for name, x in (("pool_out", pool_out), ("recent_out", recent_out)):
        if x is not None and x.dtype != seg.dtype:
            raise TypeError(f"{name} must have the dtype of seg")
    code = load_library().laser_multires_forward(
        _ptr(seg, "seg"), _ptr(lens, "lens", torch.int32), U, C, int(L), d, int(w), int(r), _dt(seg),
        _ptr(pool_out, "pool_out"), _ptr(recent_out, "recent_out"), _stream(stream))
    _check(code, "laser_multires_forward")
    return pool_out, recent_out


def laser_forward_fused(q, k, v, t0, wq, wk, wv, lens, w: int, gamma: float, seg_cnt=None, z_out=None, work=None,
                        stream=None, want_cnt: bool = True, use_work: bool = True):
    """The whole path with one GSTA layer and H' never stored. Returns (cnt [U,S] or None, z [U,C,d] fp32).
    work: device scratch for the partial results of the runs of a history (allocated here when None and use_work);
    use_work=False passes NULL, i.e. one run per user."""
    torch = _torch()
    U, C, d_q = q.shape
    L, d = v.shape[1], v.shape[2]
    S = -(-L // w)
    if tuple(wq.shape[-2:]) != (d, d) or wq.numel() != d * d:
        raise ValueError("one layer: wq, wk, wv must hold d x d elements")
    if seg_cnt is None and want_cnt:
        seg_cnt = torch.empty((U, S), dtype=torch.int32, device=q.device)
    if z_out is None:
        z_out = torch.empty((U, C, d), dtype=torch.float32, device=q.device)
    if any(x.dtype != q.dtype for x in (k, v, t0, wq, wk, wv)):
        raise TypeError("all inputs must share a dtype")
    lib = load_library()
    if work is None and use_work:
        need = lib.laser_forward_fused_work_bytes(U, C, L, d_q, d, int(w), _dt(q))
        if need:
            work = torch.empty(need, dtype=torch.uint8, device=q.device)
    code = lib.laser_forward_fused(
        _ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"), _ptr(wv, "wv"),
        _ptr(lens, "lens", torch.int32), U, C, L, d_q, d, int(w), float(gamma), _dt(q),
        _ptr(seg_cnt, "seg_cnt", torch.int32), _ptr(z_out, "z_out", torch.float32), _ptr(work, "work"),
        0 if work is None else work.numel() * work.element_size(), _stream(stream))
    _check(code, "laser_forward_fused")
    return seg_cnt, z_out


def laser_forward(q, k, v, t0, wq, wk, wv, lens, w: int, gamma: float, seg_out=None, seg_cnt=None, z_out=None,
                  stream=None, want_cnt: bool = True, want_seg: bool = True):
    """The whole path. Returns (H' [U,C,S,d], cnt [U,S] or None, z [U,C,d] fp32); with want_seg=False seg_out is passed
    as NULL (H' is never stored: the fused kernels, one layer only) and None comes back in its place."""
    torch = _torch()
    U, C, d_q = q.shape
    L, d = v.shape[1], v.shape[2]
    M = wq.shape[0]
    S = -(-L // w)
    if seg_out is None and want_seg:
        seg_out = torch.empty((U, C, S, d), dtype=q.dtype, device=q.device)
    if seg_cnt is None and want_cnt:
        seg_cnt = torch.empty((U, S), dtype=torch.int32, device=q.device)
    if z_out is None:
        z_out = torch.empty((U, C, d), dtype=torch.float32, device=q.device)
    if any(x.dtype != q.dtype for x in (k, v, t0, wq, wk, wv) + ((seg_out,) if seg_out is not None else ())):
        raise TypeError("all inputs and seg_out must share a dtype")
    code = load_library().laser_forward(
        _ptr(q, "q"), _ptr(k, "k"), _ptr(v, "v"), _ptr(t0, "t0"), _ptr(wq, "wq"), _ptr(wk, "wk"), _ptr(wv, "wv"),
        _ptr(lens, "lens", torch.int32), U, C, L, d_q, d, int(w), float(gamma), M, _dt(q), _ptr(seg_out, "seg_out"),
        _ptr(seg_cnt, "seg_cnt", torch.int32), _ptr(z_out, "z_out", torch.float32), _stream(stream))
    _check(code, "laser_forward")
    return seg_out, seg_cnt, z_out
