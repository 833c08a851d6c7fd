"""The C-ABI library without a GPU: it loads, exports every declared symbol, and rejects bad arguments
on the host before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2602_11562_amd as laser
from paper_2602_11562_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_11562_amd.build import build_library
        build_library()
    return laser.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "laser.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(laser_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert laser.laser_version() >= 100
    seen = {laser.status_string(c) for c in range(7)}
    assert len(seen) == 7 and "ok" in seen
    assert laser.status_string(99) == "unknown status"


A = 0x10000  # any 16-byte aligned non-NULL value: validation fails before it could be dereferenced


def _sta(lib, q=A, k=A, v=A, lens=None, U=2, C=3, L=64, dq=16, d=16, w=8, gamma=1.0, dt=1, out=A, cnt=None,
         variant=0):
    return lib.laser_sta_forward_variant(q, k, v, lens, U, C, L, dq, d, w, gamma, dt, out, cnt, None, variant)


def _gsta(lib, seg=A, t0=A, wq=A, wk=A, wv=A, lens=None, U=2, C=3, L=64, d=16, w=8, M=1, dt=1, z=A, variant=0):
    return lib.laser_gsta_forward_variant(seg, t0, wq, wk, wv, lens, U, C, L, d, w, M, dt, z, None, variant)


def test_sta_argument_validation(lib):
    NULL, SHAPE, DTYPE, UNSUP, ALIGN = 1, 2, 3, 4, 6
    assert _sta(lib, q=None) == NULL and _sta(lib, k=None) == NULL and _sta(lib, v=None) == NULL
    assert _sta(lib, out=None) == NULL
    assert _sta(lib, dt=2) == DTYPE and _sta(lib, dt=-1) == DTYPE
    for kw in ({"U": 0}, {"C": 0}, {"L": 0}, {"dq": 0}, {"d": 0}, {"w": 0}, {"w": -4}, {"U": -1},
               {"d": 12}, {"dq": 20}, {"d": 2048}, {"gamma": 0.0}, {"gamma": -1.0}, {"gamma": float("nan")},
               {"gamma": float("inf")},
               {"U": 1 << 20, "L": 1 << 20},                 # element count overflows int32
               {"U": 4096, "C": 4096, "L": 4096, "w": 1}):   # H' would overflow
        assert _sta(lib, **kw) == SHAPE, kw
    assert _sta(lib, q=A + 8) == ALIGN and _sta(lib, out=A + 2) == ALIGN and _sta(lib, lens=A + 2) == ALIGN
    assert _sta(lib, cnt=A + 1) == ALIGN
    assert _sta(lib, variant=7) == UNSUP and _sta(lib, variant=-1) == UNSUP
    # the plain entry point validates the same way
    assert lib.laser_sta_forward(None, A, A, None, 2, 3, 64, 16, 16, 8, 1.0, 1, A, None, None) == NULL


def test_gsta_argument_validation(lib):
    NULL, SHAPE, DTYPE, UNSUP, ALIGN = 1, 2, 3, 4, 6
    for name in ("seg", "t0", "wq", "wk", "wv", "z"):
        assert _gsta(lib, **{name: None}) == NULL
    assert _gsta(lib, dt=5) == DTYPE
    for kw in ({"M": 0}, {"M": 65}, {"d": 0}, {"d": 4}, {"w": 0}, {"L": 0}, {"U": 0}, {"C": -2},
               {"L": 8192, "w": 1}):                         # S > 4096
        assert _gsta(lib, **kw) == SHAPE, kw
    assert _gsta(lib, wk=A + 4) == ALIGN and _gsta(lib, lens=A + 1) == ALIGN
    assert _gsta(lib, variant=9) == UNSUP
    assert lib.laser_gsta_forward(A, A, A, A, None, None, 2, 3, 64, 16, 8, 1, 1, A, None) == NULL


def test_forward_validates_both_stages_before_launching(lib):
    f = lib.laser_forward
    ok_tail = (None, 2, 3, 64, 16, 16, 8, 1.0)
    assert f(A, A, A, None, A, A, A, *ok_tail, 1, 1, A, None, A, None) == 1      # t0 NULL
    # seg_out NULL asks for the fused path (H' never stored): one layer only, and validated like everything else
    assert f(A, A, A, A, A, A, A, *ok_tail, 2, 1, None, None, A, None) == 4      # seg_out NULL with two layers
    assert f(A, A, A, None, A, A, A, *ok_tail, 1, 1, None, None, A, None) == 1   # seg_out NULL, t0 NULL
    assert f(A, A, A, A, A, A, A, *ok_tail, 1, 1, None, None, None, None) == 1   # seg_out NULL, z_out NULL
    assert f(A, A, A, A, A, A, A + 8, *ok_tail, 1, 1, None, None, A, None) == 6  # seg_out NULL, wv misaligned
    assert f(A, A, A, A, A, A, A, *ok_tail, 0, 1, None, None, A, None) == 2      # seg_out NULL, M = 0
    assert f(A, A, A, A, A, A, A, *ok_tail, 1, 1, A, None, None, None) == 1      # z_out NULL
    assert f(A, A, A, A, A, A, A, *ok_tail, 0, 1, A, None, A, None) == 2         # M = 0
    assert f(A, A, A, A, A, A, A, *ok_tail, 1, 3, A, None, A, None) == 3         # dtype


def test_fused_forward_argument_validation(lib):
    NULL, SHAPE, DTYPE, ALIGN = 1, 2, 3, 6
    wb = lib.laser_forward_fused_work_bytes
    # 32 users x 256 candidates, L = 4096, w = 128, d = 128, bf16: two candidate tiles of four waves per user, four
    # runs of eight segments; per (tile of 32 candidates, run) 66 rows of 64 floats
    assert wb(32, 256, 4096, 128, 128, 128, 1) == 32 * 2 * 4 * 4 * 66 * 64 * 4
    assert wb(4096, 1, 4096, 64, 64, 256, 1) == 0          # enough users: whole histories, no scratch
    assert wb(1, 16, 1024, 64, 64, 64, 0) == 0             # fp32 storage: the generic kernel, one run per user
    assert wb(0, 16, 1024, 64, 64, 64, 1) == 0 and wb(1, 16, 1024, 64, 12, 64, 1) == 0   # invalid sizes
    f = lambda q=A, t0=A, wv=A, lens=None, U=2, C=3, L=64, dq=16, d=16, w=8, gamma=1.0, dt=1, cnt=None, z=A, work=None, \
        nbytes=0: lib.laser_forward_fused(q, A, A, t0, A, A, wv, lens, U, C, L, dq, d, w, ctypes.c_float(gamma), dt, cnt,
                                          z, work, ctypes.c_size_t(nbytes), None)
    for kw in ({"q": None}, {"t0": None}, {"wv": None}, {"z": None}):
        assert f(**kw) == NULL, kw
    assert f(dt=4) == DTYPE
    for kw in ({"U": 0}, {"C": 0}, {"w": 0}, {"d": 12}, {"gamma": 0.0}, {"L": 8192, "w": 1}):
        assert f(**kw) == SHAPE, kw
    assert f(wv=A + 8) == ALIGN and f(z=A + 4) == ALIGN and f(lens=A + 2) == ALIGN and f(cnt=A + 1) == ALIGN
    assert f(work=A + 8, nbytes=1 << 30) == ALIGN
    assert f(U=32, C=256, L=4096, dq=128, d=128, w=128, work=A, nbytes=1024) == SHAPE   # scratch too small


def test_kernel_names(lib):
    assert laser.laser_sta_kernel_name(16, 64, 64, 64, laser.LASER_F32) == "sta_generic"
    assert laser.laser_sta_kernel_name(0, 64, 64, 64, laser.LASER_F32) == "invalid"
    assert laser.laser_gsta_kernel_name(16, 16, 64, laser.LASER_F32) == "gsta_generic"
    assert laser.laser_gsta_kernel_name(128, 40, 128, laser.LASER_BF16, M=1) == "gsta_split_bf16"   # 10 row passes
    assert laser.laser_gsta_kernel_name(128, 40, 128, laser.LASER_BF16, M=2) == "gsta_tiled_bf16"   # several layers


def test_binding_refuses_host_tensors():
    import torch
    x = torch.zeros(1, 2, 8)
    with pytest.raises(ValueError):
        laser.laser_sta_forward(x, torch.zeros(1, 4, 8), torch.zeros(1, 4, 8), None, 2, 1.0,
                                seg_out=torch.zeros(1, 2, 2, 8), want_cnt=False)


def _multires(lib, seg=A, lens=None, U=2, C=3, L=64, d=16, w=8, r=2, dt=1, pool=A, recent=A):
    return lib.laser_multires_forward(seg, lens, U, C, L, d, w, r, dt, pool, recent, None)


def test_multires_argument_validation(lib):
    NULL, SHAPE, DTYPE, ALIGN = 1, 2, 3, 6
    assert _multires(lib, seg=None) == NULL
    assert _multires(lib, pool=None, recent=None, r=0) == NULL           # nothing wanted
    assert _multires(lib, dt=5) == DTYPE
    for kw in ({"U": 0}, {"C": -1}, {"L": 0}, {"d": 12}, {"w": 0}, {"r": -1}, {"r": 9},   # S = 8
               {"r": 0}, {"r": 2, "recent": None}):                                       # r and recent_out disagree
        assert _multires(lib, **kw) == SHAPE, kw
    assert _multires(lib, seg=A + 4) == ALIGN and _multires(lib, pool=A + 8) == ALIGN
    assert _multires(lib, recent=A + 2) == ALIGN and _multires(lib, lens=A + 2) == ALIGN


def test_gsta_with_views_argument_validation(lib):
    NULL, SHAPE, DTYPE, ALIGN = 1, 2, 3, 6
    f = lambda seg=A, t0=A, wv=A, lens=None, U=2, C=3, L=64, d=16, w=8, M=1, dt=1, z=A, r=2, pool=A, recent=A: \
        lib.laser_gsta_forward_multires(seg, t0, A, A, wv, lens, U, C, L, d, w, M, dt, z, r, pool, recent, None)
    for kw in ({"seg": None}, {"t0": None}, {"wv": None}, {"z": None}, {"pool": None, "recent": None, "r": 0}):
        assert f(**kw) == NULL, kw
    assert f(dt=5) == DTYPE
    for kw in ({"M": 0}, {"d": 4}, {"w": 0}, {"U": 0}, {"r": -1}, {"r": 9}, {"r": 0}, {"r": 2, "recent": None}):
        assert f(**kw) == SHAPE, kw
    assert f(pool=A + 8) == ALIGN and f(recent=A + 2) == ALIGN and f(lens=A + 2) == ALIGN and f(wv=A + 4) == ALIGN


def _ffn(lib, seg=A, lens=None, w1=A, b1=A, w2=A, b2=A, g=A, b=A, U=2, C=3, L=64, d=16, dff=32, w=8, eps=1e-5, dt=1,
         out=A, variant=0):
    return lib.laser_segment_ffn_forward_variant(seg, lens, w1, b1, w2, b2, g, b, U, C, L, d, dff, w, eps, dt, out,
                                                 None, variant)


def test_segment_ffn_argument_validation(lib):
    NULL, SHAPE, DTYPE, UNSUP, ALIGN = 1, 2, 3, 4, 6
    for kw in ({"seg": None}, {"w1": None}, {"b1": None}, {"w2": None}, {"b2": None}, {"g": None}, {"b": None},
               {"out": None}):
        assert _ffn(lib, **kw) == NULL, kw
    assert _ffn(lib, dt=7) == DTYPE
    for kw in ({"U": 0}, {"d": 12}, {"dff": 0}, {"dff": 12}, {"dff": 8192}, {"w": 0}, {"eps": -1.0},
               {"eps": float("inf")}, {"eps": float("nan")}):
        assert _ffn(lib, **kw) == SHAPE, kw
    assert _ffn(lib, seg=A + 8) == ALIGN and _ffn(lib, w2=A + 4) == ALIGN and _ffn(lib, b1=A + 2) == ALIGN
    assert _ffn(lib, variant=9) == UNSUP
    assert _ffn(lib, variant=2, d=16) == UNSUP        # the matrix-core form does not take d = 16


def _proj_kv(lib, h=A, wk=A, wv=A, U=2, L=64, din=16, dq=8, d=16, dt=1, k=A, v=A, variant=0):
    return lib.laser_project_kv_forward_variant(h, wk, wv, U, L, din, dq, d, dt, k, v, None, variant)


def _proj_q(lib, t=A, wq=A, U=2, C=3, din=16, dq=8, dt=1, q=A, variant=0):
    return lib.laser_project_q_forward_variant(t, wq, U, C, din, dq, dt, q, None, variant)


def test_projection_argument_validation(lib):
    NULL, SHAPE, DTYPE, UNSUP, ALIGN = 1, 2, 3, 4, 6
    for kw in ({"h": None}, {"wk": None}, {"wv": None}, {"k": None}, {"v": None}):
        assert _proj_kv(lib, **kw) == NULL, kw
    for kw in ({"t": None}, {"wq": None}, {"q": None}):
        assert _proj_q(lib, **kw) == NULL, kw
    assert _proj_kv(lib, dt=4) == DTYPE and _proj_q(lib, dt=-1) == DTYPE
    for kw in ({"U": 0}, {"L": 0}, {"din": 0}, {"dq": 0}, {"d": 0}, {"din": 8192}, {"d": 8192}, {"dq": -8}):
        assert _proj_kv(lib, **kw) == SHAPE, kw
    for kw in ({"U": 0}, {"C": 0}, {"din": 0}, {"dq": 0}, {"dq": 5000}):
        assert _proj_q(lib, **kw) == SHAPE, kw
    assert _proj_kv(lib, h=A + 8) == ALIGN and _proj_kv(lib, wv=A + 4) == ALIGN and _proj_kv(lib, k=A + 2) == ALIGN
    assert _proj_q(lib, wq=A + 8) == ALIGN and _proj_q(lib, q=A + 1) == ALIGN
    assert _proj_kv(lib, variant=5) == UNSUP and _proj_q(lib, variant=-1) == UNSUP
    assert _proj_kv(lib, variant=2) == UNSUP          # the matrix-core form does not take d_in = 16
    assert _proj_kv(lib, variant=2, din=128, dq=48, d=128) == UNSUP   # widths must be multiples of 32
    assert _proj_q(lib, variant=2, din=128, dq=128, dt=0) == UNSUP    # bf16 only


def test_sta_heads_argument_validation(lib):
    NULL, SHAPE, UNSUP = 1, 2, 4
    f = lambda heads=2, dq=16, d=16, variant=0, q=A, C=3: lib.laser_sta_forward_heads(
        q, A, A, None, 2, C, 64, dq, d, 8, 1.0, heads, 1, A, None, None, variant)
    assert f(q=None) == NULL
    for kw in ({"heads": 0}, {"heads": -2}, {"heads": 65}, {"heads": 3}, {"heads": 4, "dq": 16, "d": 24 + 2},
               {"heads": 2, "dq": 24, "d": 8 * 3 + 8 + 1}):
        assert f(**kw) == SHAPE, kw
    assert f(variant=9) == UNSUP
    assert f(heads=8, dq=128, d=128, C=64, variant=2) == UNSUP     # the matrix-core kernel takes 1, 2 or 4 heads
    assert f(heads=4, dq=32, d=128, C=64, variant=2) == UNSUP      # (a head needs a whole 16-wide k-step)
    assert f(heads=4, dq=32, d=128, variant=3) == UNSUP            # the streaming kernel takes one or two


def test_folded_form_argument_validation(lib):
    NULL, SHAPE, DTYPE, UNSUP, ALIGN = 1, 2, 3, 4, 6
    fold = lambda wq=A, wk=A, din=16, dq=8, heads=2, dt=1, out=A: lib.laser_fold_query_weights(wq, wk, din, dq, heads, dt, out, None)
    assert fold(wq=None) == NULL and fold(out=None) == NULL and fold(dt=9) == DTYPE
    assert fold(heads=3) == SHAPE and fold(heads=0) == SHAPE and fold(din=0) == SHAPE and fold(wk=A + 8) == ALIGN
    ph = lambda x=A, wv=A, P=4, S=5, din=16, d=16, heads=2, dt=1, y=A, variant=0: lib.laser_project_heads_forward(
        x, wv, P, S, din, d, heads, dt, y, None, variant)
    assert ph(x=None) == NULL and ph(y=None) == NULL and ph(dt=-1) == DTYPE
    for kw in ({"P": 0}, {"S": 0}, {"din": 12}, {"d": 20}, {"heads": 3}, {"heads": 0}, {"P": 1 << 20, "S": 1 << 12}):
        assert ph(**kw) == SHAPE, kw
    assert ph(wv=A + 4) == ALIGN and ph(variant=7) == UNSUP and ph(variant=2) == UNSUP   # d_in = 16: no matrix-core form
    fo = lambda t=A, h=A, a=A, wv=A, U=2, C=1, L=64, din=16, d=16, w=8, gamma=1.0, heads=2, dt=1, qf=A, g=A, out=A: \
        lib.laser_sta_folded_forward(t, h, a, wv, None, U, C, L, din, d, w, gamma, heads, dt, qf, g, out, None, None)
    for kw in ({"t": None}, {"h": None}, {"a": None}, {"wv": None}, {"qf": None}, {"g": None}, {"out": None}):
        assert fo(**kw) == NULL, kw
    for kw in ({"heads": 0}, {"heads": 3}, {"U": 0}, {"C": 0}, {"w": 0}, {"gamma": 0.0}, {"din": 12}):
        assert fo(**kw) == SHAPE, kw
    assert fo(dt=5) == DTYPE and fo(a=A + 8) == ALIGN and fo(g=A + 2) == ALIGN


def test_sta_softmax_argument_validation(lib):
    NULL, SHAPE, UNSUP = 1, 2, 4
    f = lambda heads=1, dq=16, d=16, variant=0, q=A, C=3, w=8: lib.laser_sta_forward_softmax(
        q, A, A, None, 2, C, 64, dq, d, w, 1.0, heads, 1, A, None, None, variant)
    assert f(q=None) == NULL and f(heads=0) == SHAPE and f(heads=3) == SHAPE and f(w=0) == SHAPE
    assert f(variant=9) == UNSUP
    assert f(dq=128, d=128, C=4, variant=2) == UNSUP       # the matrix-core kernel starts at nine candidates
    assert f(dq=64, d=64, C=2, w=200, variant=3) == UNSUP  # long segments: the streaming kernel's long form does not either


def test_ragged_argument_validation(lib):
    NULL, SHAPE, DTYPE, ALIGN = 1, 2, 3, 6
    sta = lambda q=A, off=A, U=3, C=8, P=10, L=64, dq=16, d=16, w=8, gamma=1.0, dt=1, out=A: \
        lib.laser_sta_forward_ragged(q, A, A, None, off, U, C, P, L, dq, d, w, gamma, dt, out, None, None)
    assert sta(q=None) == NULL and sta(off=None) == NULL and sta(out=None) == NULL and sta(dt=9) == DTYPE
    for kw in ({"P": 0}, {"P": -3}, {"P": 25}, {"U": 0}, {"C": 0}, {"w": 0}, {"gamma": 0.0}, {"d": 12}):   # 25 > U * C_max
        assert sta(**kw) == SHAPE, kw
    assert sta(off=A + 2) == ALIGN and sta(q=A + 8) == ALIGN
    gsta = lambda seg=A, off=A, U=3, C=8, P=10, M=1, z=A: \
        lib.laser_gsta_forward_ragged(seg, A, A, A, A, None, off, U, C, P, 64, 16, 8, M, 1, z, None)
    assert gsta(seg=None) == NULL and gsta(off=None) == NULL and gsta(z=None) == NULL
    assert gsta(P=0) == SHAPE and gsta(P=99) == SHAPE and gsta(M=0) == SHAPE and gsta(off=A + 1) == ALIGN
    whole = lambda off=A, P=10, t0=A, z=A: lib.laser_forward_ragged(A, A, A, t0, A, A, A, None, off, 3, 8, P, 64, 16, 16,
                                                                     8, 1.0, 1, 1, A, None, z, None)
    assert whole(off=None) == NULL and whole(t0=None) == NULL and whole(z=None) == NULL and whole(P=25) == SHAPE


def test_sta_backward_argument_validation(lib):
    NULL, SHAPE, DTYPE, UNSUP, ALIGN = 1, 2, 3, 4, 6
    lib.laser_sta_backward_work_bytes.restype = ctypes.c_size_t
    need = lib.laser_sta_backward_work_bytes(3, 2, 64, 16, 8)
    assert need >= 3 * 2 * 16 * 4 and lib.laser_sta_backward_work_bytes(0, 2, 64, 16, 8) == 0
    f = lambda q=A, dseg=A, U=3, C=2, L=64, dq=16, d=16, w=8, gamma=1.0, dt=1, dqo=A, dko=A, dvo=A, work=A, wb=1 << 20: \
        lib.laser_sta_backward(q, A, A, None, dseg, U, C, L, dq, d, w, ctypes.c_float(gamma), dt, dqo, dko, dvo, work,
                               ctypes.c_size_t(wb), None)
    for kw in ({"q": None}, {"dseg": None}, {"dqo": None}, {"dko": None}, {"dvo": None}, {"work": None}):
        assert f(**kw) == NULL, kw
    assert f(dt=6) == DTYPE
    for kw in ({"U": 0}, {"C": 0}, {"w": 0}, {"gamma": 0.0}, {"d": 12}, {"wb": 8}):
        assert f(**kw) == SHAPE, kw
    assert f(dko=A + 4) == ALIGN and f(work=A + 8) == ALIGN
    assert f(dq=512, d=512) == UNSUP


def test_gsta_backward_argument_validation(lib):
    NULL, SHAPE, DTYPE, UNSUP, ALIGN = 1, 2, 3, 4, 6
    lib.laser_gsta_backward_work_bytes.restype = ctypes.c_size_t
    assert lib.laser_gsta_backward_work_bytes(3, 2, 16, 2) >= 3 * 2 * 2 * 6 * 16 * 4
    assert lib.laser_gsta_backward_work_bytes(3, 0, 16, 2) == 0
    f = lambda seg=A, dz=A, U=3, C=2, L=64, d=16, w=8, M=2, dt=1, dseg=A, dt0=A, dwq=A, dwk=A, dwv=A, work=A, wb=1 << 20: \
        lib.laser_gsta_backward(seg, A, A, A, A, None, dz, U, C, L, d, w, M, dt, dseg, dt0, dwq, dwk, dwv, work,
                                ctypes.c_size_t(wb), None)
    for kw in ({"seg": None}, {"dz": None}, {"dseg": None}, {"dt0": None}, {"dwq": None}, {"dwk": None}, {"dwv": None},
               {"work": None}):
        assert f(**kw) == NULL, kw
    assert f(dt=8) == DTYPE
    for kw in ({"U": 0}, {"M": 0}, {"w": 0}, {"d": 12}, {"wb": 64}):
        assert f(**kw) == SHAPE, kw
    assert f(dz=A + 4) == ALIGN and f(dwk=A + 8) == ALIGN
    big = 1 << 30
    assert f(d=512, wb=big) == UNSUP and f(M=9, wb=big) == UNSUP
    assert f(L=1 << 15, w=8, d=256, wb=big) == UNSUP    # H' block too large for LDS


def test_ragged_views_and_ffn_argument_validation(lib):
    NULL, SHAPE, ALIGN = 1, 2, 6
    mr = lambda seg=A, off=A, P=10, r=2, pool=A, rec=A: lib.laser_multires_forward_ragged(
        seg, None, off, 3, 8, P, 64, 16, 8, r, 1, pool, rec, None)
    assert mr(seg=None) == NULL and mr(off=None) == NULL and mr(P=0) == SHAPE and mr(P=25) == SHAPE
    assert mr(r=9) == SHAPE and mr(off=A + 2) == ALIGN
    ffn = lambda seg=A, off=A, P=10, dff=32, out=A: lib.laser_segment_ffn_forward_ragged(
        seg, None, off, A, A, A, A, A, A, 3, 8, P, 64, 16, dff, 8, ctypes.c_float(1e-5), 1, out, None)
    assert ffn(seg=None) == NULL and ffn(off=None) == NULL and ffn(out=None) == NULL
    assert ffn(P=0) == SHAPE and ffn(P=25) == SHAPE and ffn(dff=12) == SHAPE and ffn(off=A + 1) == ALIGN


def test_host_code_under_address_and_undefined_behaviour_sanitizers(lib, tmp_path):
    """The host side of the boundary (validation, kernel selection, size arithmetic) instrumented with ASan and UBSan,
    driven by tests/abi_host_check.cpp with sizes at the edge of int: a sanitizer report aborts the run."""
    import subprocess
    from paper_2602_11562_amd.build import build_host_check
    exe = build_host_check(str(tmp_path / "abi_host_check"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "0 failure(s)" in r.stdout
