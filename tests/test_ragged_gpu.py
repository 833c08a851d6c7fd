"""GPU parity of the packed-pairs entry points (ragged candidate counts per user) against the fp64 checker, element by
element, on shapes that reach every STA and GSTA kernel family; equal counts must reproduce the dense entry points
bit for bit. Stored inputs on both sides; tolerances as everywhere (fp32 1e-5, bf16 2e-2 per output vector; GSTA reads
H' as stored)."""
import math

import numpy as np
import pytest

import oracle
import workloads

from parity_util import TOL, to_device, to_host_f64, vec_rel_err

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")

CASES = {
    # dtype, L, d_q, d, w, M, C_max, counts per user, lens per user
    "matrix_core_direct_to_lds": ("bf16", 1024 + 128, 128, 128, 128, 1, 256, [256, 100, 0, 33], [1152, 700, 1152, 129]),
    "matrix_core_direct_to_lds_four_waves": ("bf16", 1024 + 128, 128, 128, 128, 1, 128, [128, 65, 0, 33, 1],
                                             [1152, 700, 1152, 129, 1000]),
    "matrix_core_eight_waves": ("bf16", 640, 64, 128, 64, 1, 200, [200, 1, 129], [640, 65, 300]),
    "matrix_core_two_waves": ("bf16", 512, 64, 64, 64, 2, 64, [64, 33, 1, 0, 17], [512, 100, 64, 512, 0]),
    "streaming_long_segments": ("bf16", 1024, 64, 64, 256, 1, 8, [1, 8, 0, 3], [1024, 300, 1024, 257]),
    "streaming_short_segments": ("bf16", 1000, 32, 128, 10, 1, 2, [2, 0, 1, 2, 1], [1000, 1000, 404, 7, 0]),
    "many_segments_split_gsta": ("bf16", 2560, 128, 128, 64, 1, 40, [40, 7], [2560, 1000]),
    "generic_f32": ("f32", 130, 24, 48, 16, 2, 5, [5, 0, 2, 4], [130, 130, 50, 17]),
}


def _store(x, dtype):
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        bits = workloads.f32_to_bf16_bits(x)
        return bits, workloads.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


def _case(name):
    dtype, L, dq, d, w, M, cmax, counts, lens = CASES[name]
    rng = np.random.default_rng(1200 + sum(map(ord, name)))
    U, P = len(counts), sum(counts)
    t = {"q": _store(rng.normal(size=(P, dq)), dtype), "k": _store(rng.normal(size=(U, L, dq)), dtype),
         "v": _store(rng.normal(size=(U, L, d)), dtype), "t0": _store(rng.normal(size=(P, d)), dtype)}
    for nm in ("wq", "wk", "wv"):
        t[nm] = _store(rng.normal(size=(M, d, d)) / math.sqrt(d), dtype)
    off = np.cumsum([0] + counts).astype(np.int32)
    return dtype, t, np.array(lens, dtype=np.int32), off, cmax, w, math.sqrt(dq)


@pytest.mark.parametrize("name", list(CASES))
def test_ragged_path_matches_checker(name):
    import torch
    dtype, t, lens, off, cmax, w, gamma = _case(name)
    print(f"case {name}", flush=True)
    dev = {k: to_device(v[0]) for k, v in t.items()}
    val = {k: v[1] for k, v in t.items()}
    seg, cnt, z = laser.laser_forward_ragged(dev["q"], dev["k"], dev["v"], dev["t0"], dev["wq"], dev["wk"], dev["wv"],
                                             to_device(lens), to_device(off), cmax, w, gamma)
    torch.cuda.synchronize()
    Hr, cnt_ref, _ = oracle.laser_forward_ragged(val["q"], val["k"], val["v"], val["t0"], val["wq"], val["wk"], val["wv"],
                                                 lens, off, w, gamma)
    assert np.array_equal(cnt.cpu().numpy(), cnt_ref)
    err = vec_rel_err(to_host_f64(seg), Hr)
    print(f"  H': {err:.3e}", flush=True)
    assert err <= TOL[dtype]
    # GSTA on H' as stored
    U = len(lens)
    z_ref = np.zeros_like(to_host_f64(z))
    segs = to_host_f64(seg)
    for u in range(U):
        for p in range(off[u], off[u + 1]):
            z_ref[p] = oracle.gsta_pair(segs[p], val["t0"][p], val["wq"], val["wk"], val["wv"], cnt_ref[u] > 0)
    err = vec_rel_err(to_host_f64(z), z_ref)
    print(f"  z: {err:.3e}", flush=True)
    assert err <= TOL[dtype]
    # the two stages alone give the same bits as the whole path
    seg2, cnt2, _ = laser.laser_forward_ragged(dev["q"], dev["k"], dev["v"], None, None, None, None, to_device(lens),
                                               to_device(off), cmax, w, gamma, stage="sta")
    _, _, z2 = laser.laser_forward_ragged(None, dev["k"], dev["v"], dev["t0"], dev["wq"], dev["wk"], dev["wv"],
                                          to_device(lens), to_device(off), cmax, w, gamma, seg_out=seg, stage="gsta")
    torch.cuda.synchronize()
    assert torch.equal(cnt, cnt2) and torch.equal(z, z2)
    assert vec_rel_err(to_host_f64(seg2), Hr) <= TOL[dtype]


@pytest.mark.parametrize("shape", ["matrix_core", "streaming"])
def test_equal_counts_reproduce_the_dense_entry_points(shape):
    import torch
    if shape == "matrix_core":
        U, C, L, dq, d, w = 2, 256, 512, 128, 128, 128
    else:
        U, C, L, dq, d, w = 5, 2, 300, 64, 64, 10
    rng = np.random.default_rng(77)
    bf = lambda *s: to_device(workloads.f32_to_bf16_bits(rng.normal(size=s).astype(np.float32)))
    q, k, v, t0 = bf(U, C, dq), bf(U, L, dq), bf(U, L, d), bf(U, C, d)
    wq, wk, wv = (to_device(workloads.f32_to_bf16_bits((rng.normal(size=(1, d, d)) / math.sqrt(d)).astype(np.float32)))
                  for _ in range(3))
    lens = to_device(np.array([L, L // 3] + [L] * (U - 2), dtype=np.int32))
    off = to_device((np.arange(U + 1) * C).astype(np.int32))
    gamma = math.sqrt(dq)
    seg_d, cnt_d, z_d = laser.laser_forward(q, k, v, t0, wq, wk, wv, lens, w, gamma)
    seg_r, cnt_r, z_r = laser.laser_forward_ragged(q.view(U * C, dq), k, v, t0.view(U * C, d), wq, wk, wv, lens, off, C, w,
                                                   gamma)
    torch.cuda.synchronize()
    assert torch.equal(seg_d.view(torch.int16).view(U * C, -1, d), seg_r.view(torch.int16))
    assert torch.equal(cnt_d, cnt_r) and torch.equal(z_d.view(U * C, d), z_r)


def test_offsets_that_break_the_rules_stay_inside_the_buffers():
    """The host cannot see the offsets; the kernels clamp them. Counts above C_max, a first row past P and a
    decreasing pair of offsets must leave the guard bands around every output untouched."""
    import torch
    dtype, t, lens, off, cmax, w, gamma = _case("matrix_core_two_waves")
    dev = {k: to_device(v[0]) for k, v in t.items()}
    P, d = t["q"][0].shape[0], t["v"][0].shape[2]
    S = -(-t["k"][0].shape[1] // w)
    guard = 8192
    segbuf = torch.full((guard + P * S * d + guard,), 3.0, dtype=torch.bfloat16, device="cuda")
    zbuf = torch.full((guard + P * d + guard,), 3.0, dtype=torch.float32, device="cuda")
    seg = segbuf[guard:guard + P * S * d].view(P, S, d)
    z = zbuf[guard:guard + P * d].view(P, d)
    for bad in ([0, 200, 201, 90, 95, P], [P + 50, P + 60, 3, 3, 3, P], [0, 0, 0, 0, 0, 1 << 30]):
        laser.laser_forward_ragged(dev["q"], dev["k"], dev["v"], dev["t0"], dev["wq"], dev["wk"], dev["wv"],
                                   to_device(lens), to_device(np.array(bad, dtype=np.int32)), cmax, w, gamma, seg_out=seg,
                                   z_out=z)
        torch.cuda.synchronize()
        for b in (segbuf, zbuf):
            assert (b[:guard] == 3.0).all() and (b[-guard:] == 3.0).all(), bad


@pytest.mark.parametrize("name", ["matrix_core_two_waves", "streaming_short_segments", "generic_f32"])
def test_ragged_views_and_ffn_match_checker(name):
    """The views (Sec. 3.4.4) and the FFN + LayerNorm step (Sec. 3.4.2) on packed pairs: every pair against the
    checker's per-pair functions with its own user's valid segments. Views are selections of stored values: equality."""
    import torch
    dtype, t, lens, off, cmax, w, gamma = _case(name)
    dev = {k: to_device(v[0]) for k, v in t.items()}
    L = t["k"][0].shape[1]
    d = t["v"][0].shape[2]
    seg, cnt, _ = laser.laser_forward_ragged(dev["q"], dev["k"], dev["v"], None, None, None, None, to_device(lens),
                                             to_device(off), cmax, w, gamma, stage="sta")
    S = seg.shape[1]
    r = min(3, S)
    pool, recent = laser.laser_multires_forward_ragged(seg, to_device(lens), to_device(off), cmax, L, w, r)
    rng = np.random.default_rng(5)
    dff = 32
    W1s, W1v = _store(rng.normal(size=(d, dff)) / math.sqrt(d), dtype)
    W2s, W2v = _store(rng.normal(size=(dff, d)) / math.sqrt(dff), dtype)
    f32 = lambda x: np.asarray(x, dtype=np.float32)
    b1, b2 = f32(rng.normal(size=dff) * 0.3), f32(rng.normal(size=d) * 0.3)
    g, b = f32(1.0 + 0.2 * rng.normal(size=d)), f32(0.1 * rng.normal(size=d))
    out = laser.laser_segment_ffn_forward_ragged(seg, to_device(lens), to_device(off), cmax, to_device(W1s), to_device(b1),
                                                 to_device(W2s), to_device(b2), to_device(g), to_device(b), L, w, 1e-5)
    torch.cuda.synchronize()
    segh, cnth = to_host_f64(seg), cnt.cpu().numpy()
    poolh, rech, outh = to_host_f64(pool), to_host_f64(recent), to_host_f64(out)
    worst = 0.0
    for u in range(len(lens)):
        valid = cnth[u] > 0
        for p in range(off[u], off[u + 1]):
            pr, rr = oracle.multires_pair(segh[p], valid, r)
            assert np.array_equal(poolh[p], pr) and np.array_equal(rech[p], rr)
            for i in range(S):
                ref = (oracle.segment_ffn_vector(segh[p, i].copy(), W1v, b1, W2v, b2, g, b, 1e-5) if valid[i]
                       else np.zeros(d))
                worst = max(worst, vec_rel_err(outh[p, i], ref))
    print(f"  {name}: FFN + LN worst {worst:.3e}", flush=True)
    assert worst <= TOL[dtype]
