"""GPU parity of the GSTA backward pass against the fp64 checker (itself pinned to autograd and central differences),
element by element, and of the whole backward chain dz -> (dq, dk, dv) against the checker chained the same way.

The checker reads the stored inputs. Tolerances: dt0 and the weight gradients are fp32 results of fp32 arithmetic:
1e-5 (dt0 per pair vector; a weight gradient, which sums thousands of signed outer products, against the largest
entry of its matrix). dseg is rounded once to the storage type: 1e-5 for fp32, 2e-2 for bf16, per vector."""
import math

import numpy as np
import pytest

import oracle
import workloads

from parity_util import TOL, to_device, to_host_f64, vec_rel_err

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")

CASES = {
    # dtype, C, L, d, w, M, lens
    "benchmark_widths": ("bf16", 37, 1024 + 128, 128, 128, 1, [1152, 700, 0]),
    "paper_setting": ("bf16", 1, 1000, 128, 10, 1, [1000, 995, 404, 7, 0, 1000]),
    "three_layers": ("bf16", 5, 640, 64, 64, 3, [640, 65]),
    "wide": ("bf16", 2, 320, 256, 32, 2, [320, 33]),
    "f32_odd_widths": ("f32", 3, 130, 48, 16, 2, [130, 50, 0]),
}


def _store(x, dtype):
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        bits = workloads.f32_to_bf16_bits(x)
        return bits, workloads.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


def _case(name):
    dtype, C, L, d, w, M, lens = CASES[name]
    U, S = len(lens), -(-L // w)
    rng = np.random.default_rng(3100 + sum(map(ord, name)))
    lens = np.array(lens, dtype=np.int32)
    cnt = oracle.segment_counts(lens, L, w)
    Hp = rng.normal(size=(U, C, S, d)) * (cnt[:, None, :, None] > 0)     # H' as STA leaves it: empty segments are zero
    st = {"seg": _store(Hp, dtype), "t0": _store(rng.normal(size=(U, C, d)), dtype)}
    for nm in ("wq", "wk", "wv"):
        st[nm] = _store(rng.normal(size=(M, d, d)) / math.sqrt(d), dtype)
    dz = rng.normal(size=(U, C, d)).astype(np.float32)
    return dtype, st, lens, cnt, dz, L, w


@pytest.mark.parametrize("name", list(CASES))
def test_gsta_backward_matches_checker(name):
    import torch
    dtype, st, lens, cnt, dz, L, w = _case(name)
    print(f"case {name}", flush=True)
    val = {k: v[1] for k, v in st.items()}
    ref = oracle.gsta_backward(val["seg"], val["t0"], val["wq"], val["wk"], val["wv"], cnt, dz.astype(np.float64))
    dev = {k: to_device(v[0]) for k, v in st.items()}
    got = laser.laser_gsta_backward(dev["seg"], dev["t0"], dev["wq"], dev["wk"], dev["wv"], to_device(lens), to_device(dz),
                                    L, w)
    torch.cuda.synchronize()
    err = vec_rel_err(to_host_f64(got[0]), ref[0])
    print(f"  dseg: {err:.3e}", flush=True)
    assert err <= TOL[dtype]
    err = vec_rel_err(to_host_f64(got[1]), ref[1])
    print(f"  dt0: {err:.3e}", flush=True)
    assert err <= 1e-5
    for nm, a, b in zip(("dwq", "dwk", "dwv"), got[2:], ref[2:]):
        M = b.shape[0]
        err = vec_rel_err(to_host_f64(a).reshape(M, -1), b.reshape(M, -1))
        print(f"  {nm}: {err:.3e}", flush=True)
        assert err <= 1e-5, nm
    again = laser.laser_gsta_backward(dev["seg"], dev["t0"], dev["wq"], dev["wk"], dev["wv"], to_device(lens),
                                      to_device(dz), L, w)
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(got, again))      # fixed summation order


def test_backward_chain_from_dz_to_the_inputs_of_sta():
    """Forward STA -> GSTA through the library, then GSTA backward -> STA backward; the checker is chained the same way
    on the stored H' and the stored dseg (each stage held to its own tolerance)."""
    import torch
    rng = np.random.default_rng(77)
    U, C, L, dq, d, w, M = 4, 2, 300, 32, 128, 10, 1
    bf = lambda *s: _store(rng.normal(size=s), "bf16")
    (qs, qv), (ks, kv), (vs, vv), (ts, tv) = bf(U, C, dq), bf(U, L, dq), bf(U, L, d), bf(U, C, d)
    W = [_store(rng.normal(size=(M, d, d)) / math.sqrt(d), "bf16") for _ in range(3)]
    lens = np.array([300, 155, 9, 0], dtype=np.int32)
    dz = rng.normal(size=(U, C, d)).astype(np.float32)
    gamma = math.sqrt(dq)
    q, k, v, t0 = (to_device(x) for x in (qs, ks, vs, ts))
    wq, wk, wv = (to_device(x[0]) for x in W)
    lens_d = to_device(lens)
    seg, cnt = laser.laser_sta_forward(q, k, v, lens_d, w, gamma)
    dseg, dt0, dwq, dwk, dwv = laser.laser_gsta_backward(seg, t0, wq, wk, wv, lens_d, to_device(dz), L, w)
    gq, gk, gv = laser.laser_sta_backward(q, k, v, lens_d, dseg, w, gamma)
    torch.cuda.synchronize()
    cnt_h = cnt.cpu().numpy()
    ref_g = oracle.gsta_backward(to_host_f64(seg), tv, W[0][1], W[1][1], W[2][1], cnt_h, dz.astype(np.float64))
    assert vec_rel_err(to_host_f64(dseg), ref_g[0]) <= TOL["bf16"]
    assert vec_rel_err(to_host_f64(dt0), ref_g[1]) <= 1e-5
    ref_s = oracle.sta_backward(qv, kv, vv, lens, w, gamma, to_host_f64(dseg))
    assert vec_rel_err(to_host_f64(gq), ref_s[0]) <= 1e-5
    assert vec_rel_err(to_host_f64(gk).reshape(U, -1), ref_s[1].reshape(U, -1)) <= 1e-5
    assert vec_rel_err(to_host_f64(gv), ref_s[2]) <= 1e-5


def test_gsta_backward_refuses_what_it_does_not_take():
    import torch
    z = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(laser.LaserError) as e:     # d = 512
        laser.laser_gsta_backward(z(1, 1, 4, 512), z(1, 1, 512), z(1, 512, 512), z(1, 512, 512), z(1, 512, 512), None,
                                  torch.zeros(1, 1, 512, device="cuda"), 32, 8)
    assert e.value.code == 4
