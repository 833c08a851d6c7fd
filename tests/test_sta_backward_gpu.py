"""GPU parity of the STA backward pass against the fp64 checker (itself pinned to autograd and central differences),
element by element. The checker reads the stored inputs; the kernel computes in fp32 from the same values and writes
fp32 gradients, so the tolerance is the fp32 one (1e-5) for both storage types. Metric: dq and dv per output vector, as
everywhere. dk per user: with one candidate dk_j is the query times the scalar ds_j = (dH' . v_j) g (1 - g), a dot
product of d signed terms that cancels to anything between 0 and its terms' size, so an fp32 sum has an absolute, not
a relative, error bound (about d 2^-24 times the terms); a row whose dot product happens to cancel would fail a
per-row relative test at any precision short of exact. Beside the per-user figure dk is therefore also compared row by
row against max(|dk_j|, 2 % of the user's largest row) at 5e-5. Rows that must be zero must still be exactly zero."""
import math

import numpy as np
import pytest

import oracle
import workloads

from parity_util import to_device, to_host_f64, vec_rel_err

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")

BWD_TOL = 1e-5

CASES = {
    # dtype, C, L, d_q, d, w, lens
    "paper_setting": ("bf16", 1, 1000, 32, 128, 10, [1000, 995, 404, 7, 0, 1000]),
    "eight_candidates": ("bf16", 8, 300, 64, 64, 64, [300, 65, 64]),
    "wide_rows": ("bf16", 2, 520, 256, 256, 128, [520, 129]),
    "one_user_many_runs": ("bf16", 1, 4096, 64, 64, 64, [3000]),
    "three_candidates_wide_keys": ("bf16", 3, 333, 128, 64, 20, [333, 21, 20, 1]),
    "two_candidates_same_widths": ("bf16", 2, 700, 128, 128, 64, [700, 65, 64]),
    "four_candidates_narrow_keys": ("bf16", 4, 1500, 64, 128, 300, [1500, 301]),
    "odd_widths_f32": ("f32", 3, 130, 24, 48, 16, [130, 50]),
    # more than eight candidates per user: blocks of eight, one launch each, the later ones adding to dk and dv
    "nine_candidates": ("bf16", 9, 300, 64, 64, 64, [300, 65, 0]),
    "twenty_candidates_f32": ("f32", 20, 130, 24, 48, 16, [130, 50]),
    "seventeen_candidates_wide": ("bf16", 17, 200, 128, 128, 32, [200, 33]),
    "forty_candidates": ("bf16", 40, 150, 64, 128, 16, [150, 17]),            # five blocks
    "ten_candidates_very_wide": ("bf16", 10, 100, 256, 256, 32, [100]),       # rows of 256 elements, 8 + 2
    "f32_paper_setting": ("f32", 1, 200, 32, 128, 10, [200, 33, 0]),
}


def _store(x, dtype):
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        bits = workloads.f32_to_bf16_bits(x)
        return bits, workloads.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


@pytest.mark.parametrize("name", list(CASES))
def test_sta_backward_matches_checker(name):
    import torch
    dtype, C, L, dq, d, w, lens = CASES[name]
    U, S = len(lens), -(-L // w)
    rng = np.random.default_rng(2100 + sum(map(ord, name)))
    (qs, qv), (ks, kv), (vs, vv), (gs, gv) = (_store(rng.normal(size=s), dtype)
                                              for s in ((U, C, dq), (U, L, dq), (U, L, d), (U, C, S, d)))
    lens = np.array(lens, dtype=np.int32)
    gamma = math.sqrt(dq)
    print(f"case {name}", flush=True)
    ref = oracle.sta_backward(qv, kv, vv, lens, w, gamma, gv)
    got = laser.laser_sta_backward(to_device(qs), to_device(ks), to_device(vs), to_device(lens), to_device(gs), w, gamma)
    torch.cuda.synchronize()
    for nm, a, b in zip(("dq", "dk", "dv"), got, ref):
        a = to_host_f64(a)
        if nm == "dk":
            assert not a[b == 0].any()      # padding rows: exactly zero
            # row by row as well, with an absolute floor: the error of row j against max(|dk_j|, 2 % of the user's
            # largest row). A row whose scalar ds_j cancels to less than that is measured against the floor (its
            # fp32 error is absolute, see above); every other row is held to a relative bound of its own.
            row_err = np.abs(a - b).max(axis=-1)
            row_ref = np.abs(b).max(axis=-1)
            floor = 0.02 * row_ref.max(axis=-1, keepdims=True)
            per_row = float((row_err / np.maximum(np.maximum(row_ref, floor), 1e-300)).max())
            print(f"  dk: max row-wise error with a 2 % floor {per_row:.3e}", flush=True)
            assert per_row <= 5 * BWD_TOL
            a, b = a.reshape(U, -1), b.reshape(U, -1)
        err = vec_rel_err(a, b)
        print(f"  {nm}: max relative error {err:.3e}", flush=True)
        assert err <= BWD_TOL, nm
    # reproducible: a second call gives the same bits
    again = laser.laser_sta_backward(to_device(qs), to_device(ks), to_device(vs), to_device(lens), to_device(gs), w, gamma)
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(got, again))


def test_sta_backward_is_the_gradient_of_the_library_forward():
    """d/d eps of sum(H'(q + eps dq, ...) * dseg) through the library's own fp32 forward pass agrees with the inner
    product of the library's gradients with the direction (central difference; fp32 forward, so to about 1e-3)."""
    import torch
    rng = np.random.default_rng(9)
    U, C, L, dq, d, w = 3, 2, 96, 16, 32, 8
    f = lambda *s: torch.from_numpy(rng.normal(size=s).astype(np.float32)).cuda()
    q, k, v, up = f(U, C, dq), f(U, L, dq), f(U, L, d), f(U, C, L // w, d)
    lens = to_device(np.array([96, 50, 9], dtype=np.int32))
    gamma = 2.0
    gq, gk, gv = laser.laser_sta_backward(q, k, v, lens, up, w, gamma)
    dq_, dk_, dv_ = f(U, C, dq), f(U, L, dq), f(U, L, d)
    h = 1e-2
    loss = lambda s: float((laser.laser_sta_forward(q + s * dq_, k + s * dk_, v + s * dv_, lens, w, gamma,
                                                    want_cnt=False)[0].double() * up.double()).sum())
    num = (loss(h) - loss(-h)) / (2 * h)
    ana = float((gq.double() * dq_).sum() + (gk.double() * dk_).sum() + (gv.double() * dv_).sum())
    assert abs(num - ana) <= 2e-3 * max(1.0, abs(ana))


def test_sta_backward_refuses_what_it_does_not_take():
    import torch
    z = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(laser.LaserError) as e:
        laser.laser_sta_backward(z(1, 2, 512), z(1, 64, 512), z(1, 64, 32), None, z(1, 2, 8, 32), 8, 1.0)
    assert e.value.code == 4      # rows of more than 256 elements
    with pytest.raises(laser.LaserError) as e:
        laser.laser_sta_backward(z(1, 1, 32), z(1, 64, 32), z(1, 64, 32), None, z(1, 1, 8, 32), 8, 1.0,
                                 work=torch.zeros(16, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 2      # scratch too small


@pytest.mark.parametrize("name", ["paper_setting", "one_user_many_runs", "three_candidates_wide_keys",
                                  "two_candidates_same_widths", "four_candidates_narrow_keys"])
def test_sta_backward_with_bf16_gradients(name):
    """dk and dv in the storage type: the fp32 sums of the fp32-output call, rounded once to bf16 (bit for bit), so the
    error against the checker is the fp32 error plus one rounding (2^-9 relative: tolerance 2e-2 as for every bf16
    output); dq stays fp32 and identical."""
    import torch
    dtype, C, L, dq, d, w, lens = CASES[name]
    U, S = len(lens), -(-L // w)
    rng = np.random.default_rng(2100 + sum(map(ord, name)))
    (qs, qv), (ks, kv), (vs, vv), (gs, gv) = (_store(rng.normal(size=s), dtype)
                                              for s in ((U, C, dq), (U, L, dq), (U, L, d), (U, C, S, d)))
    lens = np.array(lens, dtype=np.int32)
    gamma = math.sqrt(dq)
    args = (to_device(qs), to_device(ks), to_device(vs), to_device(lens), to_device(gs), w, gamma)
    full = laser.laser_sta_backward(*args)
    low = laser.laser_sta_backward(*args, grads_bf16=True)
    torch.cuda.synchronize()
    assert low[1].dtype == torch.bfloat16 and low[2].dtype == torch.bfloat16
    assert torch.equal(full[0], low[0])
    assert torch.equal(full[1].bfloat16(), low[1]) and torch.equal(full[2].bfloat16(), low[2])
    ref = oracle.sta_backward(qv, kv, vv, lens, w, gamma, gv)
    assert vec_rel_err(to_host_f64(low[2]), ref[2]) <= 2e-2
    assert vec_rel_err(to_host_f64(low[1]).reshape(U, -1), ref[1].reshape(U, -1)) <= 2e-2


def test_bf16_gradients_need_the_wide_kernel():
    import torch
    z = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(laser.LaserError) as e:     # eight candidates: only the fp32-output kernel takes them
        laser.laser_sta_backward(z(1, 8, 32), z(1, 64, 32), z(1, 64, 32), None, z(1, 8, 8, 32), 8, 1.0, grads_bf16=True)
    assert e.value.code == 4
