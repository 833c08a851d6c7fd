"""GPU parity of the multi-resolution views (pool = max over valid segments, recent = first r segments).

Both are selections of stored values, so the comparison with the checker is exact (as numbers: -0 equals +0).
The checker is fed the H' that the GPU reads (stored values), either from the checker's own STA rounded to the
storage type or from arbitrary seeded values, so that nothing here depends on the STA kernels.
"""
import numpy as np
import pytest

import oracle
import workloads

from parity_util import to_device, to_host_f64

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")


def _stored(rng, shape, dtype):
    x = rng.normal(size=shape).astype(np.float32)
    if dtype == "bf16":
        bits = workloads.f32_to_bf16_bits(x)
        return bits, workloads.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


CASES = [
    # dtype, U, C, L, w, d, r, lens
    ("bf16", 3, 5, 1000, 100, 128, 3, [1000, 333, 0]),
    ("bf16", 2, 130, 300, 10, 64, 30, [300, 95]),
    ("bf16", 4, 1, 4096, 256, 64, 1, [4096, 64, 257, 1]),
    ("f32", 2, 7, 512, 64, 64, 8, [512, 65]),
    ("f32", 1, 3, 96, 32, 8, 0, [40]),
    ("bf16", 2, 9, 10000, 256, 128, 40, [10000, 9999]),
    ("bf16", 1, 2, 64, 8, 1024, 2, [17]),
]


@pytest.mark.parametrize("dtype,U,C,L,w,d,r,lens", CASES)
def test_multires_matches_checker_exactly(dtype, U, C, L, w, d, r, lens):
    import torch
    rng = np.random.default_rng(U * 1000 + C * 10 + r)
    S = -(-L // w)
    stored, vals = _stored(rng, (U, C, S, d), dtype)
    lens = np.array(lens, dtype=np.int32)
    cnt = oracle.segment_counts(lens, L, w)
    # segments without a valid item hold zeros after STA; put a large value in one of them first to show that the
    # pooling really leaves them out (recent copies rows as stored, so restore the zeros for that check)
    poisoned = stored.copy()
    pv = vals.copy()
    for u in range(U):
        empty = np.flatnonzero(cnt[u] == 0)
        vals[u][:, empty] = 0.0
        stored[u][:, empty] = 0
        pv[u][:, empty] = 0.0
        poisoned[u][:, empty] = (0x7f00 if dtype == "bf16" else 3.0e38)   # huge positive
    print(f"case {dtype} U={U} C={C} L={L} w={w} d={d} r={r} lens={lens.tolist()}", flush=True)
    pool_ref, recent_ref = oracle.multires_forward(vals, cnt, r)
    pool, recent = laser.laser_multires_forward(to_device(stored), to_device(lens), L, w, r)
    pool_p, _ = laser.laser_multires_forward(to_device(poisoned), to_device(lens), L, w, 0)
    torch.cuda.synchronize()
    assert np.array_equal(to_host_f64(pool), pool_ref)
    assert np.array_equal(to_host_f64(pool_p), pool_ref)
    if r > 0:
        assert np.array_equal(to_host_f64(recent), recent_ref)
    else:
        assert recent is None


def test_multires_after_sta_on_a_reduced_workload():
    """Through the path: H' from the STA kernels, views from the stored H'; lens=None means full histories."""
    import torch
    from workloads.configs import make_workload
    from parity_util import DeviceWorkload
    spec = workloads.CONFIGS["cfg3_high_fanout"].replace(U=2, L=1024 + 128)
    wl = make_workload(spec)
    dw = DeviceWorkload(wl)
    seg, cnt = laser.laser_sta_forward(dw.q, dw.k, dw.v, dw.lens, spec.w, spec.gamma)
    pool, recent = laser.laser_multires_forward(seg, dw.lens, spec.L, spec.w, 4)
    pool_n, _ = laser.laser_multires_forward(seg, None, spec.L, spec.w, 0)
    torch.cuda.synchronize()
    Hs = to_host_f64(seg)
    pool_ref, recent_ref = oracle.multires_forward(Hs, cnt.cpu().numpy(), 4)
    assert np.array_equal(to_host_f64(pool), pool_ref) and np.array_equal(to_host_f64(recent), recent_ref)
    full = np.full_like(cnt.cpu().numpy(), 1)
    assert np.array_equal(to_host_f64(pool_n), oracle.multires_forward(Hs, full, 0)[0])


@pytest.mark.parametrize("name,over,r", [
    ("cfg3_high_fanout", dict(U=2, L=1024 + 128), 3),      # bf16, M = 1: the views come out of the GSTA kernel
    ("cfg2_bf16", dict(U=6), 16),                          # same, d = 64, r = S, ragged lengths
    ("cfg5_lifelong", dict(U=1, L=2 * 256 + 16), 2),       # M = 2: third launch
    ("cfg1_tiny_f32", dict(), 5),                          # fp32: third launch
    ("cfg4_low_fanout", dict(U=48), 1),                    # one candidate per user, short histories
])
def test_whole_path_with_all_views(name, over, r):
    import torch
    from workloads.configs import make_workload
    from parity_util import DeviceWorkload
    spec = workloads.CONFIGS[name].replace(**over)
    wl = make_workload(spec)
    dw = DeviceWorkload(wl)
    print(f"case {spec}", flush=True)
    seg, cnt, z, pool, recent = laser.laser_forward_multires(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens,
                                                             spec.w, spec.gamma, r)
    seg0, cnt0, z0 = laser.laser_forward(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.w, spec.gamma)
    torch.cuda.synchronize()
    assert torch.equal(seg, seg0) and torch.equal(cnt, cnt0) and torch.equal(z, z0)   # same kernels, same bits
    pool_ref, recent_ref = oracle.multires_forward(to_host_f64(seg), cnt.cpu().numpy(), r)
    assert np.array_equal(to_host_f64(pool), pool_ref)
    assert np.array_equal(to_host_f64(recent), recent_ref)


@pytest.mark.parametrize("name,over,r", [
    ("cfg3_high_fanout", dict(U=2, L=1024 + 128), 3),      # one-kernel form: the views come out of the GSTA kernel
    ("cfg3_high_fanout", dict(U=2, C=40, L=1000, w=10), 8),   # 100 segments: split form, views from its streaming kernel
    ("cfg2_bf16", dict(U=5, C=9, L=2048, w=16), 128),      # split form, d = 64, r = S, ragged lengths (some rows invalid)
    ("cfg3_high_fanout", dict(U=3, C=5, L=1000, w=10), 100),  # split form, r = S, few pairs
    ("cfg5_lifelong", dict(U=1, L=2 * 256 + 16), 2),       # M = 2: the views take a launch of their own
    ("cfg1_tiny_f32", dict(), 5),                          # fp32: the same
])
def test_gsta_with_views_from_a_stored_h(name, over, r):
    """laser_gsta_forward_multires = laser_gsta_forward + laser_multires_forward on the same H', bit for bit, and the
    views equal to the checker's (they are exact). H' is made by STA and, so that rows without a valid item hold
    something other than zeros where lengths are ragged, left as STA wrote it (zeros there) in one run and filled
    with a marker in those rows in a second: `recent` copies rows as stored, `pool` and GSTA must not see them."""
    import torch
    from workloads.configs import make_workload
    from parity_util import DeviceWorkload
    spec = workloads.CONFIGS[name].replace(**over)
    wl = make_workload(spec)
    dw = DeviceWorkload(wl)
    print(f"case {spec} r {r}", flush=True)
    seg, cnt = laser.laser_sta_forward(dw.q, dw.k, dw.v, dw.lens, spec.w, spec.gamma)
    for marker in (False, True):
        if marker:
            seg = seg.clone()
            seg[(cnt == 0)[:, None, :].expand(-1, spec.C, -1)] = 3.0
        z, pool, recent = laser.laser_gsta_forward_multires(seg, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.L, spec.w, r)
        z0 = laser.laser_gsta_forward(seg, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.L, spec.w)
        pool0, recent0 = laser.laser_multires_forward(seg, dw.lens, spec.L, spec.w, r)
        torch.cuda.synchronize()
        assert torch.equal(z, z0) and torch.equal(pool, pool0) and torch.equal(recent, recent0)
        pool_ref, _ = oracle.multires_forward(to_host_f64(seg), cnt.cpu().numpy(), r)
        assert np.array_equal(to_host_f64(pool), pool_ref)
        assert torch.equal(recent, seg[:, :, :r])
