"""GPU parity at the full benchmark sizes, through the entry point and launch configuration that bench.py times.

The checker cannot produce every output of these workloads in reasonable time, so each one is checked three ways:
  * segment counts against the checker, bit-exact (they are cheap at any size);
  * a seeded sample of 192 (user, candidate) pairs, H'[u,c,:,:] and z[u,c,:] computed one by one by the fp64 checker
    (first/last user and candidate, the shortest and the longest history, the rest drawn at random);
  * every element of H' and z against the generic kernels (plain fp32 loops, one thread per output element, checked
    against the checker element by element at the reduced sizes): two independent kernels that are each within
    the tolerance of the exact result differ by at most twice the tolerance. This is the test that sees a fault
    confined to particular rows, segments or workgroups of the tuned kernels, which a sample may miss.
"""
import numpy as np
import pytest

import oracle
import workloads
from workloads.configs import make_workload

from parity_util import ELEM_TOL, TOL, DeviceWorkload, elem_rel_err, oracle_pair, to_host_f64, vec_rel_err

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")

FULL = ["cfg2_bf16", "cfg3_high_fanout", "cfg4_low_fanout", "cfg5_lifelong"]
N_SAMPLES = 192     # the checker takes one to a few milliseconds per pair at these sizes


def _sample_pairs(spec, lens):
    rng = np.random.default_rng(spec.seed + 77)
    pairs = {(0, 0), (spec.U - 1, spec.C - 1), (0, spec.C - 1), (spec.U - 1, 0),
             (int(np.argmin(lens)), spec.C // 2), (int(np.argmax(lens)), spec.C // 3)}
    while len(pairs) < N_SAMPLES:
        pairs.add((int(rng.integers(spec.U)), int(rng.integers(spec.C))))
    return sorted(pairs)


@pytest.fixture(scope="module", params=FULL)
def full(request):
    import torch
    spec = workloads.CONFIGS[request.param]
    print(f"generating {spec}", flush=True)
    wl = make_workload(spec)
    dw = DeviceWorkload(wl)
    print("  uploaded", flush=True)
    yield wl, dw
    del dw
    torch.cuda.empty_cache()


@pytest.mark.timeout(900)
def test_whole_path_at_full_size(full):
    import torch
    wl, dw = full
    s = wl.spec
    tol = TOL[s.dtype]
    seg, cnt, z = laser.laser_forward(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, s.w, s.gamma)
    torch.cuda.synchronize()
    print(f"case {s.name}: laser_forward done", flush=True)
    assert np.array_equal(cnt.cpu().numpy(), oracle.segment_counts(wl.lens, s.L, s.w))

    seg_h, z_h = to_host_f64(seg), to_host_f64(z)
    worst_seg = worst_z = worst_el = 0.0
    for (u, c) in _sample_pairs(s, wl.lens):
        Hp_ref, z_ref = oracle_pair(wl, u, c)
        worst_seg = max(worst_seg, vec_rel_err(seg_h[u, c], Hp_ref))
        worst_z = max(worst_z, vec_rel_err(z_h[u, c], z_ref))
        worst_el = max(worst_el, elem_rel_err(seg_h[u, c], Hp_ref), elem_rel_err(z_h[u, c], z_ref))
    print(f"  {N_SAMPLES} sampled pairs against the checker: H' err {worst_seg:.3e}  z err {worst_z:.3e}  "
          f"element-wise {worst_el:.3e}", flush=True)
    assert worst_seg <= tol and worst_z <= tol and worst_el <= ELEM_TOL[s.dtype]

    seg_g, cnt_g = laser.laser_sta_forward(dw.q, dw.k, dw.v, dw.lens, s.w, s.gamma, variant=1)
    z_g = laser.laser_gsta_forward(seg_g, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, s.L, s.w, variant=1)
    torch.cuda.synchronize()
    assert torch.equal(cnt, cnt_g)
    e_seg = vec_rel_err(seg_h, to_host_f64(seg_g))
    e_z = vec_rel_err(z_h, to_host_f64(z_g))
    print(f"  every element against the generic kernels: H' err {e_seg:.3e}  z err {e_z:.3e}", flush=True)
    assert e_seg <= 2 * tol and e_z <= 2 * tol


@pytest.mark.timeout(900)
def test_sta_alone_at_full_size(full):
    """The standalone STA entry point (its H' stores carry the non-temporal hint: a different kernel instance)."""
    import torch
    wl, dw = full
    s = wl.spec
    tol = TOL[s.dtype]
    seg, cnt = laser.laser_sta_forward(dw.q, dw.k, dw.v, dw.lens, s.w, s.gamma)
    seg_g, cnt_g = laser.laser_sta_forward(dw.q, dw.k, dw.v, dw.lens, s.w, s.gamma, variant=1)
    torch.cuda.synchronize()
    assert np.array_equal(cnt.cpu().numpy(), oracle.segment_counts(wl.lens, s.L, s.w)) and torch.equal(cnt, cnt_g)
    seg_h = to_host_f64(seg)
    e = vec_rel_err(seg_h, to_host_f64(seg_g))
    print(f"case {s.name}: laser_sta_forward against the generic kernel, every element: {e:.3e}", flush=True)
    assert e <= 2 * tol
    worst = 0.0
    for (u, c) in _sample_pairs(s, wl.lens)[:64]:
        Hp_ref, _ = oracle_pair(wl, u, c)
        worst = max(worst, vec_rel_err(seg_h[u, c], Hp_ref))
    print(f"  sampled pairs against the checker: {worst:.3e}", flush=True)
    assert worst <= tol


@pytest.mark.timeout(900)
def test_all_views_at_full_size(full):
    """laser_forward_multires: z and H' as laser_forward gives them; pool and recent exact against the checker on the
    sampled pairs and, everywhere, equal to the standalone kernel's (two different kernels where GSTA writes them)."""
    import torch
    wl, dw = full
    s = wl.spec
    r = min(4, s.S)
    seg, cnt, z, pool, recent = laser.laser_forward_multires(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens,
                                                             s.w, s.gamma, r)
    seg0, cnt0, z0 = laser.laser_forward(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, s.w, s.gamma)
    pool1, recent1 = laser.laser_multires_forward(seg, dw.lens, s.L, s.w, r)
    torch.cuda.synchronize()
    print(f"case {s.name}: laser_forward_multires done", flush=True)
    assert torch.equal(seg, seg0) and torch.equal(cnt, cnt0) and torch.equal(z, z0)
    assert torch.equal(pool.float(), pool1.float()) and torch.equal(recent, recent1)   # (as numbers: -0 == +0)
    seg_h = to_host_f64(seg)
    cnt_h = cnt.cpu().numpy()
    pool_h, recent_h = to_host_f64(pool), to_host_f64(recent)
    for (u, c) in _sample_pairs(s, wl.lens):
        p_ref, r_ref = oracle.multires_pair(seg_h[u, c], cnt_h[u] > 0, r)
        assert np.array_equal(pool_h[u, c], p_ref) and np.array_equal(recent_h[u, c], r_ref)
