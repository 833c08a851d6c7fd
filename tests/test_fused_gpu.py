"""GPU parity of the fused path (H' never stored: laser_forward with seg_out = NULL, laser_forward_fused with and
without a work buffer) against the fp64 checker's laser_forward, element by element, on reduced copies of the
benchmark workloads and on the edge cases of the method; against the two-launch path everywhere; bit-identical run to
run; and at the full size of the many-candidates workload (sampled pairs against the checker, every element against
the two-launch path). Tolerances as everywhere (1e-5 fp32, 2e-2 bf16 per output vector, the element-wise figure
beside it); the two GPU paths, each within the tolerance of the exact result, may differ by twice that."""
import numpy as np
import pytest

import oracle
import workloads
from workloads.configs import WorkloadSpec, make_workload

from parity_util import (ELEM_TOL, TOL, DeviceWorkload, elem_rel_err, oracle_batch, oracle_pair, to_device, to_host_f64,
                         vec_rel_err)

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")

C = workloads.CONFIGS
REDUCED = {
    "cfg1": C["cfg1_tiny_f32"],                                            # fp32: the generic fused kernel
    "cfg2": C["cfg2_bf16"].replace(U=6),                                   # 64 candidates, d = 64: two waves
    "cfg3": C["cfg3_high_fanout"].replace(U=2, L=1024 + 128),              # 256 candidates, d = 128: two tiles of four waves
    "cfg4": C["cfg4_low_fanout"].replace(U=48),                            # one candidate per user: the streaming kernel
}
def _spec(dtype, U, Cn, L, d, dq, w, seed):
    return WorkloadSpec(f"fused_edge_{seed}", dtype, U=U, C=Cn, L=L, d=d, d_q=dq, w=w, M=1, lens_kind="full", seed=seed)


EDGE = {
    "ragged_and_empty": (_spec("bf16", 5, 40, 700, 64, 64, 100, 31), [700, 1, 0, 399, 100]),
    "short_segments": (_spec("bf16", 3, 33, 250, 128, 32, 10, 32), [250, 95, 7]),      # w = 10: not a tile multiple
    "many_candidates_tail": (_spec("bf16", 2, 257, 300, 128, 64, 64, 33), [300, 65]),  # three candidate tiles, one nearly empty
    "one_segment": (_spec("bf16", 2, 16, 96, 64, 128, 128, 34), None),                 # w > L
    "odd_widths_f32": (_spec("f32", 3, 5, 130, 48, 24, 16, 35), [130, 50, 0]),         # the generic kernel
    "bf16_other_widths": (_spec("bf16", 2, 6, 90, 96, 40, 32, 36), [90, 33]),          # bf16 on the generic kernel
    # few candidates per user with long segments: the streaming kernel with the layer as its epilogue
    "stream_three_candidates": (_spec("bf16", 5, 3, 1500, 128, 64, 300, 37), [1500, 301, 300, 7, 0]),
    "stream_eight_candidates": (_spec("bf16", 3, 8, 700, 64, 128, 128, 38), [700, 129, 128]),
    "stream_two_wide": (_spec("bf16", 2, 2, 520, 128, 128, 256, 39), [520, 257]),
    # few candidates with short segments: not the streaming form (the matrix-core kernel takes them)
    "few_candidates_short_segments": (_spec("bf16", 3, 2, 200, 64, 64, 10, 40), [200, 95, 0]),
}


def _build(name):
    if name in REDUCED:
        return make_workload(REDUCED[name]), False
    spec, lens = EDGE[name]
    wl = make_workload(spec)
    if lens is not None:
        wl.lens = np.array(lens, dtype=np.int32)
    return wl, spec.dtype == "bf16"


@pytest.fixture(scope="module")
def cases():
    cache = {}

    def get(name):
        if name not in cache:
            wl, poison = _build(name)
            ref = oracle_batch(wl)
            if poison:   # the checker has its expected values: now poison what must never be read
                for r, n in enumerate(wl.lens):
                    wl.k[r, n:] = np.uint16(0x7FC0)
                    wl.v[r, n:] = np.uint16(0x7FC0)
            cache[name] = (wl, DeviceWorkload(wl), ref)
        return cache[name]
    return get


def _fused_all_ways(dw):
    """z by the three ways into the fused kernels: laser_forward with seg_out NULL, laser_forward_fused without and
    with a work buffer (which cuts histories into runs when there are few users)."""
    s = dw.spec
    args = (dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, s.w, s.gamma)
    none, cnt0, z0 = laser.laser_forward(*args, want_seg=False)
    assert none is None
    cnt1, z1 = laser.laser_forward_fused(*args, use_work=False)
    # with a work buffer, poisoned first: where histories are cut into runs every partial result must be written
    import torch
    from paper_2602_11562_amd import binding
    U, Cn, dq = dw.q.shape
    need = binding.load_library().laser_forward_fused_work_bytes(U, Cn, dw.k.shape[1], dq, dw.v.shape[2], s.w,
                                                                  binding.LASER_BF16 if s.dtype == "bf16" else binding.LASER_F32)
    work = torch.full((max(need, 16) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    cnt2, z2 = laser.laser_forward_fused(*args, work=work)
    torch.cuda.synchronize()
    if need:
        assert not torch.isnan(work[: need // 4]).any(), "a partial result of a run was not written"
    return (cnt0, z0), (cnt1, z1), (cnt2, z2)


@pytest.mark.parametrize("name", list(REDUCED) + list(EDGE))
def test_fused_matches_checker(cases, name):
    import torch
    wl, dw, (Hp_ref, cnt_ref, z_ref) = cases(name)
    s = wl.spec
    tol, etol = TOL[s.dtype], ELEM_TOL[s.dtype]
    print(f"case {name}: {s}", flush=True)
    ways = _fused_all_ways(dw)
    seg, cnt, z_two = laser.laser_forward(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, s.w, s.gamma)
    torch.cuda.synchronize()
    assert torch.equal(ways[0][1], ways[1][1])          # seg_out NULL is the fused entry point without a work buffer
    for label, (cnt_f, z_f) in zip(("one run per user", "same, fused entry point", "runs + merge"), ways):
        assert np.array_equal(cnt_f.cpu().numpy(), cnt_ref), label
        zf = to_host_f64(z_f)
        e, el = vec_rel_err(zf, z_ref), elem_rel_err(zf, z_ref)
        e2 = vec_rel_err(zf, to_host_f64(z_two))
        print(f"  {label}: z err {e:.3e} (element-wise {el:.3e}); against the two-launch path {e2:.3e}", flush=True)
        assert e <= tol and el <= etol and e2 <= 2 * tol, label
    # users without a valid item: z is t0, exactly
    empty = np.asarray(wl.lens) == 0
    if empty.any():
        t0 = to_host_f64(dw.t0)
        for _, z_f in ways:
            assert np.array_equal(to_host_f64(z_f)[empty], t0[empty])


def test_fused_is_bit_identical_run_to_run(cases):
    import torch
    for name in ("cfg1", "cfg2", "cfg3", "cfg4", "ragged_and_empty"):
        wl, dw, _ = cases(name)
        a, b = _fused_all_ways(dw), _fused_all_ways(dw)
        torch.cuda.synchronize()
        for (ca, za), (cb, zb) in zip(a, b):
            assert torch.equal(za.view(torch.int32), zb.view(torch.int32)) and torch.equal(ca, cb)


def test_fused_with_a_sharp_softmax(cases):
    """The default weights give a nearly uniform softmax over segments; W_q scaled up makes it sharp (a few segments
    take all the weight), which is what tells a wrong maximum, scale or merge apart."""
    import torch
    wl, dw, _ = cases("cfg3")
    s = wl.spec
    wq_sharp = (wl.f64("wq") * 50.0)
    wq_bits = workloads.f32_to_bf16_bits(wq_sharp.astype(np.float32))
    wq_dev = to_device(wq_bits)
    wq_val = workloads.bf16_bits_to_f32(wq_bits).astype(np.float64)
    Hp_ref, cnt_ref, z_ref = oracle.laser_forward(wl.f64("q"), wl.f64("k"), wl.f64("v"), wl.f64("t0"), wq_val,
                                                  wl.f64("wk"), wl.f64("wv"), wl.lens, s.w, s.gamma)
    args = (dw.q, dw.k, dw.v, dw.t0, wq_dev, dw.wk, dw.wv, dw.lens, s.w, s.gamma)
    for use_work in (False, True):
        _, z = laser.laser_forward_fused(*args, use_work=use_work)
        torch.cuda.synchronize()
        e = vec_rel_err(to_host_f64(z), z_ref)
        print(f"  sharp softmax, work buffer {use_work}: z err {e:.3e}", flush=True)
        assert e <= TOL[s.dtype]


def test_fused_refuses_what_it_does_not_take(cases):
    import torch
    wl, dw, _ = cases("cfg2")
    s = wl.spec
    two_layers = torch.cat([dw.wq, dw.wq])
    with pytest.raises(laser.LaserError) as e:      # a second layer needs H' again
        laser.laser_forward(dw.q, dw.k, dw.v, dw.t0, two_layers, two_layers, two_layers, dw.lens, s.w, s.gamma,
                            want_seg=False)
    assert e.value.code == 4
    with pytest.raises(laser.LaserError) as e:      # work buffer too small
        laser.laser_forward_fused(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, s.w, s.gamma,
                                  work=torch.zeros(64, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 2


@pytest.mark.timeout(900)
def test_fused_at_full_size_of_the_many_candidates_workload():
    """cfg3 at its full size, through laser_forward_fused with its work buffer (the launch bench.py times) and through
    laser_forward with seg_out NULL: 192 sampled pairs against the checker, every element against the two-launch path,
    a second call bit-identical."""
    import torch
    spec = workloads.CONFIGS["cfg3_high_fanout"]
    wl = make_workload(spec)
    dw = DeviceWorkload(wl)
    args = (dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.w, spec.gamma)
    cnt, z = laser.laser_forward_fused(*args)
    cnt_b, z_b = laser.laser_forward_fused(*args)
    _, cnt_n, z_n = laser.laser_forward(*args, want_seg=False)
    _, _, z_two = laser.laser_forward(*args)
    torch.cuda.synchronize()
    print("case cfg3_high_fanout: fused launches done", flush=True)
    assert torch.equal(z.view(torch.int32), z_b.view(torch.int32)) and torch.equal(cnt, cnt_b)
    assert np.array_equal(cnt.cpu().numpy(), oracle.segment_counts(wl.lens, spec.L, spec.w)) and torch.equal(cnt, cnt_n)
    zh, znh, z2h = to_host_f64(z), to_host_f64(z_n), to_host_f64(z_two)
    rng = np.random.default_rng(spec.seed + 78)
    pairs = {(0, 0), (spec.U - 1, spec.C - 1), (0, spec.C - 1), (spec.U - 1, 0)}
    while len(pairs) < 192:
        pairs.add((int(rng.integers(spec.U)), int(rng.integers(spec.C))))
    worst = worst_n = 0.0
    for (u, c) in sorted(pairs):
        _, z_ref = oracle_pair(wl, u, c)
        worst = max(worst, vec_rel_err(zh[u, c], z_ref), elem_rel_err(zh[u, c], z_ref) * TOL["bf16"] / ELEM_TOL["bf16"])
        worst_n = max(worst_n, vec_rel_err(znh[u, c], z_ref))
    e_all, e_all_n = vec_rel_err(zh, z2h), vec_rel_err(znh, z2h)
    print(f"  192 sampled pairs against the checker: {worst:.3e} (runs + merge), {worst_n:.3e} (one run per user); "
          f"every element against the two-launch path: {e_all:.3e}, {e_all_n:.3e}", flush=True)
    assert worst <= TOL["bf16"] and worst_n <= TOL["bf16"]
    assert e_all <= 2 * TOL["bf16"] and e_all_n <= 2 * TOL["bf16"]
