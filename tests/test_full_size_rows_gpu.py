"""GPU parity at full size for the entry points around the hot path, in the launch configurations bench.py times.

As in test_full_size_gpu.py the checker cannot produce every output, so each entry point is checked on a seeded sample
computed one by one by the fp64 checker and, element by element, against an independent kernel of the library (the
generic or the one-item-per-wave form, themselves checked against the checker at reduced sizes): two results that are
each within the tolerance of the exact one differ by at most twice the tolerance.
Shapes: the benchmark shape (cfg3: 32 users x 256 candidates, L = 4096, d = 128, w = 128) for the projections and the
GSTA backward pass; the paper's training setting (2048 users x 1 target, L = 1000, w = 10, 2 heads x 16, d = 128) for
heads, the folded form, the softmax variant and the STA backward pass. Inputs are seeded normal values generated on the
device (bf16), read back where the checker needs them."""
import math
import os

import numpy as np
import pytest

import oracle

from parity_util import TOL, to_host_f64, vec_rel_err

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")


def _rand(gen, *shape, scale=1.0):
    import torch
    return (torch.randn(*shape, device="cuda", generator=gen) * scale).bfloat16()


def _paper(seed=2602):
    import torch
    U, C, L, din, dq, d, w, heads = 2048, 1, 1000, 128, 32, 128, 10, 2
    gen = torch.Generator(device="cuda").manual_seed(seed)
    t, H = _rand(gen, U, C, din), _rand(gen, U, L, din)
    Wq, Wk, Wv = (_rand(gen, din, n, scale=1 / math.sqrt(din)) for n in (dq, dq, d))
    lens = torch.randint(0, L + 1, (U,), device="cuda", dtype=torch.int32, generator=gen)
    lens[:4] = torch.tensor([L, 0, 1, 9], dtype=torch.int32)
    return dict(U=U, C=C, L=L, din=din, dq=dq, d=d, w=w, heads=heads, t=t, H=H, Wq=Wq, Wk=Wk, Wv=Wv, lens=lens,
                gamma=math.sqrt(dq / heads))


@pytest.mark.timeout(600)
def test_projections_at_the_benchmark_size():
    import torch
    gen = torch.Generator(device="cuda").manual_seed(31)
    U, L, din, dq, d = 32, 4096, 128, 128, 128
    H = _rand(gen, U, L, din)
    Wk, Wv = _rand(gen, din, dq, scale=1 / math.sqrt(din)), _rand(gen, din, d, scale=1 / math.sqrt(din))
    K, V = laser.laser_project_kv_forward(H, Wk, Wv)
    Kg, Vg = laser.laser_project_kv_forward(H, Wk, Wv, variant=laser.PROJECT_GENERIC)
    torch.cuda.synchronize()
    for a, b in ((K, Kg), (V, Vg)):
        assert vec_rel_err(to_host_f64(a), to_host_f64(b)) <= 2 * TOL["bf16"]
    rng = np.random.default_rng(5)
    rows = [(0, 0), (U - 1, L - 1)] + [(int(rng.integers(U)), int(rng.integers(L))) for _ in range(62)]
    Hh, Wkh, Wvh = to_host_f64(H), to_host_f64(Wk), to_host_f64(Wv)
    Kh, Vh = to_host_f64(K), to_host_f64(V)
    for u, j in rows:
        assert vec_rel_err(Kh[u, j], oracle.project_rows(Hh[u, j], Wkh)) <= TOL["bf16"]
        assert vec_rel_err(Vh[u, j], oracle.project_rows(Hh[u, j], Wvh)) <= TOL["bf16"]


@pytest.mark.timeout(900)
def test_heads_folded_form_and_softmax_at_the_paper_setting():
    import torch
    p = _paper()
    U, L, w, heads, gamma = p["U"], p["L"], p["w"], p["heads"], p["gamma"]
    Q = laser.laser_project_q_forward(p["t"], p["Wq"])
    K, V = laser.laser_project_kv_forward(p["H"], p["Wk"], p["Wv"])
    seg, cnt = laser.laser_sta_forward(Q, K, V, p["lens"], w, gamma, heads=heads)
    seg_g, _ = laser.laser_sta_forward(Q, K, V, p["lens"], w, gamma, heads=heads, variant=laser.STA_GENERIC, want_cnt=False)
    soft, _ = laser.laser_sta_forward(Q, K, V, p["lens"], w, gamma, heads=heads, softmax=True, want_cnt=False)
    soft_g, _ = laser.laser_sta_forward(Q, K, V, p["lens"], w, gamma, heads=heads, softmax=True, variant=laser.STA_GENERIC,
                                        want_cnt=False)
    A = laser.laser_fold_query_weights(p["Wq"], p["Wk"], heads)
    fold, cnt_f = laser.laser_sta_folded_forward(p["t"], p["H"], A, p["Wv"], p["lens"], w, gamma, heads)
    torch.cuda.synchronize()
    lens_h = p["lens"].cpu().numpy()
    assert np.array_equal(cnt.cpu().numpy(), oracle.segment_counts(lens_h, L, w)) and torch.equal(cnt, cnt_f)
    segh = to_host_f64(seg)
    assert vec_rel_err(segh, to_host_f64(seg_g)) <= 2 * TOL["bf16"]
    assert vec_rel_err(to_host_f64(soft), to_host_f64(soft_g)) <= 2 * TOL["bf16"]
    assert vec_rel_err(to_host_f64(fold), segh) <= 2 * TOL["bf16"]        # two routes to the same H'
    Qh, Kh, Vh, softh = to_host_f64(Q), to_host_f64(K), to_host_f64(V), to_host_f64(soft)
    rng = np.random.default_rng(6)
    users = [0, 1, 2, 3, U - 1, int(np.argmax(lens_h))] + [int(rng.integers(U)) for _ in range(10)]
    for u in users:
        ref = oracle.sta_pair_heads(Qh[u, 0], Kh[u], Vh[u], int(lens_h[u]), w, gamma, heads)
        assert vec_rel_err(segh[u, 0], ref) <= TOL["bf16"], u
        ref = oracle.sta_pair_softmax(Qh[u, 0], Kh[u], Vh[u], int(lens_h[u]), w, gamma, heads)
        assert vec_rel_err(softh[u, 0], ref) <= TOL["bf16"], u


@pytest.mark.timeout(900)
def test_two_heads_and_softmax_on_the_matrix_cores_at_the_ranking_size():
    """Ranking at the paper's dimensions (64 users x 256 candidates, L = 1000, w = 10, 2 heads x 16, d = 128: the shape
    bench.py --project times): the matrix-core kernel with eight waves and two tile buffers against the generic kernel
    on every element, and against the checker on sampled pairs; sigmoid gates and the softmax variant."""
    import torch
    U, C, L, dq, d, w, heads = 64, 256, 1000, 32, 128, 10, 2
    gen = torch.Generator(device="cuda").manual_seed(2603)
    Q, K, V = _rand(gen, U, C, dq), _rand(gen, U, L, dq), _rand(gen, U, L, d)
    lens = torch.randint(200, L + 1, (U,), device="cuda", dtype=torch.int32, generator=gen)
    lens[:4] = torch.tensor([L, 0, 1, 11], dtype=torch.int32)
    gamma = math.sqrt(dq / heads)
    lens_h = lens.cpu().numpy()
    Qh, Kh, Vh = to_host_f64(Q), to_host_f64(K), to_host_f64(V)
    rng = np.random.default_rng(8)
    pairs = [(0, 0), (1, 5), (2, C - 1), (3, 17), (U - 1, C - 1)] + [(int(rng.integers(U)), int(rng.integers(C))) for _ in range(11)]
    for softmax in (False, True):
        print(f"softmax {softmax}", flush=True)
        seg, cnt = laser.laser_sta_forward(Q, K, V, lens, w, gamma, heads=heads, softmax=softmax)
        seg_m, _ = laser.laser_sta_forward(Q, K, V, lens, w, gamma, heads=heads, softmax=softmax,
                                           variant=laser.STA_MFMA, want_cnt=False)
        seg_g, _ = laser.laser_sta_forward(Q, K, V, lens, w, gamma, heads=heads, softmax=softmax,
                                           variant=laser.STA_GENERIC, want_cnt=False)
        assert torch.equal(seg, seg_m)                 # the matrix-core kernel is the one chosen for this shape
        torch.cuda.synchronize()
        assert np.array_equal(cnt.cpu().numpy(), oracle.segment_counts(lens_h, L, w))
        segh = to_host_f64(seg)
        assert vec_rel_err(segh, to_host_f64(seg_g)) <= 2 * TOL["bf16"]
        assert not segh[1].any()                       # no valid item: exact zeros
        one = oracle.sta_pair_softmax if softmax else oracle.sta_pair_heads
        for u, c in pairs:
            ref = one(Qh[u, c], Kh[u], Vh[u], int(lens_h[u]), w, gamma, heads)
            assert vec_rel_err(segh[u, c], ref) <= TOL["bf16"], (u, c)


@pytest.mark.timeout(900)
def test_sta_backward_at_the_paper_setting():
    import torch
    p = _paper(seed=77)
    U, L, w, gamma, dq, d = p["U"], p["L"], p["w"], math.sqrt(p["dq"]), p["dq"], p["d"]
    gen = torch.Generator(device="cuda").manual_seed(78)
    Q, K, V = _rand(gen, U, 1, dq), _rand(gen, U, L, dq), _rand(gen, U, L, d)
    dseg = _rand(gen, U, 1, L // w, d)
    wide = laser.laser_sta_backward(Q, K, V, p["lens"], dseg, w, gamma)
    os.environ["LASER_BWD_NARROW"] = "1"          # the one-item-per-wave kernel on the same inputs
    try:
        narrow = laser.laser_sta_backward(Q, K, V, p["lens"], dseg, w, gamma)
    finally:
        del os.environ["LASER_BWD_NARROW"]
    torch.cuda.synchronize()
    for nm, a, b in zip(("dq", "dk", "dv"), wide, narrow):
        a, b = to_host_f64(a), to_host_f64(b)
        if nm == "dk":
            a, b = a.reshape(U, -1), b.reshape(U, -1)
        assert vec_rel_err(a, b) <= 2e-5, nm
    lens_h = p["lens"].cpu().numpy()
    Qh, Kh, Vh, gh = to_host_f64(Q), to_host_f64(K), to_host_f64(V), to_host_f64(dseg)
    got = [to_host_f64(x) for x in wide]
    rng = np.random.default_rng(8)
    for u in [0, 1, 2, 3, U - 1] + [int(rng.integers(U)) for _ in range(5)]:
        ref = oracle.sta_backward(Qh[u:u + 1], Kh[u:u + 1], Vh[u:u + 1], lens_h[u:u + 1], w, gamma, gh[u:u + 1])
        assert vec_rel_err(got[0][u], ref[0][0]) <= 1e-5, u
        assert vec_rel_err(got[1][u].reshape(1, -1), ref[1].reshape(1, -1)) <= 1e-5, u
        assert vec_rel_err(got[2][u], ref[2][0]) <= 1e-5, u


@pytest.mark.timeout(900)
def test_gsta_backward_at_the_benchmark_size():
    import torch
    gen = torch.Generator(device="cuda").manual_seed(91)
    U, C, L, w, d = 32, 256, 4096, 128, 128
    S = L // w
    lens = torch.full((U,), L, dtype=torch.int32, device="cuda")
    lens[1], lens[2], lens[3] = 0, 1, 2000
    cnt = oracle.segment_counts(lens.cpu().numpy(), L, w)
    valid = torch.from_numpy(cnt > 0).cuda()
    seg = (_rand(gen, U, C, S, d).float() * valid[:, None, :, None]).bfloat16()     # empty segments are zero, as STA leaves them
    t0 = _rand(gen, U, C, d)
    W = [_rand(gen, 1, d, d, scale=1 / math.sqrt(d)) for _ in range(3)]
    dz = torch.randn(U, C, d, device="cuda", generator=gen)
    dseg, dt0, dwq, dwk, dwv = laser.laser_gsta_backward(seg, t0, *W, lens, dz, L, w)
    torch.cuda.synchronize()
    segh, t0h, dzh = to_host_f64(seg), to_host_f64(t0), to_host_f64(dz)
    Wh = [to_host_f64(x) for x in W]
    dsegh, dt0h = to_host_f64(dseg), to_host_f64(dt0)
    # every pair through the checker (a few seconds): the weight gradients need them all
    sums = [np.zeros((1, d, d)) for _ in range(3)]
    worst = [0.0, 0.0]
    for u in range(U):
        for c in range(C):
            ref = oracle.gsta_pair_backward(segh[u, c], t0h[u, c], *Wh, cnt[u] > 0, dzh[u, c])
            for acc, g in zip(sums, ref[2:]):
                acc += g
            if (u * C + c) % 37 == 0 or u < 4 and c < 2:
                worst[0] = max(worst[0], vec_rel_err(dsegh[u, c], ref[0]))
                worst[1] = max(worst[1], vec_rel_err(dt0h[u, c], ref[1]))
    print(f"  dseg {worst[0]:.2e} dt0 {worst[1]:.2e}", flush=True)
    assert worst[0] <= TOL["bf16"] and worst[1] <= 1e-5
    for nm, a, b in zip(("dwq", "dwk", "dwv"), (dwq, dwk, dwv), sums):
        err = vec_rel_err(to_host_f64(a).reshape(1, -1), b.reshape(1, -1))
        print(f"  {nm} {err:.2e}", flush=True)
        assert err <= 1e-5, nm
