"""GPU parity of laser_ffn_gsta_forward (segment FFN + LayerNorm feeding GSTA, Sec. 3.4.2 and 3.4.3).

Three references:
  * the fp64 checker chained as the header defines the result: segment_ffn_forward on the stored H', its result
    rounded to the storage type once, gsta_forward on that (bf16: 2e-2 per vector as for the two steps apart; the
    GPU's s and the checker's rounded s can differ by one bf16 step in single components);
  * the library's own two calls in a row (laser_segment_ffn_forward, then laser_gsta_forward): the transformed rows
    must hold the same bits (same arithmetic), z may differ by the order of fp32 sums only (1e-5, sharp softmax 1e-4);
  * itself: s wanted or not, in place or not, twice in a row -> the same bits in z.
H' rows of segments without a valid item are filled with NaN patterns before the call: nothing of them may reach s or z.
"""
import math

import numpy as np
import pytest

import oracle
import workloads

from parity_util import to_device, to_host_f64, vec_rel_err

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")


def _store(x, dtype):
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        bits = workloads.f32_to_bf16_bits(x)
        return bits, workloads.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


def _case(dtype, U, C, L, w, d, dff, M, lens, seed, sharp=1.0):
    rng = np.random.default_rng(seed)
    S = -(-L // w)
    cs = dict(S=S, lens=np.array(lens, dtype=np.int32))
    H = rng.normal(size=(U, C, S, d))
    cs["Hs"], cs["Hv"] = _store(H, dtype)
    cs["W1s"], cs["W1v"] = _store(rng.normal(size=(d, dff)) / math.sqrt(d), dtype)
    cs["W2s"], cs["W2v"] = _store(rng.normal(size=(dff, d)) / math.sqrt(dff), dtype)
    f32 = lambda x: np.asarray(x, dtype=np.float32)
    cs["b1"], cs["b2"] = f32(rng.normal(size=dff) * 0.3), f32(rng.normal(size=d) * 0.3)
    cs["g"], cs["b"] = f32(1.0 + 0.2 * rng.normal(size=d)), f32(0.1 * rng.normal(size=d))
    cs["t0s"], cs["t0v"] = _store(rng.normal(size=(U, C, d)) / math.sqrt(d), dtype)
    cs["wqs"], cs["wqv"] = _store(rng.normal(size=(M, d, d)) / math.sqrt(d) * sharp, dtype)
    cs["wks"], cs["wkv"] = _store(rng.normal(size=(M, d, d)) / math.sqrt(d), dtype)
    cs["wvs"], cs["wvv"] = _store(rng.normal(size=(M, d, d)) / math.sqrt(d), dtype)
    return cs


def _poison_empty_rows(cs, dtype, L, w):
    """NaN patterns into the stored rows of segments without a valid item (the checker never reads them)."""
    cnt = oracle.segment_counts(cs["lens"], L, w)
    Hs = cs["Hs"].copy()
    for u in range(Hs.shape[0]):
        for i in range(cs["S"]):
            if cnt[u, i] == 0:
                Hs[u, :, i, :] = 0x7fc1 if dtype == "bf16" else np.float32(np.nan)
    return Hs, cnt


def _round_like_storage(x, dtype):
    if dtype == "bf16":
        return workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))).astype(np.float64)
    return np.asarray(x, dtype=np.float32).astype(np.float64)


FUSED = {
    # dtype, U, C, L, w, d, d_ff, M, lens, sharp
    "one_tile_per_pair": ("bf16", 2, 37, 512, 16, 128, 128, 1, [512, 200], 1.0),                 # S = 32
    "few_segments": ("bf16", 3, 11, 1000, 100, 128, 128, 1, [1000, 333, 0], 1.0),               # S = 10
    "two_tiles_per_pair": ("bf16", 5, 9, 640, 16, 128, 64, 1, [640, 512, 520, 5, 0], 1.0),      # S = 40: 32 + 8 rows
    "paper_default_segments": ("bf16", 5, 3, 1000, 10, 128, 128, 1, [1000, 995, 404, 7, 0], 1.0),  # S = 100
    "one_segment": ("bf16", 2, 70, 64, 64, 128, 64, 1, [64, 1], 1.0),                            # S = 1
    "sharp_softmax": ("bf16", 2, 19, 1024, 16, 128, 128, 1, [1024, 700], 40.0),                  # S = 64, peaked weights
    "many_pairs": ("bf16", 9, 257, 256, 32, 128, 128, 1, [256, 1, 256, 33, 200, 64, 0, 255, 97], 1.0),  # every wave walks pairs
    # more than 2048 pairs: a wave walks several, and its tiles of 32 rows hold the last rows of one pair and the
    # first of the next (S = 5: two whole pairs; S = 20: 20 + 12, 8 + 20, ...; S = 100: 96 + 4 | 28 + ...)
    "packed_tiles_5": ("bf16", 6, 800, 60, 12, 128, 128, 1, [60, 13, 60, 0, 35, 59], 1.0),
    "packed_tiles_20": ("bf16", 5, 1000, 200, 10, 128, 64, 1, [200, 200, 95, 0, 151], 1.0),
    "packed_tiles_100": ("bf16", 3, 750, 1000, 10, 128, 128, 1, [1000, 1000, 637], 1.0),
}
UNFUSED = {
    "f32": ("f32", 2, 7, 512, 64, 64, 128, 1, [512, 65], 1.0),
    "d64": ("bf16", 2, 9, 300, 10, 64, 64, 1, [300, 95], 1.0),
    "two_layers": ("bf16", 2, 9, 512, 16, 128, 128, 2, [512, 100], 1.0),
    "wide_hidden": ("bf16", 1, 9, 512, 16, 128, 256, 1, [300], 1.0),
}


def _run(name, table):
    import torch
    dtype, U, C, L, w, d, dff, M, lens, sharp = table[name]
    cs = _case(dtype, U, C, L, w, d, dff, M, lens, seed=1000 + len(name) * 7 + d, sharp=sharp)
    Hs, cnt = _poison_empty_rows(cs, dtype, L, w)
    eps = 1e-5
    print(f"case {name}", flush=True)
    s_ref = oracle.segment_ffn_forward(cs["Hv"], cnt, cs["W1v"], cs["b1"], cs["W2v"], cs["b2"], cs["g"], cs["b"], eps)
    z_ref = oracle.gsta_forward(_round_like_storage(s_ref, dtype), cs["t0v"], cs["wqv"], cs["wkv"], cs["wvv"], cnt)
    seg = to_device(Hs)
    dev = {k: to_device(cs[k]) for k in ("lens", "W1s", "b1", "W2s", "b2", "g", "b", "t0s", "wqs", "wks", "wvs")}
    call = lambda s_in, **kw: laser.laser_ffn_gsta_forward(
        s_in, dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], dev["lens"], dev["W1s"], dev["b1"], dev["W2s"], dev["b2"],
        dev["g"], dev["b"], L, w, eps, **kw)
    s_out, z = call(seg)
    torch.cuda.synchronize()
    tol = {"f32": 1e-5, "bf16": 2e-2}[dtype]
    err_s = vec_rel_err(to_host_f64(s_out), s_ref)
    err_z = vec_rel_err(to_host_f64(z), z_ref)
    print(f"  against the checker: s {err_s:.3e}  z {err_z:.3e}", flush=True)
    assert err_s <= tol and err_z <= tol
    # the two calls in a row
    s2 = laser.laser_segment_ffn_forward(seg, dev["lens"], dev["W1s"], dev["b1"], dev["W2s"], dev["b2"], dev["g"],
                                         dev["b"], L, w, eps)
    z2 = laser.laser_gsta_forward(s2, dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], dev["lens"], L, w)
    torch.cuda.synchronize()
    bits = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(s_out.view(bits), s2.view(bits)), "transformed rows differ from laser_segment_ffn_forward"
    err_2 = vec_rel_err(to_host_f64(z), to_host_f64(z2))
    print(f"  against the two calls in a row: z {err_2:.3e}", flush=True)
    assert err_2 <= (1e-4 if sharp > 1.0 else 1e-5)
    return cs, seg, z, s_out, call


@pytest.mark.parametrize("name", list(FUSED))
def test_ffn_gsta_one_pass(name):
    import torch
    cs, seg, z, s_out, call = _run(name, FUSED)
    # s not wanted: z from the same arithmetic; z_out poisoned first (every row must be written)
    zp = torch.full_like(z, float("nan"))
    none, z_b = call(seg, want_seg=False, z_out=zp)
    torch.cuda.synchronize()
    assert none is None
    assert torch.equal(z.view(torch.int32), z_b.view(torch.int32))
    # in place, and a second time from the same inputs
    seg_c = seg.clone()
    s_c, z_c = call(seg_c, seg_out=seg_c)
    torch.cuda.synchronize()
    assert torch.equal(z.view(torch.int32), z_c.view(torch.int32))
    assert torch.equal(s_c.view(torch.int16), s_out.view(torch.int16))


@pytest.mark.parametrize("name", list(FUSED) + ["two_layers", "d64"])
@pytest.mark.parametrize("r", [0, 1, 5, "all"])
def test_ffn_gsta_with_views(name, r):
    """laser_ffn_gsta_forward_multires: z as without the views (same bits), max-pool and the most recent rows equal to
    those of laser_gsta_forward_multires on the stored transformed rows (bit for bit: copies and maxima of the same
    stored values) and to the checker's views of its own rounded rows wherever those rows agree."""
    import torch
    table = FUSED if name in FUSED else UNFUSED
    dtype, U, C, L, w, d, dff, M, lens, sharp = table[name]
    cs = _case(dtype, U, C, L, w, d, dff, M, lens, seed=1000 + len(name) * 7 + d, sharp=sharp)
    Hs, cnt = _poison_empty_rows(cs, dtype, L, w)
    rr = cs["S"] if r == "all" else min(r, cs["S"])
    print(f"case {name} r {rr}", flush=True)
    seg = to_device(Hs)
    dev = {k: to_device(cs[k]) for k in ("lens", "W1s", "b1", "W2s", "b2", "g", "b", "t0s", "wqs", "wks", "wvs")}
    args = (dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], dev["lens"], dev["W1s"], dev["b1"], dev["W2s"], dev["b2"],
            dev["g"], dev["b"], L, w, 1e-5)
    s_a, z_a = laser.laser_ffn_gsta_forward(seg, *args)
    s_b, z_b, pool, recent = laser.laser_ffn_gsta_forward(seg, *args, r=rr)
    z2, pool2, recent2 = laser.laser_gsta_forward_multires(s_a, dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], dev["lens"],
                                                           L, w, rr)
    torch.cuda.synchronize()
    assert torch.equal(z_a.view(torch.int32), z_b.view(torch.int32))
    assert torch.equal(s_a.view(torch.int16), s_b.view(torch.int16))
    assert torch.equal(pool.view(torch.int16), pool2.view(torch.int16))
    if rr > 0:
        assert torch.equal(recent.view(torch.int16), recent2.view(torch.int16))
    else:
        assert recent is None
    # the checker's views of the stored rows (exact operations on stored values)
    pool_ref, recent_ref = oracle.multires_forward(to_host_f64(s_a), cnt, rr)
    assert np.array_equal(to_host_f64(pool), pool_ref)
    if rr > 0:
        assert np.array_equal(to_host_f64(recent), recent_ref)
    if name in FUSED:   # rows not wanted: the views and z from the same pass, same bits
        zp = torch.full_like(z_a, float("nan"))
        none, z_c, pool_c, recent_c = laser.laser_ffn_gsta_forward(seg, *args, r=rr, want_seg=False, z_out=zp,
                                                                   pool_out=torch.full_like(pool, float("nan")),
                                                                   recent_out=None if rr == 0 else torch.full_like(recent, float("nan")))
        torch.cuda.synchronize()
        assert none is None
        assert torch.equal(z_a.view(torch.int32), z_c.view(torch.int32))
        assert torch.equal(pool.view(torch.int16), pool_c.view(torch.int16))
        if rr > 0:
            assert torch.equal(recent.view(torch.int16), recent_c.view(torch.int16))


@pytest.mark.parametrize("name", list(UNFUSED))
def test_ffn_gsta_two_launches_behind_the_same_entry_point(name):
    cs, seg, z, s_out, call = _run(name, UNFUSED)
    with pytest.raises(laser.LaserError) as e:   # no kernel takes both steps here, and there is nowhere to put s
        call(seg, want_seg=False)
    assert e.value.code == 4


def test_ffn_gsta_full_size_high_fanout():
    """32 users x 256 candidates, 32 segments of d = 128 (the shape of the benchmark's H'): every z against the two
    calls in a row, 96 sampled pairs against the checker."""
    import torch
    dtype, U, C, L, w, d, dff, M = "bf16", 32, 256, 4096, 128, 128, 128, 1
    lens = [4096] * 20 + [4095, 3000, 129, 128, 127, 1, 0, 2048, 2049, 4000, 777, 4096]
    cs = _case(dtype, U, C, L, w, d, dff, M, lens, seed=77)
    Hs, cnt = _poison_empty_rows(cs, dtype, L, w)
    seg = to_device(Hs)
    dev = {k: to_device(cs[k]) for k in ("lens", "W1s", "b1", "W2s", "b2", "g", "b", "t0s", "wqs", "wks", "wvs")}
    _, z = laser.laser_ffn_gsta_forward(seg, dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], dev["lens"], dev["W1s"],
                                        dev["b1"], dev["W2s"], dev["b2"], dev["g"], dev["b"], L, w, 1e-5, want_seg=False)
    s2 = laser.laser_segment_ffn_forward(seg, dev["lens"], dev["W1s"], dev["b1"], dev["W2s"], dev["b2"], dev["g"],
                                         dev["b"], L, w, 1e-5)
    z2 = laser.laser_gsta_forward(s2, dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], dev["lens"], L, w)
    torch.cuda.synchronize()
    zh = to_host_f64(z)
    err_2 = vec_rel_err(zh, to_host_f64(z2))
    print(f"full size against the two calls in a row: z {err_2:.3e}", flush=True)
    assert err_2 <= 1e-5
    rng = np.random.default_rng(5)
    worst = 0.0
    for _ in range(96):
        u, c = int(rng.integers(U)), int(rng.integers(C))
        s_ref = oracle.segment_ffn_forward(cs["Hv"][u:u + 1, c:c + 1], cnt[u:u + 1], cs["W1v"], cs["b1"], cs["W2v"],
                                           cs["b2"], cs["g"], cs["b"], 1e-5)
        z_ref = oracle.gsta_forward(_round_like_storage(s_ref, dtype), cs["t0v"][u:u + 1, c:c + 1], cs["wqv"], cs["wkv"],
                                    cs["wvv"], cnt[u:u + 1])
        worst = max(worst, vec_rel_err(zh[u:u + 1, c:c + 1], z_ref))
    print(f"full size against the checker (96 pairs): z {worst:.3e}", flush=True)
    assert worst <= 2e-2


def test_ffn_gsta_without_lengths_and_with_a_single_pair():
    """lens = NULL means every item is valid; one pair leaves seven waves of the workgroup without work."""
    import torch
    for (U, C, L, w, dff) in ((1, 1, 320, 8, 128), (2, 3, 96, 8, 64)):
        cs = _case("bf16", U, C, L, w, 128, dff, 1, [L] * U, seed=31 + C)
        cnt = oracle.segment_counts(cs["lens"], L, w)
        s_ref = oracle.segment_ffn_forward(cs["Hv"], cnt, cs["W1v"], cs["b1"], cs["W2v"], cs["b2"], cs["g"], cs["b"], 1e-5)
        z_ref = oracle.gsta_forward(_round_like_storage(s_ref, "bf16"), cs["t0v"], cs["wqv"], cs["wkv"], cs["wvv"], cnt)
        dev = {k: to_device(cs[k]) for k in ("Hs", "W1s", "b1", "W2s", "b2", "g", "b", "t0s", "wqs", "wks", "wvs")}
        s_out, z = laser.laser_ffn_gsta_forward(dev["Hs"], dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], None, dev["W1s"],
                                                dev["b1"], dev["W2s"], dev["b2"], dev["g"], dev["b"], L, w, 1e-5)
        torch.cuda.synchronize()
        assert vec_rel_err(to_host_f64(s_out), s_ref) <= 2e-2
        assert vec_rel_err(to_host_f64(z), z_ref) <= 2e-2


def test_ffn_gsta_seeded_random_shapes():
    """Twenty-four seeded shapes (users, candidates, segment counts from one tile's worth to several, ragged lengths with
    empty histories, both hidden sizes, with and without the views): every z and every transformed row against the
    checker, the views against the checker's views of the stored rows."""
    import torch
    rng = np.random.default_rng(20260211)
    worst = 0.0
    for case in range(24):
        U, C = int(rng.integers(1, 5)), int(rng.integers(1, 41))
        w = int(rng.choice([1, 3, 8, 10, 16]))
        S = int(rng.choice([1, 2, 7, 31, 32, 33, 40, 64, 65, 100, 130]))
        L = S * w - int(rng.integers(0, w))            # last segment short
        dff = int(rng.choice([64, 128]))
        lens = [int(x) for x in rng.integers(0, L + 1, size=U)]
        if case % 5 == 0:
            lens[0] = L
        r = int(rng.integers(0, S + 1)) if case % 2 == 0 else None
        print(f"case {case}: U {U} C {C} L {L} w {w} S {S} d_ff {dff} lens {lens} r {r}", flush=True)
        cs = _case("bf16", U, C, L, w, 128, dff, 1, lens, seed=500 + case)
        assert cs["S"] == S
        Hs, cnt = _poison_empty_rows(cs, "bf16", L, w)
        s_ref = oracle.segment_ffn_forward(cs["Hv"], cnt, cs["W1v"], cs["b1"], cs["W2v"], cs["b2"], cs["g"], cs["b"], 1e-5)
        z_ref = oracle.gsta_forward(_round_like_storage(s_ref, "bf16"), cs["t0v"], cs["wqv"], cs["wkv"], cs["wvv"], cnt)
        dev = {k: to_device(cs[k]) for k in ("lens", "W1s", "b1", "W2s", "b2", "g", "b", "t0s", "wqs", "wks", "wvs")}
        out = laser.laser_ffn_gsta_forward(to_device(Hs), dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], dev["lens"],
                                           dev["W1s"], dev["b1"], dev["W2s"], dev["b2"], dev["g"], dev["b"], L, w, 1e-5, r=r)
        torch.cuda.synchronize()
        s_out, z = out[0], out[1]
        err_s, err_z = vec_rel_err(to_host_f64(s_out), s_ref), vec_rel_err(to_host_f64(z), z_ref)
        worst = max(worst, err_s, err_z)
        assert err_s <= 2e-2 and err_z <= 2e-2, (case, err_s, err_z)
        if r is not None:
            pool_ref, recent_ref = oracle.multires_forward(to_host_f64(s_out), cnt, r)
            assert np.array_equal(to_host_f64(out[2]), pool_ref), case
            if r > 0:
                assert np.array_equal(to_host_f64(out[3]), recent_ref), case
    print(f"worst vector-relative error {worst:.3e}", flush=True)


def test_ffn_gsta_seeded_random_shapes_many_pairs():
    """Eight seeded shapes with several thousand pairs, so that every wave walks two to five of them and packs their
    valid rows into shared tiles (pairs of different users, hence of different valid lengths, meet in a tile): z, the
    transformed rows and the views against the checker."""
    import torch
    rng = np.random.default_rng(20260212)
    for case in range(8):
        U = int(rng.integers(2, 7))
        C = int(rng.integers(2100 // U + 1, 6000 // U))
        w = int(rng.choice([4, 10]))
        S = int(rng.choice([3, 7, 16, 20, 33, 50]))
        L = S * w - int(rng.integers(0, w))
        dff = int(rng.choice([64, 128]))
        lens = [int(x) for x in rng.integers(0, L + 1, size=U)]
        lens[case % U] = L
        r = int(rng.integers(0, S + 1)) if case % 2 == 0 else None
        print(f"case {case}: U {U} C {C} L {L} w {w} S {S} d_ff {dff} lens {lens} r {r}", flush=True)
        cs = _case("bf16", U, C, L, w, 128, dff, 1, lens, seed=900 + case)
        Hs, cnt = _poison_empty_rows(cs, "bf16", L, w)
        s_ref = oracle.segment_ffn_forward(cs["Hv"], cnt, cs["W1v"], cs["b1"], cs["W2v"], cs["b2"], cs["g"], cs["b"], 1e-5)
        z_ref = oracle.gsta_forward(_round_like_storage(s_ref, "bf16"), cs["t0v"], cs["wqv"], cs["wkv"], cs["wvv"], cnt)
        dev = {k: to_device(cs[k]) for k in ("lens", "W1s", "b1", "W2s", "b2", "g", "b", "t0s", "wqs", "wks", "wvs")}
        out = laser.laser_ffn_gsta_forward(to_device(Hs), dev["t0s"], dev["wqs"], dev["wks"], dev["wvs"], dev["lens"],
                                           dev["W1s"], dev["b1"], dev["W2s"], dev["b2"], dev["g"], dev["b"], L, w, 1e-5, r=r)
        torch.cuda.synchronize()
        s_out, z = out[0], out[1]
        err_s, err_z = vec_rel_err(to_host_f64(s_out), s_ref), vec_rel_err(to_host_f64(z), z_ref)
        assert err_s <= 2e-2 and err_z <= 2e-2, (case, err_s, err_z)
        # every pair on its own as well: a vector-relative error over the whole batch would hide one wrong pair
        zh = to_host_f64(z).reshape(-1, 128)
        zr = np.asarray(z_ref).reshape(-1, 128)
        per_pair = np.linalg.norm(zh - zr, axis=1) / np.maximum(np.linalg.norm(zr, axis=1), 1e-30)
        assert per_pair.max() <= 2e-2, (case, int(per_pair.argmax()), float(per_pair.max()))
        if r is not None:
            pool_ref, recent_ref = oracle.multires_forward(to_host_f64(s_out), cnt, r)
            assert np.array_equal(to_host_f64(out[2]), pool_ref), case
            if r > 0:
                assert np.array_equal(to_host_f64(out[3]), recent_ref), case
