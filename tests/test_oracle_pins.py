"""Pins for the fp64 checker: it is compared with things other than itself.

  P1  brute force written here element by element with math.exp (no numpy arithmetic)
  P2  the paper's own equivalence: per-segment loop (Sec. 3.4.2) == global gates + reshape + bmm (Sec. 3.5.1)
  P3  invariants that follow from the STA equation: permutation inside a segment, locality, silence,
      single segment == plain gated target attention
  P4  closed forms (Q=0 -> half-sum, V=1 -> sum of gates, saturated gates -> sum pooling, W_q=0 -> mean, ...)
  P5  reduction to library routines (torch softmax / scaled_dot_product_attention, scipy expit)
  P6  exact re-association of the GSTA products
  P8  planted mistakes in the checker are caught by P1 (shows the pins have teeth)
"""
import math
import types

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from oracle import laser_oracle as lo


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


# --------------------------------------------------------------------------- P1
def brute_force(q, k, v, t0, wq, wk, wv, lens, w, gamma):
    """Every output element from scalar Python arithmetic; follows Sec. 3.4.2 / 3.4.3 directly."""
    U, C, dq = len(q), len(q[0]), len(q[0][0])
    L, d = len(v[0]), len(v[0][0])
    M = len(wq)
    S = (L + w - 1) // w
    Hp = [[[[0.0] * d for _ in range(S)] for _ in range(C)] for _ in range(U)]
    cnt = [[0] * S for _ in range(U)]
    z = [[[0.0] * d for _ in range(C)] for _ in range(U)]
    for u in range(U):
        for i in range(S):
            cnt[u][i] = sum(1 for j in range(i * w, min((i + 1) * w, L)) if j < lens[u])
        for c in range(C):
            for i in range(S):
                for j in range(i * w, min((i + 1) * w, L)):
                    if j >= lens[u]:
                        continue
                    e = sum(q[u][c][a] * k[u][j][a] for a in range(dq)) / gamma
                    g = 1.0 / (1.0 + math.exp(-e))
                    for b in range(d):
                        Hp[u][c][i][b] += g * v[u][j][b]
            t = list(t0[u][c])
            for l in range(M):
                segs = [i for i in range(S) if cnt[u][i] > 0]
                if not segs:
                    continue
                qp = [sum(t[a] * wq[l][a][b] for a in range(d)) for b in range(d)]
                sc = []
                vals = []
                for i in segs:
                    kp = [sum(Hp[u][c][i][a] * wk[l][a][b] for a in range(d)) for b in range(d)]
                    vp = [sum(Hp[u][c][i][a] * wv[l][a][b] for a in range(d)) for b in range(d)]
                    sc.append(sum(qp[b] * kp[b] for b in range(d)) / math.sqrt(d))
                    vals.append(vp)
                mx = max(sc)
                ex = [math.exp(s - mx) for s in sc]
                den = sum(ex)
                for b in range(d):
                    t[b] = t[b] + sum(ex[n] / den * vals[n][b] for n in range(len(segs)))
            z[u][c] = t
    return np.array(Hp), np.array(cnt), np.array(z)


TINY = [
    # U, C, L, w, dq, d, M, lens
    (1, 2, 5, 2, 3, 2, 2, [4]),        # short last segment + one masked tail item
    (2, 3, 7, 3, 2, 4, 1, [7, 2]),     # second user: only first segment (partly) valid
    (2, 1, 6, 6, 4, 3, 3, [0, 6]),     # one user with no history at all; single segment
    (1, 2, 9, 4, 5, 5, 2, [9]),        # full length, L % w != 0
]


def _tiny_inputs(case, seed):
    U, C, L, w, dq, d, M, lens = case
    q = _rand((U, C, dq), seed + 1)
    k = _rand((U, L, dq), seed + 2)
    v = _rand((U, L, d), seed + 3)
    t0 = _rand((U, C, d), seed + 4)
    wq = _rand((M, d, d), seed + 5, 0.8)
    wk = _rand((M, d, d), seed + 6, 0.8)
    wv = _rand((M, d, d), seed + 7, 0.8)
    return q, k, v, t0, wq, wk, wv, np.array(lens), w


@pytest.mark.parametrize("case", TINY)
@pytest.mark.parametrize("gamma", [1.0, 1.7])
def test_p1_brute_force(case, gamma):
    q, k, v, t0, wq, wk, wv, lens, w = _tiny_inputs(case, 11)
    Hb, cb, zb = brute_force(q.tolist(), k.tolist(), v.tolist(), t0.tolist(), wq.tolist(), wk.tolist(),
                             wv.tolist(), lens.tolist(), w, gamma)
    Ho, co, zo = oracle.laser_forward(q, k, v, t0, wq, wk, wv, lens, w, gamma)
    assert np.array_equal(cb, co)
    np.testing.assert_allclose(Ho, Hb, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(zo, zb, rtol=1e-11, atol=1e-12)


def test_segment_counts_by_enumeration():
    for L, w in [(10, 3), (8, 4), (7, 10), (1, 1), (10000, 256), (33, 32)]:
        lens = np.minimum(np.array([0, 1, w - 1 if w > 1 else 0, w, w + 1, L - 1, L]), L)
        cnt = oracle.segment_counts(lens, L, w)
        S = oracle.num_segments(L, w)
        assert cnt.shape == (len(lens), S)
        for u, n in enumerate(lens):
            exp = [sum(1 for j in range(i * w, min((i + 1) * w, L)) if j < n) for i in range(S)]
            assert cnt[u].tolist() == exp
            assert cnt[u].sum() == n
    # out-of-range lengths are clamped to [0, L]
    assert oracle.segment_counts([-3, 99], 8, 4).tolist() == [[0, 0], [4, 4]]


# --------------------------------------------------------------------------- P2
@pytest.mark.parametrize("L,w,n", [(64, 8, 64), (70, 8, 70), (70, 8, 37), (50, 64, 50), (33, 1, 20)])
def test_p2_naive_equals_global_reshape_form(L, w, n):
    dq, d = 6, 10
    Q, K, V = _rand(dq, 1), _rand((L, dq), 2), _rand((L, d), 3)
    a = oracle.sta_pair(Q, K, V, n, w, 1.3)
    b = oracle.sta_pair_global(Q, K, V, n, w, 1.3)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-13)


# --------------------------------------------------------------------------- P3
def test_p3_permutation_inside_a_segment_leaves_output_unchanged():
    L, w, dq, d = 48, 16, 5, 7
    Q, K, V = _rand(dq, 4), _rand((L, dq), 5), _rand((L, d), 6)
    base = oracle.sta_pair(Q, K, V, L, w, 2.0)
    perm = np.arange(L)
    perm[16:32] = 16 + np.random.default_rng(0).permutation(16)
    out = oracle.sta_pair(Q, K[perm], V[perm], L, w, 2.0)
    np.testing.assert_allclose(out, base, rtol=1e-12, atol=1e-13)
    # a permutation that moves items ACROSS segments must change the result (the test can fail)
    perm2 = np.arange(L)
    perm2[[0, 40]] = [40, 0]
    out2 = oracle.sta_pair(Q, K[perm2], V[perm2], L, w, 2.0)
    assert np.abs(out2 - base).max() > 1e-3


def test_p3_perturbing_one_segment_changes_only_that_segment():
    L, w, dq, d = 40, 8, 4, 6
    Q, K, V = _rand(dq, 7), _rand((L, dq), 8), _rand((L, d), 9)
    base = oracle.sta_pair(Q, K, V, L, w, 1.0)
    K2, V2 = K.copy(), V.copy()
    K2[16:24] += 1.0
    V2[16:24] *= -2.0
    out = oracle.sta_pair(Q, K2, V2, L, w, 1.0)
    changed = np.abs(out - base).max(axis=1) > 0
    assert changed.tolist() == [False, False, True, False, False]


def test_p3_gate_driven_to_zero_silences_the_segment():
    L, w, dq, d = 24, 8, 4, 5
    Q, K, V = _rand(dq, 10), _rand((L, dq), 11), _rand((L, d), 12)
    qhat = Q / np.linalg.norm(Q)
    K[8:16] = -200.0 * qhat
    out = oracle.sta_pair(Q, K, V, L, w, 1.0)
    assert np.abs(out[1]).max() < 1e-30
    assert np.abs(out[0]).max() > 1e-2 and np.abs(out[2]).max() > 1e-2


def test_p3_single_segment_is_plain_gated_target_attention():
    L, dq, d = 30, 6, 4
    Q, K, V = _rand(dq, 13), _rand((L, dq), 14), _rand((L, d), 15)
    for w in (30, 31, 1000):
        out = oracle.sta_pair(Q, K, V, L, w, 1.5)
        assert out.shape == (1, d)
        ref = scipy.special.expit(Q @ K.T / 1.5) @ V
        np.testing.assert_allclose(out[0], ref, rtol=1e-13, atol=1e-14)


# --------------------------------------------------------------------------- P4
def test_p4_zero_query_gives_half_sum():
    L, w, dq, d = 20, 6, 3, 4
    K, V = _rand((L, dq), 16), _rand((L, d), 17)
    n = 15
    out = oracle.sta_pair(np.zeros(dq), K, V, n, w, 1.0)
    for i in range(4):
        lo, hi = i * w, min((i + 1) * w, n)
        np.testing.assert_allclose(out[i], 0.5 * V[lo:hi].sum(0) if hi > lo else 0.0, rtol=1e-14, atol=1e-15)


def test_p4_unit_values_give_sum_of_gates_and_gamma_divides_the_score():
    L, w, dq, d = 12, 4, 3, 5
    Q, K = _rand(dq, 18), _rand((L, dq), 19)
    gamma = 2.5
    out = oracle.sta_pair(Q, K, np.ones((L, d)), L, w, gamma)
    for i in range(3):
        g = sum(1.0 / (1.0 + math.exp(-float(Q @ K[j]) / gamma)) for j in range(i * w, (i + 1) * w))
        np.testing.assert_allclose(out[i], g, rtol=1e-14)


def test_p4_saturated_gates_give_sum_pooling():
    L, w, dq, d = 16, 8, 4, 3
    Q = _rand(dq, 20)
    K = np.tile(100.0 * Q / (Q @ Q), (L, 1))
    V = _rand((L, d), 21)
    out = oracle.sta_pair(Q, K, V, L, w, 1.0)
    np.testing.assert_allclose(out, V.reshape(2, 8, d).sum(1), rtol=1e-13, atol=1e-13)


def test_p4_gsta_closed_forms():
    S, d, M = 6, 5, 3
    Hp, t = _rand((S, d), 22), _rand(d, 23)
    Wq, Wk, Wv = _rand((M, d, d), 24), _rand((M, d, d), 25), _rand((M, d, d), 26)
    valid = np.array([True, True, True, True, False, False])
    # W_q = 0 -> uniform softmax -> o_l = mean over valid segments of H' W_v^l; residuals add up
    z = oracle.gsta_pair(Hp, t, np.zeros_like(Wq), Wk, Wv, valid)
    np.testing.assert_allclose(z, t + sum(Hp[:4].mean(0) @ Wv[l] for l in range(M)), rtol=1e-13, atol=1e-13)
    # exactly one valid segment -> a = 1 -> z = t + sum_l H'_0 W_v^l
    one = np.array([True] + [False] * 5)
    z = oracle.gsta_pair(Hp, t, Wq, Wk, Wv, one)
    np.testing.assert_allclose(z, t + sum(Hp[0] @ Wv[l] for l in range(M)), rtol=1e-13, atol=1e-13)
    # W_v = 0 -> z = t ; no valid segment -> z = t
    np.testing.assert_array_equal(oracle.gsta_pair(Hp, t, Wq, Wk, np.zeros_like(Wv), valid), t)
    np.testing.assert_array_equal(oracle.gsta_pair(Hp, t, Wq, Wk, Wv, np.zeros(S, bool)), t)
    # invalid segments never matter, whatever they hold
    Hp2 = Hp.copy()
    Hp2[4:] = 1e6
    np.testing.assert_array_equal(oracle.gsta_pair(Hp2, t, Wq, Wk, Wv, valid),
                                  oracle.gsta_pair(Hp, t, Wq, Wk, Wv, valid))


def test_p4_empty_history_gives_zero_segments_and_z_equals_t():
    q, k, v = _rand((1, 2, 3), 27), _rand((1, 9, 3), 28), _rand((1, 9, 4), 29)
    t0 = _rand((1, 2, 4), 30)
    W = _rand((2, 4, 4), 31)
    Hp, cnt, z = oracle.laser_forward(q, k, v, t0, W, W, W, np.array([0]), 4, 1.0)
    assert not Hp.any() and not cnt.any()
    np.testing.assert_array_equal(z, t0)


# --------------------------------------------------------------------------- P5
@pytest.mark.parametrize("sharp", [1.0, 30.0])
def test_p5_one_gsta_layer_is_masked_single_query_sdpa(sharp):
    S, d = 9, 8
    Hp, t = _rand((S, d), 32), _rand(d, 33)
    Wq, Wk, Wv = _rand((1, d, d), 34) * sharp, _rand((1, d, d), 35), _rand((1, d, d), 36)
    valid = np.array([True] * 6 + [False] * 3)
    z = oracle.gsta_pair(Hp, t, Wq, Wk, Wv, valid)
    tq = torch.from_numpy(t @ Wq[0]).reshape(1, 1, 1, d)
    tk = torch.from_numpy(Hp @ Wk[0]).reshape(1, 1, S, d)
    tv = torch.from_numpy(Hp @ Wv[0]).reshape(1, 1, S, d)
    mask = torch.from_numpy(valid).reshape(1, 1, 1, S)
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=1.0 / math.sqrt(d))
    np.testing.assert_allclose(z, t + o.reshape(d).numpy(), rtol=1e-12, atol=1e-12)
    # and the explicit softmax call
    logits = torch.from_numpy((Hp[:6] @ Wk[0]) @ (t @ Wq[0]) / math.sqrt(d))
    a = torch.softmax(logits, dim=0).numpy()
    np.testing.assert_allclose(z, t + a @ (Hp[:6] @ Wv[0]), rtol=1e-12, atol=1e-12)


def test_p5_sigmoid_matches_library_expit_over_a_wide_range():
    x = np.concatenate([np.linspace(-700, 700, 4001), _rand(1000, 37, 5.0)])
    np.testing.assert_allclose(oracle.sigmoid(x), scipy.special.expit(x), rtol=4e-16, atol=0)
    assert oracle.sigmoid(np.array([0.0]))[0] == 0.5


def test_p5_batch_sta_with_one_segment_is_two_matmuls_and_expit():
    U, C, L, dq, d = 2, 3, 17, 4, 6
    q, k, v = _rand((U, C, dq), 38), _rand((U, L, dq), 39), _rand((U, L, d), 40)
    Hp, cnt = oracle.sta_forward(q, k, v, None, L, 2.0)
    ref = scipy.special.expit(np.einsum("uca,uja->ucj", q, k) / 2.0) @ v
    np.testing.assert_allclose(Hp[:, :, 0], ref, rtol=1e-13, atol=1e-13)
    assert cnt.tolist() == [[L], [L]]


# --------------------------------------------------------------------------- P6
def test_p6_gsta_products_can_be_reassociated():
    S, d = 12, 16
    Hp, t = _rand((S, d), 41), _rand(d, 42)
    Wq, Wk, Wv = _rand((d, d), 43), _rand((d, d), 44), _rand((d, d), 45)
    e1 = (Hp @ Wk) @ (t @ Wq)
    e2 = Hp @ (Wk @ (t @ Wq))
    np.testing.assert_allclose(e1, e2, rtol=1e-12, atol=1e-12)
    a = scipy.special.softmax(e1 / math.sqrt(d))
    np.testing.assert_allclose(a @ (Hp @ Wv), (a @ Hp) @ Wv, rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------------- P8
def _p1_error(monkeypatch_fn):
    """max abs difference between (possibly sabotaged) checker and the brute force over the tiny cases."""
    worst = 0.0
    for case in TINY:
        q, k, v, t0, wq, wk, wv, lens, w = _tiny_inputs(case, 11)
        Hb, cb, zb = brute_force(q.tolist(), k.tolist(), v.tolist(), t0.tolist(), wq.tolist(), wk.tolist(),
                                 wv.tolist(), lens.tolist(), w, 1.7)
        Ho, co, zo = lo.laser_forward(q, k, v, t0, wq, wk, wv, lens, w, 1.7)
        worst = max(worst, np.abs(Ho - Hb).max(), np.abs(zo - zb).max(), float(np.abs(co - cb).max()))
    return worst


def test_p8_planted_mistakes_are_caught(monkeypatch):
    assert _p1_error(None) < 1e-11
    real_sigmoid, real_sqrt, real_segment, real_gsta = lo.sigmoid, math.sqrt, lo.sta_segment, lo.gsta_pair

    mutants = {
        "softmax instead of sigmoid": ("sigmoid", lambda x: np.exp(x - x.max()) / np.exp(x - x.max()).sum()),
        "sign of the score": ("sigmoid", lambda x: real_sigmoid(-x)),
        "gamma dropped": ("sta_segment", lambda Q, K, V, g: real_segment(Q, K, V, 1.0)),
        "gamma multiplies": ("sta_segment", lambda Q, K, V, g: real_segment(Q, K, V, 1.0 / g)),
        "transposed W_q": ("gsta_pair", lambda H, t, a, b, c, m: real_gsta(H, t, a.transpose(0, 2, 1), b, c, m)),
        "transposed W_v": ("gsta_pair", lambda H, t, a, b, c, m: real_gsta(H, t, a, b, c.transpose(0, 2, 1), m)),
        "W_k and W_v swapped": ("gsta_pair", lambda H, t, a, b, c, m: real_gsta(H, t, a, c, b, m)),
        "residual dropped": ("gsta_pair", lambda H, t, a, b, c, m: real_gsta(H, t, a, b, c, m) - t),
        "mask ignored in GSTA": ("gsta_pair", lambda H, t, a, b, c, m: real_gsta(H, t, a, b, c, np.ones_like(m))),
    }
    for name, (attr, fn) in mutants.items():
        with monkeypatch.context() as mp:
            mp.setattr(lo, attr, fn)
            assert _p1_error(None) > 1e-4, f"planted mistake not detected: {name}"
    # scale sqrt(d) -> d
    with monkeypatch.context() as mp:
        mp.setattr(lo, "math", types.SimpleNamespace(sqrt=lambda x: x))
        assert _p1_error(None) > 1e-4
    assert _p1_error(None) < 1e-11


# ------------------------------------------------------------------ multi-resolution views (Sec. 3.4.4)
def _multires_brute(Hp, valid, r):
    """Scalar Python, written independently of the checker: built-in max over the valid rows, row slices."""
    S, d = len(Hp), len(Hp[0])
    rows = [i for i in range(S) if valid[i]]
    pool = [max(Hp[i][e] for i in rows) if rows else 0.0 for e in range(d)]
    recent = [[Hp[i][e] for e in range(d)] for i in range(r)]
    return pool, recent


@pytest.mark.parametrize("S,d,r,nvalid", [(7, 5, 3, 7), (7, 5, 7, 4), (4, 3, 1, 1), (5, 2, 2, 0)])
def test_multires_brute_force(S, d, r, nvalid):
    rng = np.random.default_rng(100 * S + nvalid)
    Hp = rng.normal(size=(S, d))
    valid = np.arange(S) < nvalid            # valid segments are a prefix, as tail padding leaves them
    Hp[~valid] = 0.0                         # what STA stores for segments without a valid item
    pool, recent = lo.multires_pair(Hp, valid, r)
    bp, br = _multires_brute(Hp.tolist(), valid.tolist(), r)
    assert np.array_equal(pool, np.array(bp)) and np.array_equal(recent, np.array(br).reshape(r, d))


def test_multires_closed_forms_and_invariants():
    rng = np.random.default_rng(4242)
    S, d = 9, 6
    Hp = rng.normal(size=(S, d))
    valid = np.ones(S, dtype=bool)
    pool, recent = lo.multires_pair(Hp, valid, S)
    assert np.array_equal(recent, Hp)                                   # r = L': the whole compressed sequence
    assert np.array_equal(pool, Hp.max(axis=0))                         # the library's reduction
    assert np.array_equal(pool, torch.amax(torch.from_numpy(Hp), dim=0).numpy())
    assert (pool >= Hp).all() and all(pool[e] in Hp[:, e] for e in range(d))
    perm = rng.permutation(S)                                           # pooling ignores the order of the segments
    assert np.array_equal(lo.multires_pair(Hp[perm], valid, 1)[0], pool)
    one = np.zeros(S, dtype=bool); one[3] = True                        # a single valid segment pools to itself
    assert np.array_equal(lo.multires_pair(Hp, one, 1)[0], Hp[3])
    neg = -np.abs(Hp) - 1.0                                             # all-negative vectors: a masked zero row must
    neg[5:] = 0.0                                                       # not win the maximum
    pv = lo.multires_pair(neg, np.arange(S) < 5, 2)[0]
    assert (pv < 0).all() and np.array_equal(pv, neg[:5].max(axis=0))
    assert np.array_equal(lo.multires_pair(Hp, np.zeros(S, dtype=bool), 2)[0], np.zeros(d))   # nothing valid: 0


def test_multires_batch_matches_pairs():
    rng = np.random.default_rng(77)
    U, C, S, d, r = 3, 2, 5, 4, 2
    Hp = rng.normal(size=(U, C, S, d))
    cnt = np.array([[3, 3, 3, 3, 1], [3, 2, 0, 0, 0], [0, 0, 0, 0, 0]], dtype=np.int32)
    for u in range(U):
        Hp[u][:, cnt[u] == 0] = 0.0
    pool, recent = oracle.multires_forward(Hp, cnt, r)
    for u in range(U):
        for c in range(C):
            p1, r1 = lo.multires_pair(Hp[u, c], cnt[u] > 0, r)
            assert np.array_equal(pool[u, c], p1) and np.array_equal(recent[u, c], r1)
    assert np.array_equal(pool[2], np.zeros((C, d)))


# ------------------------------------------------------------------ segment FFN + LayerNorm (Sec. 3.4.2)
def _ffn_brute(s, W1, b1, W2, b2, g, b, eps):
    """Scalar Python with math only, written independently of the checker."""
    d, dff = len(s), len(b1)
    hid = [max(0.0, sum(s[e] * W1[e][j] for e in range(d)) + b1[j]) for j in range(dff)]
    x = [sum(hid[j] * W2[j][e] for j in range(dff)) + b2[e] + s[e] for e in range(d)]
    mu = sum(x) / d
    var = sum((t - mu) ** 2 for t in x) / d
    return [(x[e] - mu) / math.sqrt(var + eps) * g[e] + b[e] for e in range(d)]


def _ffn_params(rng, d, dff):
    return (rng.normal(size=(d, dff)) / math.sqrt(d), rng.normal(size=dff) * 0.3, rng.normal(size=(dff, d)) / math.sqrt(dff),
            rng.normal(size=d) * 0.3, 1.0 + 0.2 * rng.normal(size=d), 0.1 * rng.normal(size=d))


@pytest.mark.parametrize("d,dff,eps", [(3, 5, 1e-5), (8, 8, 1e-3), (6, 2, 1e-6)])
def test_segment_ffn_brute_force(d, dff, eps):
    rng = np.random.default_rng(31 * d + dff)
    W1, b1, W2, b2, g, b = _ffn_params(rng, d, dff)
    s = rng.normal(size=d)
    got = lo.segment_ffn_vector(s.copy(), W1, b1, W2, b2, g, b, eps)
    ref = _ffn_brute(s.tolist(), W1.tolist(), b1.tolist(), W2.tolist(), b2.tolist(), g.tolist(), b.tolist(), eps)
    assert np.allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_segment_ffn_matches_library_layers():
    """torch.nn.functional: linear, relu, layer_norm in fp64 (a reduction to library routines)."""
    import torch.nn.functional as F
    rng = np.random.default_rng(5150)
    d, dff, eps = 16, 40, 1e-5
    W1, b1, W2, b2, g, b = _ffn_params(rng, d, dff)
    s = rng.normal(size=(7, d))
    t = lambda x: torch.from_numpy(np.asarray(x, dtype=np.float64))
    y = F.linear(F.relu(F.linear(t(s), t(W1).T, t(b1))), t(W2).T, t(b2)) + t(s)
    ref = F.layer_norm(y, (d,), t(g), t(b), eps).numpy()
    got = np.stack([lo.segment_ffn_vector(s[i].copy(), W1, b1, W2, b2, g, b, eps) for i in range(7)])
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_segment_ffn_closed_forms_and_invariants():
    rng = np.random.default_rng(99)
    d, dff, eps = 12, 20, 1e-5
    W1, b1, W2, b2, g, b = _ffn_params(rng, d, dff)
    s = rng.normal(size=d)
    one, zero = np.ones(d), np.zeros(d)
    # W2 = 0, b2 = 0: FFN vanishes, the step is LN(s)
    y = lo.segment_ffn_vector(s.copy(), W1, b1, np.zeros_like(W2), zero, one, zero, 0.0)
    assert np.allclose(y, (s - s.mean()) / s.std(), rtol=1e-12) and abs(y.mean()) < 1e-12 and abs(y.var() - 1) < 1e-12
    # LN forgets a shift and a positive scale of its input: b2 + const, and (with eps = 0) x -> a x
    y0 = lo.segment_ffn_vector(s.copy(), W1, b1, W2, b2, g, b, 0.0)
    assert np.allclose(lo.segment_ffn_vector(s.copy(), W1, b1, W2, b2 + 3.7, g, b, 0.0), y0, rtol=1e-10, atol=1e-12)
    # relu: with b1 very negative every hidden unit is off, FFN(s) = b2
    yoff = lo.segment_ffn_vector(s.copy(), W1, b1 - 1e6, W2, b2, one, zero, eps)
    x = s + b2
    assert np.allclose(yoff, (x - x.mean()) / np.sqrt(x.var() + eps), rtol=1e-12)
    # with b1 very positive every unit is on: the network is affine, FFN(s) = (s W1 + b1) W2 + b2
    big = 1e3
    yon = lo.segment_ffn_vector(s.copy(), W1, b1 + big, W2, b2, one, zero, eps)
    x = (s @ W1 + b1 + big) @ W2 + b2 + s
    assert np.allclose(yon, (x - x.mean()) / np.sqrt(x.var() + eps), rtol=1e-10)
    # gain and bias act after the normalisation, component by component
    assert np.allclose(lo.segment_ffn_vector(s.copy(), W1, b1, W2, b2, 2 * g, b + 1, eps),
                       2 * (lo.segment_ffn_vector(s.copy(), W1, b1, W2, b2, g, b, eps) - b) + b + 1, rtol=1e-12)


def test_segment_ffn_batch_leaves_empty_segments_zero():
    rng = np.random.default_rng(123)
    U, C, S, d, dff = 2, 3, 4, 6, 9
    W1, b1, W2, b2, g, b = _ffn_params(rng, d, dff)
    Hp = rng.normal(size=(U, C, S, d))
    cnt = np.array([[5, 5, 2, 0], [1, 0, 0, 0]], dtype=np.int32)
    out = oracle.segment_ffn_forward(Hp, cnt, W1, b1, W2, b2, g, b, 1e-5)
    for u in range(U):
        for i in range(S):
            for c in range(C):
                if cnt[u, i] > 0:
                    assert np.array_equal(out[u, c, i], lo.segment_ffn_vector(Hp[u, c, i].copy(), W1, b1, W2, b2, g, b, 1e-5))
                else:
                    assert np.array_equal(out[u, c, i], np.zeros(d))


# ------------------------------------------------------------------ projections (Sec. 3.5.1)
def test_projection_brute_force_and_selectors():
    rng = np.random.default_rng(77)
    X, W = rng.normal(size=(5, 4)), rng.normal(size=(4, 7))
    ref = [[sum(X[i][e] * W[e][j] for e in range(4)) for j in range(7)] for i in range(5)]
    assert np.allclose(lo.project_rows(X, W), ref, rtol=1e-13, atol=1e-14)
    assert np.array_equal(lo.project_rows(X, np.eye(4)), X)                      # identity matrix
    assert np.array_equal(lo.project_rows(np.eye(4), W), W)                      # unit rows pick the rows of W
    a, b = 1.7, -0.3                                                             # linear in the rows
    X2 = rng.normal(size=(5, 4))
    assert np.allclose(lo.project_rows(a * X + b * X2, W), a * lo.project_rows(X, W) + b * lo.project_rows(X2, W), rtol=1e-12)
    with pytest.raises(ValueError):                                              # a transposed operand is refused
        lo.project_rows(X, W.T)


def test_projection_shapes_and_batch():
    rng = np.random.default_rng(78)
    U, C, L, din, dq, d = 2, 3, 6, 5, 4, 7
    t, H = rng.normal(size=(U, C, din)), rng.normal(size=(U, L, din))
    Wq, Wk, Wv = rng.normal(size=(din, dq)), rng.normal(size=(din, dq)), rng.normal(size=(din, d))
    Q, K, V = oracle.project_qkv(t, H, Wq, Wk, Wv)
    assert Q.shape == (U, C, dq) and K.shape == (U, L, dq) and V.shape == (U, L, d)
    for u in range(U):
        for j in range(L):
            assert np.allclose(K[u, j], [sum(H[u, j, e] * Wk[e, n] for e in range(din)) for n in range(dq)], rtol=1e-12)
            assert np.allclose(V[u, j], [sum(H[u, j, e] * Wv[e, n] for e in range(din)) for n in range(d)], rtol=1e-12)
        for c in range(C):
            assert np.allclose(Q[u, c], [sum(t[u, c, e] * Wq[e, n] for e in range(din)) for n in range(dq)], rtol=1e-12)


def test_projection_then_sta_equals_the_folded_form():
    """q . k_j = t (W_q W_k^T) h_j, and sum_j g_j (h_j W_v) = (sum_j g_j h_j) W_v: STA on the projected tensors equals
    STA run on the raw history with the folded query, projected afterwards (Sec. 3.5.1 with Sec. 3.4.2)."""
    rng = np.random.default_rng(79)
    L, w, n, din, dq, d, gamma = 23, 5, 19, 6, 4, 8, 2.0
    t, H = rng.normal(size=din), rng.normal(size=(L, din))
    Wq, Wk, Wv = rng.normal(size=(din, dq)), rng.normal(size=(din, dq)), rng.normal(size=(din, d))
    direct = lo.sta_pair(lo.project_rows(t, Wq), lo.project_rows(H, Wk), lo.project_rows(H, Wv), n, w, gamma)
    folded_q = lo.project_rows(lo.project_rows(t, Wq), Wk.T)
    folded = lo.project_rows(lo.sta_pair(folded_q, H, H, n, w, gamma), Wv)
    assert np.allclose(direct, folded, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ several heads (Sec. 4.1.2)
def _heads_brute(q, K, V, n, w, gamma, heads):
    """Scalar Python, written independently: every output component from its own head's scores."""
    L, dq, d = len(K), len(q), len(V[0])
    a, b = dq // heads, d // heads
    S = -(-L // w)
    out = [[0.0] * d for _ in range(S)]
    for i in range(S):
        for e in range(d):
            h = e // b
            acc = 0.0
            for j in range(i * w, min((i + 1) * w, L, n)):
                score = sum(q[h * a + x] * K[j][h * a + x] for x in range(a)) / gamma
                acc += V[j][e] / (1.0 + math.exp(-score))
            out[i][e] = acc
    return out


@pytest.mark.parametrize("heads,dq,d", [(1, 4, 6), (2, 4, 6), (3, 6, 3), (2, 2, 8)])
def test_heads_brute_force(heads, dq, d):
    rng = np.random.default_rng(100 * heads + dq)
    L, w, n, gamma = 17, 5, 13, 1.7
    q, K, V = rng.normal(size=dq), rng.normal(size=(L, dq)), rng.normal(size=(L, d))
    got = lo.sta_pair_heads(q, K, V, n, w, gamma, heads)
    assert np.allclose(got, _heads_brute(q.tolist(), K.tolist(), V.tolist(), n, w, gamma, heads), rtol=1e-12, atol=1e-13)


def test_heads_special_cases_and_invariants():
    rng = np.random.default_rng(2026)
    L, w, n, gamma, dq, d = 23, 4, 21, 2.0, 8, 12
    q, K, V = rng.normal(size=dq), rng.normal(size=(L, dq)), rng.normal(size=(L, d))
    assert np.array_equal(lo.sta_pair_heads(q, K, V, n, w, gamma, 1), lo.sta_pair(q, K, V, n, w, gamma))
    base = lo.sta_pair_heads(q, K, V, n, w, gamma, 2)
    # a head sees only its own columns of Q and K, and writes only its own columns of H'
    q2 = q.copy()
    q2[:4] += rng.normal(size=4)
    moved = lo.sta_pair_heads(q2, K, V, n, w, gamma, 2)
    assert np.array_equal(moved[:, 6:], base[:, 6:]) and not np.allclose(moved[:, :6], base[:, :6])
    K2 = K.copy()
    K2[:, 4:] *= -1.0
    moved = lo.sta_pair_heads(q, K2, V, n, w, gamma, 2)
    assert np.array_equal(moved[:, :6], base[:, :6]) and not np.allclose(moved[:, 6:], base[:, 6:])
    # two heads whose query and key columns repeat each other gate alike: the result is the one-head STA of those columns
    qq, KK = np.concatenate([q[:4], q[:4]]), np.concatenate([K[:, :4], K[:, :4]], axis=1)
    assert np.allclose(lo.sta_pair_heads(qq, KK, V, n, w, gamma, 2), lo.sta_pair(q[:4], K[:, :4], V, n, w, gamma), rtol=1e-13)
    # zero query: every gate is one half in every head
    half = lo.sta_pair_heads(np.zeros(dq), K, V, L, w, gamma, 4)
    for i in range(6):
        assert np.allclose(half[i], 0.5 * V[i * w:(i + 1) * w].sum(axis=0), rtol=1e-13)
    with pytest.raises(ValueError):
        lo.sta_pair_heads(q, K, V, n, w, gamma, 3)      # 3 does not divide d_q = 8
    # batch form
    Hb, _ = oracle.sta_forward(q[None, None], K[None], V[None], [n], w, gamma, heads=2)
    assert np.array_equal(Hb[0, 0], base)


# ------------------------------------------------------------------ folded form (Sec. 3.5.1 re-association)
def test_folded_weights_and_head_projection_brute_force():
    rng = np.random.default_rng(404)
    din, dq, d, heads, P, S = 5, 6, 4, 2, 3, 4
    Wq, Wk, Wv = rng.normal(size=(din, dq)), rng.normal(size=(din, dq)), rng.normal(size=(din, d))
    A = lo.fold_query_weights(Wq, Wk, heads)
    a, b = dq // heads, d // heads
    for h in range(heads):
        for r in range(din):
            for k in range(din):
                assert abs(A[r, h * din + k] - sum(Wq[r, h * a + x] * Wk[k, h * a + x] for x in range(a))) < 1e-13
    G = rng.normal(size=(P, heads, S, din))
    out = lo.project_heads(G, Wv, heads)
    for p in range(P):
        for i in range(S):
            for e in range(d):
                assert abs(out[p, i, e] - sum(G[p, e // b, i, k] * Wv[k, e] for k in range(din))) < 1e-13
    # the defining property of A: (t A_h) . x = (t W_q)_h . (x W_k)_h for any t, x
    t, x = rng.normal(size=din), rng.normal(size=din)
    for h in range(heads):
        lhs = (t @ A[:, h * din:(h + 1) * din]) @ x
        rhs = (t @ Wq)[h * a:(h + 1) * a] @ (x @ Wk)[h * a:(h + 1) * a]
        assert abs(lhs - rhs) < 1e-12


@pytest.mark.parametrize("heads", [1, 2, 3])
def test_folded_form_equals_projections_then_sta(heads):
    rng = np.random.default_rng(405 + heads)
    U, C, L, w, din, dq, d, gamma = 2, 3, 19, 4, 5, 6, 12, 1.3
    t, H = rng.normal(size=(U, C, din)), rng.normal(size=(U, L, din))
    Wq, Wk, Wv = rng.normal(size=(din, dq)), rng.normal(size=(din, dq)), rng.normal(size=(din, d))
    lens = [19, 6]
    Q, K, V = oracle.project_qkv(t, H, Wq, Wk, Wv)
    direct, cnt = oracle.sta_forward(Q, K, V, lens, w, gamma, heads=heads)
    folded, cnt2 = oracle.sta_folded_forward(t, H, Wq, Wk, Wv, lens, w, gamma, heads)
    assert np.array_equal(cnt, cnt2)
    assert np.allclose(direct, folded, rtol=1e-11, atol=1e-12)


# ------------------------------------------------------------------ softmax aggregation (ablation of Sec. 4.4.1)
def _softmax_brute(q, K, V, n, w, gamma, heads):
    L, dq, d = len(K), len(q), len(V[0])
    a, b = dq // heads, d // heads
    S = -(-L // w)
    out = [[0.0] * d for _ in range(S)]
    for i in range(S):
        items = range(i * w, min((i + 1) * w, L, n))
        for e in range(d):
            h = e // b
            es = [math.exp(sum(q[h * a + x] * K[j][h * a + x] for x in range(a)) / gamma) for j in items]
            if es:
                out[i][e] = sum(p * V[j][e] for p, j in zip(es, items)) / sum(es)
    return out


@pytest.mark.parametrize("heads", [1, 2])
def test_softmax_variant_brute_force_and_library(heads):
    rng = np.random.default_rng(700 + heads)
    L, w, n, gamma, dq, d = 19, 5, 17, 0.9, 4, 6
    q, K, V = rng.normal(size=dq), rng.normal(size=(L, dq)), rng.normal(size=(L, d))
    got = lo.sta_pair_softmax(q, K, V, n, w, gamma, heads)
    assert np.allclose(got, _softmax_brute(q.tolist(), K.tolist(), V.tolist(), n, w, gamma, heads), rtol=1e-12, atol=1e-13)
    if heads == 1:   # reduction to the library routine, segment by segment
        for i in range(4):
            lo_, hi_ = i * w, min((i + 1) * w, n)
            ref = scipy.special.softmax(K[lo_:hi_] @ q / gamma) @ V[lo_:hi_] if hi_ > lo_ else np.zeros(d)
            assert np.allclose(got[i], ref, rtol=1e-12, atol=1e-13)


def test_softmax_variant_invariants():
    rng = np.random.default_rng(701)
    L, w, gamma, dq, d = 24, 6, 1.1, 5, 7
    q, K, V = rng.normal(size=dq), rng.normal(size=(L, dq)), rng.normal(size=(L, d))
    base = lo.sta_pair_softmax(q, K, V, L, w, gamma)
    # a convex combination of the segment's value rows: inside their range, and rows of ones give ones
    for i in range(4):
        seg = V[i * w:(i + 1) * w]
        assert (base[i] >= seg.min(axis=0) - 1e-12).all() and (base[i] <= seg.max(axis=0) + 1e-12).all()
    assert np.allclose(lo.sta_pair_softmax(q, K, np.ones((L, d)), L, w, gamma), 1.0, rtol=1e-13)
    # zero query: the mean of the valid items (17 valid: the last segment is empty, the third holds 5 items)
    m = lo.sta_pair_softmax(np.zeros(dq), K, V, 17, w, gamma)
    assert np.allclose(m[0], V[:6].mean(axis=0)) and np.allclose(m[2], V[12:17].mean(axis=0)) and not m[3].any()
    # a score shift common to a segment cancels: one more key column that is constant, times any query entry
    K2, q2 = np.concatenate([K, np.full((L, 1), 3.0)], axis=1), np.concatenate([q, [5.0]])
    assert np.allclose(lo.sta_pair_softmax(q2, K2, V, L, w, gamma), base, rtol=1e-11)
    # one item per segment: that item's value, whatever the score; very large scores do not overflow
    assert np.allclose(lo.sta_pair_softmax(q, K, V, L, 1, gamma), V, rtol=1e-13)
    big = lo.sta_pair_softmax(1e4 * q, K, V, L, w, gamma)
    assert np.isfinite(big).all()
    for i in range(4):   # the winner takes all
        j = i * w + int(np.argmax(K[i * w:(i + 1) * w] @ q))
        assert np.allclose(big[i], V[j], rtol=1e-9)
    # differs from the sigmoid form, which is not normalised
    assert not np.allclose(base, lo.sta_pair(q, K, V, L, w, gamma))
    Hb, _ = oracle.sta_forward(q[None, None], K[None], V[None], [L], w, gamma, softmax=True)
    assert np.array_equal(Hb[0, 0], base)


# ------------------------------------------------------------------ ragged candidate counts (packed pairs)
def test_ragged_batch_is_the_dense_batch_repacked():
    rng = np.random.default_rng(811)
    U, C, L, w, dq, d, M, gamma = 3, 4, 21, 5, 4, 6, 2, 1.4
    q, t0 = rng.normal(size=(U, C, dq)), rng.normal(size=(U, C, d))
    k, v = rng.normal(size=(U, L, dq)), rng.normal(size=(U, L, d))
    wq, wk, wv = (rng.normal(size=(M, d, d)) / math.sqrt(d) for _ in range(3))
    lens = [21, 8, 0]
    Hd, cntd, zd = oracle.laser_forward(q, k, v, t0, wq, wk, wv, lens, w, gamma)
    # equal counts: the packed batch is the dense one reshaped
    Hr, cntr, zr = oracle.laser_forward_ragged(q.reshape(U * C, dq), k, v, t0.reshape(U * C, d), wq, wk, wv, lens,
                                               np.arange(U + 1) * C, w, gamma)
    assert np.array_equal(Hr, Hd.reshape(U * C, -1, d)) and np.array_equal(zr, zd.reshape(U * C, d))
    assert np.array_equal(cntr, cntd)
    # unequal counts, a user without candidates: every row equals the dense result of its (user, candidate)
    take = [[0, 2, 3], [], [1]]
    rows = [(u, c) for u in range(U) for c in take[u]]
    off = np.cumsum([0] + [len(t) for t in take])
    qp = np.stack([q[u, c] for u, c in rows])
    tp = np.stack([t0[u, c] for u, c in rows])
    Hr, cntr, zr = oracle.laser_forward_ragged(qp, k, v, tp, wq, wk, wv, lens, off, w, gamma)
    for i, (u, c) in enumerate(rows):
        assert np.array_equal(Hr[i], Hd[u, c]) and np.array_equal(zr[i], zd[u, c])
    assert np.array_equal(cntr, cntd)
    for bad in ([1, 3, 3, 4], [0, 3, 2, 4], [0, 3, 3, 5]):
        with pytest.raises(ValueError):
            oracle.laser_forward_ragged(qp, k, v, tp, wq, wk, wv, lens, bad, w, gamma)


# ------------------------------------------------------------------ STA backward
def _torch_sta(q, k, v, lens, w, gamma):
    """The forward pass in torch fp64 ops, written independently (mask + index_add), for autograd to differentiate."""
    U, C, _ = q.shape
    L, d = v.shape[1], v.shape[2]
    S = -(-L // w)
    seg_of = torch.arange(L) // w
    out = []
    for u in range(U):
        g = torch.sigmoid(q[u] @ k[u].T / gamma) * (torch.arange(L) < int(lens[u])).to(q.dtype)   # [C, L]
        contrib = g[:, :, None] * v[u][None, :, :]                                                  # [C, L, d]
        out.append(torch.zeros(C, S, d, dtype=q.dtype).index_add(1, seg_of, contrib))
    return torch.stack(out)


def test_sta_backward_matches_autograd_and_finite_differences():
    rng = np.random.default_rng(4321)
    U, C, L, w, dq, d, gamma = 2, 3, 11, 4, 5, 6, 1.3
    lens = [11, 6]
    q, k, v = rng.normal(size=(U, C, dq)), rng.normal(size=(U, L, dq)), rng.normal(size=(U, L, d))
    up = rng.normal(size=(U, C, 3, d))
    got = oracle.sta_backward(q, k, v, lens, w, gamma, up)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    # the torch forward agrees with the checker's forward, and its autograd gradients with the checker's backward
    fwd = _torch_sta(tq, tk, tv, lens, w, gamma)
    assert np.allclose(fwd.detach().numpy(), oracle.sta_forward(q, k, v, lens, w, gamma)[0], rtol=1e-12, atol=1e-13)
    (fwd * torch.tensor(up)).sum().backward()
    for mine, ref in zip(got, (tq.grad, tk.grad, tv.grad)):
        assert np.allclose(mine, ref.numpy(), rtol=1e-10, atol=1e-12)
    # items past the valid length get no gradient
    assert not got[1][1, 6:].any() and not got[2][1, 6:].any()
    # central differences of loss = sum(H' * up) in a few random directions
    loss = lambda q_, k_, v_: float((oracle.sta_forward(q_, k_, v_, lens, w, gamma)[0] * up).sum())
    for _ in range(3):
        dq_, dk_, dv_ = rng.normal(size=q.shape), rng.normal(size=k.shape), rng.normal(size=v.shape)
        h = 1e-6
        num = (loss(q + h * dq_, k + h * dk_, v + h * dv_) - loss(q - h * dq_, k - h * dk_, v - h * dv_)) / (2 * h)
        ana = (got[0] * dq_).sum() + (got[1] * dk_).sum() + (got[2] * dv_).sum()
        assert abs(num - ana) <= 1e-6 * max(1.0, abs(ana))


def test_sta_backward_closed_forms():
    rng = np.random.default_rng(4322)
    U, C, L, w, dq, d, gamma = 1, 2, 8, 4, 3, 4, 2.0
    k, v, up = rng.normal(size=(U, L, dq)), rng.normal(size=(U, L, d)), rng.normal(size=(U, C, 2, d))
    # zero query: every gate is 1/2 and g (1 - g) = 1/4
    dq_, dk_, dv_ = oracle.sta_backward(np.zeros((U, C, dq)), k, v, None, w, gamma, up)
    assert not dk_.any()                                                   # dk_j = sum_c ds q_c = 0
    for j in range(L):
        assert np.allclose(dv_[0, j], 0.5 * up[0, :, j // w].sum(axis=0))
    ref = sum(0.25 * (up[0, 0, j // w] @ v[0, j]) * k[0, j] / gamma for j in range(L))
    assert np.allclose(dq_[0, 0], ref)
    # linear in the upstream gradient
    q = rng.normal(size=(U, C, dq))
    a = oracle.sta_backward(q, k, v, None, w, gamma, up)
    b = oracle.sta_backward(q, k, v, None, w, gamma, -2.0 * up)
    assert all(np.allclose(y, -2.0 * x) for x, y in zip(a, b))


# ------------------------------------------------------------------ GSTA backward
def _torch_gsta(Hp, t, Wq, Wk, Wv, valid):
    """One pair's forward pass in torch fp64 ops with a key mask (written independently of the checker)."""
    d = Hp.shape[1]
    mask = torch.tensor(valid)
    for l in range(Wq.shape[0]):
        if not mask.any():
            break
        e = (Hp @ Wk[l]) @ (t @ Wq[l]) / math.sqrt(d)
        a = torch.softmax(e.masked_fill(~mask, float("-inf")), dim=0)
        t = t + a @ (Hp @ Wv[l])
    return t


@pytest.mark.parametrize("M,valid", [(1, [1, 1, 1, 1, 1]), (3, [1, 1, 1, 0, 0]), (2, [0, 0, 0, 0, 0]), (2, [1, 0, 0, 0, 0])])
def test_gsta_backward_matches_autograd(M, valid):
    rng = np.random.default_rng(5000 + M + sum(valid))
    S, d = 5, 6
    valid = np.array(valid, dtype=bool)
    Hp, t, dz = rng.normal(size=(S, d)), rng.normal(size=d), rng.normal(size=d)
    Wq, Wk, Wv = (rng.normal(size=(M, d, d)) / math.sqrt(d) for _ in range(3))
    got = lo.gsta_pair_backward(Hp, t, Wq, Wk, Wv, valid, dz)
    th = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Hp, t, Wq, Wk, Wv)]
    z = _torch_gsta(*th, valid)
    assert np.allclose(z.detach().numpy(), lo.gsta_pair(Hp, t, Wq, Wk, Wv, valid), rtol=1e-12)
    (z * torch.tensor(dz)).sum().backward()
    for mine, ref in zip(got, th):
        ref = np.zeros_like(mine) if ref.grad is None else ref.grad.numpy()
        assert np.allclose(mine, ref, rtol=1e-10, atol=1e-12)
    assert not got[0][~valid].any()            # segments without a valid item get no gradient


def test_gsta_backward_batch_and_finite_differences():
    rng = np.random.default_rng(5100)
    U, C, S, d, M = 2, 2, 4, 5, 2
    Hp, t0, dz = rng.normal(size=(U, C, S, d)), rng.normal(size=(U, C, d)), rng.normal(size=(U, C, d))
    Wq, Wk, Wv = (rng.normal(size=(M, d, d)) / math.sqrt(d) for _ in range(3))
    cnt = np.array([[3, 3, 1, 0], [2, 0, 0, 0]])
    dHp, dt0, dWq, dWk, dWv = oracle.gsta_backward(Hp, t0, Wq, Wk, Wv, cnt, dz)
    loss = lambda Hp_, t_, q_, k_, v_: float((oracle.gsta_forward(Hp_, t_, q_, k_, v_, cnt) * dz).sum())
    h = 1e-6
    for _ in range(3):
        dirs = [rng.normal(size=x.shape) for x in (Hp, t0, Wq, Wk, Wv)]
        plus = loss(*[x + h * dx for x, dx in zip((Hp, t0, Wq, Wk, Wv), dirs)])
        minus = loss(*[x - h * dx for x, dx in zip((Hp, t0, Wq, Wk, Wv), dirs)])
        ana = sum((g * dx).sum() for g, dx in zip((dHp, dt0, dWq, dWk, dWv), dirs))
        assert abs((plus - minus) / (2 * h) - ana) <= 1e-6 * max(1.0, abs(ana))
    # weight gradients are sums over the pairs
    one = lo.gsta_pair_backward(Hp[0, 1], t0[0, 1], Wq, Wk, Wv, cnt[0] > 0, dz[0, 1])
    rest = oracle.gsta_backward(Hp, t0, Wq, Wk, Wv, cnt, np.where(np.arange(U * C).reshape(U, C, 1) == 1, 0.0, dz))
    assert np.allclose(dWk, one[3] + rest[3], rtol=1e-11, atol=1e-13)
