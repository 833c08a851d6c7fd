"""Plain fp64 CPU checker for the STA + GSTA forward pass of LASER (arxiv 2602.11562).

TEST INFRASTRUCTURE ONLY. This module is the slow, obviously-correct statement
of what the path computes. It is imported by the tests, by the smoke check and
by the benchmark's CPU-baseline leg, never by the product package, and it shares
no code with the HIP kernels. All arithmetic is float64 numpy; `numpy.dot` /
`@` serve as the matmul step, everything else is written out.

Notation (paper, Sec. 3.1, 3.4.2, 3.4.3): one user has a history of L items; item j
has key K[j] in R^{d_q} and value V[j] in R^{d}; a candidate (target item) has query
Q in R^{d_q} (Q = t W_q) and target vector t in R^{d}; w is the segment length,
L' = S = ceil(L / w) segments, gamma the STA score scale, M = L_stack GSTA layers.

Readings where the paper is silent (listed in full in the design notes):
  * valid length: items j >= len are tail padding; their gate is exactly 0;
  * L not a multiple of w: the last segment is short;
  * GSTA: segments with no valid item are left out of the softmax; when no
    segment is valid the layer output is 0 (so z = t);
  * GSTA scale is sqrt(d) with d the embedding dim; single head; H' is the same
    in every layer; weights differ per layer; y = x @ W;
  * FFN + LayerNorm on the segment vectors (Sec. 3.4.2): two linear layers with a relu between them
    and biases, residual, LN over the d components with gain, bias and an epsilon argument; segments
    without a valid item stay zero;
  * several heads (Sec. 4.1.2): head h owns the h-th run of d_q / heads columns of Q and K and of d / heads
    columns of V; same gamma; outputs side by side;
  * softmax variant (Sec. 4.4.1): normalised over the valid items of a segment, per head;
  * projections (Sec. 3.5.1): y = x @ W with W [d_in, n], no bias;
  * multi-resolution views (Sec. 3.4.4): max-pooling runs over the segments that hold a
    valid item; "the r most recent segments" are rows 0..r-1 of H'.

Pin status: every function below is pinned by tests/test_oracle_pins.py (brute
force written independently, closed forms, invariants, and reduction to library
softmax / matmul calls). No function here is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np


def num_segments(L: int, w: int) -> int:
    """L' of split_seq (Sec. 3.4.2, first equation): windows of w consecutive items."""
    return -(-int(L) // int(w))


def segment_counts(lens, L: int, w: int) -> np.ndarray:
    """cnt[u, i] = number of valid items (j < len[u]) inside segment i = [i*w, min((i+1)*w, L))."""
    lens = np.asarray(lens, dtype=np.int64).reshape(-1)
    S = num_segments(L, w)
    cnt = np.zeros((lens.shape[0], S), dtype=np.int32)
    for u in range(lens.shape[0]):
        n = min(max(int(lens[u]), 0), L)
        for i in range(S):
            lo = i * w
            hi = min((i + 1) * w, L)
            cnt[u, i] = max(0, min(hi, n) - lo)
    return cnt


def sigmoid(x: np.ndarray) -> np.ndarray:
    """Logistic function 1 / (1 + exp(-x)), evaluated without overflow on either side."""
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    pos = x >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-x[pos]))
    ex = np.exp(x[~pos])
    out[~pos] = ex / (1.0 + ex)
    return out


def sta_segment(Q: np.ndarray, K_seg: np.ndarray, V_seg: np.ndarray, gamma: float) -> np.ndarray:
    """s_i = Sigmoid(Q K^T / gamma) V for one segment (Sec. 3.4.2, STA equation).

    Q [d_q], K_seg [n, d_q], V_seg [n, d] hold only the valid items of the segment.
    """
    d = V_seg.shape[1]
    if K_seg.shape[0] == 0:
        return np.zeros(d, dtype=np.float64)
    alpha = sigmoid((K_seg @ Q) / gamma)          # one independent gate per item
    return alpha @ V_seg


def sta_pair(Q: np.ndarray, K: np.ndarray, V: np.ndarray, length: int, w: int, gamma: float) -> np.ndarray:
    """H' [S, d] of one (user, candidate): the segment loop of Sec. 3.4.2 in its naive form."""
    L = K.shape[0]
    S = num_segments(L, w)
    n = min(max(int(length), 0), L)
    Hp = np.zeros((S, V.shape[1]), dtype=np.float64)
    for i in range(S):
        lo = i * w
        hi = min(min((i + 1) * w, L), n)
        if hi > lo:
            Hp[i] = sta_segment(Q, K[lo:hi], V[lo:hi], gamma)
    return Hp


def sta_pair_global(Q: np.ndarray, K: np.ndarray, V: np.ndarray, length: int, w: int, gamma: float) -> np.ndarray:
    """Same H', in the deployment form of Sec. 3.5.1: global gates alpha in R^{1 x L},
    reshape R(.) to (L' x 1 x w) and (L' x w x d), one batched matmul, squeeze.
    Rows past the end of the history (and past the valid length) enter with gate 0."""
    L, d = V.shape
    S = num_segments(L, w)
    n = min(max(int(length), 0), L)
    alpha = sigmoid((Q @ K.T) / gamma)            # [L]
    alpha[n:] = 0.0
    A_hat = np.zeros((S * w,), dtype=np.float64)
    A_hat[:L] = alpha
    V_hat = np.zeros((S * w, d), dtype=np.float64)
    V_hat[:L] = V
    V_hat[n:L] = 0.0                              # gate 0 must also silence non-finite padding
    A_hat = A_hat.reshape(S, 1, w)
    V_hat = V_hat.reshape(S, w, d)
    return np.matmul(A_hat, V_hat).reshape(S, d)


def sta_pair_heads(Q: np.ndarray, K: np.ndarray, V: np.ndarray, length: int, w: int, gamma: float,
                   heads: int) -> np.ndarray:
    """H' [S, d] of one (user, candidate) with several attention heads (Sec. 4.1.2 sets two heads with d_q = 16 per
    head and a value width equal to the embedding width d).

    Reading (the paper gives the head count and the widths only): as in multi-head attention, head h owns the
    h-th run of d_q / heads columns of Q and K and the h-th run of d / heads columns of V; every head is the STA of
    Sec. 3.4.2 on its own columns with the same gamma; the outputs are laid side by side, so H' keeps the width d.
    """
    dq, d = K.shape[1], V.shape[1]
    if heads < 1 or dq % heads or d % heads:
        raise ValueError("heads must divide d_q and d")
    a, b = dq // heads, d // heads
    Hp = np.zeros((num_segments(K.shape[0], w), d), dtype=np.float64)
    for h in range(heads):
        Hp[:, h * b:(h + 1) * b] = sta_pair(Q[h * a:(h + 1) * a], K[:, h * a:(h + 1) * a], V[:, h * b:(h + 1) * b],
                                            length, w, gamma)
    return Hp


def sta_pair_softmax(Q: np.ndarray, K: np.ndarray, V: np.ndarray, length: int, w: int, gamma: float,
                     heads: int = 1) -> np.ndarray:
    """H' [S, d] of one (user, candidate) in the ablation variant of Sec. 4.4.1 / Table 4: a softmax over the items
    takes the place of the sigmoid gates of Sec. 3.4.2, s_i = softmax(Q K_i^T / gamma) V_i.

    Reading: the softmax runs over the valid items of segment i (the window STA aggregates over), per head on the
    head's own columns as in sta_pair_heads; a segment without a valid item gives zeros.
    """
    L, dq = K.shape
    d = V.shape[1]
    if heads < 1 or dq % heads or d % heads:
        raise ValueError("heads must divide d_q and d")
    a, b = dq // heads, d // heads
    S = num_segments(L, w)
    n = min(max(int(length), 0), L)
    Hp = np.zeros((S, d), dtype=np.float64)
    for i in range(S):
        lo = i * w
        hi = min(min((i + 1) * w, L), n)
        if hi <= lo:
            continue
        for h in range(heads):
            score = (K[lo:hi, h * a:(h + 1) * a] @ Q[h * a:(h + 1) * a]) / gamma
            e = np.exp(score - score.max())
            Hp[i, h * b:(h + 1) * b] = (e / e.sum()) @ V[lo:hi, h * b:(h + 1) * b]
    return Hp


def gsta_pair(Hp: np.ndarray, t: np.ndarray, Wq: np.ndarray, Wk: np.ndarray, Wv: np.ndarray,
              seg_valid: np.ndarray) -> np.ndarray:
    """z = t_M for one (user, candidate) (Sec. 3.4.3, attention equation and residual update).

    Hp [S, d]; t [d]; Wq, Wk, Wv [M, d, d]; seg_valid [S] bool (segment has >= 1 valid item).
    """
    S, d = Hp.shape
    M = Wq.shape[0]
    t_l = np.array(t, dtype=np.float64)
    idx = np.flatnonzero(np.asarray(seg_valid))
    for l in range(M):
        if idx.size == 0:
            continue                                # o_l = 0
        Hv = Hp[idx]                                # valid segments only
        qp = t_l @ Wq[l]                            # t_{l-1} W_q^l
        Kp = Hv @ Wk[l]                             # H' W_k^l
        Vp = Hv @ Wv[l]                             # H' W_v^l
        e = (Kp @ qp) / math.sqrt(d)
        e = e - e.max()
        p = np.exp(e)
        a = p / p.sum()                             # softmax over segments
        o = a @ Vp
        t_l = t_l + o                               # t_l = t_{l-1} + o_l
    return t_l


def sta_forward(q, k, v, lens, w: int, gamma: float, global_form: bool = False, heads: int = 1,
                softmax: bool = False):
    """H' [U, C, S, d] and cnt [U, S] for a batch. q [U,C,d_q], k [U,L,d_q], v [U,L,d], lens [U] or None."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    U, C, _ = q.shape
    L, d = v.shape[1], v.shape[2]
    lens = np.full(U, L, dtype=np.int64) if lens is None else np.asarray(lens, dtype=np.int64)
    S = num_segments(L, w)
    one = sta_pair_global if global_form else sta_pair
    Hp = np.zeros((U, C, S, d), dtype=np.float64)
    for u in range(U):
        for c in range(C):
            if softmax:
                Hp[u, c] = sta_pair_softmax(q[u, c], k[u], v[u], int(lens[u]), w, gamma, heads)
            elif heads == 1:
                Hp[u, c] = one(q[u, c], k[u], v[u], int(lens[u]), w, gamma)
            else:
                Hp[u, c] = sta_pair_heads(q[u, c], k[u], v[u], int(lens[u]), w, gamma, heads)
    return Hp, segment_counts(lens, L, w)


def gsta_forward(Hp, t0, wq, wk, wv, cnt) -> np.ndarray:
    """z [U, C, d] for a batch. Hp [U,C,S,d], t0 [U,C,d], w* [M,d,d], cnt [U,S]."""
    Hp = np.asarray(Hp, dtype=np.float64)
    t0 = np.asarray(t0, dtype=np.float64)
    wq = np.asarray(wq, dtype=np.float64)
    wk = np.asarray(wk, dtype=np.float64)
    wv = np.asarray(wv, dtype=np.float64)
    U, C, S, d = Hp.shape
    z = np.zeros((U, C, d), dtype=np.float64)
    for u in range(U):
        valid = np.asarray(cnt[u]) > 0
        for c in range(C):
            z[u, c] = gsta_pair(Hp[u, c], t0[u, c], wq, wk, wv, valid)
    return z


def multires_pair(Hp: np.ndarray, seg_valid: np.ndarray, r: int):
    """The two other views of the multi-resolution fusion for one (user, candidate) (Sec. 3.4.4).

    Hp [S, d]; seg_valid [S] bool; r <= S. Returns (pool [d], recent [r, d]):
      pool   = max_pool(H'): component-wise maximum over the segment vectors. Reading (the paper does not
               mention padding): only segments with at least one valid item take part, as in GSTA; with no
               such segment the pooled vector is 0;
      recent = s_1 .. s_r, the r most recent segments: rows 0 .. r-1 of H' (the paper counts the history from
               its most recent item, so segment 1 is row 0). Segments without a valid item are the zero rows
               H' already holds.
    """
    S, d = Hp.shape
    pool = np.zeros(d, dtype=np.float64)
    seen = False
    for i in range(S):
        if not seg_valid[i]:
            continue
        for e in range(d):
            if not seen or Hp[i, e] > pool[e]:
                pool[e] = Hp[i, e]
        seen = True
    recent = np.array(Hp[:r], dtype=np.float64)
    return pool, recent


def multires_forward(Hp, cnt, r: int):
    """pool [U, C, d] and recent [U, C, r, d] for a batch (Sec. 3.4.4). Hp [U,C,S,d], cnt [U,S]."""
    Hp = np.asarray(Hp, dtype=np.float64)
    U, C, S, d = Hp.shape
    pool = np.zeros((U, C, d), dtype=np.float64)
    recent = np.zeros((U, C, r, d), dtype=np.float64)
    for u in range(U):
        valid = np.asarray(cnt[u]) > 0
        for c in range(C):
            pool[u, c], recent[u, c] = multires_pair(Hp[u, c], valid, r)
    return pool, recent


def segment_ffn_vector(s: np.ndarray, W1: np.ndarray, b1: np.ndarray, W2: np.ndarray, b2: np.ndarray,
                       ln_g: np.ndarray, ln_b: np.ndarray, eps: float) -> np.ndarray:
    """s <- LN(FFN(s) + s) for one segment vector (Sec. 3.4.2, the equation after the STA paragraph).

    Readings (the paper names neither the FFN's shape nor the LN's constants): FFN(s) = relu(s W1 + b1) W2 + b2
    with W1 [d, d_ff], W2 [d_ff, d] (the two-layer position-wise network of the Transformer); LN normalises
    over the d components with the biased variance, LN(x) = (x - mean) / sqrt(var + eps) * ln_g + ln_b.
    """
    d = s.shape[0]
    hidden = s @ W1 + b1                           # first layer
    for j in range(hidden.shape[0]):               # relu, written out
        if hidden[j] < 0.0:
            hidden[j] = 0.0
    x = hidden @ W2 + b2 + s                       # second layer and the residual
    mean = 0.0
    for e in range(d):
        mean += x[e]
    mean /= d
    var = 0.0
    for e in range(d):
        var += (x[e] - mean) * (x[e] - mean)
    var /= d
    return (x - mean) / math.sqrt(var + eps) * ln_g + ln_b


def segment_ffn_forward(Hp, cnt, W1, b1, W2, b2, ln_g, ln_b, eps: float) -> np.ndarray:
    """The FFN + LN step on every segment vector of a batch. Hp [U,C,S,d], cnt [U,S] -> [U,C,S,d].

    Reading: segments without a valid item stay the zero vectors they are (they are left out of everything
    downstream; LN(FFN(0)) would be a constant vector that depends on the biases only).
    """
    Hp = np.asarray(Hp, dtype=np.float64)
    W1, b1, W2, b2 = (np.asarray(x, dtype=np.float64) for x in (W1, b1, W2, b2))
    ln_g, ln_b = np.asarray(ln_g, dtype=np.float64), np.asarray(ln_b, dtype=np.float64)
    U, C, S, d = Hp.shape
    out = np.zeros_like(Hp)
    for u in range(U):
        for i in range(S):
            if cnt[u][i] <= 0:
                continue
            for c in range(C):
                out[u, c, i] = segment_ffn_vector(Hp[u, c, i], W1, b1, W2, b2, ln_g, ln_b, eps)
    return out


def project_rows(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X W for row vectors X [..., d_in] and W [d_in, n] (Sec. 3.5.1, the first two equations: every item of the
    history, and every target, goes through the same matrix)."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    if X.shape[-1] != W.shape[0]:
        raise ValueError("inner dimensions differ")
    return X @ W


def project_qkv(t, H, Wq, Wk, Wv):
    """Q = t W_q [U,C,d_q], K = H W_k [U,L,d_q], V = H W_v [U,L,d] (Sec. 3.5.1): the inputs of STA from the
    target embeddings t [U,C,d_in] and the raw history H [U,L,d_in]. No bias (the paper writes none)."""
    return project_rows(t, Wq), project_rows(H, Wk), project_rows(H, Wv)


def fold_query_weights(Wq: np.ndarray, Wk: np.ndarray, heads: int) -> np.ndarray:
    """A [d_in, heads * d_in] with A[:, h d_in + k] = sum_x W_q[:, h a + x] W_k[k, h a + x], a = d_q / heads: the
    matrix that takes a target embedding straight to the vector its head-h score is a dot product of with a raw
    history item, q_h . k_j,h = (t W_q)_h . (h_j W_k)_h = (t A_h) . h_j (Sec. 3.5.1: the matrices do not depend on
    the position, so products may be re-associated)."""
    Wq, Wk = np.asarray(Wq, dtype=np.float64), np.asarray(Wk, dtype=np.float64)
    d_in, dq = Wq.shape
    if Wk.shape != (d_in, dq) or heads < 1 or dq % heads:
        raise ValueError("W_q and W_k must be [d_in, d_q] with heads dividing d_q")
    a = dq // heads
    A = np.zeros((d_in, heads * d_in), dtype=np.float64)
    for h in range(heads):
        A[:, h * d_in:(h + 1) * d_in] = Wq[:, h * a:(h + 1) * a] @ Wk[:, h * a:(h + 1) * a].T
    return A


def project_heads(G: np.ndarray, Wv: np.ndarray, heads: int) -> np.ndarray:
    """out[p, i, h b:(h+1) b] = G[p, h, i, :] W_v[:, h b:(h+1) b], b = d / heads: the value projection applied after
    the gated sums (sum_j g_j (h_j W_v) = (sum_j g_j h_j) W_v), head h with its own columns of W_v.
    G [P, heads, S, d_in], W_v [d_in, d] -> [P, S, d]."""
    G, Wv = np.asarray(G, dtype=np.float64), np.asarray(Wv, dtype=np.float64)
    P, H, S, d_in = G.shape
    d = Wv.shape[1]
    if H != heads or Wv.shape[0] != d_in or d % heads:
        raise ValueError("shapes disagree")
    b = d // heads
    out = np.zeros((P, S, d), dtype=np.float64)
    for h in range(heads):
        out[:, :, h * b:(h + 1) * b] = G[:, h] @ Wv[:, h * b:(h + 1) * b]
    return out


def sta_folded_forward(t, H, Wq, Wk, Wv, lens, w: int, gamma: float, heads: int = 1):
    """H' [U,C,S,d] and cnt [U,S] from the raw embeddings t [U,C,d_in], H [U,L,d_in] without forming K and V: the
    folded queries t A, STA over the raw history with one pseudo-candidate per (candidate, head) and the raw items as
    keys and values, then the value projection per head. Equal, in exact arithmetic, to projections followed by STA."""
    t, H = np.asarray(t, dtype=np.float64), np.asarray(H, dtype=np.float64)
    U, C, d_in = t.shape
    qf = project_rows(t, fold_query_weights(Wq, Wk, heads)).reshape(U, C * heads, d_in)
    G, cnt = sta_forward(qf, H, H, lens, w, gamma)                    # [U, C*heads, S, d_in]
    S = G.shape[2]
    out = project_heads(G.reshape(U * C, heads, S, d_in), Wv, heads)
    return out.reshape(U, C, S, -1), cnt


def laser_forward(q, k, v, t0, wq, wk, wv, lens, w: int, gamma: float):
    """STA followed by GSTA. Returns (H' [U,C,S,d], cnt [U,S], z [U,C,d])."""
    Hp, cnt = sta_forward(q, k, v, lens, w, gamma)
    z = gsta_forward(Hp, t0, wq, wk, wv, cnt)
    return Hp, cnt, z


def laser_forward_ragged(q, k, v, t0, wq, wk, wv, lens, cand_off, w: int, gamma: float):
    """STA followed by GSTA when every user brings its own number of candidates (serving batches): the pair tensors
    are packed, q [P,d_q] and t0 [P,d], and user u owns rows cand_off[u] .. cand_off[u+1]-1 (cand_off [U+1], starts
    at 0, non-decreasing, ends at P). Each pair is computed exactly as in the dense batch (Sec. 3.4.2, 3.4.3): the
    packing changes where a pair is stored, not what it is. Returns (H' [P,S,d], cnt [U,S], z [P,d])."""
    q, k, v, t0 = (np.asarray(x, dtype=np.float64) for x in (q, k, v, t0))
    wq, wk, wv = (np.asarray(x, dtype=np.float64) for x in (wq, wk, wv))
    cand_off = np.asarray(cand_off, dtype=np.int64)
    U, L, d = v.shape
    P = q.shape[0]
    if cand_off.shape != (U + 1,) or cand_off[0] != 0 or cand_off[U] != P or (np.diff(cand_off) < 0).any():
        raise ValueError("cand_off must start at 0, end at P and not decrease")
    lens = np.full(U, L, dtype=np.int64) if lens is None else np.asarray(lens, dtype=np.int64)
    cnt = segment_counts(lens, L, w)
    Hp = np.zeros((P, num_segments(L, w), d), dtype=np.float64)
    z = np.zeros((P, d), dtype=np.float64)
    for u in range(U):
        for p in range(int(cand_off[u]), int(cand_off[u + 1])):
            Hp[p] = sta_pair(q[p], k[u], v[u], int(lens[u]), w, gamma)
            z[p] = gsta_pair(Hp[p], t0[p], wq, wk, wv, cnt[u] > 0)
    return Hp, cnt, z


def sta_backward(q, k, v, lens, w: int, gamma: float, dHp):
    """Gradients of a scalar loss through STA (Sec. 3.4.2), given dHp = d loss / d H' [U,C,S,d]: returns
    (dq [U,C,d_q], dk [U,L,d_q], dv [U,L,d]). Written out from the forward definition
        H'[c,i,:] = sum_{j in segment i, j < len} g_cj v_j,   g_cj = sigmoid(s_cj),   s_cj = q_c . k_j / gamma,
    by the chain rule, item by item:
        d loss / d v_j  = sum_c g_cj dHp[c, i(j), :]
        d loss / d s_cj = (dHp[c, i(j), :] . v_j) g_cj (1 - g_cj)
        d loss / d q_c  = sum_j (d loss / d s_cj) k_j / gamma,    d loss / d k_j = sum_c (d loss / d s_cj) q_c / gamma.
    Items at or past the valid length take no part in the forward pass, so their gradients are zero (the paper
    trains the module, Sec. 3.5.1 / 4.1.2, but prints no backward formulas: these are the derivatives of its
    forward equations)."""
    q, k, v, dHp = (np.asarray(x, dtype=np.float64) for x in (q, k, v, dHp))
    U, C, dq_dim = q.shape
    L, d = v.shape[1], v.shape[2]
    lens = np.full(U, L, dtype=np.int64) if lens is None else np.asarray(lens, dtype=np.int64)
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for u in range(U):
        n = min(max(int(lens[u]), 0), L)
        for j in range(n):
            i = j // w
            for c in range(C):
                g = float(sigmoid(np.array(q[u, c] @ k[u, j] / gamma)))
                up = dHp[u, c, i]
                dv[u, j] += g * up
                ds = (up @ v[u, j]) * g * (1.0 - g)
                dq[u, c] += ds * k[u, j] / gamma
                dk[u, j] += ds * q[u, c] / gamma
    return dq, dk, dv


def gsta_pair_backward(Hp, t, Wq, Wk, Wv, seg_valid, dz):
    """Gradients of a scalar loss through GSTA for one pair (Sec. 3.4.3), given dz = d loss / d z [d]: returns
    (dHp [S,d], dt [d], dWq, dWk, dWv [M,d,d]). The forward pass is replayed as gsta_pair defines it (projections
    K' = H' W_k, V' = H' W_v as written in the paper, softmax over the valid segments, residual update), keeping
    every layer's intermediates, and the chain rule is applied layer by layer from the last to the first:
        t_l = t_{l-1} + o,  o = a V',  a = softmax(e),  e = K' q' / sqrt(d),  q' = t_{l-1} W_q.
    Segments without a valid item take no part, so their rows of dHp are zero."""
    Hp, t, dz = (np.asarray(x, dtype=np.float64) for x in (Hp, t, dz))
    Wq, Wk, Wv = (np.asarray(x, dtype=np.float64) for x in (Wq, Wk, Wv))
    S, d = Hp.shape
    M = Wq.shape[0]
    idx = np.flatnonzero(np.asarray(seg_valid))
    dHp = np.zeros((S, d), dtype=np.float64)
    dWq, dWk, dWv = np.zeros_like(Wq), np.zeros_like(Wk), np.zeros_like(Wv)
    if idx.size == 0:
        return dHp, dz.copy(), dWq, dWk, dWv          # z = t
    Hv = Hp[idx]
    saved = []
    t_l = t.copy()
    for l in range(M):                                # forward, as in gsta_pair
        qp = t_l @ Wq[l]
        Kp = Hv @ Wk[l]
        Vp = Hv @ Wv[l]
        e = (Kp @ qp) / math.sqrt(d)
        pe = np.exp(e - e.max())
        a = pe / pe.sum()
        saved.append((t_l, qp, Kp, Vp, a))
        t_l = t_l + a @ Vp
    g = dz.copy()                                     # d loss / d t_l, walking down
    dHv = np.zeros_like(Hv)
    for l in range(M - 1, -1, -1):
        t_in, qp, Kp, Vp, a = saved[l]
        da = Vp @ g                                   # o = a V'
        dVp = np.outer(a, g)
        de = a * (da - a @ da)                        # softmax
        dKp = np.outer(de, qp) / math.sqrt(d)         # e = K' q' / sqrt(d)
        dqp = (de @ Kp) / math.sqrt(d)
        dWv[l] = Hv.T @ dVp                           # V' = H' W_v
        dWk[l] = Hv.T @ dKp                           # K' = H' W_k
        dHv += dVp @ Wv[l].T + dKp @ Wk[l].T
        dWq[l] = np.outer(t_in, dqp)                  # q' = t W_q
        g = g + dqp @ Wq[l].T                         # residual path plus the path through q'
    dHp[idx] = dHv
    return dHp, g, dWq, dWk, dWv


def gsta_backward(Hp, t0, wq, wk, wv, cnt, dz):
    """Batch form: Hp [U,C,S,d], t0 [U,C,d], dz [U,C,d] -> (dHp [U,C,S,d], dt0 [U,C,d], dWq, dWk, dWv [M,d,d]); the
    weight gradients are summed over all pairs."""
    Hp, t0, dz = (np.asarray(x, dtype=np.float64) for x in (Hp, t0, dz))
    U, C, S, d = Hp.shape
    dHp, dt0 = np.zeros_like(Hp), np.zeros_like(t0)
    dWq, dWk, dWv = (np.zeros(np.asarray(x).shape, dtype=np.float64) for x in (wq, wk, wv))
    for u in range(U):
        valid = np.asarray(cnt[u]) > 0
        for c in range(C):
            a, b, gq, gk, gv = gsta_pair_backward(Hp[u, c], t0[u, c], wq, wk, wv, valid, dz[u, c])
            dHp[u, c], dt0[u, c] = a, b
            dWq += gq
            dWk += gk
            dWv += gv
    return dHp, dt0, dWq, dWk, dWv
