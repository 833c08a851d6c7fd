#!/usr/bin/env python3
"""Benchmark of the STA + GSTA forward path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole hot path (STA, segment counts, GSTA: `laser_forward`) over one batch of
seeded synthetic input already resident in HBM. Prints ONE JSON line (see the design doc for the fields).
Order of work: (1) the fp64 CPU checker is timed on a bounded sample of the same workload, before the GPU
is touched; (2) inputs are generated on the host and uploaded (several distinct copies so the working set
exceeds the 256 MB last-level cache); (3) warm-up, then K timed steps on ONE stream, each step waiting for the
one before: `value`, `ms_per_step` and `roofline` (the whole step against max(HBM time, MFMA time) of its
algorithmic bytes and flops) all describe that loop; the same steps dealt over several streams are reported
beside it as `multi_stream`; (4) the two kernels of a step are timed on their own with HIP events over K
back-to-back launches each, in the very forms `laser_forward` launches (STA with cacheable H' stores and segment
counts); (5) sampled outputs are compared with the checker.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16
DEFAULT_WORKLOAD = "cfg3_high_fanout"   # the configuration the metric is quoted on (L=4096, 256 candidates)


def _oracle_pairs(args):
    """Worker: checker on a list of (row, candidate) pairs of a workload (CPU only)."""
    wl, pairs = args
    from parity_util import oracle_pair
    for (r, c) in pairs:
        oracle_pair(wl, r, c)
    return len(pairs)


def cpu_baseline(spec, budget_s: float = 12.0):
    """Time the fp64 checker, as it stands, on a bounded sample of the workload. Returns the JSON object."""
    import workloads
    from parity_util import oracle_pair
    try:
        from threadpoolctl import threadpool_limits
    except Exception:  # pragma: no cover
        threadpool_limits = None
    # enough users that the sample can fill the time budget (sized from a one-pair calibration)
    probe = workloads.make_workload(spec, users=[0])
    t = time.perf_counter()
    oracle_pair(probe, 0, 0)
    per_pair = max(time.perf_counter() - t, 1e-5)
    n_users = int(min(spec.U, 64, max(2, math.ceil(budget_s / per_pair / spec.C))))
    wl = workloads.make_workload(spec, users=list(range(n_users)))
    import contextlib
    with (threadpool_limits(limits=1) if threadpool_limits else contextlib.nullcontext()):
        return _cpu_baseline_timed(spec, wl, n_users, budget_s)


def _cpu_baseline_timed(spec, wl, n_users, budget_s):
    from parity_util import oracle_pair
    # calibrate on two pairs, then size the sample to the budget
    t = time.perf_counter()
    oracle_pair(wl, 0, 0)
    oracle_pair(wl, n_users - 1, spec.C - 1)
    per_pair = (time.perf_counter() - t) / 2
    n = int(max(4, min(n_users * spec.C, budget_s / max(per_pair, 1e-6))))
    pairs = [(i % n_users, (i // n_users) % spec.C) for i in range(n)]
    t = time.perf_counter()
    for (r, c) in pairs:
        oracle_pair(wl, r, c)
    one_core = time.perf_counter() - t
    out = {"value": n / one_core, "unit": "pairs/s", "cores": 1, "kind": "oracle",
           "sample": f"{n} (user, candidate) pairs of {spec.name} (users 0..{n_users - 1}), fp64 numpy, "
                     f"BLAS pinned to 1 thread, {one_core:.1f} s"}
    # the same code over all host cores (one process per core, before any GPU initialisation)
    try:
        import multiprocessing as mp
        host_cores = len(os.sched_getaffinity(0))
        cores = min(host_cores, 16)   # worker processes: the GPU machines give a job 16 cores whatever they report
        out["host_cores"] = host_cores
        out["os_cpu_count"] = os.cpu_count()
        if cores > 1:
            chunks = [pairs[i::cores] for i in range(cores)]
            with mp.get_context("fork").Pool(cores) as pool:
                t = time.perf_counter()
                done = sum(pool.map(_oracle_pairs, [(wl, ch) for ch in chunks]))
                allc = time.perf_counter() - t
            out["all_cores"] = {"value": done / allc, "cores": cores, "host_cores": host_cores,
                                "seconds": round(allc, 2)}
    except Exception as e:  # pragma: no cover
        out["all_cores"] = {"error": str(e)}
    return out


def paper_setting_chain(laser, torch, event_time):
    """Raw embeddings -> H' at the paper's own training setting (Sec. 4.1.2: batch 2048 with one target each,
    L = 1000, w = 10, 2 heads x d_q 16, d = 128; lengths uniform in [200, 1000], bf16): the direct chain
    (projections, then STA with heads) beside the folded chain, which reads the raw history once."""
    U, C, L, din, dq, d, w, heads = 2048, 1, 1000, 128, 32, 128, 10, 2
    S = -(-L // w)
    gen = torch.Generator(device="cuda").manual_seed(2602)
    rnd = lambda *shape: torch.randn(*shape, device="cuda", generator=gen)
    t, H = rnd(U, C, din).bfloat16(), rnd(U, L, din).bfloat16()
    Wq, Wk, Wv = ((rnd(din, n) / math.sqrt(din)).bfloat16() for n in (dq, dq, d))
    lens = torch.randint(200, L + 1, (U,), device="cuda", dtype=torch.int32, generator=gen)
    gamma = math.sqrt(dq / heads)
    Q = torch.empty(U, C, dq, device="cuda", dtype=torch.bfloat16)
    K = torch.empty(U, L, dq, device="cuda", dtype=torch.bfloat16)
    V = torch.empty(U, L, d, device="cuda", dtype=torch.bfloat16)
    seg = torch.empty(U, C, S, d, device="cuda", dtype=torch.bfloat16)
    A = laser.laser_fold_query_weights(Wq, Wk, heads)
    qf = torch.empty(U, C * heads, din, device="cuda", dtype=torch.bfloat16)
    gw = torch.empty(U, C * heads, S, din, device="cuda", dtype=torch.bfloat16)

    def direct(i):
        laser.laser_project_q_forward(t, Wq, q_out=Q)
        laser.laser_project_kv_forward(H, Wk, Wv, k_out=K, v_out=V)
        laser.laser_sta_forward(Q, K, V, lens, w, gamma, seg_out=seg, want_cnt=False, heads=heads)

    def folded(i):
        laser.laser_sta_folded_forward(t, H, A, Wv, lens, w, gamma, heads, qf_work=qf, g_work=gw, seg_out=seg,
                                       want_cnt=False)

    kv_ms = event_time(lambda i: laser.laser_project_kv_forward(H, Wk, Wv, k_out=K, v_out=V))
    sta_ms = event_time(lambda i: laser.laser_sta_forward(Q, K, V, lens, w, gamma, seg_out=seg, want_cnt=False,
                                                          heads=heads))
    softmax_ms = event_time(lambda i: laser.laser_sta_forward(Q, K, V, lens, w, gamma, seg_out=seg, want_cnt=False,
                                                              heads=heads, softmax=True))
    dseg = (rnd(U, C, S, d)).bfloat16()
    gq = torch.empty(U, C, dq, device="cuda")
    gk = torch.empty(U, L, dq, device="cuda")
    gv = torch.empty(U, L, d, device="cuda")
    work = torch.empty(max(16, laser.load_library().laser_sta_backward_work_bytes(U, C, L, dq, w)), dtype=torch.uint8,
                       device="cuda")
    bwd_ms = event_time(lambda i: laser.laser_sta_backward(Q, K, V, lens, dseg, w, gamma, dq_out=gq, dk_out=gk,
                                                           dv_out=gv, work=work))
    t0p = rnd(U, C, d).bfloat16()
    gw3 = [(rnd(1, d, d) / math.sqrt(d)).bfloat16() for _ in range(3)]
    zp = torch.empty(U, C, d, device="cuda")
    dzp = rnd(U, C, d)
    gwork = torch.empty(max(16, laser.load_library().laser_gsta_backward_work_bytes(U, C, d, 1)), dtype=torch.uint8,
                        device="cuda")
    laser.laser_sta_forward(Q, K, V, lens, w, gamma, seg_out=seg, want_cnt=False, heads=heads)
    gsta_ms = event_time(lambda i: laser.laser_gsta_forward(seg, t0p, *gw3, lens, L, w, z_out=zp))
    gsta_bwd_ms = event_time(lambda i: laser.laser_gsta_backward(seg, t0p, *gw3, lens, dzp, L, w, work=gwork))
    gk16, gv16 = torch.empty(U, L, dq, device="cuda", dtype=torch.bfloat16), torch.empty(U, L, d, device="cuda", dtype=torch.bfloat16)
    bwd16_ms = event_time(lambda i: laser.laser_sta_backward(Q, K, V, lens, dseg, w, gamma, dq_out=gq, dk_out=gk16,
                                                             dv_out=gv16, work=work, grads_bf16=True))
    direct_ms, folded_ms = event_time(direct), event_time(folded)
    same = float((seg.float() - 0).abs().max())   # keeps the last result alive until here
    nvalid = int(lens.sum())
    # least traffic of the job: every valid raw item once, H' once (weights and targets are noise beside them)
    alg_b = (nvalid * din + U * C * S * d) * 2
    return {"U": U, "C": C, "L": L, "w": w, "heads": heads, "d_q": dq, "d": d, "kv_projection_ms": kv_ms,
            "sta_heads_ms": sta_ms, "sta_softmax_variant_ms": softmax_ms, "direct_chain_ms": direct_ms, "folded_chain_ms": folded_ms,
            "algorithmic_bytes": alg_b, "folded_gbps": alg_b / (folded_ms * 1e-3) / 1e9,
            "folded_frac_of_hbm_peak": alg_b / (folded_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "direct_frac_of_hbm_peak": alg_b / (direct_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "pairs_per_s_folded": U * C / (folded_ms * 1e-3), "max_abs_out": same,
            # backward of STA: valid K and V rows and dH' read once (bf16), dk and dv written once (fp32, every row)
            "gsta_forward_ms": gsta_ms, "gsta_backward_ms": gsta_bwd_ms,
            "sta_backward_bf16_gradients_ms": bwd16_ms,
            "sta_backward_bf16_gradients_frac_of_hbm_peak": (nvalid * (dq + d) * 2 + U * C * S * d * 2 + U * L * (dq + d) * 2)
            / (bwd16_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "sta_backward_ms": bwd_ms,
            "sta_backward_algorithmic_bytes": nvalid * (dq + d) * 2 + U * C * S * d * 2 + U * L * (dq + d) * 4,
            "sta_backward_frac_of_hbm_peak": (nvalid * (dq + d) * 2 + U * C * S * d * 2 + U * L * (dq + d) * 4)
            / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}


def paper_setting_ranking(laser, torch, event_time):
    """Ranking at the paper's dimensions (Sec. 4.1.2: L = 1000, w = 10, 2 heads x d_q 16, d = 128) with many
    candidates per user (64 users x 256 candidates, lengths uniform in [200, 1000], bf16): raw embeddings -> K, V, Q
    -> H' (two heads, on the matrix cores) -> z, each step timed alone and the chain as a whole; the softmax variant
    and the generic kernel beside them."""
    U, C, L, din, dq, d, w, heads = 64, 256, 1000, 128, 32, 128, 10, 2
    S = -(-L // w)
    gen = torch.Generator(device="cuda").manual_seed(2603)
    rnd = lambda *shape: torch.randn(*shape, device="cuda", generator=gen)
    t, H = rnd(U, C, din).bfloat16(), rnd(U, L, din).bfloat16()
    Wq, Wk, Wv = ((rnd(din, n) / math.sqrt(din)).bfloat16() for n in (dq, dq, d))
    g3 = [(rnd(1, d, d) / math.sqrt(d)).bfloat16() for _ in range(3)]
    lens = torch.randint(200, L + 1, (U,), device="cuda", dtype=torch.int32, generator=gen)
    gamma = math.sqrt(dq / heads)
    bf = dict(device="cuda", dtype=torch.bfloat16)
    Q, K, V = torch.empty(U, C, dq, **bf), torch.empty(U, L, dq, **bf), torch.empty(U, L, d, **bf)
    seg, z = torch.empty(U, C, S, d, **bf), torch.empty(U, C, d, device="cuda")

    def sta(variant=0, softmax=False):
        return lambda i: laser.laser_sta_forward(Q, K, V, lens, w, gamma, seg_out=seg, want_cnt=False, heads=heads,
                                                 softmax=softmax, variant=variant)

    def chain(i):
        laser.laser_project_q_forward(t, Wq, q_out=Q)
        laser.laser_project_kv_forward(H, Wk, Wv, k_out=K, v_out=V)
        sta()(i)
        laser.laser_gsta_forward(seg, t, *g3, lens, L, w, z_out=z)

    # the complete head of Sec. 3.4: STA, the per-segment FFN + LayerNorm (in place, d_ff = d), GSTA, and the other two
    # views (max-pool over the segments and the r = 8 most recent segment vectors)
    d_ff, r = d, 8
    w1, w2 = (rnd(d, d_ff) / math.sqrt(d)).bfloat16(), (rnd(d_ff, d) / math.sqrt(d_ff)).bfloat16()
    b1, b2 = rnd(d_ff) * 0.3, rnd(d) * 0.3
    ln_g, ln_b = 1.0 + 0.2 * rnd(d), 0.1 * rnd(d)
    pool, recent = torch.empty(U, C, d, **bf), torch.empty(U, C, r, d, **bf)

    def ffn(i):
        laser.laser_segment_ffn_forward(seg, lens, w1, b1, w2, b2, ln_g, ln_b, L, w, 1e-5, seg_out=seg)

    def views(i):
        laser.laser_multires_forward(seg, lens, L, w, r, pool_out=pool, recent_out=recent)

    def gsta_views(i):   # GSTA and the views from one pass over H'
        laser.laser_gsta_forward_multires(seg, t, *g3, lens, L, w, r, z_out=z, pool_out=pool, recent_out=recent)

    def full_head(i):
        laser.laser_project_q_forward(t, Wq, q_out=Q)
        laser.laser_project_kv_forward(H, Wk, Wv, k_out=K, v_out=V)
        sta()(i)
        ffn(i)
        gsta_views(i)

    def ffn_gsta(i):   # FFN + LayerNorm and GSTA from one pass over H' (the transformed rows written in place)
        laser.laser_ffn_gsta_forward(seg, t, *g3, lens, w1, b1, w2, b2, ln_g, ln_b, L, w, 1e-5, seg_out=seg, z_out=z)

    def ffn_gsta_z_only(i):
        laser.laser_ffn_gsta_forward(seg, t, *g3, lens, w1, b1, w2, b2, ln_g, ln_b, L, w, 1e-5, z_out=z, want_seg=False)

    def head_one_pass(i):   # the head without the two other views: z from one pass over H'
        laser.laser_project_q_forward(t, Wq, q_out=Q)
        laser.laser_project_kv_forward(H, Wk, Wv, k_out=K, v_out=V)
        sta()(i)
        ffn_gsta_z_only(i)

    def head_one_pass_views(i):   # the complete head: z, max-pool and the most recent rows from one pass over H'
        laser.laser_project_q_forward(t, Wq, q_out=Q)
        laser.laser_project_kv_forward(H, Wk, Wv, k_out=K, v_out=V)
        sta()(i)
        laser.laser_ffn_gsta_forward(seg, t, *g3, lens, w1, b1, w2, b2, ln_g, ln_b, L, w, 1e-5, z_out=z, want_seg=False,
                                     r=r, pool_out=pool, recent_out=recent)

    def head_two_calls(i):
        laser.laser_project_q_forward(t, Wq, q_out=Q)
        laser.laser_project_kv_forward(H, Wk, Wv, k_out=K, v_out=V)
        sta()(i)
        ffn(i)
        laser.laser_gsta_forward(seg, t, *g3, lens, L, w, z_out=z)

    chain(0)
    out = {"U": U, "C": C, "L": L, "w": w, "heads": heads, "d_q": dq, "d": d,
           "kv_projection_ms": event_time(lambda i: laser.laser_project_kv_forward(H, Wk, Wv, k_out=K, v_out=V)),
           "q_projection_ms": event_time(lambda i: laser.laser_project_q_forward(t, Wq, q_out=Q)),
           "sta_heads_ms": event_time(sta()), "sta_heads_softmax_ms": event_time(sta(softmax=True)),
           "sta_heads_generic_kernel_ms": event_time(sta(variant=1)),
           "gsta_ms": event_time(lambda i: laser.laser_gsta_forward(seg, t, *g3, lens, L, w, z_out=z)),
           "chain_ms": event_time(chain)}
    sta()(0)
    out["ffn_layernorm_ms"] = event_time(ffn)     # (in place: later launches normalise normalised rows, same work)
    out["views_ms"] = event_time(views)
    out["gsta_with_views_ms"] = event_time(gsta_views)
    out["full_head_ms"] = event_time(full_head)
    out["ffn_then_gsta_one_pass_ms"] = event_time(ffn_gsta)
    out["ffn_then_gsta_one_pass_z_only_ms"] = event_time(ffn_gsta_z_only)
    out["head_z_two_calls_ms"] = event_time(head_two_calls)
    out["head_z_one_pass_ms"] = event_time(head_one_pass)
    out["full_head_one_pass_ms"] = event_time(head_one_pass_views)

    # The same chains replayed from a captured graph: a chain of four or five launches of 10-150 us each is shorter
    # than the Python binding's marshalling of their ~25 arguments apiece, so the loops above can be bound by the
    # host. (The library only enqueues kernels: nothing in it is refused by capture.)
    def graph_time(fn, replays=50):
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                fn(0)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fn(0)
            for _ in range(3):
                g.replay()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            a.record()
            for _ in range(replays):
                g.replay()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / replays
        except Exception as e:   # capture not available: the event-timed loops stand alone
            return None

    out["full_head_graph_ms"] = graph_time(full_head)
    out["full_head_one_pass_graph_ms"] = graph_time(head_one_pass_views)
    out["head_z_one_pass_graph_ms"] = graph_time(head_one_pass)
    best = out["full_head_one_pass_graph_ms"] or out["full_head_one_pass_ms"]
    out["pairs_per_s_full_head_one_pass"] = U * C / (best * 1e-3)
    out["pairs_per_s_full_head"] = U * C / (out["full_head_ms"] * 1e-3)
    nvalid = int(lens.sum())
    # STA alone: valid K and V rows, the queries, H' written once
    sta_b = nvalid * (dq + d) * 2 + U * C * dq * 2 + U * C * S * d * 2
    out["sta_algorithmic_bytes"] = sta_b
    out["sta_heads_frac_of_hbm_peak"] = sta_b / (out["sta_heads_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS
    out["pairs_per_s_chain"] = U * C / (out["chain_ms"] * 1e-3)
    out["max_abs_z"] = float(z.abs().max())
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copies", type=int, default=0, help="distinct input/output copies to rotate through (0 = auto)")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams (default priority) for the secondary \"multi_stream\" figure: consecutive steps, "
                         "which are independent batches, dealt over that many streams in turn (0 or 1 = skip it). "
                         "The headline is always the one-stream loop")
    ap.add_argument("--views", type=int, default=0, metavar="R",
                    help="also time the multi-resolution views (max-pooled H' and the R most recent segments): the "
                         "stand-alone kernel and the whole path with them; reported under \"views\"")
    ap.add_argument("--ffn", type=int, default=0, metavar="D_FF",
                    help="also time the segment FFN + LayerNorm step (hidden size D_FF) on the workload's H'; "
                         "reported under \"ffn\"")
    ap.add_argument("--project", type=int, default=0, metavar="D_IN",
                    help="also time the projections ahead of STA (Q = t W_q, K = H W_k, V = H W_v from raw embeddings "
                         "of width D_IN) and the whole path that starts from them; reported under \"project\"")
    ap.add_argument("--ragged", action="store_true",
                    help="also time the packed-pairs entry point with a seeded ragged candidate count per user "
                         "(uniform between a quarter of C and C); reported under \"ragged\"")
    ap.add_argument("--backward", action="store_true",
                    help="also time the backward pass of GSTA on the workload's H' and of STA (built for at most 8 "
                         "candidates per user; more are taken 8 at a time); reported under \"backward\"")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy 5 times (reference reading for the FETCH_SIZE / "
                         "WRITE_SIZE counters when this command runs under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (users shard across GPUs with no exchange; see DESIGN.md); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import workloads
    from paper_2602_11562_amd import cost_model as cm
    spec = workloads.CONFIGS[args.workload]

    cpu = None if args.no_cpu_baseline else cpu_baseline(spec)

    import torch
    import paper_2602_11562_amd as laser
    from parity_util import ELEM_TOL, TOL, DeviceWorkload, elem_rel_err, oracle_pair, to_host_f64, vec_rel_err
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    laser.load_library()   # fails loudly if liblaser.so is missing

    wl = workloads.make_workload(spec)
    esz = 4 if spec.dtype == "f32" else 2
    tdt = torch.float32 if spec.dtype == "f32" else torch.bfloat16
    sta_b = cm.sta_bytes(wl.lens, spec.U, spec.C, spec.L, spec.d_q, spec.d, spec.w, spec.dtype)
    sta_f = cm.sta_flops(wl.lens, spec.C, spec.d_q, spec.d)
    gsta_b = cm.gsta_bytes(wl.lens, spec.U, spec.C, spec.L, spec.d, spec.w, spec.M, spec.dtype)
    gsta_f = cm.gsta_flops(wl.lens, spec.C, spec.d, spec.w, spec.M)
    footprint = (wl.q.nbytes + wl.k.nbytes + wl.v.nbytes + wl.t0.nbytes + spec.U * spec.C * spec.S * spec.d * esz
                 + spec.U * spec.C * spec.d * 4)
    nstreams = max(1, min(4, args.streams))
    dtl_sta = 4 if (spec.dtype == "bf16" and spec.C >= 9) else 0   # LASER_STA_MFMA_CACHED where laser_forward uses it
    copies = args.copies or int(min(8, max(1, math.ceil(600e6 / footprint))))
    copies = -(-copies // nstreams) * nstreams   # a multiple of the streams: a buffer set is only ever used on one stream

    sets = []
    for _ in range(copies):
        dw = DeviceWorkload(wl)   # a fresh allocation of every input
        seg = torch.empty((spec.U, spec.C, spec.S, spec.d), dtype=tdt, device="cuda")
        cnt = torch.empty((spec.U, spec.S), dtype=torch.int32, device="cuda")
        z = torch.empty((spec.U, spec.C, spec.d), dtype=torch.float32, device="cuda")
        sets.append((dw, seg, cnt, z))

    def step(i, stream=None):
        dw, seg, cnt, z = sets[i % copies]
        laser.laser_forward(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.w, spec.gamma,
                            seg_out=seg, seg_cnt=cnt, z_out=z, stream=stream)

    def sta_only(i):   # the launch laser_forward makes: segment counts written, H' stored for a reader that follows
        dw, seg, cnt, z = sets[i % copies]
        laser.laser_sta_forward(dw.q, dw.k, dw.v, dw.lens, spec.w, spec.gamma, seg_out=seg, seg_cnt=cnt,
                                variant=dtl_sta)

    def sta_alone(i):  # what laser_sta_forward launches when nothing reads H' next (non-temporal stores, no counts)
        dw, seg, cnt, z = sets[i % copies]
        laser.laser_sta_forward(dw.q, dw.k, dw.v, dw.lens, spec.w, spec.gamma, seg_out=seg, want_cnt=False)

    def gsta_only(i):
        dw, seg, cnt, z = sets[i % copies]
        laser.laser_gsta_forward(seg, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.L, spec.w, z_out=z)

    def timed_steps(streams):
        """W warm-up steps, then K timed steps between two device synchronisations; step i goes to stream i mod n."""
        n = len(streams)
        for i in range(args.warmup):
            step(i, streams[i % n])
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for i in range(args.steps):
            step(i, streams[i % n])
        torch.cuda.synchronize()
        return time.perf_counter() - t_start

    # One stream: the latency of a step. Several: consecutive steps are independent batches (a serving process has
    # many in flight), and the tail of one step's kernels overlaps the start of the next step's.
    wall_one = timed_steps([torch.cuda.current_stream()])
    wall_multi = timed_steps([torch.cuda.Stream() for _ in range(nstreams)]) if nstreams > 1 else None
    ms_per_step = wall_one * 1e3 / args.steps

    def event_time(fn):
        """Average duration (ms) of K back-to-back launches, HIP events on the launch stream."""
        for i in range(min(args.warmup, 10)):
            fn(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for i in range(args.steps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / args.steps

    sta_ms = event_time(sta_only)
    gsta_ms = event_time(gsta_only)
    sta_alone_ms = event_time(sta_alone)
    step_event_ms = event_time(step)   # the same one-stream loop between HIP events instead of host clocks

    # The same path with H' never stored (one GSTA layer): laser_forward_fused with its work buffer
    zonly = None
    if spec.M == 1:
        lib = laser.load_library()
        need = lib.laser_forward_fused_work_bytes(spec.U, spec.C, spec.L, spec.d_q, spec.d, spec.w,
                                                  laser.LASER_F32 if spec.dtype == "f32" else laser.LASER_BF16)
        fwork = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

        def step_fused(i):
            dw, seg, cnt, z = sets[i % copies]
            laser.laser_forward_fused(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.w, spec.gamma,
                                      seg_cnt=cnt, z_out=z, work=fwork)

        zonly = {"ms_per_step": event_time(step_fused), "work_bytes": int(need)}

    views = None
    if args.views > 0:
        R = min(args.views, spec.S)
        outs = [(torch.empty((spec.U, spec.C, spec.d), dtype=tdt, device="cuda"),
                 torch.empty((spec.U, spec.C, R, spec.d), dtype=tdt, device="cuda")) for _ in range(copies)]

        def views_only(i):
            dw, seg, cnt, z = sets[i % copies]
            pool, recent = outs[i % copies]
            laser.laser_multires_forward(seg, dw.lens, spec.L, spec.w, R, pool_out=pool, recent_out=recent)

        def step_views(i):
            dw, seg, cnt, z = sets[i % copies]
            pool, recent = outs[i % copies]
            laser.laser_forward_multires(dw.q, dw.k, dw.v, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.w, spec.gamma, R,
                                         seg_out=seg, seg_cnt=cnt, z_out=z, pool_out=pool, recent_out=recent)

        mr_ms = event_time(views_only)
        path_ms = event_time(step_views)
        # algorithmic bytes of the stand-alone kernel: the valid segments of H' once, both outputs once
        nvalid = int(sum(-(-int(n) // spec.w) for n in wl.lens))
        mr_b = (nvalid * spec.C * spec.d + spec.pairs * spec.d * (1 + 2 * R)) * esz
        views = {"r": R, "kernel": "multires", "kernel_ms": mr_ms, "algorithmic_bytes": mr_b,
                 "gbps": mr_b / (mr_ms * 1e-3) / 1e9, "frac_of_hbm_peak": mr_b / (mr_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "whole_path_ms_per_step": path_ms, "whole_path_pairs_per_s": spec.pairs / (path_ms * 1e-3)}

    ffn = None
    if args.ffn > 0:
        rng = np.random.default_rng(spec.seed + 5)
        to_t = lambda x: torch.from_numpy(np.asarray(x, dtype=np.float32)).cuda()
        w1 = to_t(rng.normal(size=(spec.d, args.ffn)) / math.sqrt(spec.d)).to(tdt)
        w2 = to_t(rng.normal(size=(args.ffn, spec.d)) / math.sqrt(args.ffn)).to(tdt)
        b1, b2 = to_t(rng.normal(size=args.ffn) * 0.3), to_t(rng.normal(size=spec.d) * 0.3)
        ln_g, ln_b = to_t(1.0 + 0.2 * rng.normal(size=spec.d)), to_t(0.1 * rng.normal(size=spec.d))
        outs2 = [torch.empty_like(sets[i][1]) for i in range(copies)]

        def ffn_only(i):
            dw, seg, cnt, z = sets[i % copies]
            laser.laser_segment_ffn_forward(seg, dw.lens, w1, b1, w2, b2, ln_g, ln_b, spec.L, spec.w, 1e-5,
                                            seg_out=outs2[i % copies])

        ffn_ms = event_time(ffn_only)
        nvalid = int(sum(-(-int(n) // spec.w) for n in wl.lens))
        # algorithmic work: valid segment vectors read once, every vector written once, the weights once;
        # two products of d x d_ff per valid vector
        ffn_b = (nvalid * spec.C * spec.d + spec.pairs * spec.S * spec.d + 2 * spec.d * args.ffn) * esz
        ffn_f = 4.0 * nvalid * spec.C * spec.d * args.ffn
        t_h, t_m = ffn_b / (HBM_PEAK_GBS * 1e9), ffn_f / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        ffn = {"d_ff": args.ffn, "kernel_ms": ffn_ms, "algorithmic_bytes": ffn_b, "algorithmic_flops": ffn_f,
               "gbps": ffn_b / (ffn_ms * 1e-3) / 1e9, "tflops": ffn_f / (ffn_ms * 1e-3) / 1e12,
               "bound": "hbm" if t_h >= t_m else "mfma",
               "frac": (t_h if t_h >= t_m else t_m) / (ffn_ms * 1e-3)}
        if spec.M == 1:
            # FFN + LayerNorm and GSTA behind it: the two calls in a row (the transformed H' written and read back)
            # against laser_ffn_gsta_forward (one pass over H', transformed rows not wanted)
            def two_calls(i):
                dw, seg, cnt, z = sets[i % copies]
                laser.laser_segment_ffn_forward(seg, dw.lens, w1, b1, w2, b2, ln_g, ln_b, spec.L, spec.w, 1e-5,
                                                seg_out=outs2[i % copies])
                laser.laser_gsta_forward(outs2[i % copies], dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, spec.L, spec.w, z_out=z)

            def one_pass(i):
                dw, seg, cnt, z = sets[i % copies]
                laser.laser_ffn_gsta_forward(seg, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, w1, b1, w2, b2, ln_g, ln_b,
                                             spec.L, spec.w, 1e-5, z_out=z, want_seg=False)

            two_ms = event_time(two_calls)
            try:
                one_ms = event_time(one_pass)
            except laser.LaserError:
                one_ms = None
            # least traffic of FFN + GSTA when only z is wanted: valid segment vectors read once, t0 and z, the weights
            fg_b = (nvalid * spec.C * spec.d + spec.pairs * spec.d + (2 * args.ffn + 3 * spec.d) * spec.d) * esz \
                + spec.pairs * spec.d * 4
            ffn["then_gsta"] = {"two_calls_ms": two_ms, "one_pass_ms": one_ms, "one_pass_algorithmic_bytes": fg_b,
                                "one_pass_frac_of_hbm_peak": None if one_ms is None else
                                fg_b / (one_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    project = None
    if args.project > 0:
        din = args.project
        rng = np.random.default_rng(spec.seed + 6)
        to_t = lambda x: torch.from_numpy(np.asarray(x, dtype=np.float32)).cuda().to(tdt)
        wq_p, wk_p = (to_t(rng.normal(size=(din, spec.d_q)) / math.sqrt(din)) for _ in range(2))
        wv_p = to_t(rng.normal(size=(din, spec.d)) / math.sqrt(din))
        raws = [(to_t(rng.normal(size=(spec.U, spec.C, din))), to_t(rng.normal(size=(spec.U, spec.L, din))))
                for _ in range(min(copies, 2))]

        def kv_only(i):
            dw, seg, cnt, z = sets[i % copies]
            laser.laser_project_kv_forward(raws[i % len(raws)][1], wk_p, wv_p, k_out=dw.k, v_out=dw.v)

        def q_only(i):
            dw, seg, cnt, z = sets[i % copies]
            laser.laser_project_q_forward(raws[i % len(raws)][0], wq_p, q_out=dw.q)

        def step_from_raw(i):
            q_only(i)
            kv_only(i)
            step(i)

        kv_ms, q_ms, raw_ms = event_time(kv_only), event_time(q_only), event_time(step_from_raw)
        # algorithmic work of the K/V kernel: H read once, K and V written once, the weights once
        rows = spec.U * spec.L
        kv_b = (rows * (din + spec.d_q + spec.d) + din * (spec.d_q + spec.d)) * esz
        kv_f = 2.0 * rows * din * (spec.d_q + spec.d)
        t_h, t_m = kv_b / (HBM_PEAK_GBS * 1e9), kv_f / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        project = {"d_in": din, "kv_kernel_ms": kv_ms, "q_kernel_ms": q_ms, "algorithmic_bytes": kv_b,
                   "algorithmic_flops": kv_f, "gbps": kv_b / (kv_ms * 1e-3) / 1e9,
                   "tflops": kv_f / (kv_ms * 1e-3) / 1e12, "bound": "hbm" if t_h >= t_m else "mfma",
                   "frac": (t_h if t_h >= t_m else t_m) / (kv_ms * 1e-3),
                   "whole_path_ms_per_step": raw_ms, "whole_path_pairs_per_s": spec.pairs / (raw_ms * 1e-3)}
        project["paper_setting"] = paper_setting_chain(laser, torch, event_time)
        project["paper_setting_ranking"] = paper_setting_ranking(laser, torch, event_time)
        for (dw, seg, cnt, z) in sets:   # the timed loops above overwrote q, k, v: restore the workload's own
            fresh = DeviceWorkload(wl)
            dw.q.copy_(fresh.q), dw.k.copy_(fresh.k), dw.v.copy_(fresh.v)
        torch.cuda.synchronize()

    ragged = None
    if args.ragged:
        rng = np.random.default_rng(spec.seed + 7)
        counts = rng.integers(max(1, spec.C // 4), spec.C + 1, size=spec.U)
        off_h = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
        Pr = int(off_h[-1])
        off_d = torch.from_numpy(off_h).cuda()
        dw0 = sets[0][0]
        # the packed batch takes each user's first counts[u] candidates of the dense workload
        rows = torch.from_numpy(np.concatenate([u * spec.C + np.arange(counts[u]) for u in range(spec.U)])).cuda()
        qp = dw0.q.reshape(spec.U * spec.C, spec.d_q)[rows].contiguous()
        tp = dw0.t0.reshape(spec.U * spec.C, spec.d)[rows].contiguous()
        segp = torch.empty((Pr, spec.S, spec.d), dtype=tdt, device="cuda")
        cntp = torch.empty((spec.U, spec.S), dtype=torch.int32, device="cuda")
        zp = torch.empty((Pr, spec.d), dtype=torch.float32, device="cuda")

        def step_ragged(i):
            dw = sets[i % copies][0]
            laser.laser_forward_ragged(qp, dw.k, dw.v, tp, dw.wq, dw.wk, dw.wv, dw.lens, off_d, spec.C, spec.w,
                                       spec.gamma, seg_out=segp, seg_cnt=cntp, z_out=zp)

        rag_ms = event_time(step_ragged)
        # the same pairs against the dense result (bit for bit: the packing changes where a pair is stored only)
        step(0)
        step_ragged(0)
        torch.cuda.synchronize()
        same = bool(torch.equal(sets[0][1].reshape(spec.U * spec.C, spec.S, spec.d)[rows], segp) and
                    torch.equal(sets[0][3].reshape(spec.U * spec.C, spec.d)[rows], zp))
        ragged = {"pairs": Pr, "counts_min": int(counts.min()), "counts_max": int(counts.max()),
                  "ms_per_step": rag_ms, "pairs_per_s": Pr / (rag_ms * 1e-3),
                  "dense_padded_ms_per_step": step_event_ms, "equals_dense_rows": same}

    backward = None
    if args.backward:
        gen = torch.Generator(device="cuda").manual_seed(spec.seed + 8)
        dz = torch.randn(spec.U, spec.C, spec.d, device="cuda", generator=gen)
        lib = laser.load_library()
        gwork = torch.empty(max(16, lib.laser_gsta_backward_work_bytes(spec.U, spec.C, spec.d, spec.M)), dtype=torch.uint8,
                            device="cuda")
        step(0)
        torch.cuda.synchronize()

        def gsta_bwd(i):
            dw, seg, cnt, z = sets[i % copies]
            return laser.laser_gsta_backward(seg, dw.t0, dw.wq, dw.wk, dw.wv, dw.lens, dz, spec.L, spec.w, work=gwork)

        backward = {}
        try:
            g_ms = event_time(gsta_bwd)
            nvalid = int(sum(-(-int(n) // spec.w) for n in wl.lens))
            # H' (valid rows) read once and dH' (every row) written once in the storage type; t0, dz, dt0 and the six
            # vectors per pair and layer once; the weights once
            g_b = ((nvalid * spec.C * spec.d + spec.pairs * spec.S * spec.d + spec.pairs * spec.d) * esz
                   + spec.pairs * spec.d * 4 * (2 + 12 * spec.M) + 3 * spec.M * spec.d * spec.d * (esz + 4))
            backward["gsta"] = {"ms": g_ms, "algorithmic_bytes": g_b, "gbps": g_b / (g_ms * 1e-3) / 1e9,
                                "frac_of_hbm_peak": g_b / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        except laser.LaserError as e:
            backward["gsta"] = {"error": str(e)}
        if spec.d_q <= 256 and spec.d <= 256:
            dseg = torch.randn(spec.U, spec.C, spec.S, spec.d, device="cuda", generator=gen).to(tdt)
            swork = torch.empty(max(16, lib.laser_sta_backward_work_bytes(spec.U, spec.C, spec.L, spec.d_q, spec.w)),
                                dtype=torch.uint8, device="cuda")
            outs_b = (torch.empty(spec.U, spec.C, spec.d_q, device="cuda"), torch.empty(spec.U, spec.L, spec.d_q, device="cuda"),
                      torch.empty(spec.U, spec.L, spec.d, device="cuda"))

            def sta_bwd(i):
                dw = sets[i % copies][0]
                laser.laser_sta_backward(dw.q, dw.k, dw.v, dw.lens, dseg, spec.w, spec.gamma, dq_out=outs_b[0],
                                         dk_out=outs_b[1], dv_out=outs_b[2], work=swork)

            s_ms = event_time(sta_bwd)
            nitems = int(sum(int(n) for n in wl.lens))
            s_b = (nitems * (spec.d_q + spec.d) + spec.pairs * spec.S * spec.d) * esz + spec.U * spec.L * (spec.d_q + spec.d) * 4
            backward["sta"] = {"ms": s_ms, "algorithmic_bytes": s_b, "gbps": s_b / (s_ms * 1e-3) / 1e9,
                               "frac_of_hbm_peak": s_b / (s_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}

    if args.calibration_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # sampled parity against the checker (one-by-one pairs), in this launch configuration
    step(0)
    torch.cuda.synchronize()
    dw, seg, cnt, z = sets[0]
    rng = np.random.default_rng(0)
    worst = worst_el = 0.0
    for _ in range(4):
        r, c = int(rng.integers(spec.U)), int(rng.integers(spec.C))
        Hp_ref, z_ref = oracle_pair(wl, r, c)
        worst = max(worst, vec_rel_err(to_host_f64(seg[r, c]), Hp_ref), vec_rel_err(to_host_f64(z[r, c]), z_ref))
        worst_el = max(worst_el, elem_rel_err(to_host_f64(seg[r, c]), Hp_ref), elem_rel_err(to_host_f64(z[r, c]), z_ref))
    parity_ok = worst <= TOL[spec.dtype] and worst_el <= ELEM_TOL[spec.dtype]

    dtl = laser.LASER_F32 if spec.dtype == "f32" else laser.LASER_BF16
    sta_kernel = laser.laser_sta_kernel_name(spec.C, spec.d_q, spec.d, spec.w, dtl)
    gsta_kernel = laser.laser_gsta_kernel_name(spec.C, spec.S, spec.d, dtl, spec.M)

    def roofline_of(bytes_, flops, ms):
        """Time at the published peaks against the measured time: the larger of HBM time and bf16 MFMA time is the
        bound (fp32 storage runs on the vector ALUs and is priced against HBM only)."""
        t_h = bytes_ / (HBM_PEAK_GBS * 1e9)
        t_m = 0.0 if spec.dtype == "f32" else flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        if t_h >= t_m:
            r = {"bound": "hbm", "achieved": bytes_ / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
        else:
            r = {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                 "unit": "TFLOP/s"}
        r["frac"] = r["achieved"] / r["peak"]
        r.update({"ms": ms, "algorithmic_bytes": bytes_, "algorithmic_flops": flops,
                  "t_hbm_us": t_h * 1e6, "t_mfma_us": t_m * 1e6,
                  "gbps": bytes_ / (ms * 1e-3) / 1e9, "tflops": flops / (ms * 1e-3) / 1e12})
        return r

    # The step as timed (one stream): algorithmic bytes and flops of the whole path, H' written once and not read back
    path_b = cm.path_bytes(wl.lens, spec.U, spec.C, spec.L, spec.d_q, spec.d, spec.w, spec.M, spec.dtype)
    path_f = cm.path_flops(wl.lens, spec.C, spec.d_q, spec.d, spec.w, spec.M)
    roof = roofline_of(path_b, path_f, ms_per_step)
    roof["scope"] = "whole step (laser_forward: STA + segment counts + GSTA), one stream, host-timed"
    # HBM bytes per launch as counted by rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE) cannot be read from inside this
    # process; the figures of the profiling runs of this same command are kept under profiles/
    roof["traffic"] = None
    roof["traffic_note"] = f"not measured in this run; see profiles/bench_{spec.name}.txt"
    roof["step_event_ms"] = step_event_ms
    # the step's two launches, each timed alone in the form laser_forward launches it
    k_sta = roofline_of(sta_b, sta_f, sta_ms)
    k_sta.update({"name": sta_kernel, "form": "as launched by laser_forward: seg_cnt written, H' stored cacheable"})
    k_gsta = roofline_of(gsta_b, gsta_f, gsta_ms)
    k_gsta.update({"name": gsta_kernel})
    roof["dominant_kernel"] = k_sta if sta_ms >= gsta_ms else k_gsta
    if zonly is not None:
        zb = cm.path_bytes(wl.lens, spec.U, spec.C, spec.L, spec.d_q, spec.d, spec.w, spec.M, spec.dtype,
                           seg_out_written=False)
        zonly.update(roofline_of(zb, path_f, zonly["ms_per_step"]))
        zonly["value"] = spec.pairs / (zonly["ms_per_step"] * 1e-3)
        zonly["entry_point"] = "laser_forward_fused (H' never stored; one stream, HIP events)"
        step_fused(0)
        torch.cuda.synchronize()
        zz = to_host_f64(sets[0][3])
        rngz = np.random.default_rng(1)
        zerr = 0.0
        for _ in range(4):
            r, c = int(rngz.integers(spec.U)), int(rngz.integers(spec.C))
            zerr = max(zerr, vec_rel_err(zz[r, c], oracle_pair(wl, r, c)[1]))
        zonly["parity_max_vector_rel_err"] = zerr
        parity_ok = parity_ok and zerr <= TOL[spec.dtype]
    k_alone = roofline_of(sta_b, sta_f, sta_alone_ms)
    k_alone.update({"name": sta_kernel, "form": "as launched by laser_sta_forward: no seg_cnt, non-temporal H' stores"})

    rec = {
        "metric": "STA+GSTA (user,candidate) pairs/sec",
        "value": spec.pairs / (ms_per_step * 1e-3),
        "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": spec.name, "U": spec.U, "C": spec.C, "L": spec.L, "d": spec.d, "d_q": spec.d_q,
                   "w": spec.w, "S": spec.S, "M": spec.M, "pairs": spec.pairs, "input_copies": copies,
                   "streams": 1,
                   "footprint_mb": footprint / 1e6, "seg_out_written": True},
        "multi_stream": None if wall_multi is None else {
            "streams": nstreams, "ms_per_step": wall_multi * 1e3 / args.steps,
            "value": spec.pairs / (wall_multi / args.steps),
            "note": "consecutive steps are independent batches dealt over the streams in turn; throughput, not latency"},
        "roofline": roof,
        "cpu_baseline": cpu,
        "kernels": {"sta": k_sta, "gsta": k_gsta, "sta_standalone": k_alone},
        "z_only": zonly,
        "views": views,
        "ffn": ffn,
        "project": project,
        "ragged": ragged,
        "backward": backward,
        "parity": {"max_vector_rel_err": worst, "max_elementwise_err_floor": worst_el, "tolerance": TOL[spec.dtype],
                   "ok": bool(parity_ok), "sampled_pairs": 4},
    }
    print(json.dumps(rec))
    return 0 if parity_ok else 1


if __name__ == "__main__":
    sys.exit(main())
