"""Input generators: number formats, shapes, distributions, per-user reproducibility."""
import math

import numpy as np
import torch

import workloads
from workloads.configs import make_lens, make_user, make_weights, stored_values, TAIL_SCALE


def test_bf16_rounding_matches_torch_round_to_nearest_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 1.01171875, 3.3895e38, 1e-40, -1e-40],
                                 dtype=np.float32)])
    bits = workloads.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = workloads.bf16_bits_to_f32(bits)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy(), equal_nan=True)
    # ties go to even: 1 + 2^-8 is exactly half way between 1 and 1 + 2^-7
    assert workloads.round_to_bf16(np.array([1.00390625], np.float32))[0] == 1.0
    assert workloads.round_to_bf16(np.array([1.01171875], np.float32))[0] == 1.015625


def test_specs_match_the_five_benchmark_configs():
    c = workloads.CONFIGS
    assert [(s.U, s.C, s.L, s.d, s.w, s.S, s.M, s.dtype) for s in c.values()] == [
        (1, 16, 1024, 64, 64, 16, 1, "f32"),
        (64, 64, 2048, 64, 128, 16, 1, "bf16"),
        (32, 256, 4096, 128, 128, 32, 1, "bf16"),
        (4096, 1, 4096, 64, 256, 16, 1, "bf16"),
        (16, 128, 10000, 128, 256, 40, 2, "bf16"),
    ]


def test_lengths():
    c = workloads.CONFIGS
    l2 = make_lens(c["cfg2_bf16"])
    assert l2.dtype == np.int32 and l2.min() >= 512 and l2.max() <= 2048 and len(set(l2.tolist())) > 32
    l4 = make_lens(c["cfg4_low_fanout"])
    assert l4.min() >= 64 and l4.max() <= 4096
    # log-uniform on [64, 4096]: mean (b - a) / ln(b / a) ~ 970, median ~ sqrt(64 * 4096) = 512
    assert 900 < l4.mean() < 1040 and 440 < np.median(l4) < 590
    assert (make_lens(c["cfg3_high_fanout"]) == 4096).all()


def test_user_arrays_are_reproducible_and_scaled():
    spec = workloads.CONFIGS["cfg2_bf16"].replace(U=3)
    a = make_user(spec, 1, 700)
    b = make_user(spec, 1, 700)
    for name in a:
        assert a[name].dtype == np.uint16 and np.array_equal(a[name], b[name])
    k = stored_values(a["k"]).astype(np.float64)
    v = stored_values(a["v"]).astype(np.float64)
    assert abs(k[:700].std() - 1 / 8) < 0.01 and abs(v[:700].std() - 1 / 8) < 0.01
    assert abs(k[700:].std() - TAIL_SCALE / 8) < 0.1          # padding holds large finite values
    assert np.isfinite(k).all() and np.isfinite(v).all()
    wl = workloads.make_workload(spec, users=[1])
    n = int(make_lens(spec)[1])
    assert wl.lens.tolist() == [n]
    assert np.array_equal(wl.k[0], make_user(spec, 1, n)["k"])
    assert np.array_equal(wl.k[0][:min(n, 700)], a["k"][:min(n, 700)])
    assert np.array_equal(wl.t0, wl.q)
    w = make_weights(spec)
    assert w["wq"].shape == (1, 64, 64)
    assert abs(stored_values(w["wk"]).std() - 1 / 8) < 0.01


def test_aligned_keys_have_the_requested_cosine():
    spec = workloads.CONFIGS["cfg3_high_fanout"].replace(U=1, L=2048)
    one = make_user(spec, 0, spec.L)
    q = stored_values(one["q"]).astype(np.float64)
    k = stored_values(one["k"]).astype(np.float64)
    cos = (k / np.linalg.norm(k, axis=1, keepdims=True)) @ (q / np.linalg.norm(q, axis=1, keepdims=True)).T
    best = cos.max(axis=1)
    n_aligned = int((best > 0.7).sum())
    assert abs(n_aligned - round(0.05 * spec.L)) <= 2
    assert abs(np.median(best[best > 0.7]) - 0.8) < 0.01
