"""GPU parity of the softmax-aggregation variant of STA (the ablation of Sec. 4.4.1) against the fp64 checker, element
by element: stored inputs on both sides, tolerances as for STA (fp32 1e-5, bf16 2e-2 per output vector)."""
import math

import numpy as np
import pytest

import oracle
import workloads

from parity_util import TOL, to_device, to_host_f64, vec_rel_err

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")

VARIANTS = {"auto": 0, "generic": 1, "mfma": 2, "stream": 3}

CASES = {
    # dtype, U, C, L, d_q, d, w, heads, gamma scale, lens
    "paper_default_two_heads": ("bf16", 6, 1, 1000, 32, 128, 10, 2, 1.0, [1000, 995, 404, 7, 0, 1000]),
    "wide_same_lane_split": ("bf16", 3, 2, 700, 128, 128, 20, 1, 1.0, [700, 65, 21]),
    "eight_candidates": ("bf16", 2, 8, 400, 64, 64, 30, 2, 1.0, [400, 31]),
    "sharp_scores": ("bf16", 2, 3, 333, 64, 128, 25, 1, 0.05, [333, 100]),        # near one-hot: the maximum moves often
    "long_segments": ("bf16", 2, 2, 1024, 64, 64, 256, 1, 1.0, [1024, 300]),       # generic kernel (long-segment shape)
    "many_candidates": ("bf16", 2, 40, 256, 32, 128, 64, 1, 1.0, [256, 100]),      # matrix cores, 2 waves
    # the matrix-core kernel: online softmax per candidate and head, partial blocks masked, every workgroup size
    "mfma_paper_setting_ranking": ("bf16", 2, 200, 1000, 32, 128, 10, 2, 1.0, [1000, 404]),
    "mfma_sharp_long_segments": ("bf16", 2, 20, 700, 64, 64, 300, 1, 0.05, [700, 301]),   # the maximum moves between blocks
    "mfma_four_waves_wide": ("bf16", 3, 100, 333, 128, 128, 50, 2, 0.3, [333, 51, 0]),
    "mfma_four_heads": ("bf16", 2, 40, 300, 64, 128, 30, 4, 0.5, [300, 31]),
    "f32_three_heads": ("f32", 2, 3, 130, 24, 48, 16, 3, 1.0, [130, 50]),
    "f32_sharp": ("f32", 1, 4, 96, 16, 16, 12, 1, 0.02, [90]),
}


def _store(x, dtype):
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        bits = workloads.f32_to_bf16_bits(x)
        return bits, workloads.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


@pytest.mark.parametrize("variant", ["auto", "generic", "stream", "mfma"])
@pytest.mark.parametrize("name", list(CASES))
def test_softmax_variant_matches_checker(name, variant):
    import torch
    dtype, U, C, L, dq, d, w, heads, gscale, lens = CASES[name]
    rng = np.random.default_rng(300 + sum(map(ord, name)))
    (qs, qv), (ks, kv), (vs, vv) = (_store(rng.normal(size=s), dtype) for s in ((U, C, dq), (U, L, dq), (U, L, d)))
    lens = np.array(lens, dtype=np.int32)
    gamma = gscale * math.sqrt(dq / heads)
    print(f"case {name} variant {variant}", flush=True)
    ref, cnt_ref = oracle.sta_forward(qv, kv, vv, lens, w, gamma, heads=heads, softmax=True)
    try:
        seg, cnt = laser.laser_sta_forward(to_device(qs), to_device(ks), to_device(vs), to_device(lens), w, gamma,
                                           heads=heads, softmax=True, variant=VARIANTS[variant])
    except laser.LaserError as e:
        if e.code == 4 and variant != "auto":
            pytest.skip("variant does not take this case")
        raise
    torch.cuda.synchronize()
    assert np.array_equal(cnt.cpu().numpy(), cnt_ref)
    err = vec_rel_err(to_host_f64(seg), ref)
    print(f"  max vector-relative error {err:.3e}", flush=True)
    assert err <= TOL[dtype]
    # not the sigmoid form
    sig, _ = laser.laser_sta_forward(to_device(qs), to_device(ks), to_device(vs), to_device(lens), w, gamma, heads=heads,
                                     want_cnt=False)
    torch.cuda.synchronize()
    assert not torch.equal(sig, seg)
