"""GPU parity of STA with several heads (Sec. 4.1.2 setting: 2 heads, d_q = 16 per head, value width d) against the
fp64 checker, element by element. Inputs are stored values on both sides; tolerances as for STA (fp32 1e-5, bf16 2e-2).
"""
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
    # dtype, U, C, L, d_q, d, w, heads, lens
    "paper_default_two_heads": ("bf16", 6, 1, 1000, 32, 128, 10, 2, [1000, 995, 404, 7, 0, 1000]),
    "long_segments_same_lane_split": ("bf16", 3, 4, 1024 + 77, 64, 64, 128, 2, [1101, 640, 129]),
    "long_segments_narrow_keys": ("bf16", 2, 8, 1500, 32, 64, 300, 2, [1500, 301]),
    "short_segments_wide": ("bf16", 3, 2, 700, 128, 128, 64, 2, [700, 65, 64]),
    "short_segments_three_candidates": ("bf16", 4, 3, 333, 64, 128, 20, 2, [333, 21, 20, 1]),
    "many_candidates_two_heads": ("bf16", 2, 40, 512, 32, 128, 64, 2, [512, 100]),      # matrix cores, 2 waves
    # the matrix-core kernel with two heads: every workgroup size, short segments of the paper's setting included
    "mfma_paper_setting_ranking": ("bf16", 2, 200, 1000, 32, 128, 10, 2, [1000, 404]),   # 8 waves, 2 tile buffers
    "mfma_one_wave_wide": ("bf16", 3, 20, 300, 128, 128, 64, 2, [300, 65, 0]),
    "mfma_four_waves_narrow_values": ("bf16", 2, 100, 700, 64, 64, 128, 2, [700, 129]),
    "mfma_four_heads": ("bf16", 2, 70, 400, 64, 128, 40, 4, [400, 41]),
    "mfma_four_heads_wide_keys": ("bf16", 1, 150, 300, 128, 128, 64, 4, [290]),
    "four_heads": ("bf16", 2, 5, 200, 32, 64, 16, 4, [200, 17]),                         # generic kernel
    "f32_three_heads": ("f32", 2, 3, 130, 24, 48, 16, 3, [130, 50]),
}


def _store(x, dtype):
    x = np.asarray(x, dtype=np.float32)
    if dtype == "bf16":
        bits = workloads.f32_to_bf16_bits(x)
        return bits, workloads.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


def _case(name):
    dtype, U, C, L, dq, d, w, heads, lens = CASES[name]
    rng = np.random.default_rng(500 + sum(map(ord, name)))
    qs, qv = _store(rng.normal(size=(U, C, dq)), dtype)
    ks, kv = _store(rng.normal(size=(U, L, dq)), dtype)
    vs, vv = _store(rng.normal(size=(U, L, d)), dtype)
    return dtype, (qs, ks, vs), (qv, kv, vv), np.array(lens, dtype=np.int32), w, heads, math.sqrt(dq / heads)


@pytest.mark.parametrize("variant", ["auto", "generic", "stream", "mfma"])
@pytest.mark.parametrize("name", list(CASES))
def test_heads_match_checker(name, variant):
    import torch
    dtype, stored, values, lens, w, heads, gamma = _case(name)
    print(f"case {name} variant {variant}", flush=True)
    ref, cnt_ref = oracle.sta_forward(*values, lens, w, gamma, heads=heads)
    q, k, v = (to_device(x) for x in stored)
    try:
        seg, cnt = laser.laser_sta_forward(q, k, v, to_device(lens), w, gamma, heads=heads, variant=VARIANTS[variant])
    except laser.LaserError as e:
        if e.code == 4 and variant != "auto":
            pytest.skip("variant does not take this case")
        raise
    torch.cuda.synchronize()
    assert np.array_equal(cnt.cpu().numpy(), cnt_ref)
    err = vec_rel_err(to_host_f64(seg), ref)
    print(f"  max vector-relative error {err:.3e}", flush=True)
    assert err <= TOL[dtype]


def test_one_head_through_the_heads_entry_point_gives_the_same_bits():
    import torch
    dtype, stored, values, lens, w, heads, gamma = _case("short_segments_three_candidates")
    q, k, v = (to_device(x) for x in stored)
    lib = laser.load_library()
    U, C, dq = q.shape
    L, d = v.shape[1], v.shape[2]
    S = -(-L // w)
    a, _ = laser.laser_sta_forward(q, k, v, to_device(lens), w, gamma, want_cnt=False)
    b = torch.empty_like(a)
    code = lib.laser_sta_forward_heads(q.data_ptr(), k.data_ptr(), v.data_ptr(), to_device(lens).data_ptr(), U, C, L, dq,
                                       d, w, gamma, 1, laser.LASER_BF16, b.data_ptr(), None, None, 0)
    torch.cuda.synchronize()
    assert code == 0 and b.shape == (U, C, S, d)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_heads_differ_from_one_head():
    """A guard against a kernel that ignores the head count: with two heads the result is not the one-head result."""
    import torch
    dtype, stored, values, lens, w, heads, gamma = _case("paper_default_two_heads")
    q, k, v = (to_device(x) for x in stored)
    one, _ = laser.laser_sta_forward(q, k, v, to_device(lens), w, gamma, want_cnt=False)
    two, _ = laser.laser_sta_forward(q, k, v, to_device(lens), w, gamma, want_cnt=False, heads=2)
    torch.cuda.synchronize()
    assert not torch.equal(one.view(torch.int16), two.view(torch.int16))
