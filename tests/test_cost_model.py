"""P7: the repo's reproduction of the paper's analytic cost model against the numbers the paper prints."""
import os

import numpy as np

from paper_2602_11562_amd import cost_model as cm

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    rows = {}
    with open(os.path.join(HERE, "golden", "paper_flops.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, val, tol = line.split()[:3]
            rows[name] = (float(val), float(tol))
    return rows


def test_p7_paper_printed_flops():
    g = _golden()
    L, d, dq, w, r, M = 1000, 128, 32, 10, 4, 2
    got = {
        "self_attention": cm.c_self_attention(L, d),
        "laser": cm.c_laser(L, d, dq, w, r, M),
        "target_attention": cm.c_target_attention(L, d),
        "din_table": cm.c_target_attention(L, d),
        "rel_flops_w5": cm.c_laser(L, d, dq, 5, r, M) / cm.c_laser(L, d, dq, 10, r, M),
        "rel_flops_w10": 1.0,
        "rel_flops_w20": cm.c_laser(L, d, dq, 20, r, M) / cm.c_laser(L, d, dq, 10, r, M),
    }
    assert set(got) == set(g)
    for name, (val, tol) in g.items():
        assert abs(got[name] - val) <= tol * val + 1e-12, (name, got[name], val)


def test_cost_model_is_self_consistent():
    L, d, dq, w, r, M = 1000, 128, 32, 10, 4, 2
    # C_STA = C_proj + C_ffn (the attention term is dropped as negligible in the paper's sum)
    assert cm.c_sta(L, d, dq, w, r) == cm.c_proj(L, d, dq) + cm.c_ffn(L, d, w, r)
    # C_LASER ~ C_STA + (L/w) 2 M d^2
    assert abs(cm.c_laser(L, d, dq, w, r, M) - (cm.c_sta(L, d, dq, w, r) + (L / w) * 2 * M * d * d)) < 1e-6
    assert cm.c_attn(L, d, dq) == 1.6e5
    assert abs(cm.c_gsta(L, d, w, M) - 6.6e6) / 6.6e6 < 0.01


def test_kernel_accounting_matches_hand_numbers_for_the_headline_workload():
    # 32 users x 256 candidates, L=4096, d=d_q=128, w=128, full lengths, bf16
    lens = np.full(32, 4096)
    assert abs(cm.sta_flops(lens, 256, 128, 128) - 17.18e9) / 17.18e9 < 1e-3
    b = cm.sta_bytes(lens, 32, 256, 4096, 128, 128, 128, "bf16")
    assert abs(b - (67.1e6 + 2.1e6 + 67.1e6)) / 136.3e6 < 2e-3


def test_whole_path_accounting_for_the_headline_workload():
    # K, V 67.1 MB + Q, t0 4.2 MB + weights 0.1 MB + H' 67.1 MB + z 4.2 MB = 142.7 MB; 75.6 MB without H'
    lens = np.full(32, 4096)
    full = cm.path_bytes(lens, 32, 256, 4096, 128, 128, 128, 1, "bf16")
    zonly = cm.path_bytes(lens, 32, 256, 4096, 128, 128, 128, 1, "bf16", seg_out_written=False)
    assert abs(full - 142.7e6) / 142.7e6 < 2e-3 and abs(zonly - 75.6e6) / 75.6e6 < 2e-3
    assert abs(full - zonly - 32 * 256 * 32 * 128 * 2) < 1
    f = cm.path_flops(lens, 256, 128, 128, 128, 1)
    assert abs(f - (17.18e9 + 0.67e9)) / 17.85e9 < 0.02
