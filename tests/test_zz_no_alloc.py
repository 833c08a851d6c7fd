"""laser_sta_backward_static (the entry point for callers that cannot allocate: its scratch is a fixed array inside the
library) against laser_sta_backward (caller-owned scratch) through the C ABI: same kernels, so the three gradients
must agree bit for bit, which is stricter than the 1e-5 bar of the backward parity tests; on two calls in a row, the
second with a smaller input (the array keeps the first call's contents), and once more with the first input. The
caller-owned path is itself compared with the fp64 checker in test_sta_backward_gpu.py; one case is repeated here so
that this file also stands alone. Sizes beyond the array are refused on the host."""
import math

import numpy as np
import pytest

import oracle
import workloads

from parity_util import to_device, to_host_f64, vec_rel_err

pytestmark = pytest.mark.gpu

laser = pytest.importorskip("paper_2602_11562_amd")
from paper_2602_11562_amd import binding


def _inputs(seed, dtype, U, C, L, dq, d, w, lens):
    rng = np.random.default_rng(seed)
    S = -(-L // w)

    def store(shape):
        x = rng.normal(size=shape).astype(np.float32)
        if dtype == "bf16":
            bits = workloads.f32_to_bf16_bits(x)
            return bits, workloads.bf16_bits_to_f32(bits).astype(np.float64)
        return x, x.astype(np.float64)

    host = [store(s) for s in ((U, C, dq), (U, L, dq), (U, L, d), (U, C, S, d))]
    lens = np.asarray(lens, dtype=np.int32)
    dev = [to_device(h[0]) for h in host] + [to_device(lens)]
    return dev, [h[1] for h in host], lens


def _both(dev, w, gamma):
    import torch
    q, k, v, dseg, lens = dev
    ref = laser.laser_sta_backward(q, k, v, lens, dseg, w, gamma)
    outs = [torch.full_like(r, float("nan")) for r in ref]          # allocated by the caller, before the call
    got = laser.laser_sta_backward_static(q, k, v, lens, dseg, w, gamma, *outs)
    torch.cuda.synchronize()
    return ref, got


def test_static_scratch_matches_caller_scratch_twice_in_a_row():
    import torch
    # the paper's training shape scaled down (one target per sample, w = 10, many runs per user), then a smaller
    # batch of another shape (three candidates, fp32), then the first again
    big = dict(dtype="bf16", U=96, C=1, L=1000, dq=32, d=128, w=10, lens=[1000 - 9 * i for i in range(96)])
    small = dict(dtype="f32", U=3, C=3, L=130, dq=24, d=48, w=16, lens=[130, 50, 0])
    order = [("big", big), ("small", small), ("big again", big)]
    first = None
    for name, c in order:
        print(f"case {name}: {c['U']} users x {c['C']} candidates, L {c['L']}, w {c['w']}", flush=True)
        dev, f64, lens = _inputs(77, **c)
        gamma = math.sqrt(c["dq"])
        need = binding.load_library().laser_sta_backward_work_bytes(c["U"], c["C"], c["L"], c["dq"], c["w"])
        assert 0 < need <= binding.STATIC_SCRATCH_BYTES
        ref, got = _both(dev, c["w"], gamma)
        for nm, a, b in zip(("dq", "dk", "dv"), got, ref):
            assert torch.equal(a, b), f"{name}: {nm} differs from the caller-scratch entry point"
        if name == "small":      # against the checker as well, at the backward tests' bar
            chk = oracle.sta_backward(f64[0], f64[1], f64[2], lens, c["w"], gamma, f64[3])
            for nm, a, b in zip(("dq", "dk", "dv"), got, chk):
                a = to_host_f64(a)
                if nm == "dk":
                    a, b = a.reshape(c["U"], -1), b.reshape(c["U"], -1)
                assert vec_rel_err(a, b) <= 1e-5, nm
        if name == "big":
            first = [g.clone() for g in got]
        if name == "big again":
            assert all(torch.equal(a, b) for a, b in zip(got, first))


def test_static_scratch_refuses_sizes_beyond_the_array():
    import torch
    U, C, L, dq, d, w = 2048, 8, 1024, 256, 64, 64          # 2048 x 1 run x 8 x 256 floats = 16 MiB of partial sums
    assert binding.load_library().laser_sta_backward_work_bytes(U, C, L, dq, w) > binding.STATIC_SCRATCH_BYTES
    z = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    f = lambda *s: torch.zeros(*s, dtype=torch.float32, device="cuda")
    tiny = z(1, 1, 8)
    # the size check comes first and reads no tensor: pass the real sizes with small stand-in buffers through the raw ABI
    lib = binding.load_library()
    code = lib.laser_sta_backward_static(tiny.data_ptr(), tiny.data_ptr(), tiny.data_ptr(), None, tiny.data_ptr(), U, C,
                                         L, dq, d, w, 1.0, binding.LASER_BF16, f(4).data_ptr(), f(4).data_ptr(),
                                         f(4).data_ptr(), None)
    assert code == 2
