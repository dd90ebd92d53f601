"""Seeded random shapes and launch plans through every entry point of the C ABI, against the CPU oracle.

All paths must give the oracle's INT32 accumulators exactly, an fp32 output within 1e-5 relative of the oracle's fp64
value, and (being the same fp32 operations on the same integers) the same output bits as vlut_mpgemm.
"""
import random

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle as O
from paper_2512_06443_amd import workloads as wl

pytestmark = pytest.mark.gpu

RTOL = 1e-5
ROWS_PER_WAVE = [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16]


@pytest.fixture(scope="module")
def B(vlut_lib_path):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_06443_amd import binding
    binding.lib()
    yield binding
    binding.set_plan(0, 0, 0, 0)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def cases():
    rnd = random.Random(12345)
    out = []
    while len(out) < 80:
        M = rnd.choice([1, 3, 17, 64, 130, 257, 700, 1500, 3000, 9000])
        K = 4 * rnd.choice([1, 2, 5, 16, 33, 64, 100, 257, 640, 1088, 1728])
        N = rnd.choice([1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 24, 31, 32, 33, 64, 130, 300])
        forced = rnd.random() < 0.5
        plan = (rnd.choice([1, 2, 4, 8, 16]), rnd.choice(ROWS_PER_WAVE), rnd.choice([0, 12, 14]),
                rnd.choice([1, 1, 2, 3, 5, 8])) if forced \
            else (0, 0, 0, 0)
        if M * K * N <= 6e8:
            out.append((len(out), M, K, N, plan))
    return out


@pytest.mark.parametrize("it,M,K,N,plan", cases())
def test_random_shape_and_plan(B, it, M, K, N, plan):
    print(f"random case {it}: M={M} K={K} N={N} plan={plan}", flush=True)
    W, s, x = wl.small_case(2000 + it, M, K, N)
    _, s_ref, acc_ref, y_ref = O.mpgemm(W, s, x)
    packed = B.pack_weights(dev(W))
    a_q, a_s = B.quantize_act(dev(x))
    B.set_plan(*plan)
    try:
        try:
            y, acc = B.mpgemm(packed, float(s), a_q, a_s, M, want_acc=True)
            y1, acc1, sc = B.mpgemm_f32(packed, float(s), dev(x), M, want_acc=True, want_scales=True)
        except B.VlutError as e:                             # a plan the shape does not admit is refused, not run
            assert plan != (0, 0, 0, 0) and e.status == B.VLUT_ERR_UNSUPPORTED
            return
    finally:
        B.set_plan(0, 0, 0, 0)
    outs = [("mpgemm", y, acc), ("mpgemm_f32", y1, acc1)]
    outs.append(("mixed",) + B.mpgemm_mixed(B.pack_weights_mixed(dev(W)), float(s), a_q, a_s, M, want_acc=True))
    if K % 5 == 0:
        outs.append(("g5",) + B.mpgemm_g5(B.pack_weights_g5(dev(W)), float(s), a_q, a_s, M, want_acc=True))
    outs.append(("mfma",) + B.mpgemm(packed, float(s), a_q, a_s, M, want_acc=True, mfma=True))
    torch.cuda.synchronize()
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    for name, yy, aa in outs:
        assert np.array_equal(aa.cpu().numpy(), acc_ref), name
        yg = yy.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(yg - y_ref) <= RTOL * np.abs(y_ref)), name
        assert torch.equal(yy, y), name
