"""vlut_mpgemm_static (the entry point that allocates nothing: split-K partial sums in the library's own static
device array) against vlut_mpgemm, through the C ABI: same bits on two calls in a row, the second on a smaller input
(so the scratch still holds the larger call's partial sums), then the oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle as O
from paper_2512_06443_amd import workloads as wl

pytestmark = pytest.mark.gpu


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


PLANS = {(2560, 6912, 64): (16, 6, 0, 4), (300, 1024, 40): (16, 1, 0, 4)}    # split-K plans: both calls need the scratch


def _prepare(B, seed, M, K, N):
    B.set_plan(*PLANS.get((M, K, N), (0, 0, 0, 0)))
    W, s, x = wl.small_case(seed, M, K, N)
    packed = B.pack_weights(dev(W))
    a_q, a_s = B.quantize_act(dev(x))
    y_ref, acc_ref = B.mpgemm(packed, float(s), a_q, a_s, M, want_acc=True)      # caller-provided workspace
    y = torch.full((N, M), -7.0, dtype=torch.float32, device="cuda")
    acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    B.set_plan(0, 0, 0, 0)
    return W, s, x, packed, a_q, a_s, y_ref, acc_ref, y, acc


def test_static_scratch_entry_matches_mpgemm_on_two_calls_in_a_row(B):
    assert B.static_scratch_bytes() == 32 << 20
    # (2560, 6912, 64) with four K splits, then a smaller input (300, 1024, 40), also split four ways
    big = _prepare(B, 700, 2560, 6912, 64)
    small = _prepare(B, 701, 300, 1024, 40)
    try:
        for (M, K, N) in ((2560, 6912, 64), (300, 1024, 40)):
            B.set_plan(*PLANS[(M, K, N)])
            plan = B.query_plan(M, K, N)
            print(f"static-scratch case M={M} K={K} N={N} plan={plan} ws={B.workspace_bytes(M, K, N)}", flush=True)
            assert plan[2] > 1 and 0 < B.workspace_bytes(M, K, N) <= B.static_scratch_bytes()
        for (W, s, x, packed, a_q, a_s, y_ref, acc_ref, y, acc), shape in ((big, (2560, 6912, 64)), (small, (300, 1024, 40))):
            B.set_plan(*PLANS[shape])                                            # the override only selects the launch plan
            B.mpgemm_static(packed, float(s), a_q, a_s, shape[0], y, acc)        # back to back on one stream
        torch.cuda.synchronize()
    finally:
        B.set_plan(0, 0, 0, 0)
    for (W, s, x, packed, a_q, a_s, y_ref, acc_ref, y, acc) in (big, small):
        assert torch.equal(acc, acc_ref) and torch.equal(y.view(torch.int32), y_ref.view(torch.int32))
        _, _, acc_o, y_o = O.mpgemm(W, s, x)
        assert np.array_equal(acc.cpu().numpy(), acc_o)
        err = np.abs(y.cpu().numpy().astype(np.float64) - y_o)
        assert np.all(err <= 1e-5 * np.abs(y_o))
    # a shape without split-K needs no scratch at all and takes the same entry point
    assert B.workspace_bytes(640, 2560, 16) == 0
    W, s, x, packed, a_q, a_s, y_ref, acc_ref, y, acc = _prepare(B, 702, 640, 2560, 16)
    B.mpgemm_static(packed, float(s), a_q, a_s, 640, y, acc)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc_ref) and torch.equal(y.view(torch.int32), y_ref.view(torch.int32))


def test_static_scratch_entry_rejects_what_does_not_fit(B):
    M, K, N = 4096, 14336, 1024
    B.set_plan(16, 6, 0, 4)                                                      # four K splits: 64 MiB of partial sums
    try:
        assert B.workspace_bytes(M, K, N) == 4 * M * N * 4 > B.static_scratch_bytes()
        d = torch.empty(16, dtype=torch.uint8, device="cuda")
        rc = B.lib().vlut_mpgemm_static(d.data_ptr(), 1.0, d.data_ptr(), d.data_ptr(), M, K, N, d.data_ptr(), M, None, None)
        assert rc == B.VLUT_ERR_UNSUPPORTED
    finally:
        B.set_plan(0, 0, 0, 0)
