"""Parity of the 1.60-bit (g = 5) path against the CPU oracle, through the C ABI.

Same bar as the 2-bit path: packed bytes and INT32 accumulators bit-exact, fp32 output within 1e-5 relative of the
oracle's fp64 value.  The oracle's GEMM is the plain definition and does not know about packing at all.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import oracle as O
from paper_2512_06443_amd import workloads as wl

pytestmark = pytest.mark.gpu

RTOL = 1e-5


@pytest.fixture(scope="module")
def B(vlut_lib_path):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2512_06443_amd import binding
    binding.lib()
    yield binding
    binding.set_plan_g5(0, 0)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_y(y_gpu, y_ref):
    y_gpu = y_gpu.astype(np.float64)
    err = np.abs(y_gpu - y_ref)
    assert np.all(err <= RTOL * np.abs(y_ref)), f"max rel err {np.max(err / np.maximum(np.abs(y_ref), 1e-300))}"
    assert np.all(y_gpu[y_ref == 0.0] == 0.0)


def run_case(B, W, w_scale, x, plan=(0, 0), tag=""):
    print(f"case g5 {tag} M={W.shape[0]} K={W.shape[1]} N={x.shape[0]} plan={plan}", flush=True)
    M, K = W.shape
    _, _, acc_ref, y_ref = O.mpgemm(W, w_scale, x)
    B.set_plan_g5(*plan)
    try:
        packed = B.pack_weights_g5(dev(W))
        a_q, a_s = B.quantize_act(dev(x))
        y, acc = B.mpgemm_g5(packed, float(w_scale), a_q, a_s, M, want_acc=True)
        torch.cuda.synchronize()
    finally:
        B.set_plan_g5(0, 0)
    assert np.array_equal(acc.cpu().numpy(), acc_ref), "int32 accumulators differ"
    check_y(y.cpu().numpy(), y_ref)


def test_pack_g5_bytes_match_oracle_and_padding(B):
    L = B.lib()
    for (M, K) in [(256, 320), (10, 100), (257, 260), (4, 80)]:
        W = wl.ternary(M + K, M, K, 0.4)
        packed = B.pack_weights_g5(dev(W)).cpu().numpy()
        idx = O.pack_indices(W, 5)
        assert packed.size == L.vlut_packed_weight_bytes_g5(M, K) and packed.max() < 243
        offs = np.array([[L.vlut_packed_offset_g5(M, K, m, kg) for kg in range(K // 5)] for m in range(M)])
        assert np.array_equal(packed[offs], idx)
        pad = np.ones(packed.size, bool)
        pad[offs.ravel()] = False
        assert np.all(packed[pad] == 121)                   # padding is the all-zero pattern
    with pytest.raises(B.VlutError) as e:
        bad = wl.ternary(1, 8, 80, 0.4)
        bad[3, 17] = -2
        B.pack_weights_g5(dev(bad))
    assert e.value.status == B.VLUT_ERR_VALUE


def test_g5_small_and_ragged(B):
    W, s, x = wl.small_case(71, 257, 260, 130)              # 52 groups: not a multiple of the 64 of a dword stage
    run_case(B, W, s, x, tag="ragged")
    W, s, x = wl.small_case(72, 70, 1020, 7)
    run_case(B, W, s, x, plan=(1, 1), tag="n7")
    W, s, x = wl.small_case(73, 5, 20, 1)                   # smallest K of the whole path, GEMV
    run_case(B, W, s, x, tag="tiny")


@pytest.mark.parametrize("R", [1, 2, 4, 6, 9, 12, 14])
def test_g5_every_rows_per_wave(B, R):
    M = 48 * R * 2 - 37                                     # two row tiles, the second one ragged
    W, s, x = wl.small_case(80 + R, M, 500, 33)
    run_case(B, W, s, x, plan=(R, 1), tag=f"R{R}")


@pytest.mark.parametrize("R,S", [(1, 1), (6, 1), (4, 2), (2, 3), (9, 2), (14, 4)])
def test_g5_int32_widening_and_split_k(B, R, S):
    # K = 5120 -> 1024 groups -> 16 dword stages = 64 lookups per lane: above the block bound 51 unless split
    W, s, x = wl.small_case(90 + R + S, 300, 5120, 40)
    run_case(B, W, s, x, plan=(R, S), tag=f"widen R{R} S{S}")


def test_g5_int16_block_is_overflow_free_at_the_extremes(B):
    # all |q| = 127 and all weights equal: 48 lookups of +-635 reach +-30480 before the widening (Sec. 3.4 bound 51)
    M, K, N = 64, 5120, 16
    x = np.full((N, K), 5.0, np.float32)
    x[1::2] = -5.0
    for sign in (1, -1):
        W = np.full((M, K), sign, np.int8)
        run_case(B, W, np.float32(0.01), x, plan=(2, 1), tag=f"extreme{sign}")
        run_case(B, W[:, :2560], np.float32(0.01), x[:, :2560], plan=(9, 1), tag=f"extreme{sign}-no-widening")


def test_g5_ldy_and_acc_only(B):
    W, s, x = wl.small_case(95, 100, 260, 12)
    _, _, acc_ref, y_ref = O.mpgemm(W, s, x)
    packed = B.pack_weights_g5(dev(W))
    a_q, a_s = B.quantize_act(dev(x))
    ybig = torch.full((12, 128), -7.0, device="cuda")
    B.mpgemm_g5(packed, float(s), a_q, a_s, 100, y=ybig[:, :100])
    yb = ybig.cpu().numpy()
    check_y(yb[:, :100], y_ref)
    assert np.all(yb[:, 100:] == -7.0)                      # nothing written past M


@pytest.mark.parametrize("M,plan", [(257, (2, 1)), (257, (2, 3)), (260, (4, 2)), (262, (1, 1))])
def test_g5_output_row_stride_and_alignment(B, M, plan):
    # Outputs leave four rows at a time where y (or the split-K slots) is aligned for it, row by row otherwise and in
    # the last rows of a ragged M; the padding of y stays untouched.
    K, N = 1040, 40
    W, s, x = wl.small_case(190 + M, M, K, N)
    _, _, acc_ref, y_ref = O.mpgemm(W, s, x)
    packed = B.pack_weights_g5(dev(W))
    a_q, a_s = B.quantize_act(dev(x))
    B.set_plan_g5(*plan)
    try:
        for ldy, off in ((M, 0), ((M + 3) // 4 * 4, 0), ((M + 3) // 4 * 4 + 4, 0), (M + 5, 0), ((M + 3) // 4 * 4 + 4, 1)):
            print(f"g5 case out M={M} plan={plan} ldy={ldy} offset={off}", flush=True)
            buf = torch.full((N * ldy + 8,), -7.0, device="cuda")
            y = buf[off:off + N * ldy].view(N, ldy)[:, :M]
            _, acc = B.mpgemm_g5(packed, float(s), a_q, a_s, M, y=y, want_acc=True)
            torch.cuda.synchronize()
            assert np.array_equal(acc.cpu().numpy(), acc_ref)
            full = buf.cpu().numpy()
            yy = full[off:off + N * ldy].reshape(N, ldy)
            check_y(yy[:, :M], y_ref)
            assert np.all(yy[:, M:] == -7.0) and np.all(full[:off] == -7.0) and np.all(full[off + N * ldy:] == -7.0)
    finally:
        B.set_plan_g5(0, 0)


def test_g5_full_size_bitnet2b_ffn_up(B):
    M, K, N = 6912, 2560, 128
    W = wl.ternary(0, M, K, 0.4)
    w_scale = wl.latent_weight_scale(0, M, K)
    x = wl.activations(0, N, K)
    packed = B.pack_weights_g5(dev(W))
    a_q, a_s = B.quantize_act(dev(x))
    q_ref, s_ref = O.quantize(x)
    y, acc = B.mpgemm_g5(packed, float(w_scale), a_q, a_s, M, want_acc=True)   # automatic plan = the bench's plan
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate([rng.integers(0, M, 64), [0, 1, 2, 3, M - 1, M - 2, M // 2]]))
    acc_ref = O.gemm_acc(W[rows], q_ref)
    assert np.array_equal(acc.cpu().numpy()[rows], acc_ref)
    check_y(y.cpu().numpy()[:, rows], O.epilogue(acc_ref, w_scale, s_ref))
    colsum = W.astype(np.int64).sum(0) @ q_ref.astype(np.int64)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64).sum(0), colsum)


# ------------------------------------------------------------------ mixed 1.60-bit / 2-bit packing (Sec. 3.3)
def test_mixed_packing_blob_is_the_two_blobs(B):
    L = B.lib()
    for (M, K) in [(10, 116), (257, 4096), (33, 16), (64, 2560)]:
        W = wl.ternary(700 + M + K, M, K, 0.4)
        K5 = L.vlut_mixed_k5(K)
        assert K5 == (K // 20) * 20
        blob = B.pack_weights_mixed(dev(W)).cpu().numpy()
        b5 = L.vlut_packed_weight_bytes_g5(M, K5) if K5 else 0
        b4 = L.vlut_packed_weight_bytes(M, K - K5) if K > K5 else 0
        assert blob.size == b5 + b4 == L.vlut_packed_weight_bytes_mixed(M, K)
        if K5:                                              # bytes of the first part against the oracle's indices
            idx = O.pack_indices(np.ascontiguousarray(W[:, :K5]), 5)
            offs = np.array([[L.vlut_packed_offset_g5(M, K5, m, kg) for kg in range(K5 // 5)] for m in range(M)])
            assert np.array_equal(blob[:b5][offs], idx)
        if K > K5:
            idx = O.pack_indices(np.ascontiguousarray(W[:, K5:]), 4)
            offs = np.array([[L.vlut_packed_offset(M, K - K5, m, kg) for kg in range((K - K5) // 4)] for m in range(M)])
            assert np.array_equal(blob[b5:][offs], idx)
    with pytest.raises(B.VlutError) as e:
        bad = wl.ternary(1, 8, 36, 0.4)
        bad[3, 33] = 2                                      # in the 2-bit part
        B.pack_weights_mixed(dev(bad))
    assert e.value.status == B.VLUT_ERR_VALUE


@pytest.mark.parametrize("M,K,N", [(257, 116, 33), (300, 4096, 40), (64, 16, 8), (130, 2560, 17), (640, 6912, 1),
                                    (100, 14336, 9), (48, 36, 130)])
def test_mixed_packing_mpgemm(B, M, K, N):
    print(f"mixed case M={M} K={K} N={N}", flush=True)
    W, s, x = wl.small_case(710 + M + N, M, K, N)
    _, _, acc_ref, y_ref = O.mpgemm(W, s, x)
    blob = B.pack_weights_mixed(dev(W))
    a_q, a_s = B.quantize_act(dev(x))
    y, acc = B.mpgemm_mixed(blob, float(s), a_q, a_s, M, want_acc=True)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy(), acc_ref)
    check_y(y.cpu().numpy(), y_ref)
    # close to 1.6 bits per weight for long rows: the 2-bit part is at most 16 features (one 16-byte tile row)
    if K >= 2560 and M % 4 == 0:
        assert blob.numel() * 8 / (M * K) < 1.65
