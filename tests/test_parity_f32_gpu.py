"""Parity of vlut_mpgemm_f32 (quantisation inside the lookup kernels) against the CPU oracle, through the C ABI.

Same bar as the two-call path: token scales bitwise, INT32 accumulators bit-exact (they can only be right when every
INT8 code is), fp32 output within 1e-5 relative of the oracle's fp64 value.
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
    binding.set_plan(0, 0, 0, 0)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_y(y_gpu, y_ref):
    y_gpu = y_gpu.astype(np.float64)
    err = np.abs(y_gpu - y_ref)
    assert np.all(err <= RTOL * np.abs(y_ref)), f"max rel err {np.max(err / np.maximum(np.abs(y_ref), 1e-300))}"
    assert np.all(y_gpu[y_ref == 0.0] == 0.0)


def run_f32(B, W, w_scale, x, plan=None, fused=None, tag="", x_dev=None):
    """fused: None = the library's own choice (by cost), True/False = what the call must report.  A forced plan with
    16 sub-tables per table row always takes the fused kernel when the shape fits it."""
    M, K = W.shape
    N = x.shape[0]
    print(f"f32 case {tag} M={M} K={K} N={N} plan={plan}", flush=True)
    _, s_ref, acc_ref, y_ref = O.mpgemm(W, w_scale, x)
    B.set_plan(*(plan or (0, 0, 0, 0)))
    try:
        qp = B.query_plan_f32(M, K, N)
        assert fused is None or qp[4] == fused, qp
        packed = B.pack_weights(dev(W))
        y, acc, sc = B.mpgemm_f32(packed, float(w_scale), dev(x) if x_dev is None else x_dev, M, want_acc=True,
                                  want_scales=True)
        torch.cuda.synchronize()
    finally:
        B.set_plan(0, 0, 0, 0)
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), s_ref.view(np.uint32)), "token scales differ"
    assert np.array_equal(acc.cpu().numpy(), acc_ref), "int32 accumulators differ"
    check_y(y.cpu().numpy(), y_ref)
    return qp


def test_tiny_and_ragged(B):
    w = wl.WORKLOADS["tiny"]
    W, s, x = wl.make_case(w, w.linears[0], 8, 0)
    run_f32(B, W, s, x, tag="tiny")
    W, s, x = wl.small_case(411, 257, 260, 130)             # ragged in M, K (not a multiple of 256) and N
    run_f32(B, W, s, x, tag="ragged")
    W, s, x = wl.small_case(412, 70, 1024, 7)
    run_f32(B, W, s, x, tag="n7")
    W, s, x = wl.small_case(413, 5, 4, 3)                   # smallest K
    run_f32(B, W, s, x, tag="k4")


@pytest.mark.parametrize("R", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16])
def test_every_rows_per_wave(B, R):
    M = 48 * R * 2 - 37
    W, s, x = wl.small_case(420 + R, M, 512, 33)
    # the quantising variant of the kernel exists up to R = 14; wider forced plans take the two-launch form
    qp = run_f32(B, W, s, x, plan=(16, R, 0, 1), fused=R <= 14, tag=f"R{R}")
    assert qp[:3] == (16, R, 1)


@pytest.mark.parametrize("R,S", [(3, 1), (6, 1), (4, 3), (2, 6), (9, 2)])
def test_int32_widening_split_k_and_long_rows(B, R, S):
    # K = 4352: 17 stages; with S = 1 a lane does 68 > 64 lookups, so the INT16 blocks get widened (R <= 6); the
    # rows are longer than the 4096 values a thread keeps in registers, so the tail is read twice
    W, s, x = wl.small_case(430 + R + S, 300, 4352, 40)
    run_f32(B, W, s, x, plan=(16, R, 0, S), fused=True, tag=f"widen R{R} S{S}")


def test_split_k_ranges_past_the_register_cache(B):
    # K = 8640 in three ranges: the second and third range lie entirely in the part of the row that is read again
    W, s, x = wl.small_case(440, 200, 8640, 19)
    run_f32(B, W, s, x, plan=(16, 2, 0, 3), fused=True, tag="K8640 S3")
    run_f32(B, W, s, x, plan=(16, 4, 0, 1), fused=True, tag="K8640 S1 (34 stages: the largest range that fits)")


def test_shapes_the_fused_kernels_do_not_cover_take_two_launches(B):
    W, s, x = wl.small_case(450, 100, 9216, 40)             # 36 stages in one range do not fit next to the tables
    run_f32(B, W, s, x, plan=(16, 2, 0, 1), fused=False, tag="K9216 S1")
    run_f32(B, W, s, x, plan=(4, 2, 0, 1), fused=False, tag="J=4 forced")
    run_f32(B, W, s, x, plan=(16, 2, 0, 2), fused=True, tag="K9216 S2")
    run_f32(B, W, s, x, fused=False, tag="K9216 free plan")   # rows this long are cheaper to quantise once, ahead


def test_extremes_zero_tokens_and_outliers(B):
    M, K, N = 64, 2048, 16
    x = np.full((N, K), 5.0, np.float32)
    x[1::2] = -5.0
    for sign in (1, -1):
        run_f32(B, np.full((M, K), sign, np.int8), np.float32(0.5), x, tag=f"extreme {sign}")
    z = wl.activations(451, 11, 256)
    z[2] = 0.0                                              # a zero token: scale 0, codes 0
    z[3, :] = 3.25
    z[4, 0], z[4, 1], z[4, 2], z[4, 3] = 127.0, 0.5, 1.5, 2.5   # ties at inv == 1
    W, s, _ = wl.small_case(452, 100, 256, 11)
    run_f32(B, W, s, z, tag="zero token, ties")
    W = wl.ternary(453, 512, 1024, 0.35)
    run_f32(B, W, wl.latent_weight_scale(453, 512, 1024), wl.activations(453, 48, 1024, outlier_frac=0.01), tag="outliers")


def test_row_stride_and_unaligned_rows(B):
    W, s, x = wl.small_case(460, 100, 100, 37)
    big = np.full((37, 128), 1e9, np.float32)
    big[:, :100] = x
    run_f32(B, W, s, x, x_dev=dev(big)[:, :100], tag="ldx > K")
    odd = np.full((37, 103), 1e9, np.float32)               # rows start at odd addresses: scalar loads
    odd[:, 1:101] = x
    run_f32(B, W, s, x, x_dev=dev(odd)[:, 1:101], tag="unaligned rows")
    W1, s1, x1 = wl.small_case(461, 300, 1028, 2)
    odd = np.full((2, 1031), 1e9, np.float32)
    odd[:, 3:1031] = x1
    run_f32(B, W1, s1, x1, x_dev=dev(odd)[:, 3:1031], tag="unaligned rows, two tokens")


def test_two_kernel_quantiser_for_large_inputs(B):
    """More than about four million activation values: the quantiser inside vlut_mpgemm_f32 runs as two kernels
    (absmax per token, then chunks of 8 tokens per K range); same codes and scales, bit for bit.  Ragged last chunk,
    K ranges that do not divide K, rows that cannot be read as float4."""
    for (M, K, N, pad) in [(64, 8192, 520, 0), (40, 14336, 300, 0), (33, 8200, 515, 3)]:
        W, s, x = wl.small_case(480 + N, M, K, N)
        assert N * K >= 1 << 22
        if pad:                                              # rows start at addresses that are no multiple of 16
            big = np.full((N, K + pad + 1), 1e9, np.float32)
            big[:, 1:K + 1] = x
            run_f32(B, W, s, x, tag="two-kernel quantiser, unaligned", x_dev=dev(big)[:, 1:K + 1])
        else:
            run_f32(B, W, s, x, tag="two-kernel quantiser")


@pytest.mark.parametrize("M", [100, 5000, 10000, 20000, 40000])
def test_one_or_two_tokens_every_tile_shape(B, M):
    for N, K in ((1, 260), (2, 1028)):
        W, s, x = wl.small_case(470 + M % 97 + N, M, K, N)
        qp = run_f32(B, W, s, x, fused=True, tag=f"narrow M{M} N{N}")
        assert qp[0] == 0                                   # the one-or-two-token kernel


def test_one_or_two_tokens_long_rows(B):
    for N, K in ((1, 2560), (2, 6912), (2, 9216), (1, 14336)):   # beyond 8192 the tail of a row is read twice
        W, s, x = wl.small_case(480 + N, 130, K, N)
        run_f32(B, W, s, x, fused=True, tag=f"narrow K{K}")
    W, s, x = wl.small_case(483, 40, 36864, 2)              # 36 of at most 37 chunks of codes next to the tables
    run_f32(B, W, s, x, fused=True, tag="narrow K36864")
    # past that: two launches (the one-or-two-token kernel on the INT8 codes), or the general kernel with K split
    # into ranges whose codes fit when a plan asks for it
    W, s, x = wl.small_case(484, 40, 40000, 2)
    run_f32(B, W, s, x, fused=False, tag="K40000 at two tokens")
    qp = run_f32(B, W, s, x, plan=(16, 1, 0, 5), fused=True, tag="K40000 at two tokens, general kernel")
    assert qp[:3] == (16, 1, 5)


@pytest.mark.parametrize("N", [3, 4, 5, 6, 7, 8, 11, 16, 23, 32])
def test_few_tokens_one_launch_per_token_pair(B, N):
    # 3..32 tokens: the few-token kernel with a copy of its row tiles per token pair, while that grid is one round of
    # workgroups with few rows each; M picks the rows per workgroup, the odd N leave the last pair with one token
    for M, K in ((100, 260), (3000, 1028), (9000, 516), (130, 6912)):
        if N > 8 and M > 1000:
            continue
        W, s, x = wl.small_case(600 + 10 * N + M % 7, M, K, N)
        qp = run_f32(B, W, s, x, fused=True, tag=f"few tokens M{M} K{K} N{N}")
        assert qp[0] == 0 and qp[3] % ((N + 1) // 2) == 0
        assert qp[1] == {100: 32, 3000: 32 if N <= 4 else 64, 9000: 128 if N <= 6 else 256, 130: 32}[M] or N > 8
    M = 40000                                               # too many workgroups for one round: the general path
    W, s, x = wl.small_case(690 + N, M, 64, N)
    qp = run_f32(B, W, s, x, fused=False, tag=f"few tokens M{M} N{N}")
    assert qp[0] != 0


def test_few_tokens_long_rows_and_unaligned_rows(B):
    W, s, x = wl.small_case(695, 40, 40000, 5)              # codes do not fit next to the tables: quantiser + kernel
    run_f32(B, W, s, x, fused=False, tag="K40000 at five tokens")
    W, s, x = wl.small_case(696, 300, 1028, 7)
    odd = np.full((7, 1031), 1e9, np.float32)
    odd[:, 3:1031] = x
    run_f32(B, W, s, x, x_dev=dev(odd)[:, 3:1031], fused=True, tag="unaligned rows, seven tokens")


def test_stacked_matrices_with_row_scales(B):
    K = 516
    rows, scales = (130, 70, 71), (0.0159, 0.5, 3.25)
    Ws = [wl.ternary(490 + i, m, K, 0.4) for i, m in enumerate(rows)]
    W = np.concatenate(Ws, axis=0)
    M = W.shape[0]
    w_rows = np.concatenate([np.full(m, sc, np.float32) for m, sc in zip(rows, scales)])
    packed = B.pack_weights(dev(W))
    for plan, N in (((0, 0, 0, 0), 33), ((16, 2, 0, 3), 33), ((0, 0, 0, 0), 2), ((0, 0, 0, 0), 1), ((0, 0, 0, 0), 5),
                    ((0, 0, 0, 0), 16)):
        x = wl.activations(494 + N, N, K)
        print(f"f32 case stacked plan={plan} N={N}", flush=True)
        B.set_plan(*plan)
        try:
            y, acc, _ = B.mpgemm_f32(packed, dev(w_rows), dev(x), M, want_acc=True)
            torch.cuda.synchronize()
        finally:
            B.set_plan(0, 0, 0, 0)
        y, acc = y.cpu().numpy(), acc.cpu().numpy()
        r0 = 0
        for Wi, sc in zip(Ws, scales):
            _, _, acc_ref, y_ref = O.mpgemm(Wi, np.float32(sc), x)
            assert np.array_equal(acc[r0:r0 + Wi.shape[0]], acc_ref)
            check_y(y[:, r0:r0 + Wi.shape[0]], y_ref)
            r0 += Wi.shape[0]


def test_equals_the_two_call_path_bitwise_and_ldy(B):
    W, s, x = wl.small_case(500, 1000, 2560, 128)
    packed = B.pack_weights(dev(W))
    a_q, a_s = B.quantize_act(dev(x))
    y2, acc2 = B.mpgemm(packed, float(s), a_q, a_s, 1000, want_acc=True)
    ybig = torch.full((128, 1024), -7.0, device="cuda")
    _, acc1, sc = B.mpgemm_f32(packed, float(s), dev(x), 1000, y=ybig[:, :1000], want_acc=True, want_scales=True)
    torch.cuda.synchronize()
    assert torch.equal(acc1, acc2) and torch.equal(sc, a_s)
    assert torch.equal(ybig[:, :1000], y2)                  # the same fp32 operations in the same order
    assert bool((ybig[:, 1000:] == -7.0).all())             # nothing written past M


def test_argument_errors(B):
    W, s, x = wl.small_case(510, 64, 64, 4)
    packed = B.pack_weights(dev(W))
    xd = dev(x)
    L = B.lib()
    y = torch.empty((4, 64), device="cuda")
    args = lambda **kw: [kw.get("packed", packed.data_ptr()), 1.0, None, kw.get("x", xd.data_ptr()), kw.get("ldx", 64),
                         64, kw.get("K", 64), kw.get("N", 2), kw.get("y", y.data_ptr()), kw.get("ldy", 64), None, None,
                         None, 0, None]
    assert L.vlut_mpgemm_f32(*args()) == B.VLUT_OK
    assert L.vlut_mpgemm_f32(*args(x=None)) == B.VLUT_ERR_NULL
    assert L.vlut_mpgemm_f32(*args(packed=None)) == B.VLUT_ERR_NULL
    assert L.vlut_mpgemm_f32(*args(y=None)) == B.VLUT_ERR_NULL
    assert L.vlut_mpgemm_f32(*args(ldx=60)) == B.VLUT_ERR_SHAPE
    assert L.vlut_mpgemm_f32(*args(ldy=63)) == B.VLUT_ERR_SHAPE
    assert L.vlut_mpgemm_f32(*args(K=62)) == B.VLUT_ERR_SHAPE
    assert L.vlut_mpgemm_f32(*args(N=33)) == B.VLUT_ERR_NULL   # more than 32 tokens: the INT8 codes need a workspace
    torch.cuda.synchronize()
    # split-K needs the workspace
    B.set_plan(16, 1, 0, 2)
    try:
        W, s, x = wl.small_case(511, 64, 1024, 4)
        packed2, xd2 = B.pack_weights(dev(W)), dev(x)
        need = L.vlut_workspace_bytes_f32(64, 1024, 4)
        assert need == 256 + 2 * 64 * 4 * 4
        a2 = [packed2.data_ptr(), 1.0, None, xd2.data_ptr(), 1024, 64, 1024, 4, y.data_ptr(), 64, None, None]
        assert L.vlut_mpgemm_f32(*a2, None, 0, None) == B.VLUT_ERR_NULL
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        assert L.vlut_mpgemm_f32(*a2, ws.data_ptr(), need - 1, None) == B.VLUT_ERR_SMALL_BUFFER
        assert L.vlut_mpgemm_f32(*a2, ws.data_ptr(), need, None) == B.VLUT_OK
        torch.cuda.synchronize()
    finally:
        B.set_plan(0, 0, 0, 0)


@pytest.mark.parametrize("N", [1, 2, 5, 40])
def test_hip_graph_replays_match_eager(B, N):
    """vlut_mpgemm_f32 captured once (one kernel for a few tokens, quantiser + split-K lookup + sum otherwise)
    and replayed on changing inputs, with eager launches and synchronisations in between."""
    M, K = 300, 1024
    W = wl.ternary(585, M, K, 0.4)
    packed = B.pack_weights(dev(W))
    x_dev = torch.empty((N, K), dtype=torch.float32, device="cuda")
    y = torch.empty((N, M), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(B.lib().vlut_workspace_bytes_f32(M, K, N), 16), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    x_dev.copy_(dev(wl.activations(586, N, K)))
    with torch.cuda.stream(side):                           # warm-up outside the capture
        B.mpgemm_f32(packed, 0.02, x_dev, M, y=y, workspace=ws)
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        B.mpgemm_f32(packed, 0.02, x_dev, M, y=y, workspace=ws)
    for seed in (587, 588, 589):
        x = wl.activations(seed, N, K)
        x_dev.copy_(dev(x))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        y_graph = y.clone()
        y_eager, _, _ = B.mpgemm_f32(packed, 0.02, dev(x), M)   # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(y_graph, y_eager)
        check_y(y_graph.cpu().numpy(), O.mpgemm(W, np.float32(0.02), x)[3])


@pytest.mark.parametrize("M,K,N", [(1, 4, 1), (1, 4, 2), (1, 4, 3), (3, 8, 1), (5, 1024, 2), (1, 2560, 1), (2, 6912, 2),
                                    (7, 260, 1), (1, 4, 9), (4097, 4, 1), (33, 12, 2), (640, 2560, 3), (640, 2560, 8),
                                    (640, 2560, 9)])
def test_degenerate_shapes_through_every_entry_point(B, M, K, N):
    """Single rows, the smallest K, token counts next to the kernels' switch-over points: the one-call form, the
    two-call form and the mixed packing all give the oracle's numbers, and the first two the same bits."""
    print(f"degenerate case M={M} K={K} N={N}", flush=True)
    W, s, x = wl.small_case(900 + M + K + N, M, K, N)
    _, s_ref, acc_ref, y_ref = O.mpgemm(W, s, x)
    packed = B.pack_weights(dev(W))
    y1, acc1, sc = B.mpgemm_f32(packed, float(s), dev(x), M, want_acc=True, want_scales=True)
    a_q, a_s = B.quantize_act(dev(x))
    y2, acc2 = B.mpgemm(packed, float(s), a_q, a_s, M, want_acc=True)
    ym, accm = B.mpgemm_mixed(B.pack_weights_mixed(dev(W)), float(s), a_q, a_s, M, want_acc=True)
    torch.cuda.synchronize()
    for acc in (acc1, acc2, accm):
        assert np.array_equal(acc.cpu().numpy(), acc_ref)
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert torch.equal(y1, y2) and torch.equal(ym, y2)
    check_y(y1.cpu().numpy(), y_ref)
