"""Pins for the CPU oracle: every oracle function is checked against something
other than itself -- values the paper prints (tests/golden/paper_values.txt),
closed forms, invariants, numpy's integer matmul as an independent library
routine, and pure-Python brute force on tiny inputs."""
import itertools

import numpy as np
import pytest

from oracle import oracle as O
from paper_2512_06443_amd import workloads as wl


def _rand_q(rng, K, N, lo=-127, hi=127):
    return rng.integers(lo, hi + 1, size=(K, N), dtype=np.int64).astype(np.int8)


def _rand_w(rng, M, K):
    return rng.integers(-1, 2, size=(M, K), dtype=np.int64).astype(np.int8)


# ---------------------------------------------------------------- GetSign / pack
def test_worked_example_signs(golden):
    i = int(golden["example_index"][0])
    digits = [int(t) for t in golden["example_digits"]]
    signs = [int(t) for t in golden["example_signs"]]
    assert sum(d * 3 ** (3 - j) for j, d in enumerate(digits)) == i
    assert [O.get_sign(i, j, 4) for j in range(4)] == signs
    assert [d - 1 for d in digits] == signs


def test_pack_known_bytes(golden):
    signs = [int(t) for t in golden["example_signs"]]
    W = np.array([signs, [0, 0, 0, 0], [1, 1, 1, 1], [-1, -1, -1, -1], [0, 0, 0, 1], [1, 0, 0, 0]],
                 dtype=np.int8)
    idx = O.pack_indices(W)
    assert idx[:, 0].tolist() == [int(golden["example_index"][0]), 40, 80, 0, 41, 67]


@pytest.mark.parametrize("g,rows", [(4, 81), (5, 243)])
def test_pack_is_bijection_on_all_patterns(g, rows, golden):
    pats = np.array(list(itertools.product([-1, 0, 1], repeat=g)), dtype=np.int8)
    idx = O.pack_indices(pats, g)
    assert idx.shape == (rows, 1)
    # lexicographic order of patterns (first weight most significant) == 0..3^g-1
    assert idx[:, 0].tolist() == list(range(rows))
    assert int(idx.max()) == int(golden[f"index_max_g{g}"][0])
    assert np.array_equal(O.unpack_indices(idx, g), pats)
    # pack's digits agree with GetSign's digits
    for i in (0, 1, 23 % rows, rows // 2, rows - 1):
        assert [O.get_sign(i, j, g) for j in range(g)] == pats[i].tolist()


def test_pack_roundtrip_and_size():
    rng = np.random.default_rng(1)
    W = _rand_w(rng, 37, 52)
    idx = O.pack_indices(W)
    assert idx.dtype == np.uint8 and idx.size * 8 == 2 * W.size     # 2.00 bits per weight
    assert idx.max() < 81
    assert np.array_equal(O.unpack_indices(idx), W)


def test_pack_rejects_non_ternary():
    W = np.zeros((2, 4), dtype=np.int8)
    W[1, 2] = 2
    with pytest.raises(ValueError):
        O.pack_indices(W)
    with pytest.raises(ValueError):
        O.unpack_indices(np.array([[81]], dtype=np.uint8))


# ---------------------------------------------------------------- table T
def test_lut_worked_example_row(golden):
    rng = np.random.default_rng(2)
    q = _rand_q(rng, 12, 9)
    T = O.build_lut(q)
    c = [int(t) for t in golden["example_row_coeffs"]]
    i = int(golden["example_index"][0])
    for kg in range(3):
        a = q[4 * kg:4 * kg + 4].astype(np.int64)
        want = c[0] * a[0] + c[1] * a[1] + c[2] * a[2] + c[3] * a[3]
        assert np.array_equal(T[kg, i].astype(np.int64), want)
        assert np.array_equal(T[kg, i].astype(np.int64), -a[0] + a[1] + a[3])


def test_lut_structure_and_figure8_dependencies(golden):
    rng = np.random.default_rng(3)
    q = _rand_q(rng, 8, 33)
    T = O.build_lut(q).astype(np.int64)
    assert T.shape == (2, 81, 33)
    for kg in range(2):
        a = q[4 * kg:4 * kg + 4].astype(np.int64)
        assert not T[kg, 40].any()                                  # all-zero pattern
        assert np.array_equal(T[kg, ::-1], -T[kg])                  # row 80-i = -row i
        assert np.array_equal(T[kg, 80], a.sum(0))
        for j, p in enumerate((27, 9, 3, 1)):                       # single-trit rows
            assert np.array_equal(T[kg, 40 + p], a[j])
            assert np.array_equal(T[kg, 40 - p], -a[j])
        f, ta, tb, neg = (int(golden[k][0]) for k in ("dep_from", "dep_to_a", "dep_to_b", "dep_negated"))
        assert np.array_equal(T[kg, ta], T[kg, f] - a[3])           # 79 -> 78
        assert np.array_equal(T[kg, tb], T[kg, f] + a[3])           # 79 -> 80
        assert np.array_equal(T[kg, neg], -T[kg, tb])               # 80 -> 0
    assert np.abs(T).max() <= 4 * 127


def test_lut_equals_pattern_matrix_product():
    """Row i of a sub-table is (pattern i) . (4 activation rows): numpy matmul as the routine."""
    rng = np.random.default_rng(4)
    q = _rand_q(rng, 20, 17)
    pats = np.array(list(itertools.product([-1, 0, 1], repeat=4)), dtype=np.int64)
    T = O.build_lut(q)
    for kg in range(5):
        assert np.array_equal(T[kg].astype(np.int64), pats @ q[4 * kg:4 * kg + 4].astype(np.int64))


def test_lut_extreme_values_fit_int16():
    q = np.full((4, 3), 127, dtype=np.int8)
    q[:, 1] = -127
    T = O.build_lut(q)
    assert T[0, 80].tolist() == [508, -508, 508] and T[0, 0].tolist() == [-508, 508, -508]


def test_lut_g5():
    rng = np.random.default_rng(5)
    q = _rand_q(rng, 10, 6)
    pats = np.array(list(itertools.product([-1, 0, 1], repeat=5)), dtype=np.int64)
    T = O.build_lut(q, g=5)
    assert T.shape == (2, 243, 6)
    assert np.array_equal(T[1].astype(np.int64), pats @ q[5:10].astype(np.int64))


def test_lut_g5_structure_and_packing_density():
    """1.60-bit packing (Sec. 3.3): five weights per byte, 243 rows; the all-zero pattern is row 121, rows mirror
    around it, the extremes reach 5 * 127 and the INT16 block bound of Sec. 3.4 gives 51 lookups."""
    rng = np.random.default_rng(55)
    q = _rand_q(rng, 10, 4)
    q[:5, 0] = 127
    T = O.build_lut(q, g=5).astype(np.int64)
    assert not T[:, 121].any()
    assert np.array_equal(T[:, ::-1], -T)                                  # T[242 - i] = -T[i]
    assert np.array_equal(T[0, 242], q[:5].astype(np.int64).sum(axis=0)) and T[0, 242, 0] == 635
    for j, p3 in enumerate((81, 27, 9, 3, 1)):                             # single non-zero digit -> +-A[j]
        assert np.array_equal(T[1, 121 + p3], q[5 + j].astype(np.int64))
        assert np.array_equal(T[1, 121 - p3], -q[5 + j].astype(np.int64))
    W = _rand_w(rng, 7, 40)
    idx = O.pack_indices(W, 5)
    assert idx.size * 8 == 1.6 * W.size and idx.max() < 243
    assert 32767 // (127 * 5) == 51 and 51 * 635 <= 32767 < 52 * 635


# ---------------------------------------------------------------- integer GEMM
def test_gemm_bruteforce_tiny():
    rng = np.random.default_rng(6)
    for (M, K, N) in [(1, 4, 1), (3, 8, 2), (5, 4, 7), (8, 8, 8)]:
        W, q = _rand_w(rng, M, K), _rand_q(rng, K, N)
        acc = O.gemm_acc(W, q)
        for m in range(M):
            for n in range(N):
                assert int(acc[m, n]) == sum(int(W[m, k]) * int(q[k, n]) for k in range(K))


@pytest.mark.parametrize("M,K,N", [(17, 64, 5), (129, 256, 33), (64, 1024, 130)])
def test_gemm_matches_numpy_int64_matmul(M, K, N):
    rng = np.random.default_rng(M + K + N)
    W, q = _rand_w(rng, M, K), _rand_q(rng, K, N)
    assert np.array_equal(O.gemm_acc(W, q).astype(np.int64), W.astype(np.int64) @ q.astype(np.int64))


def test_gemm_special_weights():
    rng = np.random.default_rng(7)
    K, N = 32, 11
    q = _rand_q(rng, K, N)
    assert not O.gemm_acc(np.zeros((9, K), np.int8), q).any()
    eye = np.eye(K, dtype=np.int8)
    assert np.array_equal(O.gemm_acc(eye, q), q.astype(np.int32))
    assert np.array_equal(O.gemm_acc(-eye, q), -q.astype(np.int32))
    sel = np.zeros((4, K), np.int8)
    sel[0, 5], sel[1, 31], sel[2, 0], sel[3, 17] = 1, -1, 1, -1
    want = np.stack([q[5], -q[31].astype(np.int32), q[0], -q[17].astype(np.int32)]).astype(np.int32)
    assert np.array_equal(O.gemm_acc(sel, q), want)
    # not symmetric in its operands: a transposed-operand bug would fail here
    W = _rand_w(rng, K, K)
    assert not np.array_equal(O.gemm_acc(W, q), O.gemm_acc(W.T.copy(), q))


def test_gemm_linearity_and_permutation():
    rng = np.random.default_rng(8)
    M, K, N = 21, 48, 10
    W = _rand_w(rng, M, K)
    q1, q2 = _rand_q(rng, K, N, -60, 60), _rand_q(rng, K, N, -60, 60)
    a1, a2 = O.gemm_acc(W, q1), O.gemm_acc(W, q2)
    assert np.array_equal(O.gemm_acc(W, (q1 + q2).astype(np.int8)), a1 + a2)
    assert np.array_equal(O.gemm_acc(W, (-q1).astype(np.int8)), -a1)
    perm = rng.permutation(K)
    assert np.array_equal(O.gemm_acc(W[:, perm].copy(), q1[perm].copy()), a1)


def test_gemm_extreme_sum_and_overflow_guard():
    K = 14336
    W = np.ones((2, K), np.int8)
    W[1] = -1
    q = np.full((K, 3), 127, np.int8)
    q[:, 2] = -127
    acc = O.gemm_acc(W, q)
    assert acc.tolist() == [[127 * K, 127 * K, -127 * K], [-127 * K, -127 * K, 127 * K]]
    with pytest.raises(ValueError):
        O.gemm_acc(np.full((1, 4), 3, np.int8), q[:4])


def test_all_patterns_matrix_reproduces_table():
    """M = 81 rows enumerating every pattern, K = 4: the GEMM result is the table itself."""
    rng = np.random.default_rng(9)
    pats = np.array(list(itertools.product([-1, 0, 1], repeat=4)), dtype=np.int8)
    q = _rand_q(rng, 4, 19)
    assert np.array_equal(O.gemm_acc(pats, q), O.build_lut(q)[0].astype(np.int32))


@pytest.mark.parametrize("g", [4, 5])
def test_lookup_path_equals_definition(g):
    """Eq. 2 on the Alg. 1 table == the plain product (the method is lossless)."""
    rng = np.random.default_rng(10 + g)
    M, K, N = 23, 20 * g, 13
    W, q = _rand_w(rng, M, K), _rand_q(rng, K, N)
    acc = O.lookup_accumulate(O.pack_indices(W, g), O.build_lut(q, g), g)
    assert np.array_equal(acc, O.gemm_acc(W, q))
    assert np.array_equal(acc.astype(np.int64), W.astype(np.int64) @ q.astype(np.int64))


# ---------------------------------------------------------------- quantiser
def test_quantize_hand_cases():
    x = np.array([[1.0, -2.0, 0.5, 2.0],          # amax 2 -> inv 63.5: 63.5->64 (tie to even), 31.75->32
                  [0.0, 0.0, 0.0, 0.0],           # zero row
                  [3.0, 3.0, -3.0, 3.0],          # all equal magnitude
                  [127.0, 0.5, 1.5, 2.5],         # inv == 1: ties 0.5->0, 1.5->2, 2.5->2
                  [-127.0, -0.5, -1.5, 126.5]],   # negative ties, 126.5 -> 126
                 dtype=np.float32)
    q, s = O.quantize(x)
    assert q.shape == (4, 5) and q.dtype == np.int8 and s.dtype == np.float32
    assert q[:, 0].tolist() == [64, -127, 32, 127]
    assert q[:, 1].tolist() == [0, 0, 0, 0] and s[1] == 0.0
    assert q[:, 2].tolist() == [127, 127, -127, 127]
    assert q[:, 3].tolist() == [127, 0, 2, 2]
    assert q[:, 4].tolist() == [-127, 0, -2, 126]
    assert s[0] == np.float32(2.0) / np.float32(127.0) and s[3] == np.float32(1.0)


def test_quantize_properties_and_layout():
    x = wl.activations(3, 37, 100, outlier_frac=0.05)
    q, s = O.quantize(x)
    assert q.shape == (100, 37)                                      # token-contiguous [K][N]
    assert q.min() >= -127 and q.max() <= 127                        # -128 never produced
    amax = np.abs(x).max(axis=1)
    assert np.array_equal(s, amax / np.float32(127.0))
    k_star = np.abs(x).argmax(axis=1)
    assert np.all(np.abs(q[k_star, np.arange(37)]) == 127)           # absmax element -> +-127
    deq = q.T.astype(np.float64) * s[:, None].astype(np.float64)
    assert np.all(np.abs(deq - x) <= 0.5 * s[:, None] * (1 + 1e-5))  # error <= half a step
    assert np.array_equal(np.sign(q.T), np.sign(np.where(np.abs(x) * 127 < 0.5 * amax[:, None], 0, x)))
    # row stride (ldx > K) is honoured
    big = np.zeros((37, 128), np.float32)
    big[:, :100] = x
    big[:, 100:] = 1e9
    q2, s2 = O.quantize(big[:, :100])
    assert np.array_equal(q2, q) and np.array_equal(s2, s)


# ---------------------------------------------------------------- epilogue / whole path
def test_epilogue_exact_cases_and_layout():
    acc = np.array([[3, -5], [0, 7], [16, 1]], dtype=np.int32)       # M=3, N=2
    s = np.array([0.25, 2.0], dtype=np.float32)
    y = O.epilogue(acc, np.float32(0.5), s)
    assert y.shape == (2, 3)                                          # feature-contiguous [N][M]
    assert y.tolist() == [[0.375, 0.0, 2.0], [-5.0, 7.0, 1.0]]


def test_whole_path_vs_dequantise_and_multiply():
    W, w_scale, x = wl.small_case(5, 40, 64, 9)
    q, s, acc, y = O.mpgemm(W, w_scale, x)
    Wd = W.astype(np.float64) * float(w_scale)
    Ad = q.astype(np.float64) * s[None, :].astype(np.float64)
    ref = (Wd @ Ad).T
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-13)   # atol: cancellation in the fp64 sum
    # the integer part is recovered exactly from the dequantised product
    assert np.array_equal(np.rint(ref.T / (float(w_scale) * s[None, :].astype(np.float64))).astype(np.int64),
                          acc.astype(np.int64))
    # and the quantised product approximates the unquantised one (sanity on scales' direction)
    full = (Wd @ x.T.astype(np.float64)).T
    assert np.abs(y - full).max() <= 0.5 * float(w_scale) * float(s.max()) * 64


# ---------------------------------------------------------------- constants the paper prints
def test_paper_constants(golden):
    assert 32767 // (127 * 4) == int(golden["block_size_g4"][0])
    M, K, N = (int(golden[k][0]) for k in ("full_lut_M", "full_lut_K", "full_lut_N"))
    mib = (K // 4) * 81 * N * 2 / 2 ** 20
    assert round(mib, 1) == float(golden["full_lut_mib"][0])
    for g in (4, 5):
        assert 2 * 3 ** (g - 1) * g == int(golden[f"ops_vanilla_g{g}"][0])
        assert 3 ** g == int(golden[f"ops_topo_g{g}"][0])
    assert round(810 / 243, 1) == float(golden["speedup_g5"][0])
    assert 81 * 32 * (16 // 4) * 2 == int(golden["tile_bytes_g4"][0])
    assert 243 * 32 * (10 // 5) * 2 == int(golden["tile_bytes_g5"][0])


def test_generators_are_deterministic_and_distributed():
    a = wl.ternary(0, 64, 256, 0.4)
    assert np.array_equal(a, wl.ternary(0, 64, 256, 0.4))
    assert not np.array_equal(a, wl.ternary(1, 64, 256, 0.4))
    big = wl.ternary(0, 512, 1024, 0.4)
    assert abs((big == 0).mean() - 0.4) < 0.01 and abs((big == 1).mean() - 0.3) < 0.01
    x = wl.activations(0, 64, 1024)
    assert abs(float(x.mean())) < 0.02 and abs(float(x.std()) - 1.0) < 0.02
    s = wl.latent_weight_scale(0, 256, 256)
    assert abs(float(s) - 0.02 * np.sqrt(2 / np.pi)) < 5e-4
