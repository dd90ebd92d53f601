"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol that
include/vlut.h declares, its size helpers match the closed forms the paper gives, and every
argument error is reported before any HIP call."""
import ctypes
import os
import re

import pytest

from tests.conftest import ROOT

i64, sz, vp, ci, cf = ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_float


@pytest.fixture(scope="module")
def L(vlut_lib_path):
    lib = ctypes.CDLL(vlut_lib_path)
    lib.vlut_status_string.argtypes, lib.vlut_status_string.restype = [ci], ctypes.c_char_p
    lib.vlut_packed_weight_bytes.argtypes, lib.vlut_packed_weight_bytes.restype = [i64, i64], sz
    lib.vlut_packed_offset.argtypes, lib.vlut_packed_offset.restype = [i64, i64, i64, i64], sz
    lib.vlut_lut_bytes.argtypes, lib.vlut_lut_bytes.restype = [i64, i64], sz
    lib.vlut_act_bytes.argtypes, lib.vlut_act_bytes.restype = [i64, i64], sz
    lib.vlut_workspace_bytes.argtypes, lib.vlut_workspace_bytes.restype = [i64, i64, i64], sz
    lib.vlut_pack_weights.argtypes = [vp, i64, i64, vp, sz, vp]
    lib.vlut_quantize_act.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    lib.vlut_build_lut.argtypes = [vp, i64, i64, vp, sz, vp]
    g = [vp, cf, vp, vp, vp, i64, i64, i64, vp, i64, vp, vp, sz, vp]
    lib.vlut_mpgemm.argtypes = g
    lib.vlut_mpgemm_mfma.argtypes = g
    lib.vlut_mpgemm_rows.argtypes = [vp, vp] + g[2:]
    lib.vlut_set_plan.argtypes = [ci, ci, ci, ci]
    lib.vlut_query_lookup_waves.argtypes = [i64, i64, i64]
    lib.vlut_packed_weight_bytes_g5.argtypes, lib.vlut_packed_weight_bytes_g5.restype = [i64, i64], sz
    lib.vlut_packed_offset_g5.argtypes, lib.vlut_packed_offset_g5.restype = [i64, i64, i64, i64], sz
    lib.vlut_workspace_bytes_g5.argtypes, lib.vlut_workspace_bytes_g5.restype = [i64, i64, i64], sz
    lib.vlut_pack_weights_g5.argtypes = [vp, i64, i64, vp, sz, vp]
    lib.vlut_mpgemm_g5.argtypes = [vp, cf, vp, vp, i64, i64, i64, vp, i64, vp, vp, sz, vp]
    lib.vlut_set_plan_g5.argtypes = [ci, ci]
    lib.vlut_query_plan_g5.argtypes = [i64, i64, i64, ctypes.POINTER(ci)]
    lib.vlut_query_plan.argtypes = [i64, i64, i64, ctypes.POINTER(ci)]
    lib.vlut_mixed_k5.argtypes, lib.vlut_mixed_k5.restype = [i64], i64
    lib.vlut_packed_weight_bytes_mixed.argtypes, lib.vlut_packed_weight_bytes_mixed.restype = [i64, i64], sz
    lib.vlut_workspace_bytes_mixed.argtypes, lib.vlut_workspace_bytes_mixed.restype = [i64, i64, i64], sz
    lib.vlut_pack_weights_mixed.argtypes = [vp, i64, i64, vp, sz, vp]
    lib.vlut_mpgemm_mixed.argtypes = [vp, cf, vp, vp, i64, i64, i64, vp, i64, vp, vp, sz, vp]
    lib.vlut_workspace_bytes_f32.argtypes, lib.vlut_workspace_bytes_f32.restype = [i64, i64, i64], sz
    lib.vlut_query_plan_f32.argtypes = [i64, i64, i64, ctypes.POINTER(ci)]
    lib.vlut_mpgemm_f32.argtypes = [vp, cf, vp, vp, i64, i64, i64, i64, vp, i64, vp, vp, vp, sz, vp]
    return lib


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "vlut.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(vlut_[a-z0-9_]+)\s*\(", header)))
    assert {"vlut_pack_weights", "vlut_quantize_act", "vlut_build_lut", "vlut_mpgemm"} <= set(names)
    for n in names:
        assert hasattr(L, n), f"{n} declared in vlut.h but not exported"
    from paper_2512_06443_amd import binding
    assert set(binding.EXPORTS) == set(names)


def test_status_strings(L):
    assert L.vlut_status_string(0) == b"VLUT_OK"
    seen = {L.vlut_status_string(c) for c in range(-6, 1)}
    assert len(seen) == 7 and all(s for s in seen)
    assert L.vlut_status_string(-99).startswith(b"VLUT_ERR")


def test_size_helpers(L, golden):
    # 2.00 bits per weight when the shape needs no padding (Sec. 4: I2 = b2.00)
    assert L.vlut_packed_weight_bytes(6912, 2560) == 6912 * 2560 // 4
    assert L.vlut_packed_weight_bytes(256, 256) == 16384
    # padding to 4 rows x 16 groups
    assert L.vlut_packed_weight_bytes(257, 260) == 65 * 5 * 64
    assert L.vlut_packed_weight_bytes(1, 4) == 64
    for bad in [(0, 4), (4, 0), (4, 6), (-1, 8), (1 << 24, 4)]:
        assert L.vlut_packed_weight_bytes(*bad) == 0
    # the paper's full-table example (Sec. 1): 4096 x 14436 x 512 -> 285.5 MiB
    K, N = int(golden["full_lut_K"][0]), int(golden["full_lut_N"][0])
    assert round(L.vlut_lut_bytes(K, N) / 2 ** 20, 1) == float(golden["full_lut_mib"][0])
    assert L.vlut_lut_bytes(256, 8) == 64 * 81 * 8 * 2
    assert L.vlut_act_bytes(2560, 128) == 2560 * 128 and L.vlut_act_bytes(64, 9) == 2 * 64 * 8
    assert L.vlut_act_bytes(6, 8) == 0
    assert L.vlut_lut_bytes(6, 8) == 0 and L.vlut_lut_bytes(8, 0) == 0
    assert L.vlut_workspace_bytes(0, 8, 8) == 0


def test_packed_offset_is_a_bijection(L):
    M, K = 10, 136            # 3 row tiles (padded), 34 groups -> 3 k-tiles (padded)
    total = L.vlut_packed_weight_bytes(M, K)
    assert total == 3 * 3 * 64
    offs = {L.vlut_packed_offset(M, K, m, kg) for m in range(M) for kg in range(K // 4)}
    assert len(offs) == M * (K // 4) and max(offs) < total
    # tile structure: 4 rows x 16 groups contiguous, a row's 16 groups are 16 consecutive bytes
    assert L.vlut_packed_offset(M, K, 0, 1) - L.vlut_packed_offset(M, K, 0, 0) == 1
    assert L.vlut_packed_offset(M, K, 1, 0) - L.vlut_packed_offset(M, K, 0, 0) == 16
    assert L.vlut_packed_offset(M, K, 0, 16) - L.vlut_packed_offset(M, K, 0, 0) == 64
    assert L.vlut_packed_offset(M, K, 4, 0) - L.vlut_packed_offset(M, K, 0, 0) == 3 * 64
    for bad in [(M, 0), (-1, 0), (0, 34), (0, -1)]:
        assert L.vlut_packed_offset(M, K, *bad) == ctypes.c_size_t(-1).value


def test_argument_errors_come_before_any_device_call(L):
    d = 0x1000  # a fake non-null, 16-byte aligned "device pointer": never dereferenced on these paths
    assert L.vlut_pack_weights(None, 8, 8, d, 64, None) == -1
    assert L.vlut_pack_weights(d, 8, 8, None, 64, None) == -1
    assert L.vlut_pack_weights(d, 8, 6, d, 64, None) == -2
    assert L.vlut_pack_weights(d, 0, 8, d, 64, None) == -2
    assert L.vlut_pack_weights(d, 8, 8, d, 63, None) == -3
    assert L.vlut_quantize_act(None, 4, 8, 8, d, d, None) == -1
    assert L.vlut_quantize_act(d, 4, 8, 8, None, d, None) == -1
    assert L.vlut_quantize_act(d, 4, 8, 8, d, None, None) == -1
    assert L.vlut_quantize_act(d, 4, 8, 7, d, d, None) == -2      # ldx < K
    assert L.vlut_quantize_act(d, 0, 8, 8, d, d, None) == -2
    assert L.vlut_quantize_act(d, 4, 10, 10, d, d, None) == -2    # K % 4 != 0
    assert L.vlut_build_lut(None, 8, 4, d, 1 << 20, None) == -1
    assert L.vlut_build_lut(d, 8, 4, None, 1 << 20, None) == -1
    assert L.vlut_build_lut(d, 8, 4, d, 2 * 81 * 4 * 2 - 1, None) == -3
    assert L.vlut_build_lut(d, 9, 4, d, 1 << 20, None) == -2
    L.vlut_mfma_workspace_bytes.argtypes, L.vlut_mfma_workspace_bytes.restype = [i64, i64, i64], sz
    assert L.vlut_mfma_workspace_bytes(8, 6, 4) == 0                      # invalid shape
    assert L.vlut_mfma_workspace_bytes(8, 8, 4) == 0                      # one K step: nothing to split
    need = L.vlut_mfma_workspace_bytes(640, 2560, 16)                     # few tiles, 40 K steps: K is split
    assert need > 0 and need % (640 * 16 * 4) == 0 and need // (640 * 16 * 4) <= 16
    assert L.vlut_mfma_workspace_bytes(14336, 4096, 512) == 0             # enough tiles without a split
    assert L.vlut_mpgemm_mfma(d, 1.0, d, d, None, 640, 2560, 16, d, 640, None, None, 0, None) == -1   # needs its workspace
    assert L.vlut_mpgemm_mfma(d, 1.0, d, d, None, 640, 2560, 16, d, 640, None, d, need - 1, None) == -3
    assert L.vlut_mpgemm_mfma(d, 1.0, d, d, d, 8, 8, 4, d, 8, None, d, 1 << 20, None) == -6        # no materialised table here
    for fn in (L.vlut_mpgemm, L.vlut_mpgemm_mfma):
        assert fn(None, 1.0, d, d, None, 8, 8, 4, d, 8, None, None, 0, None) == -1
        assert fn(d, 1.0, None, d, None, 8, 8, 4, d, 8, None, None, 0, None) == -1
        assert fn(d, 1.0, d, None, None, 8, 8, 4, d, 8, None, None, 0, None) == -1
        assert fn(d, 1.0, d, d, None, 8, 8, 4, None, 8, None, None, 0, None) == -1   # neither y nor acc
        assert fn(d, 1.0, d, d, None, 8, 8, 4, d, 7, None, None, 0, None) == -2      # ldy < M
        assert fn(d, 1.0, d, d, None, 8, 7, 4, d, 8, None, None, 0, None) == -2
        assert fn(d, 1.0, d, d, None, 8, 8, 0, d, 8, None, None, 0, None) == -2
    assert L.vlut_mpgemm_rows(d, None, d, d, None, 8, 8, 4, d, 8, None, None, 0, None) == -1      # row scales are required
    assert L.vlut_mpgemm_rows(None, d, d, d, None, 8, 8, 4, d, 8, None, None, 0, None) == -1
    assert L.vlut_mpgemm_rows(d, d, d, d, None, 8, 8, 4, d, 7, None, None, 0, None) == -2
    assert L.vlut_set_plan(3, 0, 0, 0) == -6 and L.vlut_set_plan(0, 17, 0, 0) == -6
    assert L.vlut_set_plan(0, 0, 7, 0) == -6 and L.vlut_set_plan(0, 0, 0, 99) == -6
    assert L.vlut_set_plan(0, 0, 12, 0) == 0 and L.vlut_set_plan(0, 0, 14, 0) == 0 and L.vlut_set_plan(0, 0, 16, 0) == 0
    assert L.vlut_set_plan(0, 0, 0, 0) == 0
    assert L.vlut_query_plan(8, 8, 8, None) == -1


def test_split_k_needs_a_workspace(L):
    d = 0x1000
    assert L.vlut_set_plan(16, 1, 0, 2) == 0
    try:
        M, K, N = 8, 512, 8
        need = L.vlut_workspace_bytes(M, K, N)
        assert need == 2 * M * N * 4
        assert L.vlut_mpgemm(d, 1.0, d, d, None, M, K, N, d, M, None, None, 0, None) == -1
        assert L.vlut_mpgemm(d, 1.0, d, d, None, M, K, N, d, M, None, d, need - 1, None) == -3
    finally:
        assert L.vlut_set_plan(0, 0, 0, 0) == 0


def test_workspace_size_serves_the_materialised_table_variant_too(L):
    """The size vlut_workspace_bytes reports is accepted by vlut_mpgemm for lut != NULL as well, also where the
    streamed path takes the few-token kernel and needs none (the call then reaches the device step: no GPU here)."""
    d = 0x1000
    for (M, K, N) in [(70, 4352, 9), (640, 2560, 1), (2560, 2560, 4), (300, 8192, 2), (6912, 2560, 16), (300, 4352, 40)]:
        need = L.vlut_workspace_bytes(M, K, N)
        ws = d if need else None
        for lut in (None, d):
            rc = L.vlut_mpgemm(d, 1.0, d, d, lut, M, K, N, d, M, None, ws, need, None)
            assert rc not in (-1, -2, -3, -6), (M, K, N, lut, rc)


def test_override_that_does_not_fit_the_shape_is_an_error(L):
    d = 0x1000
    out = (ci * 4)()
    try:
        # K = 16384: 4096 groups; J = 1 -> 4 groups per stage, 1024 stages x 4 lookups per lane > 64 -> R <= 6 only
        assert L.vlut_set_plan(1, 9, 0, 1) == 0
        assert L.vlut_query_plan(300, 16384, 40, out) == -6
        assert L.vlut_mpgemm(d, 1.0, d, d, None, 300, 16384, 40, d, 300, None, None, 0, None) == -6
        assert L.vlut_workspace_bytes(300, 16384, 40) == 0
        # more K splits than stages: K = 256 -> 64 groups = one stage at J = 16
        assert L.vlut_set_plan(16, 2, 0, 4) == 0
        assert L.vlut_query_plan(300, 256, 40, out) == -6
        assert L.vlut_mpgemm(d, 1.0, d, d, None, 300, 256, 40, d, 300, None, d, 1 << 20, None) == -6
        assert L.vlut_set_plan(16, 2, 0, 1) == 0
        assert L.vlut_query_plan(300, 256, 40, out) == 0 and tuple(out)[:3] == (16, 2, 1)
    finally:
        assert L.vlut_set_plan(0, 0, 0, 0) == 0
    out3 = (ci * 3)()
    try:
        assert L.vlut_set_plan_g5(2, 4) == 0
        assert L.vlut_query_plan_g5(300, 320, 40, out3) == -6                  # 64 groups = one stage, four splits asked
    finally:
        assert L.vlut_set_plan_g5(0, 0) == 0


def test_packed_blob_must_be_16_byte_aligned(L):
    d, odd = 0x1000, 0x1004
    assert L.vlut_mpgemm(odd, 1.0, d, d, None, 8, 64, 40, d, 8, None, None, 0, None) == -6
    assert L.vlut_mpgemm_rows(odd, d, d, d, None, 8, 64, 40, d, 8, None, None, 0, None) == -6
    assert L.vlut_mpgemm_f32(odd, 1.0, None, d, 64, 8, 64, 40, d, 8, None, None, d, 1 << 20, None) == -6


def test_plans_cover_all_benchmark_shapes(L):
    out = (ci * 4)()
    shapes = [(256, 256, 8), (6912, 2560, 128), (8640, 3200, 256), (3200, 8640, 256), (4096, 4096, 512),
              (14336, 4096, 512), (4096, 14336, 512)]
    shapes += [(m, k, n) for (m, k) in [(2560, 2560), (640, 2560), (6912, 2560), (2560, 6912)]
               for n in (1, 2, 3, 4, 7, 8, 16, 24, 32, 33, 64, 256, 1024)]
    for (M, K, N) in shapes:
        assert L.vlut_query_plan(M, K, N, out) == 0
        J, R, S, tiles = list(out)
        if J == 0:                                     # the few-token kernel: R = rows per workgroup, a grid per token pair
            pairs = (N + 1) // 2
            assert N <= 32 and R in (32, 64, 128, 256) and S == 1 and tiles % pairs == 0 and (tiles // pairs) * R >= M
            # more than two tokens: one round of workgroups, and cheaper than the general path by the library's estimate
            per_chunk = {32: 0.9, 64: 1.35, 128: 2.0, 256: 3.4}[R]
            c = K / 1024
            assert N <= 2 or (tiles <= 256 and (3.6 + c * per_chunk) * 1.1 < 5.8 + 0.94 * c + 0.41 * M * N / 1e4)
            assert L.vlut_workspace_bytes(M, K, N) == 0 and L.vlut_query_lookup_waves(M, K, N) == 0
            continue
        assert N > 2
        assert J in (1, 2, 4, 8, 16) and 1 <= R <= 16 and 1 <= S <= 16 and tiles >= 1
        n_tile = 128 // J
        tiles_n = -(-N // n_tile)
        assert tiles % (tiles_n * S) == 0
        tiles_m = tiles // (tiles_n * S)
        waves = L.vlut_query_lookup_waves(M, K, N)
        assert waves in (12, 14)
        assert tiles_m * 4 * waves * R >= M                            # every row is covered (lookup waves x 4 rows x R)


def test_g5_host_logic(L):
    """1.60-bit packing: sizes (Sec. 3.3: 5 weights per byte, g | K), layout bijection, argument checks, plan coverage."""
    assert L.vlut_packed_weight_bytes_g5(6912, 2560) == 6912 * 512             # 1.60 bits per weight, no padding needed
    assert L.vlut_packed_weight_bytes_g5(6912, 2560) * 5 == L.vlut_packed_weight_bytes(6912, 2560) * 4
    assert L.vlut_packed_weight_bytes_g5(5, 100) == 2 * 2 * 64                 # rows padded to 4, groups to 16
    assert L.vlut_packed_weight_bytes_g5(8, 64) == 0 and L.vlut_packed_weight_bytes_g5(0, 80) == 0
    M, K = 10, 100
    offs = {L.vlut_packed_offset_g5(M, K, m, kg) for m in range(M) for kg in range(K // 5)}
    assert len(offs) == M * (K // 5) and max(offs) < L.vlut_packed_weight_bytes_g5(M, K)
    assert L.vlut_packed_offset_g5(M, K, M, 0) == 2 ** 64 - 1 and L.vlut_packed_offset_g5(M, K, 0, K // 5) == 2 ** 64 - 1
    d = ctypes.c_void_p(0x1000)                                                # never dereferenced: checks come first
    assert L.vlut_pack_weights_g5(None, 8, 80, d, 1 << 20, None) == -1
    assert L.vlut_pack_weights_g5(d, 8, 64, d, 1 << 20, None) == -2            # 5 does not divide 64
    assert L.vlut_pack_weights_g5(d, 8, 80, d, 63, None) == -3
    assert L.vlut_mpgemm_g5(None, 1.0, d, d, 8, 80, 4, d, 8, None, None, 0, None) == -1
    assert L.vlut_mpgemm_g5(d, 1.0, d, d, 8, 80, 4, None, 8, None, None, 0, None) == -1
    assert L.vlut_mpgemm_g5(d, 1.0, d, d, 8, 82, 4, d, 8, None, None, 0, None) == -2
    assert L.vlut_mpgemm_g5(d, 1.0, d, d, 8, 80, 4, d, 7, None, None, 0, None) == -2
    assert L.vlut_set_plan_g5(3, 0) == -6 and L.vlut_set_plan_g5(0, 17) == -6
    out = (ci * 3)()
    try:
        assert L.vlut_set_plan_g5(2, 4) == 0
        need = L.vlut_workspace_bytes_g5(300, 5120, 40)
        assert need == 4 * 300 * 40 * 4
        assert L.vlut_mpgemm_g5(d, 1.0, d, d, 300, 5120, 40, d, 300, None, None, 0, None) == -1
        assert L.vlut_mpgemm_g5(d, 1.0, d, d, 300, 5120, 40, d, 300, None, d, need - 1, None) == -3
    finally:
        assert L.vlut_set_plan_g5(0, 0) == 0
    for (M, K, N) in [(6912, 2560, 128), (8640, 3200, 256), (3200, 8640, 256), (2560, 2560, 1), (640, 2560, 1024)]:
        assert L.vlut_query_plan_g5(M, K, N, out) == 0
        R, S, tiles = out[0], out[1], out[2]
        assert R in (1, 2, 4, 6, 9, 12, 14) and 1 <= S <= 16 and tiles >= 1
        stages = -(-(K // 5) // 64)
        per_split = -(-stages // S)
        assert per_split * 4 <= 51 or R <= 6                                   # INT16 block bound of Sec. 3.4
        tiles_m = tiles // (S * -(-N // 8))
        assert tiles_m * 48 * R >= M                                           # the tiles cover every row


def test_f32_entry_host_logic(L):
    """vlut_mpgemm_f32: which kernels it picks, what workspace that needs, and argument errors before any device call."""
    out = (ci * 5)()
    # a few tokens: the kernel that sweeps all of K, quantising inside, a copy of the row tiles per token pair; no
    # workspace
    for (M, K, N) in [(6912, 2560, 1), (2560, 6912, 2), (640, 2560, 1), (6912, 2560, 3), (6912, 2560, 8), (640, 2560, 32)]:
        assert L.vlut_query_plan_f32(M, K, N, out) == 0
        assert out[0] == 0 and out[2] == 1 and out[4] == 1
        assert L.vlut_workspace_bytes_f32(M, K, N) == 0
    # more tokens: quantised once, by a kernel of its own ahead of the lookups; the workspace then holds the scales,
    # the INT8 activations and the split-K partial sums of the ordinary path
    for (M, K, N) in [(6912, 2560, 128), (14336, 4096, 512), (4096, 14336, 512), (3200, 8640, 256), (6912, 2560, 24), (2560, 6912, 24), (640, 2560, 33)]:
        assert L.vlut_query_plan_f32(M, K, N, out) == 0
        assert out[4] == 0
        r256 = lambda v: (v + 255) // 256 * 256
        amax = r256(4 * N) if (N * K >= 1 << 22 and N >= 64) else 0      # scratch between the two kernels of the quantiser
        assert L.vlut_workspace_bytes_f32(M, K, N) == r256(4 * N) + amax + r256(L.vlut_act_bytes(K, N)) + L.vlut_workspace_bytes(M, K, N)
    # a forced plan with 16 sub-tables per table row selects the fused kernel when the K range fits next to the
    # tables (34 stages of 256 values), with the scales in front of the split-K partial sums
    try:
        assert L.vlut_set_plan(16, 2, 0, 4) == 0
        assert L.vlut_query_plan_f32(300, 14336, 40, out) == 0 and tuple(out) == (16, 2, 4, 4 * 4 * 5, 1)
        assert L.vlut_workspace_bytes_f32(300, 14336, 40) == 256 + 4 * 300 * 40 * 4
        assert L.vlut_set_plan(16, 2, 0, 1) == 0
        assert L.vlut_query_plan_f32(300, 14336, 40, out) == 0 and out[4] == 0     # 56 stages in one range
        assert L.vlut_set_plan(8, 2, 0, 1) == 0
        assert L.vlut_query_plan_f32(300, 2560, 40, out) == 0 and out[4] == 0      # 16-token tiles
    finally:
        assert L.vlut_set_plan(0, 0, 0, 0) == 0
    d = ctypes.c_void_p(0x1000)                                                # never dereferenced: checks come first
    ok = [d, 1.0, None, d, 2560, 6912, 2560, 1, d, 6912, None, None, None, 0, None]
    def call(**kw):
        names = ["packed", "w_scale", "rows", "x", "ldx", "M", "K", "N", "y", "ldy", "acc", "scales", "ws", "ws_bytes", "stream"]
        a = list(ok)
        for k, v in kw.items():
            a[names.index(k)] = v
        return L.vlut_mpgemm_f32(*a)
    assert call(packed=None) == -1 and call(x=None) == -1 and call(y=None) == -1
    assert call(ldx=2559) == -2 and call(ldy=6911) == -2 and call(K=2562) == -2 and call(N=0) == -2
    assert call(M=14336, K=4096, N=512, ldx=4096, ldy=14336) == -1             # needs a workspace
    need = L.vlut_workspace_bytes_f32(14336, 4096, 512)
    assert call(M=14336, K=4096, N=512, ldx=4096, ldy=14336, ws=d, ws_bytes=need - 1) == -3
    assert call(M=14336, K=4096, N=512, ldx=4096, ldy=14336, ws=ctypes.c_void_p(0x1004), ws_bytes=need) == -6
    assert L.vlut_query_plan_f32(8, 8, 8, None) == -1 and L.vlut_query_plan_f32(8, 6, 8, out) == -2
    assert L.vlut_workspace_bytes_f32(8, 6, 8) == 0


def test_mixed_packing_host_logic(L):
    """Mixed 1.60-bit / 2-bit packing (Sec. 3.3): how K is divided, blob sizes, bits per weight, argument checks."""
    assert [L.vlut_mixed_k5(K) for K in (4, 16, 20, 36, 2560, 4096, 6912, 14336)] == [0, 0, 20, 20, 2560, 4080, 6900, 14320]
    assert L.vlut_mixed_k5(0) == -1 and L.vlut_mixed_k5(18) == -1
    for (M, K) in [(6912, 2560), (14336, 4096), (4096, 14336), (2560, 6912), (8, 16), (8, 36)]:
        K5 = L.vlut_mixed_k5(K)
        want = (L.vlut_packed_weight_bytes_g5(M, K5) if K5 else 0) + (L.vlut_packed_weight_bytes(M, K - K5) if K > K5 else 0)
        assert L.vlut_packed_weight_bytes_mixed(M, K) == want
        if K >= 2560:                                      # "near-1.6-bit" (Sec. 3.3): the 2-bit part is one tile column
            assert 1.6 <= want * 8 / (M * K) < 1.65
            assert want < L.vlut_packed_weight_bytes(M, K) * 0.82
        assert L.vlut_workspace_bytes_mixed(M, K, 8) >= (1 + (K > K5 > 0)) * M * 8 * 4
    assert L.vlut_packed_weight_bytes_mixed(8, 18) == 0 and L.vlut_workspace_bytes_mixed(8, 18, 8) == 0
    d = ctypes.c_void_p(0x1000)                                                # never dereferenced: checks come first
    assert L.vlut_pack_weights_mixed(None, 8, 36, d, 1 << 20, None) == -1
    assert L.vlut_pack_weights_mixed(d, 8, 18, d, 1 << 20, None) == -2
    assert L.vlut_pack_weights_mixed(d, 8, 36, d, 100, None) == -3
    assert L.vlut_mpgemm_mixed(None, 1.0, d, d, 8, 36, 4, d, 8, None, d, 1 << 20, None) == -1
    assert L.vlut_mpgemm_mixed(d, 1.0, d, d, 8, 36, 4, None, 8, None, d, 1 << 20, None) == -1
    assert L.vlut_mpgemm_mixed(d, 1.0, d, d, 8, 38, 4, d, 8, None, d, 1 << 20, None) == -2
    assert L.vlut_mpgemm_mixed(d, 1.0, d, d, 8, 36, 4, d, 7, None, d, 1 << 20, None) == -2
    assert L.vlut_mpgemm_mixed(d, 1.0, d, d, 8, 36, 4, d, 8, None, None, 0, None) == -1        # the workspace is required
    assert L.vlut_mpgemm_mixed(d, 1.0, d, d, 8, 36, 4, d, 8, None, d, 16, None) == -3
