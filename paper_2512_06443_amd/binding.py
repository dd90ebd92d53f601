"""Thin Python binding of the C ABI in include/vlut.h (argument marshalling only).

Device buffers are torch tensors on a ROCm device; this module passes their raw
pointers and the current HIP stream to libvlut.so.  Every step of the path runs
inside the library's kernels; there is no fallback: if the library is missing or
a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvlut.so")

VLUT_OK = 0
VLUT_ERR_NULL, VLUT_ERR_SHAPE, VLUT_ERR_SMALL_BUFFER = -1, -2, -3
VLUT_ERR_VALUE, VLUT_ERR_DEVICE, VLUT_ERR_UNSUPPORTED = -4, -5, -6

EXPORTS = [
    "vlut_status_string", "vlut_version", "vlut_packed_weight_bytes", "vlut_packed_offset", "vlut_act_bytes",
    "vlut_lut_bytes",
    "vlut_workspace_bytes", "vlut_pack_weights", "vlut_quantize_act", "vlut_build_lut", "vlut_mpgemm",
    "vlut_mpgemm_rows", "vlut_mpgemm_mfma", "vlut_mfma_workspace_bytes", "vlut_set_plan", "vlut_query_plan",
    "vlut_packed_weight_bytes_g5", "vlut_packed_offset_g5", "vlut_workspace_bytes_g5", "vlut_pack_weights_g5",
    "vlut_mpgemm_g5", "vlut_set_plan_g5", "vlut_query_plan_g5",
    "vlut_workspace_bytes_f32", "vlut_query_plan_f32", "vlut_mpgemm_f32",
    "vlut_build_lut_token_outer", "vlut_mpgemm_token_outer",
    "vlut_mixed_k5", "vlut_packed_weight_bytes_mixed", "vlut_workspace_bytes_mixed", "vlut_pack_weights_mixed",
    "vlut_mpgemm_mixed", "vlut_static_scratch_bytes", "vlut_mpgemm_static", "vlut_query_lookup_waves",
]

_lib = None


class VlutError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


def lib() -> ctypes.CDLL:
    """Loads libvlut.so; building it is the job of __graft_entry__.build() / paper_2512_06443_amd.build."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_06443_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        i64, sz, p, ci, cf = ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        L.vlut_status_string.argtypes, L.vlut_status_string.restype = [ci], ctypes.c_char_p
        L.vlut_version.argtypes, L.vlut_version.restype = [], ci
        L.vlut_packed_weight_bytes.argtypes, L.vlut_packed_weight_bytes.restype = [i64, i64], sz
        L.vlut_packed_offset.argtypes, L.vlut_packed_offset.restype = [i64, i64, i64, i64], sz
        L.vlut_act_bytes.argtypes, L.vlut_act_bytes.restype = [i64, i64], sz
        L.vlut_lut_bytes.argtypes, L.vlut_lut_bytes.restype = [i64, i64], sz
        L.vlut_workspace_bytes.argtypes, L.vlut_workspace_bytes.restype = [i64, i64, i64], sz
        L.vlut_mfma_workspace_bytes.argtypes, L.vlut_mfma_workspace_bytes.restype = [i64, i64, i64], sz
        L.vlut_pack_weights.argtypes, L.vlut_pack_weights.restype = [p, i64, i64, p, sz, p], ci
        L.vlut_quantize_act.argtypes, L.vlut_quantize_act.restype = [p, i64, i64, i64, p, p, p], ci
        L.vlut_build_lut.argtypes, L.vlut_build_lut.restype = [p, i64, i64, p, sz, p], ci
        gemm_args = [p, cf, p, p, p, i64, i64, i64, p, i64, p, p, sz, p]
        L.vlut_mpgemm.argtypes, L.vlut_mpgemm.restype = gemm_args, ci
        L.vlut_mpgemm_mfma.argtypes, L.vlut_mpgemm_mfma.restype = gemm_args, ci
        L.vlut_mpgemm_rows.argtypes, L.vlut_mpgemm_rows.restype = [p, p] + list(gemm_args[2:]), ci
        L.vlut_packed_weight_bytes_g5.argtypes, L.vlut_packed_weight_bytes_g5.restype = [i64, i64], sz
        L.vlut_packed_offset_g5.argtypes, L.vlut_packed_offset_g5.restype = [i64, i64, i64, i64], sz
        L.vlut_workspace_bytes_g5.argtypes, L.vlut_workspace_bytes_g5.restype = [i64, i64, i64], sz
        L.vlut_pack_weights_g5.argtypes, L.vlut_pack_weights_g5.restype = [p, i64, i64, p, sz, p], ci
        L.vlut_mpgemm_g5.argtypes, L.vlut_mpgemm_g5.restype = [p, cf, p, p, i64, i64, i64, p, i64, p, p, sz, p], ci
        L.vlut_set_plan_g5.argtypes, L.vlut_set_plan_g5.restype = [ci, ci], ci
        L.vlut_query_plan_g5.argtypes, L.vlut_query_plan_g5.restype = [i64, i64, i64, ctypes.POINTER(ci)], ci
        L.vlut_mixed_k5.argtypes, L.vlut_mixed_k5.restype = [i64], i64
        L.vlut_packed_weight_bytes_mixed.argtypes, L.vlut_packed_weight_bytes_mixed.restype = [i64, i64], sz
        L.vlut_workspace_bytes_mixed.argtypes, L.vlut_workspace_bytes_mixed.restype = [i64, i64, i64], sz
        L.vlut_pack_weights_mixed.argtypes, L.vlut_pack_weights_mixed.restype = [p, i64, i64, p, sz, p], ci
        L.vlut_mpgemm_mixed.argtypes, L.vlut_mpgemm_mixed.restype = [p, cf, p, p, i64, i64, i64, p, i64, p, p, sz, p], ci
        L.vlut_build_lut_token_outer.argtypes, L.vlut_build_lut_token_outer.restype = [p, i64, i64, p, sz, p], ci
        L.vlut_mpgemm_token_outer.argtypes = [p, cf, p, p, i64, i64, i64, p, i64, p, p]
        L.vlut_mpgemm_token_outer.restype = ci
        L.vlut_workspace_bytes_f32.argtypes, L.vlut_workspace_bytes_f32.restype = [i64, i64, i64], sz
        L.vlut_query_plan_f32.argtypes, L.vlut_query_plan_f32.restype = [i64, i64, i64, ctypes.POINTER(ci)], ci
        L.vlut_mpgemm_f32.argtypes = [p, cf, p, p, i64, i64, i64, i64, p, i64, p, p, p, sz, p]
        L.vlut_mpgemm_f32.restype = ci
        L.vlut_query_lookup_waves.argtypes, L.vlut_query_lookup_waves.restype = [i64, i64, i64], ci
        L.vlut_static_scratch_bytes.argtypes, L.vlut_static_scratch_bytes.restype = [], sz
        L.vlut_mpgemm_static.argtypes, L.vlut_mpgemm_static.restype = [p, cf, p, p, i64, i64, i64, p, i64, p, p], ci
        L.vlut_set_plan.argtypes, L.vlut_set_plan.restype = [ci, ci, ci, ci], ci
        L.vlut_query_plan.argtypes, L.vlut_query_plan.restype = [i64, i64, i64, ctypes.POINTER(ci)], ci
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().vlut_status_string(status).decode()


def _check(status: int, where: str) -> None:
    if status != VLUT_OK:
        raise VlutError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def packed_weight_bytes(M: int, K: int) -> int:
    return lib().vlut_packed_weight_bytes(M, K)


def packed_offset(M: int, K: int, m: int, kg: int) -> int:
    return lib().vlut_packed_offset(M, K, m, kg)


def act_bytes(K: int, N: int) -> int:
    return lib().vlut_act_bytes(K, N)


def act_chunked_to_kn(a_q: torch.Tensor, N: int) -> torch.Tensor:
    """View helper for checks: token-chunked int8 [ceil(N/8)][K][8] -> plain [K][N] (a copy)."""
    C, K, _ = a_q.shape
    return a_q.permute(1, 0, 2).reshape(K, C * 8)[:, :N].contiguous()


def lut_bytes(K: int, N: int) -> int:
    return lib().vlut_lut_bytes(K, N)


def workspace_bytes(M: int, K: int, N: int) -> int:
    return lib().vlut_workspace_bytes(M, K, N)


def set_plan(J: int = 0, R: int = 0, waves: int = 0, split_k: int = 0) -> None:
    _check(lib().vlut_set_plan(J, R, waves, split_k), "vlut_set_plan")


def query_plan(M: int, K: int, N: int) -> Tuple[int, int, int, int]:
    out = (ctypes.c_int * 4)()
    _check(lib().vlut_query_plan(M, K, N, out), "vlut_query_plan")
    return out[0], out[1], out[2], out[3]


def pack_weights(w_ternary: torch.Tensor) -> torch.Tensor:
    """int8 [M][K] on the GPU -> packed uint8 blob (opaque tile layout) on the GPU."""
    assert w_ternary.is_cuda and w_ternary.dtype == torch.int8 and w_ternary.is_contiguous()
    M, K = w_ternary.shape
    nbytes = packed_weight_bytes(M, K)
    if nbytes == 0:
        raise VlutError(VLUT_ERR_SHAPE, "vlut_packed_weight_bytes")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=w_ternary.device)
    _check(lib().vlut_pack_weights(_ptr(w_ternary), M, K, _ptr(packed), nbytes, _stream()), "vlut_pack_weights")
    return packed


def quantize_act(x: torch.Tensor, a_q: Optional[torch.Tensor] = None, a_scale: Optional[torch.Tensor] = None):
    """fp32 [N][K] (row stride >= K) -> (int8 token-chunked [ceil(N/8)][K][8], fp32 [N])."""
    assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.stride(1) == 1
    N, K = x.shape
    if a_q is None:
        a_q = torch.empty(((N + 7) // 8, K, 8), dtype=torch.int8, device=x.device)
    if a_scale is None:
        a_scale = torch.empty(N, dtype=torch.float32, device=x.device)
    _check(lib().vlut_quantize_act(_ptr(x), N, K, x.stride(0), _ptr(a_q), _ptr(a_scale), _stream()), "vlut_quantize_act")
    return a_q, a_scale


def build_lut(a_q: torch.Tensor, N: int, lut: Optional[torch.Tensor] = None) -> torch.Tensor:
    assert a_q.is_cuda and a_q.dtype == torch.int8 and a_q.is_contiguous() and a_q.dim() == 3
    K = a_q.shape[1]
    assert a_q.shape[0] == (N + 7) // 8
    if lut is None:
        lut = torch.empty((K // 4, 81, N), dtype=torch.int16, device=a_q.device)
    _check(lib().vlut_build_lut(_ptr(a_q), K, N, _ptr(lut), lut.numel() * 2, _stream()), "vlut_build_lut")
    return lut


def mpgemm(packed: torch.Tensor, w_scale: float, a_q: torch.Tensor, a_scale: torch.Tensor, M: int,
           y: Optional[torch.Tensor] = None, acc: Optional[torch.Tensor] = None, lut: Optional[torch.Tensor] = None,
           workspace: Optional[torch.Tensor] = None, want_acc: bool = False, mfma: bool = False):
    """Runs vlut_mpgemm (or the MFMA comparison path).  Returns (y fp32 [N][M], acc int32 [M][N] or None)."""
    K, N = a_q.shape[1], a_scale.shape[0]
    dev = a_q.device
    if y is None:
        y = torch.empty((N, M), dtype=torch.float32, device=dev)
    if acc is None and want_acc:
        acc = torch.empty((M, N), dtype=torch.int32, device=dev)
    ws_bytes = lib().vlut_mfma_workspace_bytes(M, K, N) if mfma else workspace_bytes(M, K, N)
    if workspace is None and ws_bytes:
        workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    fn = lib().vlut_mpgemm_mfma if mfma else lib().vlut_mpgemm
    rc = fn(_ptr(packed), float(w_scale), _ptr(a_q), _ptr(a_scale), _ptr(lut), M, K, N, _ptr(y), y.stride(0),
            _ptr(acc), _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
            _stream())
    _check(rc, "vlut_mpgemm_mfma" if mfma else "vlut_mpgemm")
    return y, acc


def query_lookup_waves(M: int, K: int, N: int) -> int:
    """Lookup waves per workgroup (12 or 14) of the plan vlut_mpgemm would use; 0 for the few-token kernel."""
    w = lib().vlut_query_lookup_waves(M, K, N)
    if w < 0:
        raise VlutError(w, "vlut_query_lookup_waves")
    return w


def static_scratch_bytes() -> int:
    return lib().vlut_static_scratch_bytes()


def mpgemm_static(packed: torch.Tensor, w_scale: float, a_q: torch.Tensor, a_scale: torch.Tensor, M: int,
                  y: torch.Tensor, acc: Optional[torch.Tensor] = None):
    """Runs vlut_mpgemm_static: the caller passes inputs and outputs only, the split-K scratch is the library's own
    static device array; neither this wrapper nor the call allocates anything."""
    K, N = a_q.shape[1], a_scale.shape[0]
    rc = lib().vlut_mpgemm_static(_ptr(packed), float(w_scale), _ptr(a_q), _ptr(a_scale), M, K, N, _ptr(y), y.stride(0),
                                  _ptr(acc), _stream())
    _check(rc, "vlut_mpgemm_static")
    return y, acc


def mpgemm_rows(packed: torch.Tensor, w_scale_rows: torch.Tensor, a_q: torch.Tensor, a_scale: torch.Tensor, M: int,
                y: Optional[torch.Tensor] = None, want_acc: bool = False, workspace: Optional[torch.Tensor] = None):
    """Runs vlut_mpgemm_rows: stacked weight matrices, one weight scale per output row (fp32 [M] on the GPU)."""
    assert w_scale_rows.is_cuda and w_scale_rows.dtype == torch.float32 and w_scale_rows.numel() == M
    K, N = a_q.shape[1], a_scale.shape[0]
    dev = a_q.device
    if y is None:
        y = torch.empty((N, M), dtype=torch.float32, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    ws_bytes = workspace_bytes(M, K, N)
    if workspace is None and ws_bytes:
        workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    rc = lib().vlut_mpgemm_rows(_ptr(packed), _ptr(w_scale_rows), _ptr(a_q), _ptr(a_scale), None, M, K, N, _ptr(y),
                                y.stride(0), _ptr(acc), _ptr(workspace),
                                0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "vlut_mpgemm_rows")
    return y, acc


def build_lut_token_outer(a_q: torch.Tensor, N: int) -> torch.Tensor:
    """The table with the token index outermost, int16 [N][K/4][81] (layout ablation)."""
    assert a_q.is_cuda and a_q.dtype == torch.int8 and a_q.is_contiguous() and a_q.dim() == 3
    K = a_q.shape[1]
    lut = torch.empty((N, K // 4, 81), dtype=torch.int16, device=a_q.device)
    _check(lib().vlut_build_lut_token_outer(_ptr(a_q), K, N, _ptr(lut), lut.numel() * 2, _stream()),
           "vlut_build_lut_token_outer")
    return lut


def mpgemm_token_outer(packed: torch.Tensor, w_scale: float, a_scale: torch.Tensor, lut: torch.Tensor, M: int,
                       want_acc: bool = False):
    """Runs vlut_mpgemm_token_outer on a table from build_lut_token_outer.  Returns (y [N][M], acc or None)."""
    N, G, _ = lut.shape
    y = torch.empty((N, M), dtype=torch.float32, device=lut.device)
    acc = torch.empty((M, N), dtype=torch.int32, device=lut.device) if want_acc else None
    _check(lib().vlut_mpgemm_token_outer(_ptr(packed), float(w_scale), _ptr(a_scale), _ptr(lut), M, 4 * G, N, _ptr(y),
                                         y.stride(0), _ptr(acc), _stream()), "vlut_mpgemm_token_outer")
    return y, acc


def query_plan_f32(M: int, K: int, N: int) -> Tuple[int, int, int, int, bool]:
    """(J, R, split_k, workgroups, fused) that vlut_mpgemm_f32 uses for this shape."""
    out = (ctypes.c_int * 5)()
    _check(lib().vlut_query_plan_f32(M, K, N, out), "vlut_query_plan_f32")
    return out[0], out[1], out[2], out[3], bool(out[4])


def mpgemm_f32(packed: torch.Tensor, w_scale, x: torch.Tensor, M: int, y: Optional[torch.Tensor] = None,
               want_acc: bool = False, want_scales: bool = False, workspace: Optional[torch.Tensor] = None):
    """Runs vlut_mpgemm_f32 on fp32 activations x [N][K] (row stride >= K).  w_scale: a float, or an fp32 [M]
    tensor on the GPU with one weight scale per output row.  Returns (y [N][M], acc or None, a_scale or None)."""
    assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.stride(1) == 1
    N, K = x.shape
    dev = x.device
    rows = w_scale if isinstance(w_scale, torch.Tensor) else None
    if rows is not None:
        assert rows.is_cuda and rows.dtype == torch.float32 and rows.numel() == M
    if y is None:
        y = torch.empty((N, M), dtype=torch.float32, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    scales = torch.empty(N, dtype=torch.float32, device=dev) if want_scales else None
    ws_bytes = lib().vlut_workspace_bytes_f32(M, K, N)
    if workspace is None and ws_bytes:
        workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    rc = lib().vlut_mpgemm_f32(_ptr(packed), 1.0 if rows is not None else float(w_scale), _ptr(rows), _ptr(x), x.stride(0),
                               M, K, N, _ptr(y), y.stride(0), _ptr(acc), _ptr(scales), _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "vlut_mpgemm_f32")
    return y, acc, scales


# ---- 1.60-bit packing (g = 5)
def pack_weights_g5(w_ternary: torch.Tensor) -> torch.Tensor:
    """int8 [M][K] (K % 5 == 0) on the GPU -> 1.60-bit packed blob on the GPU."""
    assert w_ternary.is_cuda and w_ternary.dtype == torch.int8 and w_ternary.is_contiguous()
    M, K = w_ternary.shape
    nbytes = lib().vlut_packed_weight_bytes_g5(M, K)
    if nbytes == 0:
        raise VlutError(VLUT_ERR_SHAPE, "vlut_packed_weight_bytes_g5")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=w_ternary.device)
    _check(lib().vlut_pack_weights_g5(_ptr(w_ternary), M, K, _ptr(packed), nbytes, _stream()), "vlut_pack_weights_g5")
    return packed


def pack_weights_mixed(w_ternary: torch.Tensor) -> torch.Tensor:
    """int8 [M][K] (K % 4 == 0) on the GPU -> blob of the mixed 1.60-bit / 2-bit packing on the GPU."""
    assert w_ternary.is_cuda and w_ternary.dtype == torch.int8 and w_ternary.is_contiguous()
    M, K = w_ternary.shape
    nbytes = lib().vlut_packed_weight_bytes_mixed(M, K)
    if nbytes == 0:
        raise VlutError(VLUT_ERR_SHAPE, "vlut_packed_weight_bytes_mixed")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=w_ternary.device)
    _check(lib().vlut_pack_weights_mixed(_ptr(w_ternary), M, K, _ptr(packed), nbytes, _stream()), "vlut_pack_weights_mixed")
    return packed


def mpgemm_mixed(packed: torch.Tensor, w_scale: float, a_q: torch.Tensor, a_scale: torch.Tensor, M: int,
                 y: Optional[torch.Tensor] = None, want_acc: bool = False):
    """Runs vlut_mpgemm_mixed on a blob from pack_weights_mixed.  Returns (y [N][M], acc or None)."""
    K, N = a_q.shape[1], a_scale.shape[0]
    dev = a_q.device
    if y is None:
        y = torch.empty((N, M), dtype=torch.float32, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    ws = torch.empty(max(lib().vlut_workspace_bytes_mixed(M, K, N), 16), dtype=torch.uint8, device=dev)
    _check(lib().vlut_mpgemm_mixed(_ptr(packed), float(w_scale), _ptr(a_q), _ptr(a_scale), M, K, N, _ptr(y), y.stride(0),
                                   _ptr(acc), _ptr(ws), ws.numel(), _stream()), "vlut_mpgemm_mixed")
    return y, acc


def set_plan_g5(R: int = 0, split_k: int = 0) -> None:
    _check(lib().vlut_set_plan_g5(R, split_k), "vlut_set_plan_g5")


def query_plan_g5(M: int, K: int, N: int) -> Tuple[int, int, int]:
    out = (ctypes.c_int * 3)()
    _check(lib().vlut_query_plan_g5(M, K, N, out), "vlut_query_plan_g5")
    return out[0], out[1], out[2]


def mpgemm_g5(packed: torch.Tensor, w_scale: float, a_q: torch.Tensor, a_scale: torch.Tensor, M: int,
              y: Optional[torch.Tensor] = None, want_acc: bool = False, workspace: Optional[torch.Tensor] = None):
    """Runs vlut_mpgemm_g5.  Returns (y fp32 [N][M], acc int32 [M][N] or None)."""
    K, N = a_q.shape[1], a_scale.shape[0]
    dev = a_q.device
    if y is None:
        y = torch.empty((N, M), dtype=torch.float32, device=dev)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    ws_bytes = lib().vlut_workspace_bytes_g5(M, K, N)
    if workspace is None and ws_bytes:
        workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    rc = lib().vlut_mpgemm_g5(_ptr(packed), float(w_scale), _ptr(a_q), _ptr(a_scale), M, K, N, _ptr(y), y.stride(0),
                              _ptr(acc), _ptr(workspace),
                              0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "vlut_mpgemm_g5")
    return y, acc
