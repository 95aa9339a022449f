"""ctypes binding to libatk.so -- argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
device pointers and the current HIP stream through the C ABI declared in
``include/atk.h`` and returns torch tensors.  No step of the method runs here;
if the shared library is missing the import fails loudly (there is no CPU
fallback).
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# ATK_LIB_PATH lets a developer point the binding at an experimental build of the same library
LIB_PATH = os.environ.get("ATK_LIB_PATH") or os.path.join(_PKG, "libatk.so")

F32, BF16, F16, I32, U32 = 0, 1, 2, 3, 4
_CODES = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16, torch.int32: I32,
          torch.uint32: U32}
OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR = range(5)
OP_APPROX_TOPK, OP_TOPK, OP_STAGE1 = 0, 1, 2
SIZE_MAX = ctypes.c_size_t(-1).value

EXPORTS = [
    "atk_approx_topk", "atk_approx_mink", "atk_mink", "atk_approx_topk_noalloc", "atk_topk", "atk_approx_topk_stage1", "atk_workspace_bytes",
    "atk_expected_recall", "atk_select_params", "atk_recall_params", "atk_set_option", "atk_approx_topk_recall", "atk_approx_mink_recall", "atk_describe_plan", "atk_describe_topk_plan", "atk_valu_probe", "atk_read_probe",
    "atk_mips_approx_topk", "atk_mips_workspace_bytes", "atk_mips_describe_plan", "atk_mips_select_params", "atk_mips_approx_topk_recall", "atk_status_string", "atk_last_hip_error",
    "atk_version",
]


class AtkError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        name = status_string(status)
        extra = f": {last_hip_error()}" if status == HIP_ERROR else ""
        super().__init__(f"{what} failed with {name}{extra}")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2506_04165_amd.build` "
            "(this package has no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.atk_approx_topk.argtypes = [vp, ci, i64, i64, i64, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.atk_approx_topk.restype = ci
    lib.atk_approx_mink.argtypes = [vp, ci, i64, i64, i64, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.atk_approx_mink.restype = ci
    lib.atk_mink.argtypes = [vp, ci, i64, i64, i64, ci, vp, vp, vp, sz, vp]
    lib.atk_mink.restype = ci
    lib.atk_approx_topk_noalloc.argtypes = [vp, ci, i64, i64, i64, ci, ci, ci, vp, vp, vp]
    lib.atk_approx_topk_noalloc.restype = ci
    lib.atk_topk.argtypes = [vp, ci, i64, i64, i64, ci, vp, vp, vp, sz, vp]
    lib.atk_topk.restype = ci
    lib.atk_approx_topk_stage1.argtypes = [vp, ci, i64, i64, i64, ci, ci, vp, vp, vp]
    lib.atk_approx_topk_stage1.restype = ci
    lib.atk_workspace_bytes.argtypes = [ci, ci, i64, i64, ci, ci, ci]
    lib.atk_workspace_bytes.restype = sz
    lib.atk_expected_recall.argtypes = [i64, i64, i64, i64]
    lib.atk_expected_recall.restype = ctypes.c_double
    ip, dp = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double)
    lib.atk_select_params.argtypes = [i64, ci, ctypes.c_double, ci, ci, ip, ip, dp]
    lib.atk_select_params.restype = ci
    lib.atk_recall_params.argtypes = [ci, i64, i64, ci, ctypes.c_double, ip, ip, dp]
    lib.atk_recall_params.restype = ci
    lib.atk_set_option.argtypes = [ctypes.c_char_p, ci]
    lib.atk_set_option.restype = ci
    lib.atk_approx_topk_recall.argtypes = [vp, ci, i64, i64, i64, ci, ctypes.c_double, vp, vp, vp, sz, vp, ip, ip]
    lib.atk_approx_topk_recall.restype = ci
    lib.atk_approx_mink_recall.argtypes = lib.atk_approx_topk_recall.argtypes
    lib.atk_approx_mink_recall.restype = ci
    lib.atk_valu_probe.argtypes = [ci, vp, vp, vp, sz, ci, vp]
    lib.atk_valu_probe.restype = ci
    lib.atk_read_probe.argtypes = [vp, sz, vp, vp]
    lib.atk_read_probe.restype = ci
    lib.atk_describe_plan.argtypes = [ci, i64, i64, ci, ci, ci, ctypes.c_char_p, sz]
    lib.atk_describe_plan.restype = ci
    lib.atk_describe_topk_plan.argtypes = [ci, i64, i64, ci, ctypes.c_char_p, sz]
    lib.atk_describe_topk_plan.restype = ci
    lib.atk_mips_approx_topk.argtypes = [vp, vp, ci, i64, i64, i64, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.atk_mips_approx_topk.restype = ci
    lib.atk_mips_workspace_bytes.argtypes = [ci, i64, i64, i64, ci, ci, ci]
    lib.atk_mips_workspace_bytes.restype = sz
    lib.atk_mips_describe_plan.argtypes = [ci, i64, i64, i64, ci, ci, ci, ctypes.c_char_p, sz]
    lib.atk_mips_describe_plan.restype = ci
    lib.atk_mips_approx_topk_recall.argtypes = [vp, vp, ci, i64, i64, i64, ci, ctypes.c_double, vp, vp, vp, sz, vp, ip, ip]
    lib.atk_mips_approx_topk_recall.restype = ci
    lib.atk_mips_select_params.argtypes = [i64, ci, ctypes.c_double, ip, ip, dp]
    lib.atk_mips_select_params.restype = ci
    lib.atk_status_string.argtypes = [ci]
    lib.atk_status_string.restype = ctypes.c_char_p
    lib.atk_last_hip_error.restype = ctypes.c_char_p
    lib.atk_version.restype = ctypes.c_char_p
    return lib


lib = _load()


def status_string(status: int) -> str:
    return lib.atk_status_string(int(status)).decode()


def last_hip_error() -> str:
    return lib.atk_last_hip_error().decode()


def version() -> str:
    return lib.atk_version().decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.int32:
        return I32
    if t.dtype == torch.uint32:
        return U32
    raise TypeError(f"unsupported dtype {t.dtype}: float32, bfloat16, float16, int32 or uint32")


def _check_input(values: torch.Tensor):
    if values.dim() != 2:
        raise ValueError("values must be [rows, N]")
    if not values.is_cuda:
        raise ValueError("values must live on the GPU (this library has no CPU path)")
    if values.stride(1) != 1:
        raise ValueError("values must be contiguous along the last axis")
    rows, N = values.shape
    stride = values.stride(0) if rows > 1 else max(values.stride(0), N)
    return rows, N, stride


def _stream_ptr(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def workspace_bytes(op: int, dtype: torch.dtype, rows: int, N: int, K: int, Kprime: int, B: int) -> int:
    code = _CODES[dtype]
    return int(lib.atk_workspace_bytes(op, code, rows, N, K, Kprime, B))


def describe_plan(dtype: torch.dtype, rows: int, N: int, K: int, Kprime: int, B: int):
    code = _CODES[dtype]
    buf = ctypes.create_string_buffer(512)
    st = lib.atk_describe_plan(code, rows, N, K, Kprime, B, buf, 512)
    return st, buf.value.decode()


def describe_topk_plan(dtype: torch.dtype, rows: int, N: int, K: int):
    buf = ctypes.create_string_buffer(512)
    st = lib.atk_describe_topk_plan(_CODES[dtype], rows, N, K, buf, 512)
    return st, buf.value.decode()


def expected_recall(N: int, B: int, K: int, Kprime: int) -> float:
    return float(lib.atk_expected_recall(N, B, K, Kprime))


def select_params(N: int, K: int, recall_target: float, max_kprime: int = 4, bucket_multiple: int = 64):
    """(K', B, expected recall) with the fewest stage-1 survivors meeting the recall target."""
    kp, b, r = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_double(0.0)
    st = lib.atk_select_params(N, K, recall_target, max_kprime, bucket_multiple,
                               ctypes.byref(kp), ctypes.byref(b), ctypes.byref(r))
    if st != OK:
        raise AtkError(st, "atk_select_params")
    return kp.value, b.value, r.value


def recall_params(dtype: torch.dtype, rows: int, N: int, K: int, recall_target: float):
    """(K', B, expected recall) that approx_topk_recall uses for this problem."""
    kp, b, r = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_double(0.0)
    st = lib.atk_recall_params(_CODES[dtype], rows, N, K, recall_target, ctypes.byref(kp), ctypes.byref(b),
                               ctypes.byref(r))
    if st != OK:
        raise AtkError(st, "atk_recall_params")
    return kp.value, b.value, r.value


def set_option(name: str, value: int) -> None:
    """Developer option of the library (launch geometry only); value < 0 restores the default."""
    st = lib.atk_set_option(name.encode(), int(value))
    if st != OK:
        raise AtkError(st, f"atk_set_option({name!r}, {value})")


def _check_out(out, rows: int, K: int, val_dtype: torch.dtype, device):
    """A caller's (vals, idx) pair must be exactly what the library writes: dense [rows, K] of the
    value type and of int32, on the input's device."""
    out_vals, out_idx = out
    for t, dt, what in ((out_vals, val_dtype, "out values"), (out_idx, torch.int32, "out indices")):
        if not isinstance(t, torch.Tensor) or t.dtype != dt or tuple(t.shape) != (rows, K) \
                or t.device != device or not t.is_contiguous():
            raise ValueError(f"{what} must be a contiguous [{rows}, {K}] {dt} tensor on {device}")
    return out_vals, out_idx


def _workspace_ptr(workspace, device):
    """(pointer, bytes) of a caller's workspace: a dense tensor on the input's device."""
    if not isinstance(workspace, torch.Tensor) or workspace.device != device or not workspace.is_contiguous():
        raise ValueError(f"workspace must be a contiguous tensor on {device}")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def approx_topk_recall(values: torch.Tensor, K: int, recall_target: float, workspace=None, smallest: bool = False):
    """approx_top_k(array, K, recall_target) (smallest: the K smallest): returns (vals, idx, K' used, B used)."""
    rows, N, stride = _check_input(values)
    code = _dtype_code(values)
    kp, b, _ = recall_params(values.dtype, rows, N, K, recall_target)
    out_vals = torch.empty((rows, K), dtype=values.dtype, device=values.device)
    out_idx = torch.empty((rows, K), dtype=torch.int32, device=values.device)
    ws_ptr, ws_bytes = None, 0
    # (K' = K, B = 1 -- the exact fallback -- is sized like the exact entry)
    need = (lib.atk_workspace_bytes(OP_TOPK, code, rows, N, K, 0, 0) if (kp == K and b == 1)
            else lib.atk_workspace_bytes(OP_APPROX_TOPK, code, rows, N, K, kp, b))
    if need != SIZE_MAX and need > 0:
        if workspace is None or workspace.numel() * workspace.element_size() < need:
            workspace = torch.empty(need, dtype=torch.uint8, device=values.device)
        ws_ptr, ws_bytes = _workspace_ptr(workspace, values.device)
    kp_used, b_used = ctypes.c_int(0), ctypes.c_int(0)
    entry = lib.atk_approx_mink_recall if smallest else lib.atk_approx_topk_recall
    st = entry(values.data_ptr(), code, rows, N, stride, K, recall_target,
               out_vals.data_ptr(), out_idx.data_ptr(), ws_ptr, ws_bytes,
               _stream_ptr(values.device), ctypes.byref(kp_used), ctypes.byref(b_used))
    if st != OK:
        raise AtkError(st, "atk_approx_mink_recall" if smallest else "atk_approx_topk_recall")
    return out_vals, out_idx, kp_used.value, b_used.value


def approx_topk(values: torch.Tensor, K: int, Kprime: int, B: int, out=None, workspace=None,
                smallest: bool = False):
    """Two-stage approximate Top-K of every row (smallest: min-K, the K smallest, smallest first).
    Returns (vals[rows,K], idx[rows,K] int32)."""
    rows, N, stride = _check_input(values)
    code = _dtype_code(values)
    if out is None:
        out_vals = torch.empty((rows, K), dtype=values.dtype, device=values.device)
        out_idx = torch.empty((rows, K), dtype=torch.int32, device=values.device)
    else:
        out_vals, out_idx = _check_out(out, rows, K, values.dtype, values.device)
    need = lib.atk_workspace_bytes(OP_APPROX_TOPK, code, rows, N, K, Kprime, B)
    ws_ptr, ws_bytes = None, 0
    if need != SIZE_MAX and need > 0:
        if workspace is None or workspace.numel() * workspace.element_size() < need:
            workspace = torch.empty(need, dtype=torch.uint8, device=values.device)
        ws_ptr, ws_bytes = _workspace_ptr(workspace, values.device)
    entry = lib.atk_approx_mink if smallest else lib.atk_approx_topk
    st = entry(values.data_ptr(), code, rows, N, stride, K, Kprime, B,
               out_vals.data_ptr(), out_idx.data_ptr(), ws_ptr, ws_bytes, _stream_ptr(values.device))
    if st != OK:
        raise AtkError(st, "atk_approx_mink" if smallest else "atk_approx_topk")
    return out_vals, out_idx


def approx_topk_noalloc(values: torch.Tensor, K: int, Kprime: int, B: int, out):
    """atk_approx_topk_noalloc: the caller's `out` pair is required (this wrapper allocates nothing
    either), the library's own scratch array stands in for the workspace."""
    rows, N, stride = _check_input(values)
    out_vals, out_idx = _check_out(out, rows, K, values.dtype, values.device)
    st = lib.atk_approx_topk_noalloc(values.data_ptr(), _dtype_code(values), rows, N, stride, K, Kprime, B,
                                     out_vals.data_ptr(), out_idx.data_ptr(), _stream_ptr(values.device))
    if st != OK:
        raise AtkError(st, "atk_approx_topk_noalloc")
    return out_vals, out_idx


def topk(values: torch.Tensor, K: int, out=None, smallest: bool = False, workspace=None):
    """Exact Top-K (smallest: min-K) of every row under the library's total order.  workspace:
    a uint8 device tensor of workspace_bytes(OP_TOPK, ...) bytes, allocated here when omitted;
    False: none (the radix-selection kernel)."""
    rows, N, stride = _check_input(values)
    code = _dtype_code(values)
    if out is None:
        out_vals = torch.empty((rows, K), dtype=values.dtype, device=values.device)
        out_idx = torch.empty((rows, K), dtype=torch.int32, device=values.device)
    else:
        out_vals, out_idx = _check_out(out, rows, K, values.dtype, values.device)
    ws_ptr, ws_bytes = None, 0
    if workspace is None:
        need = int(lib.atk_workspace_bytes(OP_TOPK, code, rows, N, K, 0, 0))
        if need not in (0, SIZE_MAX):
            workspace = torch.empty(need, dtype=torch.uint8, device=values.device)
    if workspace is not None and workspace is not False:
        ws_ptr, ws_bytes = _workspace_ptr(workspace, values.device)
    entry = lib.atk_mink if smallest else lib.atk_topk
    st = entry(values.data_ptr(), code, rows, N, stride, K, out_vals.data_ptr(), out_idx.data_ptr(),
               ws_ptr, ws_bytes, _stream_ptr(values.device))
    if st != OK:
        raise AtkError(st, "atk_mink" if smallest else "atk_topk")
    return out_vals, out_idx


def mips_workspace_bytes(Q: int, N: int, D: int, K: int, Kprime: int, B: int) -> int:
    return int(lib.atk_mips_workspace_bytes(BF16, Q, N, D, K, Kprime, B))


def mips_describe_plan(Q: int, N: int, D: int, K: int, Kprime: int, B: int):
    buf = ctypes.create_string_buffer(512)
    st = lib.atk_mips_describe_plan(BF16, Q, N, D, K, Kprime, B, buf, 512)
    return st, buf.value.decode()


def mips_select_params(N: int, K: int, recall_target: float):
    """Fusion-aware (K', B) for the fused entry: smallest K', then smallest B.  Returns
    (K', B, expected recall); raises AtkError when no legal setting reaches the target."""
    kp, b, r = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_double(0.0)
    st = lib.atk_mips_select_params(N, K, recall_target, ctypes.byref(kp), ctypes.byref(b), ctypes.byref(r))
    if st != OK:
        raise AtkError(st, "atk_mips_select_params")
    return kp.value, b.value, r.value


def mips_approx_topk(queries: torch.Tensor, database: torch.Tensor, K: int, Kprime: int, B: int,
                     out=None, workspace=None):
    """Approximate Top-K of queries @ database.T without storing the scores (bf16 [Q,D], [N,D]).
    Returns (scores[Q,K] float32, idx[Q,K] int32)."""
    for t in (queries, database):
        if not t.is_cuda:
            raise ValueError("vectors must live on the GPU")
        if t.dim() != 2 or t.dtype not in (torch.bfloat16, torch.float16) or not t.is_contiguous():
            raise ValueError("vectors must be contiguous bf16 or fp16 [count, D] tensors")
    if queries.shape[1] != database.shape[1] or queries.dtype != database.dtype:
        raise ValueError("queries and database differ in D or in type")
    code = _CODES[queries.dtype]
    Q, D = queries.shape
    N = database.shape[0]
    if out is None:
        out_vals = torch.empty((Q, K), dtype=torch.float32, device=queries.device)
        out_idx = torch.empty((Q, K), dtype=torch.int32, device=queries.device)
    else:
        out_vals, out_idx = _check_out(out, Q, K, torch.float32, queries.device)
    need = lib.atk_mips_workspace_bytes(code, Q, N, D, K, Kprime, B)
    ws_ptr, ws_bytes = None, 0
    if need != SIZE_MAX and need > 0:
        if workspace is None or workspace.numel() * workspace.element_size() < need:
            workspace = torch.empty(need, dtype=torch.uint8, device=queries.device)
        ws_ptr, ws_bytes = _workspace_ptr(workspace, queries.device)
    st = lib.atk_mips_approx_topk(queries.data_ptr(), database.data_ptr(), code, Q, N, D, K, Kprime,
                                  B, out_vals.data_ptr(), out_idx.data_ptr(), ws_ptr, ws_bytes,
                                  _stream_ptr(queries.device))
    if st != OK:
        raise AtkError(st, "atk_mips_approx_topk")
    return out_vals, out_idx


def mips_approx_topk_recall(queries: torch.Tensor, database: torch.Tensor, K: int, recall_target: float):
    """Fused entry with fusion-aware parameters for a recall target.  Returns (scores, idx, K', B)."""
    kp, b, _ = mips_select_params(database.shape[0], K, recall_target)
    Q, D = queries.shape
    ws = torch.empty(max(1, mips_workspace_bytes(Q, database.shape[0], D, K, kp, b)), dtype=torch.uint8,
                     device=queries.device)
    out_vals = torch.empty((Q, K), dtype=torch.float32, device=queries.device)
    out_idx = torch.empty((Q, K), dtype=torch.int32, device=queries.device)
    kp_used, b_used = ctypes.c_int(0), ctypes.c_int(0)
    st = lib.atk_mips_approx_topk_recall(queries.data_ptr(), database.data_ptr(), _CODES[queries.dtype], Q,
                                         database.shape[0], D, K, recall_target, out_vals.data_ptr(),
                                         out_idx.data_ptr(), ws.data_ptr(), ws.numel(),
                                         _stream_ptr(queries.device), ctypes.byref(kp_used), ctypes.byref(b_used))
    if st != OK:
        raise AtkError(st, "atk_mips_approx_topk_recall")
    return out_vals, out_idx, kp_used.value, b_used.value


def valu_probe(kind: int, x: torch.Tensor, y, ops: int, out=None):
    """Run the vector-ALU probe on int32 tensors (kind 0: fibonacci steps, 1: squarings)."""
    if out is None:
        out = torch.empty_like(x)
    st = lib.atk_valu_probe(kind, x.data_ptr(), None if y is None else y.data_ptr(), out.data_ptr(),
                            x.numel(), ops, _stream_ptr(x.device))
    if st != OK:
        raise AtkError(st, "atk_valu_probe")
    return out


READ_PROBE_WORDS = 256


def read_probe(data: torch.Tensor, checksum: torch.Tensor | None = None):
    """Stream `data` (contiguous, on the GPU) once, read only.  Returns the int32 tensor of
    READ_PROBE_WORDS words whose exclusive-or is that of all 32-bit words of `data` (pass a zeroed
    one to reuse it)."""
    if not data.is_cuda or not data.is_contiguous():
        raise ValueError("data must be a contiguous GPU tensor")
    if checksum is None:
        checksum = torch.zeros(READ_PROBE_WORDS, dtype=torch.int32, device=data.device)
    elif checksum.dtype != torch.int32 or checksum.numel() != READ_PROBE_WORDS or not checksum.is_contiguous() \
            or checksum.device != data.device:
        raise ValueError(f"checksum must be a contiguous int32 tensor of {READ_PROBE_WORDS} words on {data.device}")
    st = lib.atk_read_probe(data.data_ptr(), data.numel() * data.element_size(), checksum.data_ptr(),
                            _stream_ptr(data.device))
    if st != OK:
        raise AtkError(st, "atk_read_probe")
    return checksum


def approx_topk_stage1(values: torch.Tensor, Kprime: int, B: int):
    """Stage 1 only: survivors (vals[rows,K',B], idx[rows,K',B] int32)."""
    rows, N, stride = _check_input(values)
    code = _dtype_code(values)
    sv = torch.empty((rows, Kprime, B), dtype=values.dtype, device=values.device)
    si = torch.empty((rows, Kprime, B), dtype=torch.int32, device=values.device)
    st = lib.atk_approx_topk_stage1(values.data_ptr(), code, rows, N, stride, Kprime, B,
                                    sv.data_ptr(), si.data_ptr(), _stream_ptr(values.device))
    if st != OK:
        raise AtkError(st, "atk_approx_topk_stage1")
    return sv, si
