"""ctypes binding of libfp8mm.so: same names as the C ABI (include/fp8mm.h), argument
marshalling only.  Tensors are torch tensors used as device buffers; every computation
happens in the HIP kernels.  There is no fallback: a missing library is an error."""
from __future__ import annotations

import ctypes
import os

import torch

FP8_E4M3, FP8_E5M2 = 0, 1
FP8_F32, FP8_BF16 = 0, 1
FP8_OK, FP8_ERR_INVALID_ARG, FP8_ERR_UNSUPPORTED, FP8_ERR_DEVICE = 0, 1, 2, 3
FP8_QUANT_NOSAT = 1
FP8_AMAX_WORKSPACE_BYTES = 16384
FP8_SPLITK_STATIC_BYTES = 64 << 20
FP8_GEMM_MFMA8 = 1
FP8_OUT_F32, FP8_OUT_BF16, FP8_OUT_E4M3, FP8_OUT_E5M2 = 0, 1, 2, 3
FP8_PLAN_NO_GEMM, FP8_PLAN_FMA_KERNEL, FP8_PLAN_TILED_256x256, FP8_PLAN_TILED_256x128, FP8_PLAN_MFMA_ANY, FP8_PLAN_TILED_MIXED = 0, 1, 2, 3, 4, 5
FP8_PLAN_ELEMENTWISE_STORES = 16
FP8_MULTI_MAX = 4
FP8_PLAN_PERSISTENT = 32
FP8_KNOB_CAST_PATH, FP8_KNOB_TILE_N, FP8_KNOB_GROUP_M, FP8_KNOB_GEMM_KERNEL, FP8_KNOB_SPLIT_K, FP8_KNOB_CAST_RUN, FP8_KNOB_PERSIST, FP8_KNOB_MIXED = 0, 1, 2, 3, 4, 5, 6, 7

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libfp8mm.so")

EXPORTS = (
    "fp8_amax", "fp8_amax_scale", "fp8_amax_scale_multi", "fp8_quantize_multi", "fp8_scale_from_amax_host", "fp8_scale_from_amax", "fp8_quantize",
    "fp8_quantize_dscale", "fp8_quantize_ex", "fp8_dequantize", "fp8_quantize_amax", "fp8_quantize_sr",
    "fp8_scale_from_amax_history", "fp8_scale_from_amax_n", "fp8_amax_rows", "fp8_quantize_rows",
    "fp8_quantize_transpose", "fp8_gemm", "fp8_gemm_dscale", "fp8_gemm_mfma8",
    "fp8_gemm_mfma8_dscale", "fp8_gemm_ex", "fp8_gemm_splitk", "fp8_gemm_splitk_workspace_size", "fp8_gemm_splitk_static", "fp8_gemm_fused", "fp8_scaled_gemm", "fp8_gemm_plan", "fp8_set_knob", "fp8_get_knob",
    "fp8_last_error", "fp8_version",
)

_lib = None


class Fp8Error(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("fp8mm status %d: %s" % (status, message))
        self.status = status


def lib() -> ctypes.CDLL:
    """Loads the built library (build it first: python -m paper_2209_05433_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s is missing: build the HIP library with __graft_entry__.build() or "
            "`python paper_2209_05433_amd/build.py`; there is no CPU fallback" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, sz, i, i64, f = c.c_void_p, c.c_size_t, c.c_int, c.c_int64, c.c_float
    L.fp8_amax.argtypes, L.fp8_amax.restype = [vp, sz, i, vp, vp], i
    L.fp8_amax_scale.argtypes, L.fp8_amax_scale.restype = [vp, sz, i, i, vp, vp, vp, vp], i
    L.fp8_amax_scale_multi.argtypes, L.fp8_amax_scale_multi.restype = [i, vp, vp, i, vp, vp, vp, vp, vp], i
    L.fp8_quantize_multi.argtypes, L.fp8_quantize_multi.restype = [i, vp, vp, i, vp, vp, vp, vp], i
    L.fp8_scale_from_amax_host.argtypes, L.fp8_scale_from_amax_host.restype = [f, i], f
    L.fp8_scale_from_amax.argtypes, L.fp8_scale_from_amax.restype = [vp, i, vp, vp], i
    L.fp8_quantize.argtypes, L.fp8_quantize.restype = [vp, sz, i, i, f, vp, vp], i
    L.fp8_quantize_dscale.argtypes, L.fp8_quantize_dscale.restype = [vp, sz, i, i, vp, vp, vp], i
    L.fp8_quantize_ex.argtypes, L.fp8_quantize_ex.restype = [vp, sz, i, i, f, vp, i, vp, vp], i
    L.fp8_dequantize.argtypes, L.fp8_dequantize.restype = [vp, sz, i, f, vp, i, vp, vp], i
    L.fp8_gemm.argtypes, L.fp8_gemm.restype = [vp, i, f, vp, i, f, vp, i64, i64, i64, i, vp], i
    L.fp8_gemm_dscale.argtypes, L.fp8_gemm_dscale.restype = [vp, i, vp, vp, i, vp, vp, i64, i64, i64, i, vp], i
    L.fp8_gemm_mfma8.argtypes, L.fp8_gemm_mfma8.restype = L.fp8_gemm.argtypes, i
    L.fp8_gemm_mfma8_dscale.argtypes, L.fp8_gemm_mfma8_dscale.restype = L.fp8_gemm_dscale.argtypes, i
    L.fp8_gemm_ex.argtypes, L.fp8_gemm_ex.restype = [vp, i, i, vp, i, i, vp, i64, i64, i64, i, f, f, vp, vp, i, vp], i
    L.fp8_scaled_gemm.argtypes, L.fp8_scaled_gemm.restype = [vp, vp, i, i, i, i64, i64, i64, i, i, vp, vp, vp, vp, vp, vp, i, i, vp], i
    L.fp8_gemm_splitk.argtypes, L.fp8_gemm_splitk.restype = [vp, i, i, vp, i, i, vp, i64, i64, i64, i, f, f, vp, vp, i, i, vp, sz, vp], i
    L.fp8_gemm_splitk_static.argtypes, L.fp8_gemm_splitk_static.restype = [vp, i, i, vp, i, i, vp, i64, i64, i64, i, f, f, vp, vp, i, i, vp], i
    L.fp8_gemm_splitk_workspace_size.argtypes, L.fp8_gemm_splitk_workspace_size.restype = [i64, i64, i64, i, i, i], sz
    L.fp8_gemm_fused.argtypes, L.fp8_gemm_fused.restype = [vp, i, i, vp, i, i, vp, i, i64, i64, i64, vp, i64, vp, i64, vp, vp, i, vp], i
    L.fp8_quantize_sr.argtypes, L.fp8_quantize_sr.restype = [vp, sz, i, i, f, vp, c.c_uint64, vp, vp], i
    L.fp8_quantize_amax.argtypes, L.fp8_quantize_amax.restype = [vp, sz, i, i, vp, vp, vp, vp], i
    L.fp8_scale_from_amax_history.argtypes, L.fp8_scale_from_amax_history.restype = [vp, sz, i, vp, vp], i
    L.fp8_scale_from_amax_n.argtypes, L.fp8_scale_from_amax_n.restype = [vp, sz, i, vp, vp], i
    L.fp8_amax_rows.argtypes, L.fp8_amax_rows.restype = [vp, i64, i64, i, vp, vp], i
    L.fp8_quantize_rows.argtypes, L.fp8_quantize_rows.restype = [vp, i64, i64, i, i, vp, vp, vp], i
    L.fp8_quantize_transpose.argtypes, L.fp8_quantize_transpose.restype = [vp, i64, i64, i, i, vp, vp, vp, vp], i
    L.fp8_gemm_plan.argtypes, L.fp8_gemm_plan.restype = [vp, i, vp, i, vp, i64, i64, i64, vp], i
    L.fp8_set_knob.argtypes, L.fp8_set_knob.restype = [i, i], i
    L.fp8_get_knob.argtypes, L.fp8_get_knob.restype = [i], i
    L.fp8_last_error.argtypes, L.fp8_last_error.restype = [], c.c_char_p
    L.fp8_version.argtypes, L.fp8_version.restype = [], c.c_char_p
    _lib = L
    return L


def _check(status: int) -> None:
    if status != FP8_OK:
        raise Fp8Error(status, lib().fp8_last_error().decode())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: torch.Tensor, what: str) -> int:
    if not t.is_cuda:
        raise ValueError("%s must live in device memory" % what)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    return t.data_ptr()


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FP8_F32
    if t.dtype == torch.bfloat16:
        return FP8_BF16
    raise TypeError("expected a float32 or bfloat16 tensor, got %s" % t.dtype)


def fp8_last_error() -> str:
    return lib().fp8_last_error().decode()


def fp8_version() -> str:
    return lib().fp8_version().decode()


def fp8_set_knob(knob: int, value: int) -> int:
    """Sets a tuning knob (fp8_knob_t) and returns its previous value."""
    old = lib().fp8_set_knob(int(knob), int(value))
    if old < 0:
        raise Fp8Error(-old, lib().fp8_last_error().decode())
    return old


def fp8_get_knob(knob: int) -> int:
    v = lib().fp8_get_knob(int(knob))
    if v < 0:
        raise Fp8Error(-v, lib().fp8_last_error().decode())
    return v


def fp8_gemm_plan(A: torch.Tensor, transA: bool, B: torch.Tensor, transB: bool, C: torch.Tensor, sB_per_column=None) -> int:
    """Which kernel the GEMM entry points would run for these tensors (an fp8_plan_t, possibly ORed
    with FP8_PLAN_ELEMENTWISE_STORES); nothing is launched."""
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    N = B.shape[0] if transB else B.shape[1]
    plan = lib().fp8_gemm_plan(A.data_ptr(), int(bool(transA)), B.data_ptr(), int(bool(transB)), C.data_ptr(), M, N, K,
                               None if sB_per_column is None else sB_per_column.data_ptr())
    if plan < 0:
        raise Fp8Error(-plan, lib().fp8_last_error().decode())
    return plan


def fp8_amax(x: torch.Tensor, amax_out: torch.Tensor, stream=None) -> None:
    _check(lib().fp8_amax(_dev(x, "x") if x.numel() else None, x.numel(), dtype_code(x),
                          _dev(amax_out, "amax_out"), _stream(stream)))


def fp8_amax_scale(x: torch.Tensor, fmt: int, amax_out: torch.Tensor, scale_out, workspace: torch.Tensor, stream=None) -> None:
    """amax and scale = fmt_max / amax in one launch; workspace: device tensor of at least
    FP8_AMAX_WORKSPACE_BYTES bytes, zero-filled once before its first use."""
    if workspace.numel() * workspace.element_size() < FP8_AMAX_WORKSPACE_BYTES:
        raise ValueError("workspace must hold FP8_AMAX_WORKSPACE_BYTES bytes")
    _check(lib().fp8_amax_scale(_dev(x, "x") if x.numel() else None, x.numel(), dtype_code(x), fmt,
                                _dev(amax_out, "amax_out"), _dev(scale_out, "scale_out") if scale_out is not None else None,
                                _dev(workspace, "workspace"), _stream(stream)))


def _host_arrays(tensors, fmts, what):
    """The host-side argument arrays of the multi-tensor entry points: device pointers, element counts, formats."""
    count = len(tensors)
    if count > FP8_MULTI_MAX or len(fmts) != count:
        raise ValueError("%s: at most %d tensors, one format each" % (what, FP8_MULTI_MAX))
    codes = {dtype_code(t) for t in tensors}
    if len(codes) > 1:
        raise TypeError("%s: all tensors must have one element type" % what)
    ptrs = (ctypes.c_void_p * count)(*[(_dev(t, "x") if t.numel() else None) for t in tensors])
    ns = (ctypes.c_size_t * count)(*[t.numel() for t in tensors])
    fm = (ctypes.c_int * count)(*[int(f) for f in fmts])
    return count, ptrs, ns, (codes.pop() if codes else FP8_BF16), fm


def fp8_amax_scale_multi(xs, fmts, amax_out: torch.Tensor, scale_out, workspace: torch.Tensor, stream=None) -> None:
    """fp8_amax_scale for up to FP8_MULTI_MAX tensors of one element type in one launch: amax_out and
    scale_out are fp32 device tensors of len(xs) values, workspace holds len(xs) * FP8_AMAX_WORKSPACE_BYTES bytes."""
    count, ptrs, ns, code, fm = _host_arrays(xs, fmts, "fp8_amax_scale_multi")
    if workspace.numel() * workspace.element_size() < count * FP8_AMAX_WORKSPACE_BYTES:
        raise ValueError("workspace must hold FP8_AMAX_WORKSPACE_BYTES bytes per tensor")
    _check(lib().fp8_amax_scale_multi(count, ptrs, ns, code, fm, _f32_cells(amax_out, "amax_out", count),
                                      _f32_cells(scale_out, "scale_out", count) if scale_out is not None else None,
                                      _dev(workspace, "workspace"), _stream(stream)))


def fp8_quantize_multi(xs, fmts, scale: torch.Tensor, q_outs, stream=None) -> None:
    """fp8_quantize_dscale for up to FP8_MULTI_MAX tensors of one element type in one launch; scale is an
    fp32 device tensor of len(xs) factors, q_outs the uint8 outputs."""
    count, ptrs, ns, code, fm = _host_arrays(xs, fmts, "fp8_quantize_multi")
    if len(q_outs) != count or any(q.dtype != torch.uint8 or q.numel() != x.numel() for q, x in zip(q_outs, xs)):
        raise ValueError("q_outs must be uint8 tensors with as many elements as their inputs")
    qs = (ctypes.c_void_p * count)(*[(_dev(q, "q_out") if q.numel() else None) for q in q_outs])
    _check(lib().fp8_quantize_multi(count, ptrs, ns, code, fm, _f32_cells(scale, "scale", count), qs, _stream(stream)))


def fp8_scale_from_amax_host(amax: float, fmt: int) -> float:
    return float(lib().fp8_scale_from_amax_host(float(amax), fmt))


def fp8_scale_from_amax(amax: torch.Tensor, fmt: int, scale_out: torch.Tensor, stream=None) -> None:
    _check(lib().fp8_scale_from_amax(_dev(amax, "amax"), fmt, _dev(scale_out, "scale_out"),
                                     _stream(stream)))


def fp8_quantize(x: torch.Tensor, fmt: int, scale: float, q_out: torch.Tensor, stream=None) -> None:
    if q_out.dtype != torch.uint8 or q_out.numel() != x.numel():
        raise ValueError("q_out must be uint8 with as many elements as x")
    _check(lib().fp8_quantize(_dev(x, "x") if x.numel() else None, x.numel(), dtype_code(x), fmt,
                              float(scale), _dev(q_out, "q_out") if x.numel() else None,
                              _stream(stream)))


def fp8_quantize_dscale(x: torch.Tensor, fmt: int, scale: torch.Tensor, q_out: torch.Tensor,
                        stream=None) -> None:
    if q_out.dtype != torch.uint8 or q_out.numel() != x.numel():
        raise ValueError("q_out must be uint8 with as many elements as x")
    _check(lib().fp8_quantize_dscale(_dev(x, "x") if x.numel() else None, x.numel(), dtype_code(x),
                                     fmt, _dev(scale, "scale"),
                                     _dev(q_out, "q_out") if x.numel() else None, _stream(stream)))


def fp8_quantize_ex(x: torch.Tensor, fmt: int, scale, flags: int, q_out: torch.Tensor, stream=None) -> None:
    """`scale` is a float or a one-element device tensor."""
    if q_out.dtype != torch.uint8 or q_out.numel() != x.numel():
        raise ValueError("q_out must be uint8 with as many elements as x")
    dev = isinstance(scale, torch.Tensor)
    _check(lib().fp8_quantize_ex(_dev(x, "x") if x.numel() else None, x.numel(), dtype_code(x), fmt,
                                 0.0 if dev else float(scale), _dev(scale, "scale") if dev else None,
                                 int(flags), _dev(q_out, "q_out") if x.numel() else None, _stream(stream)))


def fp8_dequantize(q: torch.Tensor, fmt: int, scale, out: torch.Tensor, stream=None) -> None:
    """`scale` is a float or a one-element device tensor; out is float32 or bfloat16."""
    if q.dtype != torch.uint8 or out.numel() != q.numel():
        raise ValueError("q must be uint8 and out must have as many elements")
    dev = isinstance(scale, torch.Tensor)
    _check(lib().fp8_dequantize(_dev(q, "q") if q.numel() else None, q.numel(), fmt,
                                0.0 if dev else float(scale), _dev(scale, "scale") if dev else None,
                                dtype_code(out), _dev(out, "out") if q.numel() else None, _stream(stream)))


def _gemm_dims(A, B, C):
    if A.dtype != torch.uint8 or B.dtype != torch.uint8 or A.dim() != 2 or B.dim() != 2:
        raise ValueError("A and B must be 2-D uint8 tensors of FP8 bytes")
    M, K = A.shape
    K2, N = B.shape
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("shapes do not form C[M,N] = A[M,K] B[K,N]")
    return M, N, K


def _gemm(fn, A, fmtA, sA, B, fmtB, sB, C, stream):
    M, N, K = _gemm_dims(A, B, C)
    _check(fn(_dev(A, "A") if A.numel() else None, fmtA, sA,
              _dev(B, "B") if B.numel() else None, fmtB, sB,
              _dev(C, "C") if C.numel() else None, M, N, K, dtype_code(C), _stream(stream)))


def fp8_gemm(A, fmtA: int, sA: float, B, fmtB: int, sB: float, C, stream=None) -> None:
    _gemm(lib().fp8_gemm, A, fmtA, float(sA), B, fmtB, float(sB), C, stream)


def fp8_gemm_dscale(A, fmtA: int, sA: torch.Tensor, B, fmtB: int, sB: torch.Tensor, C,
                    stream=None) -> None:
    _gemm(lib().fp8_gemm_dscale, A, fmtA, _dev(sA, "sA"), B, fmtB, _dev(sB, "sB"), C, stream)


def fp8_gemm_mfma8(A, fmtA: int, sA: float, B, fmtB: int, sB: float, C, stream=None) -> None:
    _gemm(lib().fp8_gemm_mfma8, A, fmtA, float(sA), B, fmtB, float(sB), C, stream)


def fp8_gemm_mfma8_dscale(A, fmtA: int, sA: torch.Tensor, B, fmtB: int, sB: torch.Tensor, C,
                          stream=None) -> None:
    _gemm(lib().fp8_gemm_mfma8_dscale, A, fmtA, _dev(sA, "sA"), B, fmtB, _dev(sB, "sB"), C, stream)


def fp8_gemm_ex(A, fmtA: int, transA: bool, B, fmtB: int, transB: bool, C, sA, sB, flags: int = 0,
                stream=None) -> None:
    """A is [M, K] (or [K, M] if transA), B is [K, N] (or [N, K] if transB); sA and sB are both
    floats or both one-element device tensors."""
    if A.dtype != torch.uint8 or B.dtype != torch.uint8 or A.dim() != 2 or B.dim() != 2:
        raise ValueError("A and B must be 2-D uint8 tensors of FP8 bytes")
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    N, K2 = (B.shape[0], B.shape[1]) if transB else (B.shape[1], B.shape[0])
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("shapes do not form C[M,N] = op(A)[M,K] op(B)[K,N]")
    dev = isinstance(sA, torch.Tensor)
    if dev != isinstance(sB, torch.Tensor):
        raise ValueError("sA and sB must both be floats or both device tensors")
    _check(lib().fp8_gemm_ex(_dev(A, "A") if A.numel() else None, fmtA, int(bool(transA)),
                             _dev(B, "B") if B.numel() else None, fmtB, int(bool(transB)),
                             _dev(C, "C") if C.numel() else None, M, N, K, dtype_code(C),
                             0.0 if dev else float(sA), 0.0 if dev else float(sB),
                             _dev(sA, "sA") if dev else None, _dev(sB, "sB") if dev else None,
                             int(flags), _stream(stream)))


def fp8_scaled_gemm(a, fmtA: int, transA: bool, b, fmtB: int, transB: bool, qa_out, qb_out, amax_out, scale_out,
                    workspace, C, flags: int = 0, stream=None) -> None:
    """amax + scale + cast of both operands and their FP8 product in one call.  a is [M, K] (or
    [K, M] if transA), b is [K, N] (or [N, K] if transB), both bf16 or both fp32; qa_out / qb_out are
    uint8 tensors of the operands' shapes; amax_out and scale_out hold two floats ([0]: a, [1]: b);
    workspace: 2 * FP8_AMAX_WORKSPACE_BYTES bytes, zero-filled once."""
    if a.dim() != 2 or b.dim() != 2 or a.dtype != b.dtype:
        raise ValueError("a and b must be 2-D tensors of one element type")
    M, K = (a.shape[1], a.shape[0]) if transA else a.shape
    N, K2 = (b.shape[0], b.shape[1]) if transB else (b.shape[1], b.shape[0])
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("shapes do not form C[M,N] = op(a)[M,K] op(b)[K,N]")
    for q, x in ((qa_out, a), (qb_out, b)):
        if q.dtype != torch.uint8 or tuple(q.shape) != tuple(x.shape):
            raise ValueError("qa_out / qb_out must be uint8 tensors of the operands' shapes")
    if workspace.numel() * workspace.element_size() < 2 * FP8_AMAX_WORKSPACE_BYTES:
        raise ValueError("workspace must hold 2 * FP8_AMAX_WORKSPACE_BYTES bytes")
    _check(lib().fp8_scaled_gemm(_dev(a, "a") if a.numel() else None, _dev(b, "b") if b.numel() else None, dtype_code(a),
                                 int(bool(transA)), int(bool(transB)), M, N, K, fmtA, fmtB,
                                 _dev(qa_out, "qa_out") if qa_out.numel() else None, _dev(qb_out, "qb_out") if qb_out.numel() else None,
                                 _f32_cells(amax_out, "amax_out", 2), _f32_cells(scale_out, "scale_out", 2), _dev(workspace, "workspace"),
                                 _dev(C, "C") if C.numel() else None, dtype_code(C), int(flags), _stream(stream)))


def _gemm_ex_dims(A, transA, B, transB, C):
    if A.dtype != torch.uint8 or B.dtype != torch.uint8 or A.dim() != 2 or B.dim() != 2:
        raise ValueError("A and B must be 2-D uint8 tensors of FP8 bytes")
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    N, K2 = (B.shape[0], B.shape[1]) if transB else (B.shape[1], B.shape[0])
    if K != K2 or tuple(C.shape) != (M, N):
        raise ValueError("shapes do not form C[M,N] = op(A)[M,K] op(B)[K,N]")
    return M, N, K


def fp8_gemm_splitk_workspace_size(M: int, N: int, K: int, transA: bool, transB: bool, splits: int = 0) -> int:
    return int(lib().fp8_gemm_splitk_workspace_size(M, N, K, int(bool(transA)), int(bool(transB)), int(splits)))


def fp8_gemm_splitk(A, fmtA: int, transA: bool, B, fmtB: int, transB: bool, C, sA, sB, workspace, flags: int = 0,
                    splits: int = 0, stream=None) -> None:
    """fp8_gemm_ex with K cut into slices; `workspace` is a device tensor (any dtype) of at least
    fp8_gemm_splitk_workspace_size(...) bytes, or None where that is 0."""
    M, N, K = _gemm_ex_dims(A, transA, B, transB, C)
    dev = isinstance(sA, torch.Tensor)
    if dev != isinstance(sB, torch.Tensor):
        raise ValueError("sA and sB must both be floats or both device tensors")
    _check(lib().fp8_gemm_splitk(_dev(A, "A") if A.numel() else None, fmtA, int(bool(transA)),
                                 _dev(B, "B") if B.numel() else None, fmtB, int(bool(transB)),
                                 _dev(C, "C") if C.numel() else None, M, N, K, dtype_code(C),
                                 0.0 if dev else float(sA), 0.0 if dev else float(sB),
                                 _dev(sA, "sA") if dev else None, _dev(sB, "sB") if dev else None,
                                 int(flags), int(splits),
                                 _dev(workspace, "workspace") if workspace is not None else None,
                                 workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                 _stream(stream)))


def fp8_gemm_splitk_static(A, fmtA: int, transA: bool, B, fmtB: int, transB: bool, C, sA, sB, flags: int = 0,
                           splits: int = 0, stream=None) -> None:
    """fp8_gemm_splitk with the library's own scratch array in place of a workspace; allocates nothing."""
    M, N, K = _gemm_ex_dims(A, transA, B, transB, C)
    dev = isinstance(sA, torch.Tensor)
    if dev != isinstance(sB, torch.Tensor):
        raise ValueError("sA and sB must both be floats or both device tensors")
    _check(lib().fp8_gemm_splitk_static(_dev(A, "A") if A.numel() else None, fmtA, int(bool(transA)),
                                        _dev(B, "B") if B.numel() else None, fmtB, int(bool(transB)),
                                        _dev(C, "C") if C.numel() else None, M, N, K, dtype_code(C),
                                        0.0 if dev else float(sA), 0.0 if dev else float(sB),
                                        _dev(sA, "sA") if dev else None, _dev(sB, "sB") if dev else None,
                                        int(flags), int(splits), _stream(stream)))


def fp8_gemm_fused(A, fmtA: int, transA: bool, B, fmtB: int, transB: bool, D, out_kind: int, sA, sB,
                   sD=None, amax_out=None, flags: int = 0, stream=None) -> None:
    """A is [M, K] (or [K, M] if transA), B is [K, N] (or [N, K] if transB), D is [M, N] of the
    element type of out_kind (uint8 for the FP8 kinds).  sA: fp32 device tensor of 1 or M values,
    sB: of 1 or N values; sD: None or one value; amax_out: None or one fp32 cell."""
    if A.dtype != torch.uint8 or B.dtype != torch.uint8 or A.dim() != 2 or B.dim() != 2:
        raise ValueError("A and B must be 2-D uint8 tensors of FP8 bytes")
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    N, K2 = (B.shape[0], B.shape[1]) if transB else (B.shape[1], B.shape[0])
    if K != K2 or tuple(D.shape) != (M, N):
        raise ValueError("shapes do not form D[M,N] = op(A)[M,K] op(B)[K,N]")
    want = {FP8_OUT_F32: torch.float32, FP8_OUT_BF16: torch.bfloat16}.get(out_kind, torch.uint8)
    if D.dtype != want:
        raise ValueError("D must be %s for out_kind %d" % (want, out_kind))
    for name, t in (("sA", sA), ("sB", sB), ("sD", sD), ("amax_out", amax_out)):
        if t is not None and t.dtype != torch.float32:
            raise ValueError("%s must be an fp32 device tensor" % name)
    _check(lib().fp8_gemm_fused(_dev(A, "A") if A.numel() else None, fmtA, int(bool(transA)),
                                _dev(B, "B") if B.numel() else None, fmtB, int(bool(transB)),
                                _dev(D, "D") if D.numel() else None, int(out_kind), M, N, K,
                                _dev(sA, "sA"), sA.numel(), _dev(sB, "sB"), sB.numel(),
                                _dev(sD, "sD") if sD is not None else None,
                                _dev(amax_out, "amax_out") if amax_out is not None else None,
                                int(flags), _stream(stream)))


def _f32_cells(t, what, count=None):
    if t.dtype != torch.float32 or (count is not None and t.numel() != count):
        raise ValueError("%s must be an fp32 device tensor%s" % (what, "" if count is None else " of %d values" % count))
    return _dev(t, what)


def fp8_quantize_amax(x, fmt: int, scale, q_out, amax_out, stream=None) -> None:
    """Cast x with the one-element device tensor `scale` and write max |x| into amax_out."""
    if q_out.dtype != torch.uint8 or q_out.numel() != x.numel():
        raise ValueError("q_out must be uint8 with as many elements as x")
    _check(lib().fp8_quantize_amax(_dev(x, "x") if x.numel() else None, x.numel(), dtype_code(x), fmt,
                                   _f32_cells(scale, "scale", 1), _dev(q_out, "q_out") if x.numel() else None,
                                   _f32_cells(amax_out, "amax_out", 1), _stream(stream)))


def fp8_scale_from_amax_history(amax_history, fmt: int, scale_out, stream=None) -> None:
    _check(lib().fp8_scale_from_amax_history(_f32_cells(amax_history, "amax_history") if amax_history.numel() else None,
                                             amax_history.numel(), fmt, _f32_cells(scale_out, "scale_out", 1),
                                             _stream(stream)))


def fp8_scale_from_amax_n(amax, fmt: int, scale_out, stream=None) -> None:
    n = amax.numel()
    _check(lib().fp8_scale_from_amax_n(_f32_cells(amax, "amax") if n else None, n, fmt,
                                       _f32_cells(scale_out, "scale_out", n) if n else None, _stream(stream)))


def _matrix(x, what):
    if x.dim() != 2:
        raise ValueError("%s must be a 2-D tensor" % what)
    return x.shape[0], x.shape[1]


def fp8_amax_rows(x, amax_out, stream=None) -> None:
    rows, cols = _matrix(x, "x")
    _check(lib().fp8_amax_rows(_dev(x, "x") if x.numel() else None, rows, cols, dtype_code(x),
                               _f32_cells(amax_out, "amax_out", rows) if rows else None, _stream(stream)))


def fp8_quantize_rows(x, fmt: int, scale, q_out, stream=None) -> None:
    rows, cols = _matrix(x, "x")
    if q_out.dtype != torch.uint8 or tuple(q_out.shape) != (rows, cols):
        raise ValueError("q_out must be a uint8 tensor of the shape of x")
    _check(lib().fp8_quantize_rows(_dev(x, "x") if x.numel() else None, rows, cols, dtype_code(x), fmt,
                                   _f32_cells(scale, "scale", rows) if x.numel() else None,
                                   _dev(q_out, "q_out") if x.numel() else None, _stream(stream)))


def fp8_quantize_transpose(x, fmt: int, scale, q_out, qt_out, stream=None) -> None:
    """q_out (rows x cols, may be None) and qt_out (cols x rows) receive the FP8 bytes of x."""
    rows, cols = _matrix(x, "x")
    if qt_out.dtype != torch.uint8 or tuple(qt_out.shape) != (cols, rows):
        raise ValueError("qt_out must be a uint8 tensor of shape (cols, rows)")
    if q_out is not None and (q_out.dtype != torch.uint8 or tuple(q_out.shape) != (rows, cols)):
        raise ValueError("q_out must be None or a uint8 tensor of the shape of x")
    _check(lib().fp8_quantize_transpose(_dev(x, "x") if x.numel() else None, rows, cols, dtype_code(x), fmt,
                                        _f32_cells(scale, "scale", 1) if x.numel() else None,
                                        _dev(q_out, "q_out") if (q_out is not None and x.numel()) else None,
                                        _dev(qt_out, "qt_out") if x.numel() else None, _stream(stream)))


def fp8_quantize_sr(x, fmt: int, scale, seed: int, q_out, stream=None) -> None:
    """Stochastic-rounding cast; scale is a float or a one-element fp32 device tensor."""
    if q_out.dtype != torch.uint8 or q_out.numel() != x.numel():
        raise ValueError("q_out must be uint8 with as many elements as x")
    dev = isinstance(scale, torch.Tensor)
    _check(lib().fp8_quantize_sr(_dev(x, "x") if x.numel() else None, x.numel(), dtype_code(x), fmt,
                                 1.0 if dev else float(scale), _f32_cells(scale, "scale", 1) if dev else None,
                                 int(seed) & 0xFFFFFFFFFFFFFFFF, _dev(q_out, "q_out") if x.numel() else None,
                                 _stream(stream)))
