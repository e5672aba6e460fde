"""Thin ctypes binding of libslidesparse.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/slidesparse.h; tensors are torch CUDA tensors used purely as device
memory, and work is enqueued on torch's current stream.  There is no CPU
fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libslidesparse.so")

SS_I8, SS_FP8_E4M3, SS_BF16, SS_FP16 = 0, 1, 2, 3
SS_IN_F32, SS_IN_BF16 = 0, 1
DTYPE_CODE = {"i8": SS_I8, "fp8": SS_FP8_E4M3, "bf16": SS_BF16, "fp16": SS_FP16}
EXPORTS = ("slide_lifted_k", "slide_lifted_ld", "slide_packed_sizes", "slide_prune_quant", "slide_decompose",
           "slide_decompose_canonical", "act_lift_quant", "slide_sparse_gemm", "dense_gemm",
           "slide_gemm_workspace_bytes", "slide_sparse_gemm_ws", "dense_gemm_ws",
           "slide_packed_sizes_fused", "slide_decompose_fused", "slide_sparse_gemm_fused", "slide_sparse_gemm_fused_ws",
           "slide_static_scratch_bytes", "slide_sparse_gemm_static",
           "ss_status_string", "slide_format_version")

_lib = None


class SlideSparseError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (status {code})")


def load():
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it first (python -m paper_2603_05232_amd.build)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, vp, sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.slide_lifted_k.argtypes = [i64, i32]
    lib.slide_lifted_k.restype = i64
    lib.slide_lifted_ld.argtypes = [i64, i32, i32]
    lib.slide_lifted_ld.restype = i64
    lib.slide_packed_sizes.argtypes = [i64, i64, i32, i32, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.slide_prune_quant.argtypes = [vp, i32, i64, i64, i32, i32, vp, vp, vp]
    lib.slide_decompose.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
    lib.slide_decompose_canonical.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
    lib.act_lift_quant.argtypes = [vp, i32, i64, i64, i64, i32, i32, vp, vp, vp]
    lib.slide_sparse_gemm.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, i64, vp]
    lib.dense_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, i64, vp]
    lib.slide_sparse_gemm_ws.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, i64, vp, sz, vp]
    lib.dense_gemm_ws.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, vp, i64, vp, sz, vp]
    lib.slide_packed_sizes_fused.argtypes = [i64, i64, i32, i32, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.slide_decompose_fused.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp]
    lib.slide_sparse_gemm_fused.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, i32, vp, i64, vp]
    lib.slide_sparse_gemm_fused_ws.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, i32, i32, vp, i64, vp, sz, vp]
    lib.slide_static_scratch_bytes.argtypes = []
    lib.slide_static_scratch_bytes.restype = sz
    lib.slide_sparse_gemm_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, i64, vp]
    lib.slide_sparse_gemm_static.restype = i32
    lib.slide_gemm_workspace_bytes.argtypes = [i64, i64, i64, i32]
    lib.slide_gemm_workspace_bytes.restype = sz
    for name in ("slide_packed_sizes", "slide_prune_quant", "slide_decompose", "slide_decompose_canonical",
                 "act_lift_quant", "slide_sparse_gemm", "dense_gemm", "slide_sparse_gemm_ws", "dense_gemm_ws",
                 "slide_packed_sizes_fused", "slide_decompose_fused", "slide_sparse_gemm_fused"):
        getattr(lib, name).restype = i32
    lib.ss_status_string.argtypes = [i32]
    lib.ss_status_string.restype = ctypes.c_char_p
    lib.slide_format_version.restype = i32
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load().ss_status_string(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != 0:
        raise SlideSparseError(code, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _in_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SS_IN_F32
    if t.dtype == torch.bfloat16:
        return SS_IN_BF16
    raise TypeError(f"activations/weights must be float32 or bfloat16, got {t.dtype}")


def _storage_dtype(dtype: str) -> torch.dtype:
    return {"i8": torch.int8, "fp8": torch.uint8, "bf16": torch.bfloat16, "fp16": torch.float16}[dtype]


def slide_lifted_k(K: int, N: int) -> int:
    return int(load().slide_lifted_k(K, N))


def slide_lifted_ld(K: int, N: int, dtype: str) -> int:
    return int(load().slide_lifted_ld(K, N, DTYPE_CODE[dtype]))


def slide_packed_sizes(O: int, K: int, N: int, dtype: str):
    v, m = ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().slide_packed_sizes(O, K, N, DTYPE_CODE[dtype], ctypes.byref(v), ctypes.byref(m)), "slide_packed_sizes")
    return int(v.value), int(m.value)


def slide_prune_quant(W: torch.Tensor, N: int, dtype: str):
    """W[O,K] fp32/bf16 on the GPU -> (Wq[O,K], s_w[O] or None)."""
    O, K = W.shape
    assert W.is_cuda and W.is_contiguous()
    Wq = torch.empty((O, K), dtype=_storage_dtype(dtype), device=W.device)
    s_w = None if dtype in ("bf16", "fp16") else torch.empty((O,), dtype=torch.float32, device=W.device)
    _check(load().slide_prune_quant(_ptr(W), _in_code(W), O, K, N, DTYPE_CODE[dtype], _ptr(Wq), _ptr(s_w), _stream()),
           "slide_prune_quant")
    return Wq, s_w


def slide_decompose(Wq: torch.Tensor, N: int, dtype: str, count_violations: bool = False):
    """Wq[O,K] -> (w_vals, w_meta[, violations]) in the packed layout."""
    O, K = Wq.shape
    assert Wq.is_cuda and Wq.is_contiguous()
    vb, mb = slide_packed_sizes(O, K, N, dtype)
    w_vals = torch.empty((vb,), dtype=torch.uint8, device=Wq.device)
    w_meta = torch.empty((mb,), dtype=torch.uint8, device=Wq.device)
    viol = torch.zeros((1,), dtype=torch.int32, device=Wq.device) if count_violations else None
    _check(load().slide_decompose(_ptr(Wq), O, K, N, DTYPE_CODE[dtype], _ptr(w_vals), _ptr(w_meta), _ptr(viol), _stream()),
           "slide_decompose")
    return (w_vals, w_meta, viol) if count_violations else (w_vals, w_meta)


def slide_decompose_canonical(Wq: torch.Tensor, N: int, dtype: str):
    """Wq[O,K] -> (vals[O,K'/2], idx[O,K'/4] uint8, violations[1] int32)."""
    O, K = Wq.shape
    assert Wq.is_cuda and Wq.is_contiguous()
    Kp = slide_lifted_k(K, N)
    if Kp < 0:
        raise SlideSparseError(3 if 2 <= N <= 8 else 2, "slide_decompose_canonical")
    vals = torch.empty((O, Kp // 2), dtype=Wq.dtype, device=Wq.device)
    idx = torch.empty((O, Kp // 4), dtype=torch.uint8, device=Wq.device)
    viol = torch.zeros((1,), dtype=torch.int32, device=Wq.device)
    _check(load().slide_decompose_canonical(_ptr(Wq), O, K, N, DTYPE_CODE[dtype], _ptr(vals), _ptr(idx), _ptr(viol), _stream()),
           "slide_decompose_canonical")
    return vals, idx, viol


def act_lift_quant(X: torch.Tensor, N: int, dtype: str, out=None, s_x=None):
    """X[M,K] fp32/bf16 (row stride allowed) -> (X_lifted[M,Kld], s_x[M] or None)."""
    M, K = X.shape
    assert X.is_cuda and X.stride(1) == 1
    Kp = slide_lifted_ld(K, N, dtype)
    if Kp < 0:
        raise SlideSparseError(3 if 2 <= N <= 8 else 2, "act_lift_quant")
    if out is None:
        out = torch.empty((M, Kp), dtype=_storage_dtype(dtype), device=X.device)
    if s_x is None and dtype not in ("bf16", "fp16"):
        s_x = torch.empty((M,), dtype=torch.float32, device=X.device)
    ldx = X.stride(0) if M > 1 else K
    _check(load().act_lift_quant(_ptr(X), _in_code(X), M, K, ldx, N, DTYPE_CODE[dtype], _ptr(out), _ptr(s_x), _stream()),
           "act_lift_quant")
    return out, s_x


def slide_gemm_workspace_bytes(M: int, O: int, K: int, dtype: str) -> int:
    return int(load().slide_gemm_workspace_bytes(M, O, K, DTYPE_CODE[dtype]))


def slide_sparse_gemm(X_lifted, s_x, w_vals, w_meta, s_w, O: int, dtype: str, out=None, workspace=None):
    """Y[M,O] bf16 = epilogue(X_lifted[M,Kld] . W'^T); workspace: optional uint8 device tensor (slide_sparse_gemm_ws)."""
    M, Kp = X_lifted.shape
    assert X_lifted.is_contiguous()
    if out is None:
        out = torch.empty((M, O), dtype=torch.bfloat16, device=X_lifted.device)
    if workspace is None:
        _check(load().slide_sparse_gemm(_ptr(X_lifted), _ptr(s_x), _ptr(w_vals), _ptr(w_meta), _ptr(s_w), M, O, Kp,
                                        DTYPE_CODE[dtype], _ptr(out), out.stride(0), _stream()), "slide_sparse_gemm")
    else:
        _check(load().slide_sparse_gemm_ws(_ptr(X_lifted), _ptr(s_x), _ptr(w_vals), _ptr(w_meta), _ptr(s_w), M, O, Kp,
                                           DTYPE_CODE[dtype], _ptr(out), out.stride(0), _ptr(workspace),
                                           workspace.numel() * workspace.element_size(), _stream()), "slide_sparse_gemm_ws")
    return out


def dense_gemm(Xq, s_x, Wq, s_w, dtype: str, out=None, workspace=None):
    """Y[M,O] bf16 = epilogue(Xq[M,K] . Wq[O,K]^T); workspace: optional uint8 device tensor (dense_gemm_ws)."""
    M, K = Xq.shape
    O = Wq.shape[0]
    assert Xq.is_contiguous() and Wq.is_contiguous() and Wq.shape[1] == K
    if out is None:
        out = torch.empty((M, O), dtype=torch.bfloat16, device=Xq.device)
    if workspace is None:
        _check(load().dense_gemm(_ptr(Xq), _ptr(s_x), _ptr(Wq), _ptr(s_w), M, O, K, DTYPE_CODE[dtype], _ptr(out),
                                 out.stride(0), _stream()), "dense_gemm")
    else:
        _check(load().dense_gemm_ws(_ptr(Xq), _ptr(s_x), _ptr(Wq), _ptr(s_w), M, O, K, DTYPE_CODE[dtype], _ptr(out),
                                    out.stride(0), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
               "dense_gemm_ws")
    return out


def slide_packed_sizes_fused(O: int, K: int, N: int, dtype: str):
    v, m = ctypes.c_size_t(), ctypes.c_size_t()
    _check(load().slide_packed_sizes_fused(O, K, N, DTYPE_CODE[dtype], ctypes.byref(v), ctypes.byref(m)), "slide_packed_sizes_fused")
    return int(v.value), int(m.value)


def slide_decompose_fused(Wq: torch.Tensor, N: int, dtype: str, count_violations: bool = False):
    """Wq[O,K] -> (w_vals, w_meta[, violations]) in the window order of slide_sparse_gemm_fused."""
    O, K = Wq.shape
    assert Wq.is_cuda and Wq.is_contiguous()
    vb, mb = slide_packed_sizes_fused(O, K, N, dtype)
    w_vals = torch.empty((vb,), dtype=torch.uint8, device=Wq.device)
    w_meta = torch.empty((mb,), dtype=torch.uint8, device=Wq.device)
    viol = torch.zeros((1,), dtype=torch.int32, device=Wq.device) if count_violations else None
    _check(load().slide_decompose_fused(_ptr(Wq), O, K, N, DTYPE_CODE[dtype], _ptr(w_vals), _ptr(w_meta), _ptr(viol), _stream()),
           "slide_decompose_fused")
    return (w_vals, w_meta, viol) if count_violations else (w_vals, w_meta)


def slide_sparse_gemm_fused(Xq, s_x, w_vals, w_meta, s_w, O: int, K: int, N: int, dtype: str, out=None, workspace=None):
    """Y[M,O] bf16 = epilogue(Psi(Xq[M, :K]) . W'^T) from unlifted quantised activations (row stride = Xq.stride(0)).
    workspace: optional uint8 device tensor (slide_gemm_workspace_bytes(M, O, K, dtype) bytes) that lets the kernels for
    small and medium M split the k range."""
    M = Xq.shape[0]
    assert Xq.is_cuda and Xq.stride(1) == 1 and Xq.shape[1] >= K
    if out is None:
        out = torch.empty((M, O), dtype=torch.bfloat16, device=Xq.device)
    ldx = Xq.stride(0) if M > 1 else Xq.shape[1]
    if workspace is None:
        _check(load().slide_sparse_gemm_fused(_ptr(Xq), _ptr(s_x), _ptr(w_vals), _ptr(w_meta), _ptr(s_w), M, O, K, ldx, N,
                                              DTYPE_CODE[dtype], _ptr(out), out.stride(0), _stream()), "slide_sparse_gemm_fused")
    else:
        _check(load().slide_sparse_gemm_fused_ws(_ptr(Xq), _ptr(s_x), _ptr(w_vals), _ptr(w_meta), _ptr(s_w), M, O, K, ldx, N,
                                                 DTYPE_CODE[dtype], _ptr(out), out.stride(0), _ptr(workspace), workspace.numel(),
                                                 _stream()), "slide_sparse_gemm_fused_ws")
    return out


def slide_static_scratch_bytes() -> int:
    return int(load().slide_static_scratch_bytes())


def slide_sparse_gemm_static(X_lifted, s_x, w_vals, w_meta, s_w, O: int, dtype: str, out):
    """slide_sparse_gemm with the split-k scratch in the library's static device array; `out` is required: this call
    path allocates nothing."""
    M, Kp = X_lifted.shape
    assert X_lifted.is_contiguous() and out is not None
    _check(load().slide_sparse_gemm_static(_ptr(X_lifted), _ptr(s_x), _ptr(w_vals), _ptr(w_meta), _ptr(s_w), M, O, Kp,
                                           DTYPE_CODE[dtype], _ptr(out), out.stride(0), _stream()), "slide_sparse_gemm_static")
    return out
