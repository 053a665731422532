"""ctypes binding of librotq.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI (include/rotq.h); PyTorch
is used for device memory and streams.  There is no CPU fallback: if the library has not
been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librotq.so")

RQ_OK, RQ_ERR_ARG, RQ_ERR_NO_ORDER, RQ_ERR_HIP, RQ_ERR_NOMEM, RQ_ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5
RQ_NOALLOC_SCRATCH_BYTES = 4 << 20
RQ_BF16, RQ_F32, RQ_F16 = 0, 1, 2
RQ_MAX_CLIPS = 64

_lib = None


class RotqError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().rq_strerror(code).decode()} ({code})")


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2504_13989_amd.build` "
            "(hipcc, gfx950); there is no fallback path")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, f32p = C.c_void_p, C.c_int, C.c_int64, C.POINTER(C.c_float)
    ip = C.POINTER(C.c_int)
    L.rq_hadamard_build.argtypes = [i32, C.POINTER(vp)]
    L.rq_hadamard_free.argtypes = [vp]
    L.rq_hadamard_free.restype = None
    L.rq_hadamard_info.argtypes = [vp, ip, ip, ip, ip, ip]
    L.rq_hadamard_dense.argtypes = [vp, vp]
    L.rq_next_order.argtypes = [i32, ip]
    L.rq_rotate_quantize.argtypes = [vp, vp, i32, i64, i32, i64, i32, C.c_float, vp, vp, vp]
    L.rq_rotate_quantize_asym.argtypes = [vp, vp, i32, i64, i32, i64, i32, C.c_float, vp, vp, vp, vp]
    L.rq_quantize.argtypes = [vp, i32, i64, i32, i64, i32, C.c_float, vp, vp, vp]
    L.rq_quantize_asym.argtypes = [vp, i32, i64, i32, i64, i32, C.c_float, vp, vp, vp, vp]
    L.rq_rotate.argtypes = [vp, vp, i32, i64, i32, i64, i32, vp, i32, i32, i64, vp]
    L.rq_stream_reference.argtypes = [vp, i64, i32, i64, i32, vp, vp, vp]
    L.rq_dequantize_rotate.argtypes = [vp, vp, vp, vp, i64, i32, i32, vp, i32, i32, i64, vp]
    L.rq_expand_limit.argtypes = [i32, i32, i32, C.POINTER(C.c_int64)]
    L.rq_quant_error_workspace.argtypes = [i64, i32]
    L.rq_quant_error_workspace.restype = C.c_size_t
    L.rq_quant_error.argtypes = [vp, vp, i32, i64, i32, i64, i32, f32p, i32, vp, vp, C.c_size_t, vp]
    L.rq_quant_error_asym.argtypes = L.rq_quant_error.argtypes
    L.rq_quant_error_noalloc.argtypes = [vp, vp, i32, i64, i32, i64, i32, f32p, i32, vp, vp]
    L.rq_dequantize.argtypes = [vp, vp, vp, i64, i32, vp, vp]
    L.rq_dequantize_asym.argtypes = [vp, vp, vp, vp, i64, i32, vp, vp]
    L.rq_gbs_workspace.argtypes = [i64]
    L.rq_gbs_workspace.restype = C.c_size_t
    L.rq_gbs_search.argtypes = [vp, vp, i32, i64, i32, i64, i32, C.c_float, i32, vp, C.c_size_t, vp,
                                f32p, f32p, f32p, f32p, ip]
    L.rq_gbs_search_asym.argtypes = L.rq_gbs_search.argtypes
    L.rq_hadamard_set_variant.argtypes = [vp, i32]
    L.rq_hadamard_last_kernel.argtypes = [vp]
    L.rq_hadamard_last_kernel.restype = C.c_char_p
    L.rq_strerror.argtypes = [i32]
    L.rq_strerror.restype = C.c_char_p
    for name in ("rq_hadamard_build", "rq_hadamard_info", "rq_hadamard_dense", "rq_next_order",
                 "rq_rotate_quantize", "rq_quant_error", "rq_hadamard_set_variant", "rq_gbs_search"):
        getattr(L, name).restype = i32
    _lib = L
    return L


def _check(code: int, where: str) -> None:
    if code != RQ_OK:
        raise RotqError(code, where)


class Hadamard:
    """Handle returned by rq_hadamard_build (owns the library-side object)."""

    def __init__(self, n: int):
        h = C.c_void_p()
        _check(lib().rq_hadamard_build(int(n), C.byref(h)), f"rq_hadamard_build({n})")
        self._h = h
        v = [C.c_int() for _ in range(5)]
        _check(lib().rq_hadamard_info(h, *[C.byref(x) for x in v]), "rq_hadamard_info")
        self.n, self.p, self.kind, self.q, self.log2m = (x.value for x in v)

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().rq_hadamard_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def dense(self):
        import numpy as np
        out = np.empty((self.n, self.n), dtype=np.int8)
        _check(lib().rq_hadamard_dense(self._h, out.ctypes.data_as(C.c_void_p)), "rq_hadamard_dense")
        return out

    def set_variant(self, variant: int) -> None:
        _check(lib().rq_hadamard_set_variant(self._h, int(variant)), "rq_hadamard_set_variant")

    @property
    def last_kernel(self) -> str:
        return lib().rq_hadamard_last_kernel(self._h).decode()


def hadamard_build(n: int) -> Hadamard:
    return Hadamard(n)


def next_order(d: int) -> int:
    out = C.c_int()
    _check(lib().rq_next_order(int(d), C.byref(out)), f"rq_next_order({d})")
    return out.value


def _dtype_code(x) -> int:
    import torch
    if x.dtype == torch.bfloat16:
        return RQ_BF16
    if x.dtype == torch.float32:
        return RQ_F32
    if x.dtype == torch.float16:
        return RQ_F16
    raise TypeError(f"unsupported input dtype {x.dtype}")


def _rows_view(x):
    """(rows, d, ld) of a tensor whose last dimension is contiguous and whose leading dimensions
    collapse to one row index with a single stride."""
    if x.stride(-1) != 1:
        raise ValueError("last dimension must be contiguous")
    d = x.shape[-1]
    x2 = x.reshape(-1, d) if x.is_contiguous() else x
    if x2.dim() != 2:
        raise ValueError("non-contiguous input must be 2-D")
    return x2, x2.shape[0], d, (x2.stride(0) if x2.shape[0] > 1 else max(d, x2.stride(0)))


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def rotate_quantize(h: Hadamard, x, bits: int, clip: float, codes=None, scales=None, stream=None):
    """rq_rotate_quantize on a CUDA tensor x [..., d]; returns (codes uint8 [rows, n*bits/8],
    scales float32 [rows]).  Output tensors are allocated with torch unless given."""
    import torch
    if not x.is_cuda:
        raise ValueError("x must be a device tensor")
    x2, rows, d, ld = _rows_view(x)
    nbytes = h.n * bits // 8
    if codes is None:
        codes = torch.empty((rows, nbytes), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows,), dtype=torch.float32, device=x.device)
    rc = lib().rq_rotate_quantize(h._h, C.c_void_p(x2.data_ptr()), _dtype_code(x2), rows, d, ld,
                                  int(bits), C.c_float(clip), C.c_void_p(codes.data_ptr()),
                                  C.c_void_p(scales.data_ptr()), _stream_ptr(stream))
    _check(rc, "rq_rotate_quantize")
    return codes, scales


GROUP = 128


def rotate_quantize_asym(h: Hadamard, x, bits: int, clip: float, codes=None, scales=None, mins=None,
                         stream=None):
    """rq_rotate_quantize_asym on a CUDA tensor x [..., d]; returns (codes uint8 [rows, n*bits/8],
    scales float32 [rows, n/128], mins float32 [rows, n/128])."""
    import torch
    if not x.is_cuda:
        raise ValueError("x must be a device tensor")
    x2, rows, d, ld = _rows_view(x)
    groups = max(h.n // GROUP, 1)
    if codes is None:
        codes = torch.empty((rows, h.n * bits // 8), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows, groups), dtype=torch.float32, device=x.device)
    if mins is None:
        mins = torch.empty((rows, groups), dtype=torch.float32, device=x.device)
    rc = lib().rq_rotate_quantize_asym(h._h, C.c_void_p(x2.data_ptr()), _dtype_code(x2), rows, d, ld,
                                       int(bits), C.c_float(clip), C.c_void_p(codes.data_ptr()),
                                       C.c_void_p(scales.data_ptr()), C.c_void_p(mins.data_ptr()),
                                       _stream_ptr(stream))
    _check(rc, "rq_rotate_quantize_asym")
    return codes, scales, mins


def quantize(x, bits: int, clip: float, codes=None, scales=None, stream=None):
    """rq_quantize (no rotation) on a CUDA tensor x [..., d]; returns (codes uint8 [rows, d*bits/8],
    scales float32 [rows])."""
    import torch
    if not x.is_cuda:
        raise ValueError("x must be a device tensor")
    x2, rows, d, ld = _rows_view(x)
    if codes is None:
        codes = torch.empty((rows, d * bits // 8), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows,), dtype=torch.float32, device=x.device)
    rc = lib().rq_quantize(C.c_void_p(x2.data_ptr()), _dtype_code(x2), rows, d, ld, int(bits),
                           C.c_float(clip), C.c_void_p(codes.data_ptr()),
                           C.c_void_p(scales.data_ptr()), _stream_ptr(stream))
    _check(rc, "rq_quantize")
    return codes, scales


def quantize_asym(x, bits: int, clip: float, codes=None, scales=None, mins=None, stream=None):
    """rq_quantize_asym (no rotation, asymmetric groups of 128) on a CUDA tensor x [..., d]; returns
    (codes uint8 [rows, d*bits/8], scales float32 [rows, d/128], mins float32 [rows, d/128])."""
    import torch
    if not x.is_cuda:
        raise ValueError("x must be a device tensor")
    x2, rows, d, ld = _rows_view(x)
    groups = max(d // GROUP, 1)
    if codes is None:
        codes = torch.empty((rows, d * bits // 8), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows, groups), dtype=torch.float32, device=x.device)
    if mins is None:
        mins = torch.empty((rows, groups), dtype=torch.float32, device=x.device)
    rc = lib().rq_quantize_asym(C.c_void_p(x2.data_ptr()), _dtype_code(x2), rows, d, ld, int(bits),
                                C.c_float(clip), C.c_void_p(codes.data_ptr()),
                                C.c_void_p(scales.data_ptr()), C.c_void_p(mins.data_ptr()),
                                _stream_ptr(stream))
    _check(rc, "rq_quantize_asym")
    return codes, scales, mins


def stream_reference(x, bits: int, codes=None, scales=None, stream=None):
    """rq_stream_reference: the traffic of rotate_quantize on 16-bit rows [rows, n] without the
    arithmetic (measurement aid; the outputs are not a quantization)."""
    import torch
    if not x.is_cuda:
        raise ValueError("x must be a device tensor")
    x2, rows, n, ld = _rows_view(x)
    if codes is None:
        codes = torch.empty((rows, n * bits // 8), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows,), dtype=torch.float32, device=x.device)
    rc = lib().rq_stream_reference(C.c_void_p(x2.data_ptr()), rows, n, ld, int(bits),
                                   C.c_void_p(codes.data_ptr()), C.c_void_p(scales.data_ptr()),
                                   _stream_ptr(stream))
    _check(rc, "rq_stream_reference")
    return codes, scales


def _out_code(torch, dtype):
    if dtype == torch.float32:
        return RQ_F32
    if dtype == torch.bfloat16:
        return RQ_BF16
    if dtype == torch.float16:
        return RQ_F16
    raise ValueError("output dtype must be float32, bfloat16 or float16")


def rotate(h: Hadamard, x, transpose: bool = False, d_out: Optional[int] = None, out_dtype=None,
           out=None, stream=None):
    """rq_rotate on a CUDA tensor x [..., d]: (H_n pad(x) / sqrt(n))[:, :d_out] per row (H_n^T with
    transpose), as float32 (default) or bfloat16.  Applied to the rows of a weight stored
    [out_features, in_features] it is the offline input-side fusion of section 4.2."""
    import torch
    if not x.is_cuda:
        raise ValueError("x must be a device tensor")
    x2, rows, d, ld = _rows_view(x)
    d_out = h.n if d_out is None else int(d_out)
    if out is None:
        out = torch.empty((rows, d_out), dtype=out_dtype or torch.float32, device=x.device)
    rc = lib().rq_rotate(h._h, C.c_void_p(x2.data_ptr()), _dtype_code(x2), rows, d, ld,
                         1 if transpose else 0, C.c_void_p(out.data_ptr()), _out_code(torch, out.dtype),
                         d_out, out.stride(0) if rows > 1 else max(d_out, out.stride(0)),
                         _stream_ptr(stream))
    _check(rc, "rq_rotate")
    return out


def dequantize_rotate(h: Hadamard, codes, scales, bits: int, mins=None, transpose: bool = True,
                      d_out: Optional[int] = None, out_dtype=None, out=None, stream=None):
    """rq_dequantize_rotate: packed codes (+ scales, + mins for the asymmetric variant) back to
    rows in the original basis, (H_n^T y^ / sqrt(n))[:, :d_out]."""
    import torch
    rows = codes.shape[0]
    d_out = h.n if d_out is None else int(d_out)
    if out is None:
        out = torch.empty((rows, d_out), dtype=out_dtype or torch.float32, device=codes.device)
    rc = lib().rq_dequantize_rotate(h._h, C.c_void_p(codes.data_ptr()), C.c_void_p(scales.data_ptr()),
                                    C.c_void_p(mins.data_ptr()) if mins is not None else None, rows,
                                    int(bits), 1 if transpose else 0, C.c_void_p(out.data_ptr()),
                                    _out_code(torch, out.dtype), d_out,
                                    out.stride(0) if rows > 1 else max(d_out, out.stride(0)),
                                    _stream_ptr(stream))
    _check(rc, "rq_dequantize_rotate")
    return out


def dequantize(h: Hadamard, codes, scales, bits: int, mins=None, out=None, stream=None):
    """rq_dequantize (rq_dequantize_asym when mins is given): packed codes and scales to float32
    values [rows, n] in the rotated domain."""
    import torch
    rows = codes.shape[0]
    if out is None:
        out = torch.empty((rows, h.n), dtype=torch.float32, device=codes.device)
    if mins is None:
        rc = lib().rq_dequantize(h._h, C.c_void_p(codes.data_ptr()), C.c_void_p(scales.data_ptr()), rows,
                                 int(bits), C.c_void_p(out.data_ptr()), _stream_ptr(stream))
        _check(rc, "rq_dequantize")
    else:
        rc = lib().rq_dequantize_asym(h._h, C.c_void_p(codes.data_ptr()), C.c_void_p(scales.data_ptr()),
                                      C.c_void_p(mins.data_ptr()), rows, int(bits),
                                      C.c_void_p(out.data_ptr()), _stream_ptr(stream))
        _check(rc, "rq_dequantize_asym")
    return out


def expand_limit(n: int, bits: int, bits_reduced: int) -> int:
    """rq_expand_limit: floor(n (bits - bits_reduced) / bits_reduced) (Lemma "Expanding limit")."""
    out = C.c_int64(0)
    _check(lib().rq_expand_limit(int(n), int(bits), int(bits_reduced), C.byref(out)), "rq_expand_limit")
    return int(out.value)


def quant_error_workspace(rows: int, n_clips: int) -> int:
    return int(lib().rq_quant_error_workspace(int(rows), int(n_clips)))


def quant_error(h: Hadamard, x, bits: int, clips: Sequence[float], mse=None, workspace=None,
                stream=None, asym: bool = False):
    """rq_quant_error (rq_quant_error_asym with asym=True) on a CUDA tensor x [..., d]; returns mse
    float32 [len(clips)] (device)."""
    import torch
    if not x.is_cuda:
        raise ValueError("x must be a device tensor")
    x2, rows, d, ld = _rows_view(x)
    k = len(clips)
    arr = (C.c_float * k)(*[float(c) for c in clips])
    if mse is None:
        mse = torch.empty((k,), dtype=torch.float32, device=x.device)
    need = quant_error_workspace(rows, k)
    if workspace is None:
        workspace = torch.empty((max(need, 8) + 7) // 8, dtype=torch.float64, device=x.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    fn = lib().rq_quant_error_asym if asym else lib().rq_quant_error
    rc = fn(h._h, C.c_void_p(x2.data_ptr()), _dtype_code(x2), rows, d, ld, int(bits), arr, k,
            C.c_void_p(mse.data_ptr()), C.c_void_p(workspace.data_ptr()), ws_bytes, _stream_ptr(stream))
    _check(rc, "rq_quant_error_asym" if asym else "rq_quant_error")
    return mse


def quant_error_noalloc(h: Hadamard, x, bits: int, clips: Sequence[float], mse, stream=None):
    """rq_quant_error_noalloc on a CUDA tensor x [..., d]: rq_quant_error with the library's static
    scratch array in place of a workspace.  `mse` (float32 [len(clips)], device) is the caller's: the
    call itself allocates nothing."""
    x2, rows, d, ld = _rows_view(x)
    k = len(clips)
    arr = (C.c_float * k)(*[float(c) for c in clips])
    rc = lib().rq_quant_error_noalloc(h._h, C.c_void_p(x2.data_ptr()), _dtype_code(x2), rows, d, ld, int(bits),
                                      arr, k, C.c_void_p(mse.data_ptr()), _stream_ptr(stream))
    _check(rc, "rq_quant_error_noalloc")
    return mse


def gbs_search(h: Hadamard, x, bits: int, eps: float, max_evals: int = 64, workspace=None, stream=None,
               asym: bool = False):
    """rq_gbs_search (rq_gbs_search_asym with asym=True) on a CUDA tensor x [..., d]; returns
    (clip, mse, trace) with trace a list of (probe, objective) pairs in the algorithm's order.
    Synchronises the stream once per batch of probes."""
    import torch
    if not x.is_cuda:
        raise ValueError("x must be a device tensor")
    x2, rows, d, ld = _rows_view(x)
    need = int(lib().rq_gbs_workspace(rows))
    if workspace is None:
        workspace = torch.empty((need + 7) // 8, dtype=torch.float64, device=x.device)
    clip, mse, n = C.c_float(), C.c_float(), C.c_int()
    tc, tm = (C.c_float * max_evals)(), (C.c_float * max_evals)()
    fn = lib().rq_gbs_search_asym if asym else lib().rq_gbs_search
    rc = fn(h._h, C.c_void_p(x2.data_ptr()), _dtype_code(x2), rows, d, ld, int(bits),
            C.c_float(eps), int(max_evals), C.c_void_p(workspace.data_ptr()),
            workspace.numel() * workspace.element_size(), _stream_ptr(stream),
            C.byref(clip), C.byref(mse), tc, tm, C.byref(n))
    _check(rc, "rq_gbs_search_asym" if asym else "rq_gbs_search")
    return clip.value, mse.value, [(tc[i], tm[i]) for i in range(n.value)]
