"""ctypes binding of libiconv_mi355.so: argument marshalling only.

Function names and argument order follow include/iconv.h.  Tensors are torch CUDA tensors used
purely as device buffers (their data_ptr() is passed through); every step of the convolution
runs inside the library's HIP kernels.  There is no CPU fallback: if the library is missing
the import fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ICONV_LIB") or os.path.join(_PKG, "libiconv_mi355.so")

F32_F32, BF16_F32, F16_F32, BF16_BF16, F16_F16 = 0, 1, 2, 3, 4
ALGO_IMPLICIT, ALGO_EXPLICIT = 0, 1
DTYPE_CODES = {"f32": F32_F32, "bf16": BF16_F32, "f16": F16_F32, "bf16_bf16": BF16_BF16, "f16_f16": F16_F16}
_IN_TORCH = {F32_F32: torch.float32, BF16_F32: torch.bfloat16, F16_F32: torch.float16,
             BF16_BF16: torch.bfloat16, F16_F16: torch.float16}
_OUT_TORCH = {F32_F32: torch.float32, BF16_F32: torch.float32, F16_F32: torch.float32,
              BF16_BF16: torch.bfloat16, F16_F16: torch.float16}

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2110_03901_amd.build` "
                      "(there is no fallback path)")
_lib = ctypes.CDLL(LIB_PATH)

_i, _p, _sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
_lib.iconv_out_shape.restype = _i
_lib.iconv_out_shape.argtypes = [_i] * 7 + [ctypes.POINTER(_i)] * 2
_lib.iconv_fwd.restype = _i
_lib.iconv_fwd.argtypes = [_p, _p, _p] + [_i] * 11 + [_p]
_lib.iconv_workspace_bytes.restype = _sz
_lib.iconv_workspace_bytes.argtypes = [_i] * 12
_lib.iconv_fwd_explicit.restype = _i
_lib.iconv_fwd_explicit.argtypes = [_p, _p, _p, _p, _sz] + [_i] * 11 + [_p]
_lib.iconv_fwd_explicit_noalloc.restype = _i
_lib.iconv_fwd_explicit_noalloc.argtypes = [_p, _p, _p] + [_i] * 11 + [_p]
_lib.iconv_fwd_channel_last.restype = _i
_lib.iconv_fwd_channel_last.argtypes = [_p, _p, _p] + [_i] * 11 + [_p]
_lib.iconv_im2col.restype = _i
_lib.iconv_im2col.argtypes = [_p, _p, _sz] + [_i] * 10 + [_p]
_lib.iconv_probe_copy.restype = _i
_lib.iconv_probe_copy.argtypes = [_p, _p, _sz, _p]
_lib.iconv_probe_copy_wt.restype = _i
_lib.iconv_probe_copy_wt.argtypes = [_p, _p, _sz, _p]
_lib.iconv_probe_mfma.restype = _i
_lib.iconv_probe_mfma.argtypes = [_p, _sz, _i, _i, _p]
_lib.iconv_probe_lds.restype = _i
_lib.iconv_probe_lds.argtypes = [_p, _sz, _i, _i, _p]
_lib.iconv_lds_swizzle.restype = _i
_lib.iconv_lds_swizzle.argtypes = [_i, _i, _i]
_lib.iconv_lds_stage_offset.restype = _i
_lib.iconv_lds_stage_offset.argtypes = [_i, _i]
_lib.iconv_fwd_ex.restype = _i
_lib.iconv_fwd_ex.argtypes = [_p, _p, _p] + [_i] * 13 + [_p]
_lib.iconv_num_variants.restype = _i
_lib.iconv_variant_accepts.restype = _i
_lib.iconv_variant_accepts.argtypes = [_i] * 12
_lib.iconv_variant_name.restype = ctypes.c_char_p
_lib.iconv_variant_name.argtypes = [_i]
_lib.iconv_kernel_for.restype = ctypes.c_char_p
_lib.iconv_kernel_for.argtypes = [_i] * 11
_lib.iconv_status_string.restype = ctypes.c_char_p
_lib.iconv_status_string.argtypes = [_i]

# symbols declared in include/iconv.h and include/iconv_bench.h
NOALLOC_WORKSPACE_BYTES = 16 << 20
EXPORTS = ["iconv_out_shape", "iconv_fwd", "iconv_fwd_channel_last", "iconv_workspace_bytes", "iconv_fwd_explicit",
           "iconv_fwd_explicit_noalloc", "iconv_im2col",
           "iconv_kernel_for", "iconv_status_string"]
EXPORTS_BENCH = ["iconv_fwd_ex", "iconv_num_variants", "iconv_variant_name", "iconv_variant_accepts", "iconv_probe_copy", "iconv_probe_copy_wt", "iconv_probe_mfma", "iconv_probe_lds", "iconv_lds_swizzle", "iconv_lds_stage_offset"]


class IconvError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"iconv status {status}: {iconv_status_string(status)}")


def _ptr(t) -> int:
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def iconv_status_string(status: int) -> str:
    return _lib.iconv_status_string(status).decode()


def iconv_out_shape(H, W, R, S, stride, pad, dilation):
    P, Q = _i(0), _i(0)
    rc = _lib.iconv_out_shape(H, W, R, S, stride, pad, dilation, ctypes.byref(P), ctypes.byref(Q))
    if rc != 0:
        raise IconvError(rc)
    return P.value, Q.value


def iconv_fwd_raw(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream=None) -> int:
    """Direct pass-through of the C call; returns the status code (no exception)."""
    return _lib.iconv_fwd(_ptr(x), _ptr(w), _ptr(y), N, H, W, C, K, R, S, stride, pad, dilation, dtype,
                          _stream(stream))


def iconv_fwd(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream=None) -> None:
    rc = iconv_fwd_raw(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream)
    if rc != 0:
        raise IconvError(rc)


def iconv_fwd_ex_raw(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, variant=-1, max_workgroups=0, stream=None) -> int:
    return _lib.iconv_fwd_ex(_ptr(x), _ptr(w), _ptr(y), N, H, W, C, K, R, S, stride, pad, dilation, dtype,
                             variant, max_workgroups, _stream(stream))


def iconv_fwd_ex(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, variant=-1, max_workgroups=0, stream=None) -> None:
    """iconv_fwd with a forced kernel-table entry and/or a cap on the workgroups, for this call only."""
    rc = iconv_fwd_ex_raw(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, variant, max_workgroups, stream)
    if rc != 0:
        raise IconvError(rc)


def iconv_fwd_channel_last(x_nchw, w_kcrs, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream=None) -> None:
    rc = _lib.iconv_fwd_channel_last(_ptr(x_nchw), _ptr(w_kcrs), _ptr(y), N, H, W, C, K, R, S, stride, pad, dilation, dtype,
                                     _stream(stream))
    if rc != 0:
        raise IconvError(rc)


def iconv_workspace_bytes(algo, N, H, W, C, K, R, S, stride, pad, dilation, dtype) -> int:
    return _lib.iconv_workspace_bytes(algo, N, H, W, C, K, R, S, stride, pad, dilation, dtype)


def iconv_fwd_explicit_raw(x, w, y, workspace, workspace_bytes, N, H, W, C, K, R, S, stride, pad, dilation, dtype,
                           stream=None) -> int:
    return _lib.iconv_fwd_explicit(_ptr(x), _ptr(w), _ptr(y), _ptr(workspace), workspace_bytes, N, H, W, C, K, R, S,
                                   stride, pad, dilation, dtype, _stream(stream))


def iconv_fwd_explicit(x, w, y, workspace, workspace_bytes, N, H, W, C, K, R, S, stride, pad, dilation, dtype,
                       stream=None) -> None:
    rc = iconv_fwd_explicit_raw(x, w, y, workspace, workspace_bytes, N, H, W, C, K, R, S, stride, pad, dilation,
                                dtype, stream)
    if rc != 0:
        raise IconvError(rc)


def iconv_fwd_explicit_noalloc_raw(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream=None) -> int:
    return _lib.iconv_fwd_explicit_noalloc(_ptr(x), _ptr(w), _ptr(y), N, H, W, C, K, R, S, stride, pad, dilation, dtype,
                                           _stream(stream))


def iconv_fwd_explicit_noalloc(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream=None) -> None:
    rc = iconv_fwd_explicit_noalloc_raw(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream)
    if rc != 0:
        raise IconvError(rc)


def iconv_im2col(x, workspace, workspace_bytes, N, H, W, C, R, S, stride, pad, dilation, dtype, stream=None) -> None:
    rc = _lib.iconv_im2col(_ptr(x), _ptr(workspace), workspace_bytes, N, H, W, C, R, S, stride, pad, dilation, dtype,
                           _stream(stream))
    if rc != 0:
        raise IconvError(rc)


def iconv_probe_copy(dst, src, nbytes, stream=None) -> None:
    rc = _lib.iconv_probe_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream))
    if rc != 0:
        raise IconvError(rc)


def iconv_probe_copy_wt(dst, src, nbytes, stream=None) -> None:
    rc = _lib.iconv_probe_copy_wt(_ptr(dst), _ptr(src), nbytes, _stream(stream))
    if rc != 0:
        raise IconvError(rc)


MFMA_PROBE_GROUPS = 1024


def iconv_probe_mfma(out, out_bytes, iters, random_operands=False, stream=None) -> None:
    rc = _lib.iconv_probe_mfma(_ptr(out), out_bytes, iters, int(bool(random_operands)), _stream(stream))
    if rc != 0:
        raise IconvError(rc)


LDS_PROBE_PATTERNS = ("read_linear", "write_linear", "read_operand_rows64_unswizzled", "read_operand_rows64",
                      "read_operand_rows128", "write_staging_deposit_16_pixels", "write_staging_deposit_32_pixels",
                      "write_deposit_read_friendly_layout")


def iconv_probe_lds(out, out_bytes, iters, pattern, stream=None) -> None:
    rc = _lib.iconv_probe_lds(_ptr(out), out_bytes, iters, pattern, _stream(stream))
    if rc != 0:
        raise IconvError(rc)


def iconv_lds_swizzle(chunks_per_row, row, chunk) -> int:
    return _lib.iconv_lds_swizzle(chunks_per_row, row, chunk)


def iconv_lds_stage_offset(pixel, piece) -> int:
    return _lib.iconv_lds_stage_offset(pixel, piece)


def iconv_num_variants() -> int:
    return _lib.iconv_num_variants()


def iconv_variant_accepts(variant, N, H, W, C, K, R, S, stride, pad, dilation, dtype) -> bool:
    return bool(_lib.iconv_variant_accepts(variant, N, H, W, C, K, R, S, stride, pad, dilation, dtype))


def iconv_variant_name(variant: int) -> str:
    return _lib.iconv_variant_name(variant).decode()


def iconv_kernel_for(N, H, W, C, K, R, S, stride, pad, dilation, dtype):
    """Name of the kernel iconv_fwd runs for this layer without an override, or None for invalid arguments."""
    r = _lib.iconv_kernel_for(N, H, W, C, K, R, S, stride, pad, dilation, dtype)
    return r.decode() if r is not None else None


# ---- device-buffer helpers (plumbing: upload, allocate, download) ---------------------------

def to_device(a, dtype: int, device="cuda:0"):
    """numpy fp32 array (values representable in the input type) -> device tensor of that type."""
    return torch.from_numpy(a).to(device=device, dtype=_IN_TORCH[dtype]).contiguous()


def empty_output(N, P, Q, K, dtype: int, device="cuda:0"):
    return torch.empty((N, P, Q, K), dtype=_OUT_TORCH[dtype], device=device)


def conv2d_nhwc(x, w, stride=1, pad=0, dilation=1, dtype=BF16_F32, explicit=False, stream=None):
    """x: device tensor [N,H,W,C], w: device tensor [K,R,S,C] (element type of `dtype`).
    Allocates y [N,P,Q,K] and runs iconv_fwd (or the explicit variant)."""
    N, H, W, C = x.shape
    K, R, S, C2 = w.shape
    if C2 != C:
        raise ValueError("channel mismatch")
    if x.dtype != _IN_TORCH[dtype] or w.dtype != _IN_TORCH[dtype] or not (x.is_contiguous() and w.is_contiguous()):
        raise ValueError("x and w must be contiguous tensors of the input element type")
    P, Q = iconv_out_shape(H, W, R, S, stride, pad, dilation)
    y = empty_output(N, P, Q, K, dtype, x.device)
    if explicit:
        nbytes = iconv_workspace_bytes(ALGO_EXPLICIT, N, H, W, C, K, R, S, stride, pad, dilation, dtype)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=x.device)
        if stream is not None and not isinstance(stream, int):
            ws.record_stream(stream)        # the block must not be handed out again before the two kernels have run
        iconv_fwd_explicit(x, w, y, ws, nbytes, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream)
        if isinstance(stream, int) and stream != torch.cuda.current_stream().cuda_stream:
            torch.cuda.synchronize()        # a raw stream handle cannot be recorded: finish before ws is dropped
    else:
        iconv_fwd(x, w, y, N, H, W, C, K, R, S, stride, pad, dilation, dtype, stream)
    return y
