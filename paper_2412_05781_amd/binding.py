"""ctypes binding of libwino.so — argument marshalling only.

Function names and argument order mirror ``include/wino.h``.  Tensors are torch
tensors on the GPU (torch is used for device memory and streams only); every
step of the path runs inside the library's HIP kernels.  There is no fallback:
if the library is missing, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libwino.so")

WINO_OK = 0
WINO_ERR_NULL, WINO_ERR_DIM, WINO_ERR_DTYPE, WINO_ERR_VARIANT = 1, 2, 3, 4
WINO_ERR_ALIGN, WINO_ERR_WORKSPACE, WINO_ERR_ALIAS, WINO_ERR_HIP, WINO_ERR_LAYOUT, WINO_ERR_SCRATCH = 5, 6, 7, 8, 9, 10
WINO_F32, WINO_F16, WINO_BF16 = 0, 1, 2
WINO_AUTO, WINO_DIRECT, WINO_F2, WINO_F4, WINO_FUSED_F2, WINO_FUSED_F4 = 0, 1, 2, 4, 12, 14
WINO_NCHW, WINO_NHWC = 0, 1

DTYPE_OF = {torch.float32: WINO_F32, torch.float16: WINO_F16, torch.bfloat16: WINO_BF16}
TORCH_OF = {WINO_F32: torch.float32, WINO_F16: torch.float16, WINO_BF16: torch.bfloat16}

EXPORTS = [
    "wino_version", "wino_status_string", "wino_resolve_variant", "wino_transformed_dims",
    "wino_filter_bytes", "wino_workspace_bytes", "wino_filter_transform", "wino_conv2d",
    "wino_conv2d_ex", "wino_input_transform", "wino_batched_gemm", "wino_output_transform",
    "wino_direct_conv2d", "wino_groupnorm_stats_bytes", "wino_groupnorm_stats", "wino_conv2d_fused",
    "wino_igemm_filter_bytes", "wino_igemm_filter_repack", "wino_igemm_workspace_bytes", "wino_igemm_conv2d",
    "wino_recommend_variant",
    "wino_fp8_filter_bytes", "wino_fp8_filter_quantize", "wino_fp8_workspace_bytes", "wino_fp8_conv2d",
    "wino_fused_gemm_output", "wino_batched_gemm_shape", "wino_static_scratch_bytes", "wino_conv2d_static",
    "wino_i8_filter_bytes", "wino_i8_filter_transform", "wino_i8_workspace_bytes", "wino_i8_conv2d",
    "wino_i8_input_transform", "wino_i8_batched_gemm", "wino_fused_f4_gemm_output",
]


class wino_filter(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("K", ctypes.c_int), ("C", ctypes.c_int),
                ("dtype", ctypes.c_int), ("variant", ctypes.c_int)]


class wino_fusion(ctypes.Structure):
    _fields_ = [("gn_stats", ctypes.c_void_p), ("gn_gamma", ctypes.c_void_p), ("gn_beta", ctypes.c_void_p),
                ("gn_groups", ctypes.c_int), ("addvec", ctypes.c_void_p), ("residual", ctypes.c_void_p),
                ("upsample", ctypes.c_int), ("product_fp16", ctypes.c_int)]


class WinoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Open libwino.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2412_05781_amd.build` "
                               "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        i, vp, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        ip = ctypes.POINTER(ctypes.c_int)
        fp = ctypes.POINTER(wino_filter)
        L.wino_version.restype = i; L.wino_version.argtypes = []
        L.wino_status_string.restype = ctypes.c_char_p; L.wino_status_string.argtypes = [i]
        L.wino_resolve_variant.restype = i; L.wino_resolve_variant.argtypes = [i] * 7
        L.wino_transformed_dims.restype = i; L.wino_transformed_dims.argtypes = [i] * 6 + [ip, ip, ip]
        L.wino_filter_bytes.restype = sz; L.wino_filter_bytes.argtypes = [i] * 4
        L.wino_workspace_bytes.restype = sz; L.wino_workspace_bytes.argtypes = [i] * 7
        L.wino_filter_transform.restype = i
        L.wino_filter_transform.argtypes = [vp, vp, i, i, i, i, fp, vp]
        L.wino_conv2d.restype = i
        L.wino_conv2d.argtypes = [vp, fp, vp, vp, i, i, i, i, i, vp]
        L.wino_conv2d_ex.restype = i
        L.wino_conv2d_ex.argtypes = [vp, fp, vp, vp, i, i, i, i, i, i, vp, sz, vp]
        L.wino_input_transform.restype = i
        L.wino_input_transform.argtypes = [vp, vp, i, i, i, i, i, i, i, vp]
        L.wino_batched_gemm.restype = i
        L.wino_batched_gemm.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        L.wino_static_scratch_bytes.restype = sz; L.wino_static_scratch_bytes.argtypes = []
        L.wino_conv2d_static.restype = i
        L.wino_conv2d_static.argtypes = [vp, fp, vp, vp, i, i, i, i, i, i, vp]
        L.wino_batched_gemm_shape.restype = i
        L.wino_batched_gemm_shape.argtypes = [vp, vp, vp, i, i, i, i, i, i, vp]
        L.wino_fused_gemm_output.restype = i
        L.wino_fused_gemm_output.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, i, vp]
        L.wino_fused_f4_gemm_output.restype = i
        L.wino_fused_f4_gemm_output.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, i, vp]
        L.wino_output_transform.restype = i
        L.wino_output_transform.argtypes = [vp, vp, vp, i, i, i, i, i, i, i, vp]
        L.wino_direct_conv2d.restype = i
        L.wino_direct_conv2d.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp]
        L.wino_groupnorm_stats_bytes.restype = sz; L.wino_groupnorm_stats_bytes.argtypes = [i, i]
        L.wino_groupnorm_stats.restype = i
        L.wino_groupnorm_stats.argtypes = [vp, vp, i, i, i, i, i, ctypes.c_float, i, i, vp]
        L.wino_conv2d_fused.restype = i
        L.wino_conv2d_fused.argtypes = [vp, fp, vp, vp, i, i, i, i, i, i, ctypes.POINTER(wino_fusion), vp, sz, vp]
        L.wino_fp8_filter_bytes.restype = sz; L.wino_fp8_filter_bytes.argtypes = [i] * 3
        L.wino_fp8_filter_quantize.restype = i
        L.wino_fp8_filter_quantize.argtypes = [vp, vp, i, i, i, i, ctypes.c_float, vp]
        L.wino_fp8_workspace_bytes.restype = sz; L.wino_fp8_workspace_bytes.argtypes = [i] * 7
        L.wino_fp8_conv2d.restype = i
        L.wino_fp8_conv2d.argtypes = [vp, vp, vp, vp] + [i] * 9 + [ctypes.c_float, ctypes.c_float, ctypes.POINTER(wino_fusion), vp, sz, vp]
        L.wino_recommend_variant.restype = i; L.wino_recommend_variant.argtypes = [i] * 6
        L.wino_i8_filter_bytes.restype = sz; L.wino_i8_filter_bytes.argtypes = [i, i]
        L.wino_i8_filter_transform.restype = i; L.wino_i8_filter_transform.argtypes = [vp, vp, i, i, i, vp]
        L.wino_i8_workspace_bytes.restype = sz; L.wino_i8_workspace_bytes.argtypes = [i] * 5
        L.wino_i8_conv2d.restype = i; L.wino_i8_conv2d.argtypes = [vp, vp, vp, vp] + [i] * 7 + [vp, sz, vp]
        L.wino_i8_input_transform.restype = i; L.wino_i8_input_transform.argtypes = [vp, vp, vp] + [i] * 6 + [vp]
        L.wino_i8_batched_gemm.restype = i; L.wino_i8_batched_gemm.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, vp]
        L.wino_igemm_filter_bytes.restype = sz; L.wino_igemm_filter_bytes.argtypes = [i] * 4
        L.wino_igemm_filter_repack.restype = i
        L.wino_igemm_filter_repack.argtypes = [vp, vp, i, i, i, i, vp]
        L.wino_igemm_workspace_bytes.restype = sz; L.wino_igemm_workspace_bytes.argtypes = [i] * 9
        L.wino_igemm_conv2d.restype = i
        L.wino_igemm_conv2d.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, i, i, i, vp, sz, vp]
        _lib = L
    return _lib


# ---- helpers -------------------------------------------------------------------------------
def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream: Optional[torch.cuda.Stream]):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev(t: torch.Tensor, name: str):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous GPU tensor")


def _check(status: int, where: str):
    if status != WINO_OK:
        raise WinoError(status, where)


def _unpack(x, layout):
    """(N, C, H, W) of an activation tensor stored as NCHW or NHWC."""
    if x.dim() != 4:
        raise ValueError("activation tensors are 4-D")
    if layout == WINO_NHWC:
        N, H, W, C = map(int, x.shape)
    elif layout == WINO_NCHW:
        N, C, H, W = map(int, x.shape)
    else:
        raise WinoError(WINO_ERR_LAYOUT, "layout")
    return N, C, H, W


def _act_shape(N, C, H, W, layout):
    return (N, H, W, C) if layout == WINO_NHWC else (N, C, H, W)


def _conv_shapes(x, w_t, bias, y, layout=WINO_NCHW, upsample=False):
    """Host-side shape/dtype agreement (the C side cannot see tensor extents).  H and W are those
    of y: twice x's when x is read through the 2x upsampling."""
    N, C, H, W = _unpack(x, layout)
    if upsample:
        H, W = 2 * H, 2 * W
    K = int(w_t.desc.K)
    dt = TORCH_OF[w_t.desc.dtype]
    if tuple(y.shape) != _act_shape(N, K, H, W, layout) or x.dtype != dt or y.dtype != dt:
        raise ValueError(f"expected y{_act_shape(N, K, H, W, layout)} and dtype {dt} for x and y")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != K or not bias.is_cuda):
        raise ValueError("bias must be a GPU fp32 tensor of K elements")
    return N, C, H, W, K


# ---- same names as the C ABI ------------------------------------------------------------------
def wino_version() -> int:
    return lib().wino_version()


def status_string(status: int) -> str:
    return lib().wino_status_string(int(status)).decode()


wino_status_string = status_string


def wino_resolve_variant(N, C, H, W, K, dtype, variant) -> int:
    return lib().wino_resolve_variant(N, C, H, W, K, dtype, variant)


def wino_recommend_variant(N, C, H, W, K, dtype) -> int:
    return lib().wino_recommend_variant(N, C, H, W, K, dtype)


def wino_transformed_dims(N, C, H, W, K, variant):
    a, cp, t = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib().wino_transformed_dims(N, C, H, W, K, variant, ctypes.byref(a), ctypes.byref(cp), ctypes.byref(t)),
           "wino_transformed_dims")
    return a.value, cp.value, t.value


def wino_filter_bytes(K, C, dtype, variant) -> int:
    return lib().wino_filter_bytes(K, C, dtype, variant)


def wino_workspace_bytes(N, C, H, W, K, dtype, variant) -> int:
    return lib().wino_workspace_bytes(N, C, H, W, K, dtype, variant)


class Filter:
    """A transformed filter: the device buffer (kept alive here) plus the host descriptor."""

    def __init__(self, buf: torch.Tensor, desc: wino_filter):
        self.buf, self.desc = buf, desc

    @property
    def variant(self):
        return self.desc.variant


def wino_filter_transform(w: torch.Tensor, variant: int, stream=None) -> Filter:
    """w[K,C,3,3] (GPU) -> Filter holding U[alpha^2][K][Cp] (WINO_DIRECT: the re-laid filter of the direct path)."""
    _dev(w, "w")
    K, C = int(w.shape[0]), int(w.shape[1])
    if tuple(w.shape) != (K, C, 3, 3):
        raise ValueError("w must be [K,C,3,3]")
    dt = DTYPE_OF[w.dtype]
    nbytes = wino_filter_bytes(K, C, dt, variant)
    if nbytes == 0:
        raise WinoError(WINO_ERR_VARIANT, "wino_filter_bytes")
    buf = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    desc = wino_filter()
    _check(lib().wino_filter_transform(_ptr(w), _ptr(buf), K, C, dt, variant, ctypes.byref(desc), _stream(stream)),
           "wino_filter_transform")
    return Filter(buf, desc)


def wino_conv2d(x: torch.Tensor, w_t: Filter, bias: Optional[torch.Tensor], y: torch.Tensor, stream=None) -> torch.Tensor:
    _dev(x, "x"); _dev(y, "y")
    N, C, H, W, K = _conv_shapes(x, w_t, bias, y)
    _check(lib().wino_conv2d(_ptr(x), ctypes.byref(w_t.desc), _ptr(bias), _ptr(y), N, C, H, W, K, _stream(stream)),
           "wino_conv2d")
    return y


def wino_conv2d_ex(x, w_t: Filter, bias, y, workspace: torch.Tensor, layout: int = WINO_NCHW, stream=None):
    _dev(x, "x"); _dev(y, "y"); _dev(workspace, "workspace")
    N, C, H, W, K = _conv_shapes(x, w_t, bias, y, layout)
    _check(lib().wino_conv2d_ex(_ptr(x), ctypes.byref(w_t.desc), _ptr(bias), _ptr(y), N, C, H, W, K, layout,
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "wino_conv2d_ex")
    return y


def wino_static_scratch_bytes() -> int:
    return lib().wino_static_scratch_bytes()


def wino_conv2d_static(x, w_t: Filter, bias, y, layout: int = WINO_NCHW, stream=None):
    """wino_conv2d_ex with the scratch in the library's own device array: allocates nothing."""
    _dev(x, "x"); _dev(y, "y")
    N, C, H, W, K = _conv_shapes(x, w_t, bias, y, layout)
    _check(lib().wino_conv2d_static(_ptr(x), ctypes.byref(w_t.desc), _ptr(bias), _ptr(y), N, C, H, W, K, layout,
                                    _stream(stream)), "wino_conv2d_static")
    return y


def wino_input_transform(x: torch.Tensor, variant: int, layout: int = WINO_NCHW, stream=None, out=None) -> torch.Tensor:
    """x[N,C,H,W] (or [N,H,W,C] for NHWC) -> V[alpha^2, T, Cp] (same dtype)."""
    _dev(x, "x")
    N, C, H, W = _unpack(x, layout)
    alpha, Cp, T = wino_transformed_dims(N, C, H, W, 1, variant)
    V = out if out is not None else torch.empty((alpha * alpha, T, Cp), dtype=x.dtype, device=x.device)
    if V.numel() < alpha * alpha * T * Cp or V.dtype != x.dtype:
        raise ValueError("V buffer too small or of the wrong dtype")
    _check(lib().wino_input_transform(_ptr(x), _ptr(V), N, C, H, W, DTYPE_OF[x.dtype], variant, layout, _stream(stream)),
           "wino_input_transform")
    return V


def wino_batched_gemm(U: torch.Tensor, V: torch.Tensor, K: int, C: int, T: int, variant: int, stream=None, out=None,
                      block_shape: Optional[int] = None) -> torch.Tensor:
    """U[alpha^2,K,Cp], V[alpha^2,T,Cp] -> M[alpha^2,K,T] fp32.  block_shape names one of the kernel's block shapes
    (wino_batched_gemm_shape); None leaves the choice to the library (wino_batched_gemm)."""
    _dev(U, "U"); _dev(V, "V")
    a2 = (variant + 2) ** 2
    Cp = (C + 7) // 8 * 8
    if U.numel() < a2 * K * Cp or V.numel() < a2 * T * Cp or U.dtype != V.dtype:
        raise ValueError("U or V buffer too small for these dimensions")
    M = out if out is not None else torch.empty((a2, K, T), dtype=torch.float32, device=U.device)
    if M.numel() < a2 * K * T or M.dtype != torch.float32:
        raise ValueError("M buffer too small or not fp32")
    if block_shape is None:
        _check(lib().wino_batched_gemm(_ptr(U), _ptr(V), _ptr(M), K, C, T, DTYPE_OF[U.dtype], variant, _stream(stream)),
               "wino_batched_gemm")
    else:
        _check(lib().wino_batched_gemm_shape(_ptr(U), _ptr(V), _ptr(M), K, C, T, DTYPE_OF[U.dtype], variant, int(block_shape),
                                             _stream(stream)), "wino_batched_gemm_shape")
    return M


wino_batched_gemm_shape = wino_batched_gemm


def wino_fused_gemm_output(U: torch.Tensor, V: torch.Tensor, bias, N: int, C: int, H: int, W: int, K: int,
                           layout: int = WINO_NCHW, block_shape: int = -1, stream=None, out=None, m: int = 2) -> torch.Tensor:
    """U[a2,K,Cp], V[a2,T,Cp] -> y: steps (ii) and (iii) + bias in one kernel; m = 2: F(2x2,3x3), a2 = 16 (wino_fused_gemm_output),
    m = 4: F(4x4,3x3), a2 = 36 (wino_fused_f4_gemm_output)."""
    _dev(U, "U"); _dev(V, "V")
    if m not in (2, 4):
        raise WinoError(WINO_ERR_VARIANT, "m")
    a2 = (m + 2) ** 2
    Cp = (C + 7) // 8 * 8
    T = N * (-(-H // m)) * (-(-W // m))
    if U.numel() < a2 * K * Cp or V.numel() < a2 * T * Cp or U.dtype != V.dtype:
        raise ValueError("U or V buffer too small for these dimensions")
    if layout not in (WINO_NCHW, WINO_NHWC):
        raise WinoError(WINO_ERR_LAYOUT, "layout")
    y = out if out is not None else torch.empty(_act_shape(N, K, H, W, layout), dtype=U.dtype, device=U.device)
    if y.numel() < N * K * H * W or y.dtype != U.dtype:
        raise ValueError("y buffer too small or of the wrong dtype")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != K or not bias.is_cuda):
        raise ValueError("bias must be a GPU fp32 tensor of K elements")
    fn = lib().wino_fused_gemm_output if m == 2 else lib().wino_fused_f4_gemm_output
    _check(fn(_ptr(U), _ptr(V), _ptr(bias), _ptr(y), N, C, H, W, K, DTYPE_OF[U.dtype], layout, int(block_shape), _stream(stream)),
           "wino_fused_gemm_output" if m == 2 else "wino_fused_f4_gemm_output")
    return y


def wino_output_transform(M: torch.Tensor, bias, N: int, K: int, H: int, W: int, dtype: torch.dtype,
                          variant: int, layout: int = WINO_NCHW, stream=None, out=None) -> torch.Tensor:
    _dev(M, "M")
    m = variant
    if M.numel() < (m + 2) ** 2 * K * N * (-(-H // m)) * (-(-W // m)) or M.dtype != torch.float32:
        raise ValueError("M buffer too small or not fp32")
    y = out if out is not None else torch.empty(_act_shape(N, K, H, W, layout), dtype=dtype, device=M.device)
    if layout not in (WINO_NCHW, WINO_NHWC):
        raise WinoError(WINO_ERR_LAYOUT, "layout")
    if y.numel() < N * K * H * W or y.dtype != dtype:
        raise ValueError("y buffer too small or of the wrong dtype")
    _check(lib().wino_output_transform(_ptr(M), _ptr(bias), _ptr(y), N, K, H, W, DTYPE_OF[dtype], variant, layout,
                                       _stream(stream)), "wino_output_transform")
    return y


def wino_direct_conv2d(x: torch.Tensor, w: torch.Tensor, bias, y: torch.Tensor, stream=None) -> torch.Tensor:
    _dev(x, "x"); _dev(w, "w"); _dev(y, "y")
    N, C, H, W = map(int, x.shape)
    K = int(w.shape[0])
    if tuple(w.shape) != (K, C, 3, 3) or tuple(y.shape) != (N, K, H, W) or w.dtype != x.dtype or y.dtype != x.dtype:
        raise ValueError("direct conv: need w[K,C,3,3], y[N,K,H,W], one dtype")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != K or not bias.is_cuda):
        raise ValueError("bias must be a GPU fp32 tensor of K elements")
    _check(lib().wino_direct_conv2d(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), N, C, H, W, K, DTYPE_OF[x.dtype], _stream(stream)),
           "wino_direct_conv2d")
    return y


def wino_groupnorm_stats_bytes(N, groups) -> int:
    return lib().wino_groupnorm_stats_bytes(N, groups)


def wino_groupnorm_stats(x: torch.Tensor, groups: int, eps: float = 1e-5, layout: int = WINO_NCHW, stream=None,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """(mean, rstd) per (image, group) for the fused GroupNorm.  Returns the raw byte buffer; its
    first N*groups*2 floats are the statistics (`stats_view`)."""
    _dev(x, "x")
    N, C, H, W = _unpack(x, layout)
    nbytes = wino_groupnorm_stats_bytes(N, groups)
    if nbytes == 0 or C % groups:
        raise WinoError(WINO_ERR_DIM, "wino_groupnorm_stats_bytes")
    buf = out if out is not None else torch.empty(nbytes, dtype=torch.uint8, device=x.device)
    if buf.numel() * buf.element_size() < nbytes:
        raise ValueError("stats buffer too small")
    _check(lib().wino_groupnorm_stats(_ptr(x), _ptr(buf), N, C, H, W, groups, ctypes.c_float(eps), DTYPE_OF[x.dtype],
                                      layout, _stream(stream)), "wino_groupnorm_stats")
    return buf


def stats_view(buf: torch.Tensor, N: int, groups: int) -> torch.Tensor:
    return buf[: N * groups * 8].view(torch.float32).view(N, groups, 2)


def wino_conv2d_fused(x, w_t: Filter, bias, y, workspace, layout: int = WINO_NCHW, gn_stats=None, gn_gamma=None,
                      gn_beta=None, gn_groups: int = 32, addvec=None, residual=None, upsample: bool = False,
                      product_fp16: bool = False, stream=None):
    """wino_conv2d_ex with SiLU(GroupNorm(x)) and an optional 2x nearest-neighbour upsampling on the way in
    and + addvec[n,k] + residual on the way out."""
    _dev(x, "x"); _dev(y, "y"); _dev(workspace, "workspace")
    N, C, H, W, K = _conv_shapes(x, w_t, bias, y, layout, upsample)
    f = wino_fusion()
    f.upsample = 1 if upsample else 0
    f.product_fp16 = 1 if product_fp16 else 0
    if gn_stats is not None:
        for t, n, cnt in ((gn_gamma, "gn_gamma", C), (gn_beta, "gn_beta", C)):
            if t is None or not t.is_cuda or t.dtype != torch.float32 or t.numel() != cnt or not t.is_contiguous():
                raise ValueError(f"{n} must be a contiguous GPU fp32 tensor of {cnt} elements")
        if C % gn_groups or gn_stats.numel() * gn_stats.element_size() < N * gn_groups * 8 or not gn_stats.is_cuda:
            raise ValueError("gn_stats too small for N x gn_groups, or gn_groups does not divide C")
        f.gn_stats, f.gn_gamma, f.gn_beta, f.gn_groups = gn_stats.data_ptr(), gn_gamma.data_ptr(), gn_beta.data_ptr(), gn_groups
    if addvec is not None:
        if not addvec.is_cuda or addvec.dtype != torch.float32 or tuple(addvec.shape) != (N, K) or not addvec.is_contiguous():
            raise ValueError("addvec must be a contiguous GPU fp32 tensor [N, K]")
        f.addvec = addvec.data_ptr()
    if residual is not None:
        _dev(residual, "residual")
        if tuple(residual.shape) != tuple(y.shape) or residual.dtype != y.dtype:
            raise ValueError("residual must have the shape and dtype of y")
        f.residual = residual.data_ptr()
    _check(lib().wino_conv2d_fused(_ptr(x), ctypes.byref(w_t.desc), _ptr(bias), _ptr(y), N, C, H, W, K, layout,
                                   ctypes.byref(f), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream(stream)), "wino_conv2d_fused")
    return y


def wino_igemm_filter_bytes(K, C, R, dtype) -> int:
    return lib().wino_igemm_filter_bytes(K, C, R, dtype)


def wino_igemm_filter_repack(w: torch.Tensor, stream=None) -> torch.Tensor:
    """w[K,C,R,R] -> the re-laid filter Wr[R*R,K,Cp] followed by a row of zeros (raw byte buffer)."""
    _dev(w, "w")
    K, C, R = int(w.shape[0]), int(w.shape[1]), int(w.shape[2])
    if w.dim() != 4 or int(w.shape[3]) != R or w.dtype not in DTYPE_OF:
        raise ValueError("w must be [K,C,R,R], fp16 or fp32")
    nbytes = wino_igemm_filter_bytes(K, C, R, DTYPE_OF[w.dtype])
    if nbytes == 0:
        raise WinoError(WINO_ERR_DIM, "wino_igemm_filter_bytes")
    buf = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    _check(lib().wino_igemm_filter_repack(_ptr(w), _ptr(buf), K, C, R, DTYPE_OF[w.dtype], _stream(stream)),
           "wino_igemm_filter_repack")
    return buf


def wino_igemm_workspace_bytes(N, C, H, W, K, R, stride, dtype, layout) -> int:
    return lib().wino_igemm_workspace_bytes(N, C, H, W, K, R, stride, dtype, layout)


def wino_igemm_conv2d(x: torch.Tensor, w_r: torch.Tensor, bias, y: torch.Tensor, K: int, R: int, stride: int,
                      workspace: Optional[torch.Tensor], layout: int = WINO_NCHW, stream=None) -> torch.Tensor:
    _dev(x, "x"); _dev(w_r, "w_r"); _dev(y, "y")
    N, C, H, W = _unpack(x, layout)
    pad = (R - 1) // 2
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    if tuple(y.shape) != _act_shape(N, K, Ho, Wo, layout) or y.dtype != x.dtype:
        raise ValueError(f"expected y{_act_shape(N, K, Ho, Wo, layout)} of dtype {x.dtype}")
    if w_r.numel() * w_r.element_size() < wino_igemm_filter_bytes(K, C, R, DTYPE_OF[x.dtype]):
        raise ValueError("re-laid filter buffer too small")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != K or not bias.is_cuda):
        raise ValueError("bias must be a GPU fp32 tensor of K elements")
    wsb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().wino_igemm_conv2d(_ptr(x), _ptr(w_r), _ptr(bias), _ptr(y), N, C, H, W, K, R, stride, DTYPE_OF[x.dtype],
                                   layout, _ptr(workspace), wsb, _stream(stream)), "wino_igemm_conv2d")
    return y


def wino_fp8_filter_bytes(K, C, R) -> int:
    return lib().wino_fp8_filter_bytes(K, C, R)


def wino_fp8_filter_quantize(w: torch.Tensor, scale_w: float, stream=None) -> torch.Tensor:
    """w[K,C,R,R] -> e4m3(w * scale_w), re-laid [R*R,K,Cq] plus a row of zeros (raw byte buffer)."""
    _dev(w, "w")
    K, C, R = int(w.shape[0]), int(w.shape[1]), int(w.shape[2])
    if w.dim() != 4 or int(w.shape[3]) != R or w.dtype not in DTYPE_OF:
        raise ValueError("w must be [K,C,R,R] in one of the storage types")
    nbytes = wino_fp8_filter_bytes(K, C, R)
    if nbytes == 0:
        raise WinoError(WINO_ERR_DIM, "wino_fp8_filter_bytes")
    buf = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    _check(lib().wino_fp8_filter_quantize(_ptr(w), _ptr(buf), K, C, R, DTYPE_OF[w.dtype], ctypes.c_float(scale_w), _stream(stream)),
           "wino_fp8_filter_quantize")
    return buf


def wino_fp8_workspace_bytes(N, C, H, W, K, R, stride) -> int:
    return lib().wino_fp8_workspace_bytes(N, C, H, W, K, R, stride)


def wino_fp8_conv2d(x: torch.Tensor, w_q: torch.Tensor, bias, y: torch.Tensor, K: int, R: int, stride: int, scale_x: float,
                    scale_w: float, workspace: torch.Tensor, layout: int = WINO_NCHW, gn_stats=None, gn_gamma=None, gn_beta=None,
                    gn_groups: int = 32, addvec=None, residual=None, upsample: bool = False, stream=None) -> torch.Tensor:
    _dev(x, "x"); _dev(w_q, "w_q"); _dev(y, "y"); _dev(workspace, "workspace")
    N, C, H, W = _unpack(x, layout)
    if upsample:
        H, W = 2 * H, 2 * W
    pad = (R - 1) // 2
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    if tuple(y.shape) != _act_shape(N, K, Ho, Wo, layout) or y.dtype != x.dtype:
        raise ValueError(f"expected y{_act_shape(N, K, Ho, Wo, layout)} of dtype {x.dtype}")
    if w_q.numel() * w_q.element_size() < wino_fp8_filter_bytes(K, C, R):
        raise ValueError("quantised filter buffer too small")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != K or not bias.is_cuda):
        raise ValueError("bias must be a GPU fp32 tensor of K elements")
    f = wino_fusion()
    f.upsample = 1 if upsample else 0
    if gn_stats is not None:
        for t, cnt in ((gn_gamma, C), (gn_beta, C)):
            if t is None or not t.is_cuda or t.dtype != torch.float32 or t.numel() != cnt or not t.is_contiguous():
                raise ValueError("gn_gamma / gn_beta must be contiguous GPU fp32 tensors of C elements")
        f.gn_stats, f.gn_gamma, f.gn_beta, f.gn_groups = gn_stats.data_ptr(), gn_gamma.data_ptr(), gn_beta.data_ptr(), gn_groups
    if addvec is not None:
        if not addvec.is_cuda or addvec.dtype != torch.float32 or tuple(addvec.shape) != (N, K) or not addvec.is_contiguous():
            raise ValueError("addvec must be a contiguous GPU fp32 tensor [N, K]")
        f.addvec = addvec.data_ptr()
    if residual is not None:
        _dev(residual, "residual")
        if tuple(residual.shape) != tuple(y.shape) or residual.dtype != y.dtype:
            raise ValueError("residual must have the shape and dtype of y")
        f.residual = residual.data_ptr()
    _check(lib().wino_fp8_conv2d(_ptr(x), _ptr(w_q), _ptr(bias), _ptr(y), N, C, H, W, K, R, stride, DTYPE_OF[x.dtype], layout,
                                 ctypes.c_float(scale_x), ctypes.c_float(scale_w), ctypes.byref(f), _ptr(workspace),
                                 workspace.numel() * workspace.element_size(), _stream(stream)), "wino_fp8_conv2d")
    return y


def _align256(v: int) -> int:
    return (v + 255) // 256 * 256


def wino_i8_filter_bytes(K, C) -> int:
    return lib().wino_i8_filter_bytes(K, C)


def wino_i8_filter_transform(w: torch.Tensor, stream=None) -> torch.Tensor:
    """w[K,C,3,3] -> raw byte buffer: codes Uq[16][K][Cq] int8, then (256-byte aligned) steps dU[16][K] fp32."""
    _dev(w, "w")
    if w.dim() != 4 or tuple(w.shape[2:]) != (3, 3) or w.dtype not in DTYPE_OF:
        raise ValueError("w must be [K,C,3,3] in one of the storage types")
    K, C = int(w.shape[0]), int(w.shape[1])
    nbytes = wino_i8_filter_bytes(K, C)
    if nbytes == 0:
        raise WinoError(WINO_ERR_DIM, "wino_i8_filter_bytes")
    buf = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    _check(lib().wino_i8_filter_transform(_ptr(w), _ptr(buf), K, C, DTYPE_OF[w.dtype], _stream(stream)), "wino_i8_filter_transform")
    return buf


def i8_filter_views(u_q: torch.Tensor, K: int, C: int):
    """(Uq[16][K][Cq] int8, dU[16][K] fp32) as views of the buffer wino_i8_filter_transform wrote."""
    Cq = (C + 15) // 16 * 16
    n = 16 * K * Cq
    return u_q[:n].view(torch.int8).view(16, K, Cq), u_q[_align256(n):_align256(n) + 64 * K].view(torch.float32).view(16, K)


def wino_i8_workspace_bytes(N, C, H, W, K) -> int:
    return lib().wino_i8_workspace_bytes(N, C, H, W, K)


def wino_i8_conv2d(x: torch.Tensor, u_q: torch.Tensor, bias, y: torch.Tensor, K: int, workspace: torch.Tensor,
                   layout: int = WINO_NCHW, stream=None) -> torch.Tensor:
    _dev(x, "x"); _dev(u_q, "u_q"); _dev(y, "y"); _dev(workspace, "workspace")
    N, C, H, W = _unpack(x, layout)
    if tuple(y.shape) != _act_shape(N, K, H, W, layout) or y.dtype != x.dtype or x.dtype not in DTYPE_OF:
        raise ValueError(f"expected y{_act_shape(N, K, H, W, layout)} of dtype {x.dtype}")
    if u_q.numel() * u_q.element_size() < wino_i8_filter_bytes(K, C):
        raise ValueError("quantised filter buffer too small")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != K or not bias.is_cuda):
        raise ValueError("bias must be a GPU fp32 tensor of K elements")
    _check(lib().wino_i8_conv2d(_ptr(x), _ptr(u_q), _ptr(bias), _ptr(y), N, C, H, W, K, DTYPE_OF[x.dtype], layout, _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)), "wino_i8_conv2d")
    return y


def wino_i8_input_transform(x: torch.Tensor, layout: int = WINO_NCHW, stream=None):
    """x -> (Vq[16][T][Cq] int8, dV[16][T] fp32)."""
    _dev(x, "x")
    N, C, H, W = _unpack(x, layout)
    T, Cq = N * ((H + 1) // 2) * ((W + 1) // 2), (C + 15) // 16 * 16
    Vq = torch.empty((16, T, Cq), dtype=torch.int8, device=x.device)
    dV = torch.empty((16, T), dtype=torch.float32, device=x.device)
    _check(lib().wino_i8_input_transform(_ptr(x), _ptr(Vq), _ptr(dV), N, C, H, W, DTYPE_OF[x.dtype], layout, _stream(stream)),
           "wino_i8_input_transform")
    return Vq, dV


def wino_i8_batched_gemm(Uq: torch.Tensor, dU: torch.Tensor, Vq: torch.Tensor, dV: torch.Tensor, K: int, C: int, T: int,
                         block_shape: int = -1, stream=None) -> torch.Tensor:
    """M[16][K][T] fp32 = float(sum_c Uq * Vq) * dU[b][k] * dV[b][t]; called as (Vq, dV, Uq, dU, T, C, K) it writes M[16][T][K]."""
    for t, name in ((Uq, "Uq"), (dU, "dU"), (Vq, "Vq"), (dV, "dV")):
        _dev(t, name)
    Cq = (C + 15) // 16 * 16
    if Uq.dtype != torch.int8 or Vq.dtype != torch.int8 or Uq.numel() != 16 * K * Cq or Vq.numel() != 16 * T * Cq:
        raise ValueError("Uq / Vq must be int8 tensors of 16*K*Cq and 16*T*Cq elements")
    if dU.dtype != torch.float32 or dV.dtype != torch.float32 or dU.numel() != 16 * K or dV.numel() != 16 * T:
        raise ValueError("dU / dV must be fp32 tensors of 16*K and 16*T elements")
    M = torch.empty((16, K, T), dtype=torch.float32, device=Uq.device)
    _check(lib().wino_i8_batched_gemm(_ptr(Uq), _ptr(dU), _ptr(Vq), _ptr(dV), _ptr(M), K, C, T, block_shape, _stream(stream)),
           "wino_i8_batched_gemm")
    return M


# ---- convenience (allocation only) ------------------------------------------------------------
def conv2d_i8(x: torch.Tensor, w: torch.Tensor, bias=None, layout: int = WINO_NCHW) -> torch.Tensor:
    """Quantise the transformed filter, allocate workspace and output, run the Winograd path with 8-bit integer U and V."""
    N, C, H, W = _unpack(x, layout)
    K = int(w.shape[0])
    y = torch.empty(_act_shape(N, K, H, W, layout), dtype=x.dtype, device=x.device)
    u_q = wino_i8_filter_transform(w)
    ws = torch.empty(max(16, wino_i8_workspace_bytes(N, C, H, W, K)), dtype=torch.uint8, device=x.device)
    return wino_i8_conv2d(x, u_q, bias, y, K, ws, layout)


def conv2d_fp8(x: torch.Tensor, w: torch.Tensor, bias, scale_x: float, scale_w: float, stride: int = 1, layout: int = WINO_NCHW,
               **fused) -> torch.Tensor:
    """Quantise the filter, allocate workspace and output, run the 8-bit direct path (fused operators by keyword)."""
    N, C, H, W = _unpack(x, layout)
    if fused.get("upsample"):
        H, W = 2 * H, 2 * W
    K, R = int(w.shape[0]), int(w.shape[2])
    pad = (R - 1) // 2
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    y = torch.empty(_act_shape(N, K, Ho, Wo, layout), dtype=x.dtype, device=x.device)
    w_q = wino_fp8_filter_quantize(w, scale_w)
    ws = torch.empty(max(16, wino_fp8_workspace_bytes(N, C, H, W, K, R, stride)), dtype=torch.uint8, device=x.device)
    if fused.get("gn_gamma") is not None and fused.get("gn_stats") is None:
        fused["gn_stats"] = wino_groupnorm_stats(x, fused.get("gn_groups", 32), fused.pop("eps", 1e-5), layout)
    fused.pop("eps", None)
    return wino_fp8_conv2d(x, w_q, bias, y, K, R, stride, scale_x, scale_w, ws, layout, **fused)


def conv2d_igemm(x: torch.Tensor, w: torch.Tensor, bias=None, stride: int = 1, layout: int = WINO_NCHW) -> torch.Tensor:
    """1x1 or 3x3 convolution with stride 1 or 2 through the implicit-GEMM path (filter re-layout, workspace, call)."""
    N, C, H, W = _unpack(x, layout)
    K, R = int(w.shape[0]), int(w.shape[2])
    pad = (R - 1) // 2
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    y = torch.empty(_act_shape(N, K, Ho, Wo, layout), dtype=x.dtype, device=x.device)
    w_r = wino_igemm_filter_repack(w)
    nb = wino_igemm_workspace_bytes(N, C, H, W, K, R, stride, DTYPE_OF[x.dtype], layout)
    ws = torch.empty(nb, dtype=torch.uint8, device=x.device) if nb else None
    return wino_igemm_conv2d(x, w_r, bias, y, K, R, stride, ws, layout)


def conv2d(x: torch.Tensor, w: torch.Tensor, bias=None, variant: int = WINO_AUTO, layout: int = WINO_NCHW) -> torch.Tensor:
    """Transform the filter, allocate workspace and output, run the chosen variant."""
    N, C, H, W = _unpack(x, layout)
    K = int(w.shape[0])
    y = torch.empty(_act_shape(N, K, H, W, layout), dtype=x.dtype, device=x.device)
    # WINO_AUTO here means "whatever the library recommends for this shape", the direct variant included
    v = (wino_recommend_variant(N, C, H, W, K, DTYPE_OF[x.dtype]) if variant == WINO_AUTO
         else wino_resolve_variant(N, C, H, W, K, DTYPE_OF[x.dtype], variant))
    if v < 0:
        raise WinoError(WINO_ERR_DIM, "wino_resolve_variant")
    w_t = wino_filter_transform(w, v)          # WINO_DIRECT: the re-laid filter of the implicit-GEMM path
    ws = torch.empty(wino_workspace_bytes(N, C, H, W, K, DTYPE_OF[x.dtype], v), dtype=torch.uint8, device=x.device)
    return wino_conv2d_ex(x, w_t, bias, y, ws, layout)


def conv2d_fused(x, w, bias=None, variant: int = WINO_AUTO, layout: int = WINO_NCHW, gn_gamma=None, gn_beta=None,
                 gn_groups: int = 32, eps: float = 1e-5, addvec=None, residual=None, upsample: bool = False,
                 product_fp16: bool = False) -> torch.Tensor:
    """Statistics (if GroupNorm is asked for), filter transform, workspace, then the fused call."""
    N, C, H, W = _unpack(x, layout)
    if upsample:
        H, W = 2 * H, 2 * W
    K = int(w.shape[0])
    y = torch.empty(_act_shape(N, K, H, W, layout), dtype=x.dtype, device=x.device)
    v = (wino_recommend_variant(N, C, H, W, K, DTYPE_OF[x.dtype]) if variant == WINO_AUTO
         else wino_resolve_variant(N, C, H, W, K, DTYPE_OF[x.dtype], variant))
    if v not in (WINO_F2, WINO_F4, WINO_FUSED_F2, WINO_FUSED_F4, WINO_DIRECT):
        raise WinoError(WINO_ERR_VARIANT, "conv2d_fused")
    stats = wino_groupnorm_stats(x, gn_groups, eps, layout) if gn_gamma is not None else None
    w_t = wino_filter_transform(w, v)
    ws = torch.empty(wino_workspace_bytes(N, C, H, W, K, DTYPE_OF[x.dtype], v), dtype=torch.uint8, device=x.device)
    return wino_conv2d_fused(x, w_t, bias, y, ws, layout, stats, gn_gamma, gn_beta, gn_groups, addvec, residual, upsample,
                             product_fp16)
