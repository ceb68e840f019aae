"""Thin Python front end of libcg.so (the C-ABI declared in include/cg.h).

Argument marshalling only: tensors are torch int64 tensors on the GPU whose
bits are the uint64 ring elements; every function forwards pointers and sizes
to the C entry point of the same name and raises on a non-zero status.  There
is no fallback: if the library has not been built, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcg.so")

(CG_OK, CG_ERR_NULL, CG_ERR_SHAPE, CG_ERR_ALIGN, CG_ERR_ALIAS, CG_ERR_UNSUPPORTED, CG_ERR_DEVICE,
 CG_ERR_WORKSPACE) = range(8)

EXPORTS = ("cg_status_string", "cg_version", "cg_share_matmul", "cg_share_conv2d", "cg_share_add",
           "cg_share_mul_public", "cg_share_add_public", "cg_reconstruct",
           "cg_share_matmul_ws", "cg_share_conv2d_ws", "cg_zero_share", "cg_reshare", "cg_share_matmul_t",
           "cg_share_mul", "cg_share_sum_pool2d", "cg_share_conv2d_dgrad", "cg_share_conv2d_wgrad",
           "cg_trunc1_local", "cg_prf_words", "cg_bshare_xor", "cg_bshare_and", "cg_bshare_prefix_stage",
           "cg_bzero_share", "cg_breshare", "cg_share_bias_add", "cg_share_col_sum",
           "cg_bit_transpose64", "cg_bshare_carry_level", "cg_bits_unpack", "cg_bshare_csa", "cg_bshare_half_adder",
           "cg_share_matmul_acc", "cg_share_conv2d_acc", "cg_share_matmul_f64limb", "cg_share_matmul_static",
           "cg_share_matmul_prefers_workspace", "cg_share_conv2d_prefers_workspace",
           "cg_share_matmul_workspace_bytes", "cg_share_conv2d_workspace_bytes")
SIZE_EXPORTS = 2      # the last entries return size_t, the first two a string and an int, the rest cg_status


class ConvDesc(ctypes.Structure):
    """Mirror of cg_conv2d_desc."""
    _fields_ = [(n, ctypes.c_int64) for n in
                ("B", "H", "W", "Cin", "Cout", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w")]


class PoolDesc(ctypes.Structure):
    """Mirror of cg_pool2d_desc."""
    _fields_ = [(n, ctypes.c_int64) for n in
                ("B", "H", "W", "C", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w")]


class CgError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Load libcg.so (built by paper_2104_10949_amd.build.build()); no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2104_10949_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, u64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64, ctypes.c_size_t
        L.cg_status_string.argtypes = [ctypes.c_int]
        L.cg_status_string.restype = ctypes.c_char_p
        L.cg_version.argtypes = []
        L.cg_version.restype = ctypes.c_int
        L.cg_share_matmul.argtypes = [vp] * 5 + [i64] * 3 + [vp]
        L.cg_share_conv2d.argtypes = [vp] * 5 + [ctypes.POINTER(ConvDesc), vp]
        L.cg_share_matmul_acc.argtypes = L.cg_share_matmul.argtypes
        L.cg_share_matmul_f64limb.argtypes = L.cg_share_matmul.argtypes
        L.cg_share_matmul_static.argtypes = L.cg_share_matmul.argtypes
        L.cg_share_conv2d_acc.argtypes = L.cg_share_conv2d.argtypes
        L.cg_share_add.argtypes = [vp] * 6 + [sz, vp]
        L.cg_share_mul_public.argtypes = [vp, vp, u64, vp, vp, sz, vp]
        L.cg_share_add_public.argtypes = [vp, vp, u64, ctypes.c_int, vp, vp, sz, vp]
        L.cg_reconstruct.argtypes = [vp] * 4 + [sz, vp]
        L.cg_share_matmul_ws.argtypes = [vp] * 5 + [i64] * 3 + [vp, sz, vp]
        L.cg_share_conv2d_ws.argtypes = [vp] * 5 + [ctypes.POINTER(ConvDesc), vp, sz, vp]
        L.cg_share_matmul_workspace_bytes.argtypes = [i64] * 3
        L.cg_share_conv2d_workspace_bytes.argtypes = [ctypes.POINTER(ConvDesc)]
        L.cg_share_matmul_prefers_workspace.argtypes = [i64] * 3
        L.cg_share_conv2d_prefers_workspace.argtypes = [ctypes.POINTER(ConvDesc)]
        key = ctypes.c_char_p
        L.cg_zero_share.argtypes = [key, key, u64, u64, vp, sz, vp]
        L.cg_reshare.argtypes = [vp, key, key, u64, u64, vp, sz, vp]
        L.cg_share_matmul_t.argtypes = [vp] * 5 + [i64] * 3 + [ctypes.c_int] * 2 + [vp]
        L.cg_share_mul.argtypes = [vp] * 5 + [sz, sz, vp]
        L.cg_share_sum_pool2d.argtypes = [vp] * 4 + [ctypes.POINTER(PoolDesc), vp]
        L.cg_share_bias_add.argtypes = [vp] * 6 + [sz, sz, vp]
        L.cg_share_col_sum.argtypes = [vp] * 4 + [sz, sz, vp]
        L.cg_bshare_csa.argtypes = [vp] * 9 + [sz, vp]
        L.cg_bshare_half_adder.argtypes = [vp] * 7 + [sz, vp]
        L.cg_bit_transpose64.argtypes = [vp, vp, sz, vp]
        L.cg_bshare_carry_level.argtypes = [vp] * 6 + [sz, sz, vp]
        L.cg_bits_unpack.argtypes = [vp, vp, sz, vp]
        L.cg_bshare_xor.argtypes = [vp] * 6 + [sz, vp]
        L.cg_bshare_and.argtypes = [vp] * 5 + [sz, vp]
        L.cg_bshare_prefix_stage.argtypes = [vp] * 4 + [ctypes.c_int, vp, vp, sz, vp]
        L.cg_bzero_share.argtypes = [key, key, u64, u64, vp, sz, vp]
        L.cg_breshare.argtypes = [vp, key, key, u64, u64, vp, sz, vp]
        L.cg_trunc1_local.argtypes = [vp, vp, key, key, u64, u64, ctypes.c_int, key, u64, vp, sz, vp]
        L.cg_prf_words.argtypes = [key, u64, u64, vp, sz, vp]
        L.cg_share_conv2d_dgrad.argtypes = [vp] * 5 + [ctypes.POINTER(ConvDesc), vp]
        L.cg_share_conv2d_wgrad.argtypes = [vp] * 5 + [ctypes.POINTER(ConvDesc), vp]
        for name in EXPORTS[2:-SIZE_EXPORTS]:
            getattr(L, name).restype = ctypes.c_int
        for name in EXPORTS[-SIZE_EXPORTS:]:
            getattr(L, name).restype = sz
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().cg_status_string(int(status)).decode()


def version() -> int:
    return int(lib().cg_version())


def _ptr(t: torch.Tensor) -> int:
    if t.dtype != torch.int64:
        raise TypeError(f"ring tensors are torch.int64 (uint64 bit patterns), got {t.dtype}")
    if not t.is_cuda:
        raise ValueError("ring tensors must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("ring tensors must be contiguous")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _check(status: int, where: str) -> None:
    if status != CG_OK:
        raise CgError(status, where)


def cg_share_matmul(x_i, x_ip1, y_i, y_ip1, z_i=None, stream=None) -> torch.Tensor:
    """z_i = x_i y_i^T + x_ip1 y_i^T + x_i y_ip1^T mod 2^64; x [M,K], y [N,K], z [M,N]."""
    M, K = x_i.shape
    N = y_i.shape[0]
    if x_ip1.shape != x_i.shape or y_ip1.shape != y_i.shape or y_i.shape[1] != K:
        raise ValueError("operand shapes do not match")
    if z_i is None:
        z_i = torch.empty((M, N), dtype=torch.int64, device=x_i.device)
    elif tuple(z_i.shape) != (M, N):
        raise ValueError("output shape does not match")
    _check(lib().cg_share_matmul(_ptr(x_i), _ptr(x_ip1), _ptr(y_i), _ptr(y_ip1), _ptr(z_i),
                                 M, N, K, _stream(stream)), "cg_share_matmul")
    return z_i


def cg_share_matmul_t(x_i, x_ip1, y_i, y_ip1, trans_x: bool, trans_y: bool, z_i=None, stream=None) -> torch.Tensor:
    """Three-term product of L [M,K] and R [N,K] where x holds L ([M,K]) or L^T ([K,M], trans_x) and
    y holds R ([N,K]) or R^T ([K,N], trans_y)."""
    if trans_x:
        K, M = x_i.shape
    else:
        M, K = x_i.shape
    if trans_y:
        K2, N = y_i.shape
    else:
        N, K2 = y_i.shape
    if x_ip1.shape != x_i.shape or y_ip1.shape != y_i.shape or K2 != K:
        raise ValueError("operand shapes do not match")
    if z_i is None:
        z_i = torch.empty((M, N), dtype=torch.int64, device=x_i.device)
    elif tuple(z_i.shape) != (M, N):
        raise ValueError("output shape does not match")
    _check(lib().cg_share_matmul_t(_ptr(x_i), _ptr(x_ip1), _ptr(y_i), _ptr(y_ip1), _ptr(z_i),
                                   M, N, K, int(bool(trans_x)), int(bool(trans_y)), _stream(stream)),
           "cg_share_matmul_t")
    return z_i


def cg_share_matmul_f64limb(x_i, x_ip1, y_i, y_ip1, z_i=None, stream=None) -> torch.Tensor:
    """cg_share_matmul on the float64 matrix instruction with 16-bit blocks (comparator for the limb choice)."""
    M, K = x_i.shape
    N = y_i.shape[0]
    if x_ip1.shape != x_i.shape or y_ip1.shape != y_i.shape or y_i.shape[1] != K:
        raise ValueError("operand shapes do not match")
    if z_i is None:
        z_i = torch.empty((M, N), dtype=torch.int64, device=x_i.device)
    elif tuple(z_i.shape) != (M, N):
        raise ValueError("output shape does not match")
    _check(lib().cg_share_matmul_f64limb(_ptr(x_i), _ptr(x_ip1), _ptr(y_i), _ptr(y_ip1), _ptr(z_i), M, N, K,
                                         _stream(stream)), "cg_share_matmul_f64limb")
    return z_i


def cg_share_matmul_acc(x_i, x_ip1, y_i, y_ip1, z_i, stream=None) -> torch.Tensor:
    """z_i += party-local product of x [M,K] and y [N,K]; z_i [M,N] holds a value on entry (e.g. the zero share)."""
    M, K = x_i.shape
    N = y_i.shape[0]
    if x_ip1.shape != x_i.shape or y_ip1.shape != y_i.shape or y_i.shape[1] != K:
        raise ValueError("operand shapes do not match")
    if tuple(z_i.shape) != (M, N):
        raise ValueError("output shape does not match")
    _check(lib().cg_share_matmul_acc(_ptr(x_i), _ptr(x_ip1), _ptr(y_i), _ptr(y_ip1), _ptr(z_i), M, N, K,
                                     _stream(stream)), "cg_share_matmul_acc")
    return z_i


def cg_share_conv2d_acc(x_i, x_ip1, w_i, w_ip1, z_i, stride=(1, 1), pad=(0, 0), stream=None) -> torch.Tensor:
    """z_i += party-local convolution on shares; z_i NHWC holds a value on entry (e.g. the zero share)."""
    B, H, W, Cin = x_i.shape
    Cout, kh, kw, Cin2 = w_i.shape
    if x_ip1.shape != x_i.shape or w_ip1.shape != w_i.shape or Cin2 != Cin:
        raise ValueError("operand shapes do not match")
    d = ConvDesc(B, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1])
    if tuple(z_i.shape) != conv_out_shape(x_i.shape, w_i.shape, stride, pad):
        raise ValueError("output shape does not match")
    _check(lib().cg_share_conv2d_acc(_ptr(x_i), _ptr(x_ip1), _ptr(w_i), _ptr(w_ip1), _ptr(z_i),
                                     ctypes.byref(d), _stream(stream)), "cg_share_conv2d_acc")
    return z_i


def cg_share_matmul_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().cg_share_matmul_workspace_bytes(M, N, K))


def _ws(workspace) -> Tuple[int, int]:
    if workspace is None:
        return 0, 0
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def cg_share_matmul_ws(x_i, x_ip1, y_i, y_ip1, workspace, z_i=None, stream=None) -> torch.Tensor:
    """cg_share_matmul with caller-supplied scratch memory (any contiguous GPU tensor)."""
    M, K = x_i.shape
    N = y_i.shape[0]
    if x_ip1.shape != x_i.shape or y_ip1.shape != y_i.shape or y_i.shape[1] != K:
        raise ValueError("operand shapes do not match")
    if z_i is None:
        z_i = torch.empty((M, N), dtype=torch.int64, device=x_i.device)
    elif tuple(z_i.shape) != (M, N):
        raise ValueError("output shape does not match")
    wp, wb = _ws(workspace)
    _check(lib().cg_share_matmul_ws(_ptr(x_i), _ptr(x_ip1), _ptr(y_i), _ptr(y_ip1), _ptr(z_i),
                                    M, N, K, wp, wb, _stream(stream)), "cg_share_matmul_ws")
    return z_i


STATIC_SCRATCH_BYTES = 64 << 20   # CG_STATIC_SCRATCH_BYTES of include/cg.h


def cg_share_matmul_static(x_i, x_ip1, y_i, y_ip1, z_i=None, stream=None) -> torch.Tensor:
    """cg_share_matmul on the library's own fixed scratch array: the call allocates nothing."""
    M, K = x_i.shape
    N = y_i.shape[0]
    if x_ip1.shape != x_i.shape or y_ip1.shape != y_i.shape or y_i.shape[1] != K:
        raise ValueError("operand shapes do not match")
    if z_i is None:
        z_i = torch.empty((M, N), dtype=torch.int64, device=x_i.device)
    elif tuple(z_i.shape) != (M, N):
        raise ValueError("output shape does not match")
    _check(lib().cg_share_matmul_static(_ptr(x_i), _ptr(x_ip1), _ptr(y_i), _ptr(y_ip1), _ptr(z_i),
                                        M, N, K, _stream(stream)), "cg_share_matmul_static")
    return z_i


def conv_out_shape(x_shape: Sequence[int], w_shape: Sequence[int], stride: Tuple[int, int],
                   pad: Tuple[int, int]) -> Tuple[int, int, int, int]:
    B, H, W, _ = x_shape
    Cout, kh, kw, _ = w_shape
    return (B, (H + 2 * pad[0] - kh) // stride[0] + 1, (W + 2 * pad[1] - kw) // stride[1] + 1, Cout)


def cg_share_conv2d(x_i, x_ip1, w_i, w_ip1, stride=(1, 1), pad=(0, 0), z_i=None, stream=None) -> torch.Tensor:
    """Party-local convolution on shares; x NHWC [B,H,W,Cin], w [Cout,kh,kw,Cin], z NHWC."""
    B, H, W, Cin = x_i.shape
    Cout, kh, kw, Cin2 = w_i.shape
    if x_ip1.shape != x_i.shape or w_ip1.shape != w_i.shape or Cin2 != Cin:
        raise ValueError("operand shapes do not match")
    d = ConvDesc(B, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1])
    zs = conv_out_shape(x_i.shape, w_i.shape, stride, pad)
    if z_i is None:
        if zs[1] < 1 or zs[2] < 1:
            _check(CG_ERR_SHAPE, "cg_share_conv2d")
        z_i = torch.empty(zs, dtype=torch.int64, device=x_i.device)
    elif tuple(z_i.shape) != zs:
        raise ValueError("output shape does not match")
    _check(lib().cg_share_conv2d(_ptr(x_i), _ptr(x_ip1), _ptr(w_i), _ptr(w_ip1), _ptr(z_i),
                                 ctypes.byref(d), _stream(stream)), "cg_share_conv2d")
    return z_i


def cg_share_matmul_prefers_workspace(M: int, N: int, K: int) -> bool:
    return bool(lib().cg_share_matmul_prefers_workspace(M, N, K))


def cg_share_conv2d_prefers_workspace(x_shape, w_shape, stride=(1, 1), pad=(0, 0)) -> bool:
    B, H, W, Cin = x_shape
    Cout, kh, kw, _ = w_shape
    d = ConvDesc(B, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1])
    return bool(lib().cg_share_conv2d_prefers_workspace(ctypes.byref(d)))


def cg_share_conv2d_workspace_bytes(x_shape, w_shape, stride=(1, 1), pad=(0, 0)) -> int:
    B, H, W, Cin = x_shape
    Cout, kh, kw, _ = w_shape
    d = ConvDesc(B, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1])
    return int(lib().cg_share_conv2d_workspace_bytes(ctypes.byref(d)))


def cg_share_conv2d_ws(x_i, x_ip1, w_i, w_ip1, workspace, stride=(1, 1), pad=(0, 0), z_i=None,
                       stream=None) -> torch.Tensor:
    """cg_share_conv2d with caller-supplied scratch memory (any contiguous GPU tensor)."""
    B, H, W, Cin = x_i.shape
    Cout, kh, kw, Cin2 = w_i.shape
    if x_ip1.shape != x_i.shape or w_ip1.shape != w_i.shape or Cin2 != Cin:
        raise ValueError("operand shapes do not match")
    d = ConvDesc(B, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1])
    zs = conv_out_shape(x_i.shape, w_i.shape, stride, pad)
    if z_i is None:
        if zs[1] < 1 or zs[2] < 1:
            _check(CG_ERR_SHAPE, "cg_share_conv2d_ws")
        z_i = torch.empty(zs, dtype=torch.int64, device=x_i.device)
    elif tuple(z_i.shape) != zs:
        raise ValueError("output shape does not match")
    wp, wb = _ws(workspace)
    _check(lib().cg_share_conv2d_ws(_ptr(x_i), _ptr(x_ip1), _ptr(w_i), _ptr(w_ip1), _ptr(z_i),
                                    ctypes.byref(d), wp, wb, _stream(stream)), "cg_share_conv2d_ws")
    return z_i


def cg_share_conv2d_dgrad(g_i, g_ip1, w_i, w_ip1, x_shape, stride=(1, 1), pad=(0, 0), dx_i=None,
                          stream=None) -> torch.Tensor:
    """Party-local input gradient of a convolution layer; g NHWC [B,Ho,Wo,Cout], w [Cout,kh,kw,Cin],
    x_shape = (B,H,W,Cin) of the layer input, result NHWC of that shape."""
    B, H, W, Cin = (int(v) for v in x_shape)
    Cout, kh, kw, Cin2 = w_i.shape
    if g_ip1.shape != g_i.shape or w_ip1.shape != w_i.shape or Cin2 != Cin:
        raise ValueError("operand shapes do not match")
    if tuple(g_i.shape) != conv_out_shape((B, H, W, Cin), w_i.shape, stride, pad):
        raise ValueError("gradient shape does not match the layer")
    d = ConvDesc(B, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1])
    if dx_i is None:
        dx_i = torch.empty((B, H, W, Cin), dtype=torch.int64, device=g_i.device)
    elif tuple(dx_i.shape) != (B, H, W, Cin):
        raise ValueError("output shape does not match")
    _check(lib().cg_share_conv2d_dgrad(_ptr(g_i), _ptr(g_ip1), _ptr(w_i), _ptr(w_ip1), _ptr(dx_i),
                                       ctypes.byref(d), _stream(stream)), "cg_share_conv2d_dgrad")
    return dx_i


def cg_share_conv2d_wgrad(g_i, g_ip1, x_i, x_ip1, w_shape, stride=(1, 1), pad=(0, 0), dw_i=None,
                          stream=None) -> torch.Tensor:
    """Party-local weight gradient of a convolution layer; g NHWC [B,Ho,Wo,Cout], x NHWC [B,H,W,Cin],
    w_shape = (Cout,kh,kw,Cin), result of that shape."""
    B, H, W, Cin = x_i.shape
    Cout, kh, kw, Cin2 = (int(v) for v in w_shape)
    if g_ip1.shape != g_i.shape or x_ip1.shape != x_i.shape or Cin2 != Cin:
        raise ValueError("operand shapes do not match")
    if tuple(g_i.shape) != conv_out_shape(x_i.shape, (Cout, kh, kw, Cin), stride, pad):
        raise ValueError("gradient shape does not match the layer")
    d = ConvDesc(B, H, W, Cin, Cout, kh, kw, stride[0], stride[1], pad[0], pad[1])
    if dw_i is None:
        dw_i = torch.empty((Cout, kh, kw, Cin), dtype=torch.int64, device=g_i.device)
    elif tuple(dw_i.shape) != (Cout, kh, kw, Cin):
        raise ValueError("output shape does not match")
    _check(lib().cg_share_conv2d_wgrad(_ptr(g_i), _ptr(g_ip1), _ptr(x_i), _ptr(x_ip1), _ptr(dw_i),
                                       ctypes.byref(d), _stream(stream)), "cg_share_conv2d_wgrad")
    return dw_i


def cg_share_add(xa, xb, ya, yb, za=None, zb=None, stream=None):
    za = torch.empty_like(xa) if za is None else za
    zb = torch.empty_like(xb) if zb is None else zb
    if not (xa.shape == xb.shape == ya.shape == yb.shape == za.shape == zb.shape):
        raise ValueError("operand shapes do not match")
    _check(lib().cg_share_add(_ptr(xa), _ptr(xb), _ptr(ya), _ptr(yb), _ptr(za), _ptr(zb),
                              xa.numel(), _stream(stream)), "cg_share_add")
    return za, zb


def cg_share_mul_public(xa, xb, alpha: int, za=None, zb=None, stream=None):
    za = torch.empty_like(xa) if za is None else za
    zb = torch.empty_like(xb) if zb is None else zb
    if not (xa.shape == xb.shape == za.shape == zb.shape):
        raise ValueError("operand shapes do not match")
    _check(lib().cg_share_mul_public(_ptr(xa), _ptr(xb), int(alpha) % (1 << 64), _ptr(za), _ptr(zb),
                                     xa.numel(), _stream(stream)), "cg_share_mul_public")
    return za, zb


def cg_share_add_public(xa, xb, gamma: int, party: int, za=None, zb=None, stream=None):
    za = torch.empty_like(xa) if za is None else za
    zb = torch.empty_like(xb) if zb is None else zb
    if not (xa.shape == xb.shape == za.shape == zb.shape):
        raise ValueError("operand shapes do not match")
    _check(lib().cg_share_add_public(_ptr(xa), _ptr(xb), int(gamma) % (1 << 64), int(party), _ptr(za), _ptr(zb),
                                     xa.numel(), _stream(stream)), "cg_share_add_public")
    return za, zb


def cg_share_mul(x_i, x_ip1, y_i, y_ip1, z_i=None, stream=None) -> torch.Tensor:
    """Element-wise three-term product; y (y.numel() divides x.numel()) is broadcast along x's leading dims."""
    if x_ip1.shape != x_i.shape or y_ip1.shape != y_i.shape:
        raise ValueError("operand shapes do not match")
    z_i = torch.empty_like(x_i) if z_i is None else z_i
    if z_i.shape != x_i.shape:
        raise ValueError("output shape does not match")
    n = x_i.numel()
    _check(lib().cg_share_mul(_ptr(x_i) if n else 0, _ptr(x_ip1) if n else 0, _ptr(y_i) if n else 0,
                              _ptr(y_ip1) if n else 0, _ptr(z_i) if n else 0, n, y_i.numel(), _stream(stream)),
           "cg_share_mul")
    return z_i


def cg_share_sum_pool2d(xa, xb, window, stride, pad=(0, 0), za=None, zb=None, stream=None):
    """Window sums (zero padded) of both components of a replicated pair, NHWC."""
    B, H, W, C = xa.shape
    if xb.shape != xa.shape:
        raise ValueError("operand shapes do not match")
    d = PoolDesc(B, H, W, C, window[0], window[1], stride[0], stride[1], pad[0], pad[1])
    Ho = (H + 2 * pad[0] - window[0]) // stride[0] + 1
    Wo = (W + 2 * pad[1] - window[1]) // stride[1] + 1
    if Ho < 1 or Wo < 1:
        _check(CG_ERR_SHAPE, "cg_share_sum_pool2d")
    za = torch.empty((B, Ho, Wo, C), dtype=torch.int64, device=xa.device) if za is None else za
    zb = torch.empty((B, Ho, Wo, C), dtype=torch.int64, device=xa.device) if zb is None else zb
    _check(lib().cg_share_sum_pool2d(_ptr(xa), _ptr(xb), _ptr(za), _ptr(zb), ctypes.byref(d), _stream(stream)),
           "cg_share_sum_pool2d")
    return za, zb


def _key16(key: bytes) -> bytes:
    key = bytes(key)
    if len(key) != 16:
        raise ValueError("PRF keys are 16 bytes (AES-128)")
    return key


def cg_zero_share(key_self: bytes, key_prev: bytes, nonce: int, first: int, n: int, out=None,
                  stream=None) -> torch.Tensor:
    """alpha[j] = F(key_self, first + j) - F(key_prev, first + j) for j < n."""
    if out is None:
        out = torch.empty((n,), dtype=torch.int64, device="cuda")
    elif out.numel() != n:
        raise ValueError("output size does not match")
    _check(lib().cg_zero_share(_key16(key_self), _key16(key_prev), nonce % (1 << 64), first % (1 << 64),
                               _ptr(out) if n else 0, n, _stream(stream)), "cg_zero_share")
    return out


def cg_reshare(z_i, key_self: bytes, key_prev: bytes, nonce: int, first: int = 0, out=None,
               stream=None) -> torch.Tensor:
    """out = z_i + alpha_i, the blinded additive share sent to the next party."""
    out = torch.empty_like(z_i) if out is None else out
    if out.shape != z_i.shape:
        raise ValueError("output shape does not match")
    n = z_i.numel()
    _check(lib().cg_reshare(_ptr(z_i) if n else 0, _key16(key_self), _key16(key_prev), nonce % (1 << 64),
                            first % (1 << 64), _ptr(out) if n else 0, n, _stream(stream)), "cg_reshare")
    return out


def cg_trunc1_local(z_i, msg, key_self: bytes, key_prev: bytes, nonce: int, first: int, d: int,
                    key_mask=None, mask_nonce: int = 0, out=None, stream=None) -> torch.Tensor:
    """One party's local step of the share truncation: asr(z_i + alpha + msg, d) - F(key_mask, .)."""
    if msg is not None and msg.shape != z_i.shape:
        raise ValueError("message shape does not match")
    if out is None:
        out = torch.empty_like(z_i)
    _check(lib().cg_trunc1_local(_ptr(z_i), None if msg is None else _ptr(msg), _key16(key_self), _key16(key_prev),
                                 nonce, first, d, None if key_mask is None else _key16(key_mask), mask_nonce,
                                 _ptr(out), z_i.numel(), _stream(stream)), "cg_trunc1_local")
    return out


def cg_prf_words(key: bytes, nonce: int, first: int, n: int, out=None, stream=None) -> torch.Tensor:
    """F(key, first + j) for j < n as a GPU tensor."""
    if out is None:
        out = torch.empty((n,), dtype=torch.int64, device="cuda")
    elif out.numel() != n:
        raise ValueError("output size does not match")
    _check(lib().cg_prf_words(_key16(key), nonce, first, _ptr(out) if n else None, n, _stream(stream)), "cg_prf_words")
    return out


def cg_share_bias_add(xa, xb, ba, bb, za=None, zb=None, stream=None):
    """(xa + ba, xb + bb) with the bias pair [cols] broadcast over the leading dimensions of x [..., cols]."""
    if xa.shape != xb.shape or ba.shape != bb.shape or ba.dim() != 1 or xa.shape[-1] != ba.shape[0]:
        raise ValueError("operand shapes do not match")
    za = torch.empty_like(xa) if za is None else za
    zb = torch.empty_like(xb) if zb is None else zb
    n = xa.numel()
    _check(lib().cg_share_bias_add(*(_ptr(t) if n else 0 for t in (xa, xb, ba, bb, za, zb)), n, ba.numel(),
                                   _stream(stream)), "cg_share_bias_add")
    return za, zb


def cg_share_col_sum(xa, xb, za=None, zb=None, stream=None):
    """Column sums of both components of x [..., cols] over all leading dimensions."""
    if xa.shape != xb.shape:
        raise ValueError("operand shapes do not match")
    cols = xa.shape[-1]
    rows = xa.numel() // cols if cols else 0
    za = torch.empty((cols,), dtype=torch.int64, device=xa.device) if za is None else za
    zb = torch.empty((cols,), dtype=torch.int64, device=xa.device) if zb is None else zb
    _check(lib().cg_share_col_sum(_ptr(xa) if rows else 0, _ptr(xb) if rows else 0, _ptr(za) if cols else 0,
                                  _ptr(zb) if cols else 0, rows, cols, _stream(stream)), "cg_share_col_sum")
    return za, zb


def cg_bshare_xor(xa, xb, ya, yb, za=None, zb=None, stream=None):
    """XOR gate on binary replicated pairs: (xa ^ ya, xb ^ yb)."""
    za = torch.empty_like(xa) if za is None else za
    zb = torch.empty_like(xb) if zb is None else zb
    n = xa.numel()
    _check(lib().cg_bshare_xor(*(_ptr(t) if n else 0 for t in (xa, xb, ya, yb, za, zb)), n, _stream(stream)),
           "cg_bshare_xor")
    return za, zb


def cg_bshare_and(x_i, x_ip1, y_i, y_ip1, z_i=None, stream=None) -> torch.Tensor:
    """Local step of an AND gate on binary replicated pairs (64 gates per word)."""
    if not (x_i.shape == x_ip1.shape == y_i.shape == y_ip1.shape):
        raise ValueError("operand shapes do not match")
    z_i = torch.empty_like(x_i) if z_i is None else z_i
    n = x_i.numel()
    _check(lib().cg_bshare_and(*(_ptr(t) if n else 0 for t in (x_i, x_ip1, y_i, y_ip1, z_i)), n, _stream(stream)),
           "cg_bshare_and")
    return z_i


def cg_bshare_prefix_stage(p_i, p_ip1, g_i, g_ip1, shift: int, last: bool = False, p_out=None, g_out=None,
                           stream=None):
    """Local step of one parallel-prefix adder stage; returns (p_out or None, g_out)."""
    if not (p_i.shape == p_ip1.shape == g_i.shape == g_ip1.shape):
        raise ValueError("operand shapes do not match")
    g_out = torch.empty_like(g_i) if g_out is None else g_out
    if not last and p_out is None:
        p_out = torch.empty_like(p_i)
    n = p_i.numel()
    _check(lib().cg_bshare_prefix_stage(*(_ptr(t) if n else 0 for t in (p_i, p_ip1, g_i, g_ip1)), shift,
                                        None if last else (_ptr(p_out) if n else 0), _ptr(g_out) if n else 0, n,
                                        _stream(stream)), "cg_bshare_prefix_stage")
    return (None if last else p_out), g_out


def cg_bshare_csa(a_i, a_ip1, b_i, b_ip1, c_i, c_ip1, s_i=None, s_ip1=None, carry_i=None, stream=None):
    """Local step of a carry-save adder: returns (s_i, s_ip1, carry_i).  An input given as None is a component
    that is zero everywhere (a party's view of a sharing whose only non-zero share it does not hold)."""
    ins = (a_i, a_ip1, b_i, b_ip1, c_i, c_ip1)
    given = [t for t in ins if t is not None]
    if not given and s_i is None:
        raise ValueError("no operand to take the shape from")
    like = given[0] if given else s_i
    if any(t.shape != like.shape for t in given):
        raise ValueError("operand shapes do not match")
    s_i = torch.empty_like(like) if s_i is None else s_i
    s_ip1 = torch.empty_like(like) if s_ip1 is None else s_ip1
    carry_i = torch.empty_like(like) if carry_i is None else carry_i
    n = like.numel()
    _check(lib().cg_bshare_csa(*(_ptr(t) if (n and t is not None) else 0 for t in ins + (s_i, s_ip1, carry_i)), n,
                               _stream(stream)), "cg_bshare_csa")
    return s_i, s_ip1, carry_i


def cg_bshare_half_adder(s_i, s_ip1, t_i, t_ip1, p_i=None, p_ip1=None, g_i=None, stream=None):
    """Local step of a half adder: returns (p_i, p_ip1, g_i)."""
    ins = (s_i, s_ip1, t_i, t_ip1)
    if any(t.shape != s_i.shape for t in ins):
        raise ValueError("operand shapes do not match")
    p_i = torch.empty_like(s_i) if p_i is None else p_i
    p_ip1 = torch.empty_like(s_i) if p_ip1 is None else p_ip1
    g_i = torch.empty_like(s_i) if g_i is None else g_i
    n = s_i.numel()
    _check(lib().cg_bshare_half_adder(*(_ptr(t) if n else 0 for t in ins + (p_i, p_ip1, g_i)), n, _stream(stream)),
           "cg_bshare_half_adder")
    return p_i, p_ip1, g_i


def cg_bit_transpose64(x, out=None, stream=None) -> torch.Tensor:
    """Bit planes [64, m] of a flat tensor of 64 m words."""
    n = x.numel()
    if n % 64:
        _check(CG_ERR_SHAPE, "cg_bit_transpose64")
    out = torch.empty((64, n // 64), dtype=torch.int64, device=x.device) if out is None else out
    _check(lib().cg_bit_transpose64(_ptr(x) if n else 0, _ptr(out) if n else 0, n, _stream(stream)), "cg_bit_transpose64")
    return out


def cg_bshare_carry_level(p_i, p_ip1, g_i, g_ip1, last: bool = False, stream=None):
    """Local step of one level of the carry tree on planes [2k, m]; returns (p_out or None, g_out), each [k, m]."""
    if not (p_i.shape == p_ip1.shape == g_i.shape == g_ip1.shape) or p_i.dim() != 2 or p_i.shape[0] % 2:
        raise ValueError("operands must be [2k, m] tensors of one shape")
    k, m = p_i.shape[0] // 2, p_i.shape[1]
    g_out = torch.empty((k, m), dtype=torch.int64, device=p_i.device)
    p_out = None if last else torch.empty((k, m), dtype=torch.int64, device=p_i.device)
    _check(lib().cg_bshare_carry_level(_ptr(p_i), _ptr(p_ip1), _ptr(g_i), _ptr(g_ip1),
                                       None if last else _ptr(p_out), _ptr(g_out), k, m, _stream(stream)),
           "cg_bshare_carry_level")
    return p_out, g_out


def cg_bits_unpack(plane, n: int, out=None, stream=None) -> torch.Tensor:
    """One word per element (0 or 1) from a packed plane of at least ceil(n / 64) words."""
    if plane.numel() * 64 < n:
        raise ValueError("plane too short")
    out = torch.empty((n,), dtype=torch.int64, device=plane.device) if out is None else out
    _check(lib().cg_bits_unpack(_ptr(plane) if n else 0, _ptr(out) if n else 0, n, _stream(stream)), "cg_bits_unpack")
    return out


def cg_bzero_share(key_self: bytes, key_prev: bytes, nonce: int, first: int, n: int, out=None,
                   stream=None) -> torch.Tensor:
    if out is None:
        out = torch.empty((n,), dtype=torch.int64, device="cuda")
    _check(lib().cg_bzero_share(_key16(key_self), _key16(key_prev), nonce, first, _ptr(out) if n else 0, n,
                                _stream(stream)), "cg_bzero_share")
    return out


def cg_breshare(z_i, key_self: bytes, key_prev: bytes, nonce: int, first: int = 0, out=None,
                stream=None) -> torch.Tensor:
    """out = z_i ^ beta_i, the blinded XOR share passed on after an AND gate; out may be z_i."""
    out = torch.empty_like(z_i) if out is None else out
    n = z_i.numel()
    _check(lib().cg_breshare(_ptr(z_i) if n else 0, _key16(key_self), _key16(key_prev), nonce, first,
                             _ptr(out) if n else 0, n, _stream(stream)), "cg_breshare")
    return out


def cg_reconstruct(s0, s1, s2, out=None, stream=None) -> torch.Tensor:
    out = torch.empty_like(s0) if out is None else out
    if not (s0.shape == s1.shape == s2.shape == out.shape):
        raise ValueError("operand shapes do not match")
    _check(lib().cg_reconstruct(_ptr(s0), _ptr(s1), _ptr(s2), _ptr(out), s0.numel(), _stream(stream)),
           "cg_reconstruct")
    return out


def to_device(a) -> torch.Tensor:
    """numpy uint64 array -> int64 GPU tensor with the same bits."""
    import numpy as np
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint64:
        raise TypeError("expected uint64")
    return torch.from_numpy(a.view(np.int64)).cuda()


def to_host(t: torch.Tensor):
    """int64 GPU tensor -> numpy uint64 array with the same bits."""
    import numpy as np
    return t.cpu().numpy().view(np.uint64)
