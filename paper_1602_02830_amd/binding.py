"""ctypes binding of the C ABI in ``include/bnn.h``; same names, same argument order.

Only marshalling happens here: shapes and strides are read off the tensors,
outputs are allocated with torch on the inputs' device, and the call is
enqueued on torch's current stream.  No arithmetic of the method is done in
Python, and nothing falls back to the CPU.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libbnn_hip.so")

(KERNEL_AUTO, KERNEL_NAIVE, KERNEL_TILED128, KERNEL_KSPLIT, KERNEL_TILED64, KERNEL_MFMA, KERNEL_MFMA128,
 KERNEL_MFMA_SHORTK, KERNEL_MFMA_PERSIST, KERNEL_MFMA_BIG, KERNEL_MFMA_SPLITK) = range(11)

_i64 = ctypes.c_int64
_int = ctypes.c_int
_ptr = ctypes.c_void_p
_f32 = ctypes.c_float

_SIGNATURES = {
    "bnn_version": (_int, []),
    "bnn_status_string": (ctypes.c_char_p, [_int]),
    "bnn_words_per_row": (_i64, [_i64]),
    "bnn_pack_sign": (_int, [_ptr, _i64, _i64, _i64, _ptr, _i64, _ptr]),
    "bnn_xnor_gemm": (_int, [_ptr, _i64, _ptr, _i64, _ptr, _i64, _i64, _i64, _i64, _ptr]),
    "bnn_xnor_gemm_kernel": (_int, [_ptr, _i64, _ptr, _i64, _ptr, _i64, _i64, _i64, _i64, _int, _ptr]),
    "bnn_xnor_gemm_bn_sign_pack": (_int, [_ptr, _i64, _ptr, _i64, _i64, _i64, _i64, _ptr, _ptr, _ptr, _i64, _ptr]),
    "bnn_xnor_gemm_bn_sign_pack_kernel": (_int, [_ptr, _i64, _ptr, _i64, _i64, _i64, _i64, _ptr, _ptr, _ptr, _i64,
                                                 _int, _ptr]),
    "bnn_pack_bitplanes": (_int, [_ptr, _i64, _i64, _i64, _ptr, _i64, _ptr]),
    "bnn_bitplane_gemm": (_int, [_ptr, _i64, _ptr, _i64, _ptr, _i64, _i64, _i64, _i64, _ptr]),
    "bnn_bitplane_gemm_bn_sign_pack": (_int, [_ptr, _i64, _ptr, _i64, _i64, _i64, _i64, _ptr, _ptr, _ptr, _i64, _ptr]),
    "bnn_bn_fold": (_int, [_ptr, _ptr, _ptr, _ptr, _f32, _i64, _i64, _ptr, _ptr]),
    "bnn_bn_sign_pack": (_int, [_ptr, _i64, _i64, _i64, _ptr, _ptr, _ptr, _i64, _ptr]),
    "bnn_conv_im2col_pack": (_int, [_ptr, _i64, _i64, _i64, _i64, _int, _int, _int, _int, _ptr, _i64, _ptr]),
    "bnn_conv_xnor": (_int, [_ptr, _i64, _i64, _i64, _i64, _ptr, _i64, _i64, _int, _int, _int, _int, _ptr, _i64, _ptr]),
    "bnn_conv_bn_sign_pack": (_int, [_ptr, _i64, _i64, _i64, _i64, _ptr, _i64, _i64, _int, _int, _int, _int, _ptr,
                                     _ptr, _ptr, _i64, _ptr]),
    "bnn_conv_pool_bn_sign_pack": (_int, [_ptr, _i64, _i64, _i64, _i64, _ptr, _i64, _i64, _int, _int, _int, _int, _int,
                                          _ptr, _ptr, _ptr, _i64, _ptr]),
    "bnn_maxpool_bits": (_int, [_ptr, _i64, _i64, _i64, _i64, _int, _int, _int, _ptr, _ptr, _ptr]),
    "bnn_gemm_i8_mfma": (_int, [_ptr, _i64, _ptr, _i64, _ptr, _i64, _i64, _i64, _i64, _ptr]),
    "bnn_unpack_i8": (_int, [_ptr, _i64, _i64, _i64, _ptr, _i64, _ptr]),
}

_lib = None


class BnnError(RuntimeError):
    def __init__(self, fn: str, status: int):
        msg = load_library().bnn_status_string(status).decode()
        super().__init__(f"{fn} failed with status {status} ({msg})")
        self.status = status


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libbnn_hip.so (built in-tree by ``build.build_library``).  Raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is not built; run `python -m paper_1602_02830_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def exported_symbols():
    return sorted(_SIGNATURES)


def _check(fn: str, status: int):
    if status != 0:
        raise BnnError(fn, status)


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(t: torch.Tensor):
    """torch's current stream on the device of `t`, as the ABI's `void* stream`."""
    if _raw_stream is not None:            # the handle itself, without building a Stream object
        return _raw_stream(t.device.index)
    return torch.cuda.current_stream(t.device).cuda_stream


def _dev(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with unit stride along its rows")
    return t


def _ld(t: torch.Tensor) -> int:
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def version() -> int:
    return int(load_library().bnn_version())


def words_per_row(K: int) -> int:
    """bnn_words_per_row: 32-bit words of a packed row of K values (the layout rule of the ABI, restated
    here so that the wrappers do not pay a foreign call for it; a host test compares the two)."""
    K = int(K)
    return -1 if K < 0 else (K + 31) // 32


def _alloc_words(rows: int, kw: int, device, ld: int | None = None) -> torch.Tensor:
    ld = kw if ld is None else ld
    if ld < kw:
        raise ValueError("ld smaller than the packed row")
    if ld == kw:
        return torch.empty((rows, kw), dtype=torch.int32, device=device)
    # Words between the packed row and ld are never written by the library: define them.
    return torch.zeros((rows, ld), dtype=torch.int32, device=device)[:, :kw]


def pack_sign(x: torch.Tensor, out: torch.Tensor | None = None, ld_out: int | None = None) -> torch.Tensor:
    """bnn_pack_sign: float32 [rows][cols] -> packed int32 words [rows][ceil(cols/32)]."""
    lib = load_library()
    _dev(x, torch.float32, "x")
    rows, cols = x.shape
    kw = words_per_row(cols)
    if out is None:
        out = _alloc_words(rows, kw, x.device, ld_out)
    _dev(out, torch.int32, "out")
    _check("bnn_pack_sign", lib.bnn_pack_sign(x.data_ptr(), rows, cols, _ld(x), out.data_ptr(), _ld(out),
                                             _stream(out)))
    return out


def xnor_gemm(A: torch.Tensor, B: torch.Tensor, K: int, out: torch.Tensor | None = None,
              kernel: int = KERNEL_AUTO) -> torch.Tensor:
    """bnn_xnor_gemm: packed A [M][Kw], packed B [N][Kw] -> int32 C [M][N]."""
    lib = load_library()
    _dev(A, torch.int32, "A")
    _dev(B, torch.int32, "B")
    M, N = A.shape[0], B.shape[0]
    kw = words_per_row(K)
    if A.shape[1] < kw or B.shape[1] < kw:
        raise ValueError("packed operands have fewer words per row than K needs")
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _dev(out, torch.int32, "out")
    if kernel == KERNEL_AUTO:
        st = lib.bnn_xnor_gemm(A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), out.data_ptr(), _ld(out), M, N, K,
                               _stream(out))
    else:
        st = lib.bnn_xnor_gemm_kernel(A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), out.data_ptr(), _ld(out),
                                      M, N, K, kernel, _stream(out))
    _check("bnn_xnor_gemm", st)
    return out


def bn_fold(gamma, beta, mean, var, eps: float, K: int):
    """bnn_bn_fold (host): float32 arrays [N] -> (thr int32 [N], flip_bits uint32 [ceil(N/32)]) numpy."""
    lib = load_library()
    arrs = [np.ascontiguousarray(a, dtype=np.float32) for a in (gamma, beta, mean, var)]
    N = arrs[0].shape[0]
    for a in arrs:
        if a.shape != (N,):
            raise ValueError("BatchNorm parameter arrays must all be [N]")
    thr = np.empty(N, np.int32)
    flip = np.empty((N + 31) // 32, np.uint32)
    st = lib.bnn_bn_fold(*(a.ctypes.data for a in arrs), eps, N, K, thr.ctypes.data, flip.ctypes.data)
    _check("bnn_bn_fold", st)
    return thr, flip


def bn_sign_pack(C: torch.Tensor, thr: torch.Tensor, flip_bits: torch.Tensor,
                 out: torch.Tensor | None = None, ld_out: int | None = None) -> torch.Tensor:
    """bnn_bn_sign_pack: int32 C [M][N] + folded thresholds -> packed bits [M][ceil(N/32)]."""
    lib = load_library()
    _dev(C, torch.int32, "C")
    M, N = C.shape
    nw = words_per_row(N)
    if thr.dtype != torch.int32 or flip_bits.dtype != torch.int32 or not thr.is_cuda or not flip_bits.is_cuda:
        raise ValueError("thr and flip_bits must be int32 device tensors")
    if thr.numel() != N or flip_bits.numel() != nw or not thr.is_contiguous() or not flip_bits.is_contiguous():
        raise ValueError("thr must be [N] and flip_bits [ceil(N/32)], contiguous")
    if out is None:
        out = _alloc_words(M, nw, C.device, ld_out)
    _dev(out, torch.int32, "out")
    _check("bnn_bn_sign_pack", lib.bnn_bn_sign_pack(C.data_ptr(), _ld(C), M, N, thr.data_ptr(),
                                                   flip_bits.data_ptr(), out.data_ptr(), _ld(out), _stream(out)))
    return out


def xnor_gemm_bn_sign_pack(A: torch.Tensor, B: torch.Tensor, K: int, thr: torch.Tensor, flip_bits: torch.Tensor,
                           out: torch.Tensor | None = None, ld_out: int | None = None,
                           kernel: int = KERNEL_AUTO) -> torch.Tensor:
    """bnn_xnor_gemm_bn_sign_pack: packed A [M][Kw], packed B [N][Kw], thresholds -> packed bits [M][ceil(N/32)]."""
    lib = load_library()
    _dev(A, torch.int32, "A")
    _dev(B, torch.int32, "B")
    M, N = A.shape[0], B.shape[0]
    kw = words_per_row(K)
    nw = words_per_row(N)
    if A.shape[1] < kw or B.shape[1] < kw:
        raise ValueError("packed operands have fewer words per row than K needs")
    if thr.dtype != torch.int32 or flip_bits.dtype != torch.int32 or not thr.is_cuda or not flip_bits.is_cuda:
        raise ValueError("thr and flip_bits must be int32 device tensors")
    if thr.numel() != N or flip_bits.numel() != nw or not thr.is_contiguous() or not flip_bits.is_contiguous():
        raise ValueError("thr must be [N] and flip_bits [ceil(N/32)], contiguous")
    if out is None:
        out = _alloc_words(M, nw, A.device, ld_out)
    _dev(out, torch.int32, "out")
    if kernel == KERNEL_AUTO:
        st = lib.bnn_xnor_gemm_bn_sign_pack(A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), M, N, K, thr.data_ptr(),
                                            flip_bits.data_ptr(), out.data_ptr(), _ld(out), _stream(out))
    else:
        st = lib.bnn_xnor_gemm_bn_sign_pack_kernel(A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), M, N, K,
                                                   thr.data_ptr(), flip_bits.data_ptr(), out.data_ptr(),
                                                   _ld(out), kernel, _stream(out))
    _check("bnn_xnor_gemm_bn_sign_pack", st)
    return out


def pack_bitplanes(x: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """bnn_pack_bitplanes: uint8 [rows][cols] -> packed planes int32 [rows][8*ceil(cols/32)] (word 8*w + p)."""
    lib = load_library()
    _dev(x, torch.uint8, "x")
    rows, cols = x.shape
    kw8 = 8 * words_per_row(cols)
    if out is None:
        out = torch.empty((rows, kw8), dtype=torch.int32, device=x.device)
    _dev(out, torch.int32, "out")
    _check("bnn_pack_bitplanes", lib.bnn_pack_bitplanes(x.data_ptr(), rows, cols, _ld(x), out.data_ptr(), _ld(out),
                                                       _stream(out)))
    return out


def bitplane_gemm(Xp: torch.Tensor, B: torch.Tensor, K: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """bnn_bitplane_gemm: bit planes Xp [M][8*Kw], packed +-1 rows B [N][Kw] -> int32 [M][N] = x @ w^T."""
    lib = load_library()
    _dev(Xp, torch.int32, "Xp")
    _dev(B, torch.int32, "B")
    M, N = Xp.shape[0], B.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=Xp.device)
    _dev(out, torch.int32, "out")
    _check("bnn_bitplane_gemm", lib.bnn_bitplane_gemm(Xp.data_ptr(), _ld(Xp), B.data_ptr(), _ld(B), out.data_ptr(),
                                                     _ld(out), M, N, K, _stream(out)))
    return out


def bitplane_gemm_bn_sign_pack(Xp: torch.Tensor, B: torch.Tensor, K: int, thr: torch.Tensor, flip_bits: torch.Tensor,
                               out: torch.Tensor | None = None, ld_out: int | None = None) -> torch.Tensor:
    """bnn_bitplane_gemm_bn_sign_pack: first layer on 8-bit inputs, fused with Sign(BatchNorm)."""
    lib = load_library()
    _dev(Xp, torch.int32, "Xp")
    _dev(B, torch.int32, "B")
    M, N = Xp.shape[0], B.shape[0]
    nw = words_per_row(N)
    if thr.dtype != torch.int32 or flip_bits.dtype != torch.int32 or not thr.is_cuda or not flip_bits.is_cuda:
        raise ValueError("thr and flip_bits must be int32 device tensors")
    if thr.numel() != N or flip_bits.numel() != nw or not thr.is_contiguous() or not flip_bits.is_contiguous():
        raise ValueError("thr must be [N] and flip_bits [ceil(N/32)], contiguous")
    if out is None:
        out = _alloc_words(M, nw, Xp.device, ld_out)
    _dev(out, torch.int32, "out")
    _check("bnn_bitplane_gemm_bn_sign_pack",
           lib.bnn_bitplane_gemm_bn_sign_pack(Xp.data_ptr(), _ld(Xp), B.data_ptr(), _ld(B), M, N, K,
                                              thr.data_ptr(), flip_bits.data_ptr(), out.data_ptr(), _ld(out),
                                              _stream(out)))
    return out


def conv_im2col_pack(x_bits: torch.Tensor, Cin: int, kh: int = 3, kw: int = 3, stride: int = 1, pad: int = 1,
                     out: torch.Tensor | None = None, ld_out: int | None = None) -> torch.Tensor:
    """bnn_conv_im2col_pack: packed NHWC int32 [B][H][W][ceil(Cin/32)] -> [B*Ho*Wo][ceil(kh*kw*Cin/32)]."""
    lib = load_library()
    if not x_bits.is_cuda or x_bits.dtype != torch.int32 or x_bits.dim() != 4 or not x_bits.is_contiguous():
        raise ValueError("x_bits must be a contiguous int32 device tensor [B][H][W][ceil(Cin/32)]")
    B, H, W, Cw = x_bits.shape
    if Cw != words_per_row(Cin):
        raise ValueError("last dimension does not match Cin")
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    kwords = words_per_row(kh * kw * Cin)
    if out is None:
        out = _alloc_words(B * max(Ho, 0) * max(Wo, 0), kwords, x_bits.device, ld_out)
    _dev(out, torch.int32, "out")
    _check("bnn_conv_im2col_pack",
           lib.bnn_conv_im2col_pack(x_bits.data_ptr(), B, H, W, Cin, kh, kw, stride, pad, out.data_ptr(),
                                    _ld(out), _stream(out)))
    return out


def _check_nhwc_bits(x_bits: torch.Tensor, Cin: int):
    if not x_bits.is_cuda or x_bits.dtype != torch.int32 or x_bits.dim() != 4 or not x_bits.is_contiguous():
        raise ValueError("x_bits must be a contiguous int32 device tensor [B][H][W][ceil(Cin/32)]")
    if x_bits.shape[3] != words_per_row(Cin):
        raise ValueError("last dimension does not match the channel count")


def conv_xnor(x_bits: torch.Tensor, Cin: int, w_bits: torch.Tensor, kh: int = 3, kw: int = 3, stride: int = 1,
              pad: int = 1, out: torch.Tensor | None = None) -> torch.Tensor:
    """bnn_conv_xnor: packed NHWC input, packed filters [Cout][kh*kw*Cin/32] -> int32 [B*Ho*Wo][Cout]."""
    lib = load_library()
    _check_nhwc_bits(x_bits, Cin)
    _dev(w_bits, torch.int32, "w_bits")
    B, H, W, _ = x_bits.shape
    Cout = w_bits.shape[0]
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    if out is None:
        out = torch.empty((B * Ho * Wo, Cout), dtype=torch.int32, device=x_bits.device)
    _dev(out, torch.int32, "out")
    _check("bnn_conv_xnor", lib.bnn_conv_xnor(x_bits.data_ptr(), B, H, W, Cin, w_bits.data_ptr(), _ld(w_bits), Cout,
                                             kh, kw, stride, pad, out.data_ptr(), _ld(out), _stream(out)))
    return out


def conv_bn_sign_pack(x_bits: torch.Tensor, Cin: int, w_bits: torch.Tensor, thr: torch.Tensor,
                      flip_bits: torch.Tensor, kh: int = 3, kw: int = 3, stride: int = 1, pad: int = 1,
                      out: torch.Tensor | None = None) -> torch.Tensor:
    """bnn_conv_bn_sign_pack: binary conv + Sign(BatchNorm) -> packed bits [B*Ho*Wo][ceil(Cout/32)]."""
    lib = load_library()
    _check_nhwc_bits(x_bits, Cin)
    _dev(w_bits, torch.int32, "w_bits")
    B, H, W, _ = x_bits.shape
    Cout = w_bits.shape[0]
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    nw = words_per_row(Cout)
    if thr.dtype != torch.int32 or flip_bits.dtype != torch.int32 or not thr.is_cuda or not flip_bits.is_cuda:
        raise ValueError("thr and flip_bits must be int32 device tensors")
    if thr.numel() != Cout or flip_bits.numel() != nw or not thr.is_contiguous() or not flip_bits.is_contiguous():
        raise ValueError("thr must be [Cout] and flip_bits [ceil(Cout/32)], contiguous")
    if out is None:
        out = torch.empty((B * Ho * Wo, nw), dtype=torch.int32, device=x_bits.device)
    _dev(out, torch.int32, "out")
    _check("bnn_conv_bn_sign_pack",
           lib.bnn_conv_bn_sign_pack(x_bits.data_ptr(), B, H, W, Cin, w_bits.data_ptr(), _ld(w_bits), Cout, kh, kw,
                                     stride, pad, thr.data_ptr(), flip_bits.data_ptr(), out.data_ptr(), _ld(out),
                                     _stream(out)))
    return out


def conv_pool_bn_sign_pack(x_bits: torch.Tensor, Cin: int, w_bits: torch.Tensor, thr: torch.Tensor,
                           flip_bits: torch.Tensor, kh: int = 3, kw: int = 3, stride: int = 1, pad: int = 1,
                           pool: int = 2, out: torch.Tensor | None = None) -> torch.Tensor:
    """bnn_conv_pool_bn_sign_pack: binary conv + max pooling + Sign(BatchNorm) in one launch ->
    packed bits [B*(Ho/pool)*(Wo/pool)][ceil(Cout/32)].  Raises BnnError with status 3 (unsupported)
    for geometries the fused kernel does not take."""
    lib = load_library()
    _check_nhwc_bits(x_bits, Cin)
    _dev(w_bits, torch.int32, "w_bits")
    B, H, W, _ = x_bits.shape
    Cout = w_bits.shape[0]
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
    nw = words_per_row(Cout)
    if thr.dtype != torch.int32 or flip_bits.dtype != torch.int32 or not thr.is_cuda or not flip_bits.is_cuda:
        raise ValueError("thr and flip_bits must be int32 device tensors")
    if thr.numel() != Cout or flip_bits.numel() != nw or not thr.is_contiguous() or not flip_bits.is_contiguous():
        raise ValueError("thr must be [Cout] and flip_bits [ceil(Cout/32)], contiguous")
    if pool < 1:
        raise ValueError("pool must be positive")
    if out is None:
        out = torch.empty((B * (Ho // pool) * (Wo // pool), nw), dtype=torch.int32, device=x_bits.device)
    _dev(out, torch.int32, "out")
    if out.shape[0] != B * (Ho // pool) * (Wo // pool) or out.shape[1] != nw:
        raise ValueError("out must be [B*(Ho/pool)*(Wo/pool)][ceil(Cout/32)]")
    _check("bnn_conv_pool_bn_sign_pack",
           lib.bnn_conv_pool_bn_sign_pack(x_bits.data_ptr(), B, H, W, Cin, w_bits.data_ptr(), _ld(w_bits), Cout, kh,
                                          kw, stride, pad, pool, thr.data_ptr(), flip_bits.data_ptr(),
                                          out.data_ptr(), _ld(out), _stream(out)))
    return out


def maxpool_bits(x_bits: torch.Tensor, C: int, flip_bits: torch.Tensor | None, ph: int = 2, pw: int = 2,
                 stride: int = 2, out: torch.Tensor | None = None) -> torch.Tensor:
    """bnn_maxpool_bits: packed NHWC [B][H][W][Cw] -> [B][Hp][Wp][Cw]; OR where flip = 0, AND where flip = 1."""
    lib = load_library()
    _check_nhwc_bits(x_bits, C)
    B, H, W, Cw = x_bits.shape
    Hp, Wp = (H - ph) // stride + 1, (W - pw) // stride + 1
    if flip_bits is not None and (flip_bits.dtype != torch.int32 or not flip_bits.is_cuda or
                                  flip_bits.numel() != Cw or not flip_bits.is_contiguous()):
        raise ValueError("flip_bits must be a contiguous int32 device tensor [ceil(C/32)]")
    if out is None:
        out = torch.empty((B, Hp, Wp, Cw), dtype=torch.int32, device=x_bits.device)
    if not out.is_cuda or out.dtype != torch.int32 or not out.is_contiguous() or out.numel() != B * Hp * Wp * Cw:
        raise ValueError("out must be a contiguous int32 device tensor [B][Hp][Wp][Cw]")
    _check("bnn_maxpool_bits", lib.bnn_maxpool_bits(x_bits.data_ptr(), B, H, W, C, ph, pw, stride,
                                                   flip_bits.data_ptr() if flip_bits is not None else None,
                                                   out.data_ptr(), _stream(out)))
    return out


def gemm_i8_mfma(A: torch.Tensor, B: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """bnn_gemm_i8_mfma: int8 A [M][K], int8 B [N][K] -> int32 C [M][N]."""
    lib = load_library()
    _dev(A, torch.int8, "A")
    _dev(B, torch.int8, "B")
    M, K = A.shape
    N, K2 = B.shape
    if K != K2:
        raise ValueError("A and B disagree on K")
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _dev(out, torch.int32, "out")
    _check("bnn_gemm_i8_mfma", lib.bnn_gemm_i8_mfma(A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), out.data_ptr(),
                                                   _ld(out), M, N, K, _stream(out)))
    return out


def unpack_i8(bits: torch.Tensor, K: int, ld_out: int | None = None) -> torch.Tensor:
    """bnn_unpack_i8: packed rows -> int8 +-1 [rows][K] (row stride ld_out, default K rounded up to 16)."""
    lib = load_library()
    _dev(bits, torch.int32, "bits")
    rows = bits.shape[0]
    ld = ld_out if ld_out is not None else (K + 15) // 16 * 16
    buf = torch.empty((rows, ld), dtype=torch.int8, device=bits.device)
    _check("bnn_unpack_i8", lib.bnn_unpack_i8(bits.data_ptr(), _ld(bits), rows, K, buf.data_ptr(), ld, _stream(buf)))
    return buf[:, :K] if ld != K else buf
