"""ctypes/numpy wrapper around ``bnn_oracle.c`` and the network drivers.

TEST INFRASTRUCTURE ONLY: the GPU library never imports or links this.

Array conventions (all numpy, C-contiguous, host memory):
  * +-1 values are ``int8``;
  * a dense weight matrix is given in the math layout ``Bm[K][N]`` of
    ``s = a W`` (Alg. 1 forward pass / Alg. 4 of the paper);
  * feature maps are NHWC, conv weights ``[Cout][kh][kw][Cin]``;
  * packed words are ``uint32``, bit = 1 <=> +1, element k in word k//32 at
    bit k%32, pad bits zero (Sec. 4 fixes only "32 variables per word"; the
    polarity and order are this build's declared convention).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bnn_oracle.c")
_LIB = os.path.join(_HERE, "libbnn_oracle.so")

# The paper never states BatchNorm's epsilon; this build reads it as 1e-4.
EPS_DEFAULT = 1e-4

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle into ``libbnn_oracle.so`` next to its source."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O3", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-std=c99", "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    """Loads the oracle library, building it first.  BNN_ORACLE_LIB names another build of it to load
    instead: the mutation tests use that to check that the pins reject a deliberately broken oracle."""
    global _lib
    if _lib is None:
        override = os.environ.get("BNN_ORACLE_LIB")
        if override:
            _lib = ctypes.CDLL(override)
        else:
            build()
            _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


_i64 = ctypes.c_int64


def num_threads() -> int:
    lib = _load()
    lib.oracle_num_threads.restype = ctypes.c_int
    return int(lib.oracle_num_threads())


def sign(x: np.ndarray) -> np.ndarray:
    """Eq. (1): +1 where x >= 0, else -1.  Returns int8 of x's shape."""
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.int8)
    _load().oracle_sign(_p(x), _i64(x.size), _p(out))
    return out


def matmul_pm1(A: np.ndarray, Bm: np.ndarray) -> np.ndarray:
    """Literal +-1 integer product: A[M][K] @ Bm[K][N] -> int32 [M][N]."""
    A = _c(A, np.int8)
    Bm = _c(Bm, np.int8)
    M, K = A.shape
    K2, N = Bm.shape
    assert K == K2
    C = np.empty((M, N), np.int32)
    _load().oracle_matmul_pm1(_p(A), _p(Bm), _p(C), _i64(M), _i64(N), _i64(K))
    return C


def _bn_args(N, gamma, beta, mean, var):
    arrs = [_c(a, np.float32) for a in (gamma, beta, mean, var)]
    for a in arrs:
        assert a.shape == (N,)
    return arrs


def bn_float(S, gamma, beta, mean, var, eps=EPS_DEFAULT) -> np.ndarray:
    """Inference BatchNorm per column, float32: gamma*((s-mean)/sqrt(var+eps))+beta."""
    S = _c(S, np.int32)
    M, N = S.shape
    g, b, mu, v = _bn_args(N, gamma, beta, mean, var)
    Y = np.empty((M, N), np.float32)
    _load().oracle_bn_float(_p(S), _i64(M), _i64(N), _p(g), _p(b), _p(mu), _p(v),
                            ctypes.c_float(eps), _p(Y))
    return Y


def bn_sign(S, gamma, beta, mean, var, eps=EPS_DEFAULT) -> np.ndarray:
    """Alg. 4: Sign(BatchNorm(s)) per column, as int8 +-1."""
    S = _c(S, np.int32)
    M, N = S.shape
    g, b, mu, v = _bn_args(N, gamma, beta, mean, var)
    out = np.empty((M, N), np.int8)
    _load().oracle_bn_sign(_p(S), _i64(M), _i64(N), _p(g), _p(b), _p(mu), _p(v),
                           ctypes.c_float(eps), _p(out))
    return out


def pack_bits(v: np.ndarray) -> np.ndarray:
    """int8 +-1 [rows][cols] -> uint32 [rows][ceil(cols/32)]."""
    v = _c(v, np.int8)
    rows, cols = v.shape
    words = np.empty((rows, (cols + 31) // 32), np.uint32)
    _load().oracle_pack_bits(_p(v), _i64(rows), _i64(cols), _p(words))
    return words


def unpack_bits(words: np.ndarray, cols: int) -> np.ndarray:
    """uint32 [rows][ceil(cols/32)] -> int8 +-1 [rows][cols] (pad bits ignored)."""
    words = _c(words, np.uint32)
    rows, kw = words.shape
    assert kw == (cols + 31) // 32
    v = np.empty((rows, cols), np.int8)
    _load().oracle_unpack_bits(_p(words), _i64(rows), _i64(cols), _p(v))
    return v


def conv_out_size(H, W, kh, kw, stride, pad):
    return (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1


def conv_direct(x, Wt, stride=1, pad=1) -> np.ndarray:
    """Direct +-1 convolution, out-of-image inputs = +1.

    x: int8 [B][H][W][Cin]; Wt: int8 [Cout][kh][kw][Cin] -> int32 [B][Ho][Wo][Cout].
    """
    x = _c(x, np.int8)
    Wt = _c(Wt, np.int8)
    B, H, W, Cin = x.shape
    Cout, kh, kw, Cin2 = Wt.shape
    assert Cin == Cin2
    Ho, Wo = conv_out_size(H, W, kh, kw, stride, pad)
    S = np.empty((B, Ho, Wo, Cout), np.int32)
    _load().oracle_conv_direct(_p(x), _i64(B), _i64(H), _i64(W), _i64(Cin), _p(Wt),
                               _i64(Cout), _i64(kh), _i64(kw), _i64(stride), _i64(pad),
                               _p(S))
    return S


def im2col(x, kh=3, kw=3, stride=1, pad=1) -> np.ndarray:
    """Receptive-field matrix int8 [B*Ho*Wo][kh*kw*Cin], K index (ky*kw+kx)*Cin+ci."""
    x = _c(x, np.int8)
    B, H, W, Cin = x.shape
    Ho, Wo = conv_out_size(H, W, kh, kw, stride, pad)
    cols = np.empty((B * Ho * Wo, kh * kw * Cin), np.int8)
    _load().oracle_im2col(_p(x), _i64(B), _i64(H), _i64(W), _i64(Cin), _i64(kh),
                          _i64(kw), _i64(stride), _i64(pad), _p(cols))
    return cols


def maxpool2d(S, ph=2, pw=2, stride=2) -> np.ndarray:
    """Window maximum of int32 maps [B][H][W][C] -> [B][Hp][Wp][C], no padding."""
    S = _c(S, np.int32)
    B, H, W, C = S.shape
    Hp, Wp = (H - ph) // stride + 1, (W - pw) // stride + 1
    P = np.empty((B, Hp, Wp, C), np.int32)
    _load().oracle_maxpool2d(_p(S), _i64(B), _i64(H), _i64(W), _i64(C), _i64(ph), _i64(pw), _i64(stride), _p(P))
    return P


def first_layer_bitplanes(X, Wb) -> np.ndarray:
    """Sec. 1.6 / Alg. 4 step 1: uint8 X[M][K], +-1 Wb[K][N] -> sum_p 2^(p-1) <x^p, w>."""
    X = _c(X, np.uint8)
    Wb = _c(Wb, np.int8)
    M, K = X.shape
    K2, N = Wb.shape
    assert K == K2
    S = np.empty((M, N), np.int32)
    _load().oracle_first_layer_bitplanes(_p(X), _p(Wb), _p(S), _i64(M), _i64(N), _i64(K))
    return S


# --------------------------------------------------------------------------
# Drivers: the steps above chained in the order of Alg. 4.
# --------------------------------------------------------------------------

def dense_layer(a_b, Wb, bn, eps=EPS_DEFAULT):
    """One hidden layer of Alg. 4: s = a^b W^b; a^b_next = Sign(BatchNorm(s)).

    Returns (s int32 [M][N], a^b_next int8 [M][N]).  ``bn`` = (gamma, beta, mean, var).
    """
    s = matmul_pm1(a_b, Wb)
    return s, bn_sign(s, *bn, eps=eps)


def mlp_forward(x_real, weights, bns, eps=EPS_DEFAULT):
    """Fully binarized MLP: Sign on the real input, hidden layers of Alg. 4,
    last layer emits the int32 pre-activations.

    weights: list of int8 Bm[K_l][N_l]; bns: one (gamma,beta,mean,var) per hidden layer.
    Returns dict with per-layer 's' (int32) and 'a' (int8 +-1, a[0] = Sign(x)).
    """
    assert len(bns) == len(weights) - 1
    a = sign(x_real)
    trace = {"a": [a], "s": []}
    for l, Wb in enumerate(weights):
        s = matmul_pm1(a, Wb)
        trace["s"].append(s)
        if l < len(bns):
            a = bn_sign(s, *bns[l], eps=eps)
            trace["a"].append(a)
    return trace


def mlp_forward_uint8(x_u8, weights, bns, eps=EPS_DEFAULT):
    """Alg. 4 as printed: 8-bit inputs, first layer as the sum over bit planes weighted 2^(n-1)
    (step 1), hidden layers XnorDotProduct -> Sign(BatchNorm) (step 2), last layer's int32
    pre-activations.  Same return structure as mlp_forward; a[0] is the raw uint8 input."""
    assert len(bns) == len(weights) - 1
    trace = {"a": [np.asarray(x_u8)], "s": []}
    a = None
    for l, Wb in enumerate(weights):
        s = first_layer_bitplanes(x_u8, Wb) if l == 0 else matmul_pm1(a, Wb)
        trace["s"].append(s)
        if l < len(bns):
            a = bn_sign(s, *bns[l], eps=eps)
            trace["a"].append(a)
    return trace


def conv_pool_layer(x_b, Wt, bn, pool=2, stride=1, pad=1, eps=EPS_DEFAULT):
    """Binary conv layer with max pooling in the paper's order: convolution, max pooling of the
    pre-activations, BatchNorm, Sign.  Returns (pooled S int32, a^b int8), both [B][Hp][Wp][Cout]."""
    S = conv_direct(x_b, Wt, stride=stride, pad=pad)
    P = maxpool2d(S, pool, pool, pool)
    B, Hp, Wp, Cout = P.shape
    a = bn_sign(P.reshape(-1, Cout), *bn, eps=eps).reshape(B, Hp, Wp, Cout)
    return P, a


def conv_layer(x_b, Wt, bn, stride=1, pad=1, eps=EPS_DEFAULT):
    """Binary conv layer: direct convolution, then Sign(BatchNorm) per output channel.

    Returns (S int32 [B][Ho][Wo][Cout], a^b int8 same shape).
    """
    S = conv_direct(x_b, Wt, stride=stride, pad=pad)
    B, Ho, Wo, Cout = S.shape
    a = bn_sign(S.reshape(-1, Cout), *bn, eps=eps).reshape(B, Ho, Wo, Cout)
    return S, a
