"""CPU-only tests of the product's host side: the C-ABI library loads without a
GPU, exports what include/bnn.h declares, validates arguments before touching
the device, and its BatchNorm fold agrees with the oracle's float BatchNorm+Sign
on every admissible pre-activation."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_1602_02830_amd as bnn
from paper_1602_02830_amd import binding
from workloads import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# tests/test_sanitizers.py runs the fold and size-helper tests of this file in a child process against a
# build of the library's host-only sources (bn_fold.cpp, api.cpp) under AddressSanitizer and
# UndefinedBehaviorSanitizer; BNN_HOST_LIB names that build, which exports only the host functions.
_HOST_LIB = os.environ.get("BNN_HOST_LIB")
if _HOST_LIB:
    _lib = ctypes.CDLL(_HOST_LIB)
    for _name in ("bnn_version", "bnn_status_string", "bnn_words_per_row", "bnn_bn_fold"):
        getattr(_lib, _name).restype, getattr(_lib, _name).argtypes = binding._SIGNATURES[_name]
    binding._lib = _lib


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "bnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bnn_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = bnn.load_library()
    declared = _declared_symbols()
    assert "bnn_xnor_gemm" in declared and "bnn_pack_sign" in declared
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in bnn.h but not exported"
    assert sorted(binding.exported_symbols()) == declared
    assert bnn.version() == 100
    assert lib.bnn_status_string(1) == b"invalid argument"


def test_words_per_row():
    assert [bnn.words_per_row(k) for k in (0, 1, 31, 32, 33, 784, 4096)] == [0, 1, 1, 1, 2, 25, 128]
    assert bnn.words_per_row(-1) == -1
    # the binding restates the rule; the library's own answer must agree
    lib = binding.load_library()
    for k in (-5, -1, 0, 1, 31, 32, 33, 63, 64, 65, 784, 4097, 2**31 - 2, 2**40 + 1):
        assert lib.bnn_words_per_row(k) == bnn.words_per_row(k)


def test_argument_validation_happens_before_any_launch():
    lib = bnn.load_library()
    buf = (ctypes.c_uint32 * 64)()
    p = ctypes.addressof(buf)
    INVALID, ALIGN = 1, 2
    # negative sizes, short leading dimensions, null pointers, misalignment
    assert lib.bnn_pack_sign(p, -1, 4, 4, p, 1, None) == INVALID
    assert lib.bnn_pack_sign(p, 2, 40, 39, p, 2, None) == INVALID
    assert lib.bnn_pack_sign(p, 2, 40, 40, p, 1, None) == INVALID
    assert lib.bnn_pack_sign(None, 2, 40, 40, p, 2, None) == INVALID
    assert lib.bnn_pack_sign(p + 2, 2, 40, 40, p, 2, None) == ALIGN
    assert lib.bnn_pack_sign(p, 0, 40, 40, p, 2, None) == 0          # empty problem
    assert lib.bnn_xnor_gemm(p, 1, p, 1, p, 4, 4, 4, 33, None) == INVALID      # lda < ceil(K/32)
    assert lib.bnn_xnor_gemm(p, 2, p, 2, p, 3, 4, 4, 33, None) == INVALID      # ldc < N
    assert lib.bnn_xnor_gemm(p, 2, p, 2, p, 4, 4, 4, 2 ** 31 - 1, None) == INVALID
    assert lib.bnn_xnor_gemm(p, 2 ** 26, p, 2 ** 26, p, 4, 4, 4, 2 ** 31 - 31, None) == INVALID   # (K + 31) / 32 must fit 32 bits
    assert lib.bnn_xnor_gemm(None, 2, p, 2, p, 4, 4, 4, 33, None) == INVALID
    assert lib.bnn_xnor_gemm(p, 2, p, 2, p, 4, 0, 4, 33, None) == 0
    assert lib.bnn_xnor_gemm_kernel(p, 2, p, 2, p, 4, 4, 4, 33, 99, None) == INVALID
    assert lib.bnn_xnor_gemm(p, 2, p, 2, p, 4, 2 ** 31 - 100, 4, 33, None) == 3            # rows within a tile of 2^31: unsupported
    assert lib.bnn_bn_sign_pack(p, 3, 4, 4, p, p, p, 1, None) == INVALID
    assert lib.bnn_bn_sign_pack(p, 4, 4, 4, None, p, p, 1, None) == INVALID
    assert lib.bnn_conv_im2col_pack(p, 1, 4, 4, 32, 3, 3, 0, 1, p, 9, None) == INVALID   # stride 0
    assert lib.bnn_conv_im2col_pack(p, 1, 4, 4, 32, 3, 3, 1, 1, p, 8, None) == INVALID   # ld_out short
    assert lib.bnn_conv_im2col_pack(p, 1, 1, 1, 32, 3, 3, 1, 0, p, 9, None) == INVALID   # no output pixel
    assert lib.bnn_gemm_i8_mfma(p, 16, p, 16, p, 4, 4, 4, 17, None) == INVALID           # lda < K
    assert lib.bnn_gemm_i8_mfma(p, 24, p, 32, p, 4, 4, 4, 17, None) == ALIGN             # lda % 16
    assert lib.bnn_unpack_i8(p, 1, 2, 33, p, 36, None) == INVALID


def test_argument_validation_of_the_fused_bitplane_and_conv_entry_points():
    lib = bnn.load_library()
    buf = (ctypes.c_uint32 * 64)()
    p = ctypes.addressof(buf)
    INVALID, ALIGN, UNSUPPORTED = 1, 2, 3
    # fused hidden layer: short leading dimensions, null thresholds, unknown kernel id, empty problem
    assert lib.bnn_xnor_gemm_bn_sign_pack(p, 1, p, 2, 4, 4, 33, p, p, p, 1, None) == INVALID     # lda < ceil(K/32)
    assert lib.bnn_xnor_gemm_bn_sign_pack(p, 2, p, 2, 4, 40, 33, p, p, p, 1, None) == INVALID    # ld_out < ceil(N/32)
    assert lib.bnn_xnor_gemm_bn_sign_pack(p, 2, p, 2, 4, 4, 33, None, p, p, 1, None) == INVALID
    assert lib.bnn_xnor_gemm_bn_sign_pack(p, 2, p, 2, 4, 4, 33, p, p, p + 2, 1, None) == ALIGN
    assert lib.bnn_xnor_gemm_bn_sign_pack(p, 2, p, 2, 0, 4, 33, p, p, p, 1, None) == 0
    assert lib.bnn_xnor_gemm_bn_sign_pack_kernel(p, 2, p, 2, 4, 4, 33, p, p, p, 1, 3, None) == INVALID   # no fused K-split
    assert lib.bnn_xnor_gemm_bn_sign_pack_kernel(p, 2, p, 2, 4, 4, 33, p, p, p, 1, 99, None) == INVALID
    # kernel 9 (256 x 256 tiles, fused product only) refuses, launching nothing: the int32 product; K not a
    # multiple of 512; N / 256 = 3 column tiles, which do not divide the compute units; strips under 256 rows
    assert lib.bnn_xnor_gemm_kernel(p, 128, p, 128, p, 4096, 10000, 4096, 4096, 9, None) == UNSUPPORTED
    assert lib.bnn_xnor_gemm_bn_sign_pack_kernel(p, 128, p, 128, 10000, 4096, 4000, p, p, p, 128, 9, None) == UNSUPPORTED
    assert lib.bnn_xnor_gemm_bn_sign_pack_kernel(p, 128, p, 128, 10000, 768, 4096, p, p, p, 24, 9, None) == UNSUPPORTED
    assert lib.bnn_xnor_gemm_bn_sign_pack_kernel(p, 128, p, 128, 4000, 4096, 4096, p, p, p, 128, 9, None) == UNSUPPORTED
    assert lib.bnn_xnor_gemm_bn_sign_pack_kernel(p, 128, p, 128, 10000, 4096, 4096, p, p, p, 129, 9, None) == UNSUPPORTED  # ld_out odd
    # kernel id 10: K a multiple of 128, rows that allow 16-byte loads
    assert lib.bnn_xnor_gemm_kernel(p, 32, p, 32, p, 64, 64, 64, 1000, 10, None) == UNSUPPORTED
    assert lib.bnn_xnor_gemm_kernel(p, 34, p, 34, p, 64, 64, 64, 1024, 10, None) == UNSUPPORTED
    assert lib.bnn_xnor_gemm_bn_sign_pack_kernel(p, 32, p, 32, 64, 64, 1000, p, p, p, 2, 10, None) == UNSUPPORTED
    assert lib.bnn_xnor_gemm_bn_sign_pack_kernel(p, 34, p, 34, 64, 64, 1024, p, p, p, 2, 10, None) == UNSUPPORTED
    assert lib.bnn_xnor_gemm_kernel(p, 32, p, 32, p, 64, 64, 64, 1024, 11, None) == INVALID
    # 8-bit first layer: a row holds 8 words per K-word
    assert lib.bnn_pack_bitplanes(p, -1, 4, 4, p, 8, None) == INVALID
    assert lib.bnn_pack_bitplanes(p, 2, 40, 40, p, 15, None) == INVALID                           # ld_out < 8 * ceil(cols/32)
    assert lib.bnn_pack_bitplanes(p, 2, 40, 39, p, 16, None) == INVALID                           # ld_x < cols
    assert lib.bnn_pack_bitplanes(p, 0, 40, 40, p, 16, None) == 0
    assert lib.bnn_bitplane_gemm(p, 15, p, 2, p, 4, 4, 4, 33, None) == INVALID                    # ldx < 8 * ceil(K/32)
    assert lib.bnn_bitplane_gemm(p, 16, p, 2, p, 3, 4, 4, 33, None) == INVALID                    # ldc < N
    assert lib.bnn_bitplane_gemm(p, 16, p, 2, p, 4, 0, 4, 33, None) == 0
    assert lib.bnn_bitplane_gemm(p, 8 * 2 ** 19, p, 2 ** 19, p, 4, 4, 4, 2 ** 24, None) == INVALID       # 255 K beyond int32
    assert lib.bnn_bitplane_gemm_bn_sign_pack(p, 16, p, 2, 4, 4, 33, None, p, p, 1, None) == INVALID
    # implicit-GEMM convolution: geometry, leading dimensions, channel granularity
    assert lib.bnn_conv_xnor(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 0, 1, p, 4, None) == INVALID        # stride 0
    assert lib.bnn_conv_xnor(p, 1, 4, 4, 128, p, 35, 4, 3, 3, 1, 1, p, 4, None) == INVALID        # ldw < 9 * Cin / 32
    assert lib.bnn_conv_xnor(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 1, 1, p, 3, None) == INVALID        # lds < Cout
    assert lib.bnn_conv_xnor(p, 1, 1, 1, 128, p, 36, 4, 3, 3, 1, 0, p, 4, None) == INVALID        # no output pixel
    assert lib.bnn_conv_xnor(p, 1, 4, 4, 48, p, 14, 4, 3, 3, 1, 1, p, 4, None) == UNSUPPORTED     # Cin % 32 != 0
    assert lib.bnn_conv_xnor(p, 1, 4, 4, 64, p, 20, 4, 3, 3, 2, 1, p, 4, None) == UNSUPPORTED     # Cin % 128 != 0 at stride 2
    assert lib.bnn_conv_xnor(p, 1, 4, 4, 64, p, 18, 4, 3, 3, 1, 1, p, 4, None) == UNSUPPORTED     # ... or with ldw % 4 != 0
    assert lib.bnn_conv_xnor(p, 0, 4, 4, 128, p, 36, 4, 3, 3, 1, 1, p, 4, None) == 0
    # output maps or paddings beyond the 15-bit coordinates of the tile loaders are refused, not mis-addressed
    assert lib.bnn_conv_xnor(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 1, 20000, p, 4, None) == UNSUPPORTED   # Ho = 40002
    assert lib.bnn_conv_xnor(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 1, 40000, p, 4, None) == UNSUPPORTED   # pad itself
    assert lib.bnn_conv_bn_sign_pack(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 1, 2 ** 30, p, p, p, 1, None) == UNSUPPORTED
    assert lib.bnn_conv_bn_sign_pack(p, 1, 4, 4, 128, p, 36, 40, 3, 3, 1, 1, p, p, p, 1, None) == INVALID   # ld_out < ceil(Cout/32)
    assert lib.bnn_conv_bn_sign_pack(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 1, 1, None, p, p, 1, None) == INVALID
    # pooled layer in one launch: pool size, output leading dimension, what its tiles cannot hold
    assert lib.bnn_conv_pool_bn_sign_pack(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 1, 1, 0, p, p, p, 1, None) == INVALID
    assert lib.bnn_conv_pool_bn_sign_pack(p, 1, 4, 4, 128, p, 36, 40, 3, 3, 1, 1, 2, p, p, p, 1, None) == INVALID
    assert lib.bnn_conv_pool_bn_sign_pack(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 1, 1, 2, None, p, p, 1, None) == INVALID
    assert lib.bnn_conv_pool_bn_sign_pack(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 1, 1, 3, p, p, p, 1, None) == UNSUPPORTED
    assert lib.bnn_conv_pool_bn_sign_pack(p, 1, 6, 6, 128, p, 36, 4, 3, 3, 1, 1, 2, p, p, p, 1, None) == UNSUPPORTED
    assert lib.bnn_conv_pool_bn_sign_pack(p, 1, 4, 4, 128, p, 36, 4, 3, 3, 2, 1, 2, p, p, p, 1, None) == UNSUPPORTED
    assert lib.bnn_conv_pool_bn_sign_pack(p, 0, 4, 4, 128, p, 36, 4, 3, 3, 1, 1, 2, p, p, p, 1, None) == 0
    # pooling on bits: window larger than the map, zero stride, empty batch
    assert lib.bnn_maxpool_bits(p, 1, 2, 2, 32, 3, 3, 1, None, p, None) == INVALID
    assert lib.bnn_maxpool_bits(p, 1, 4, 4, 32, 2, 2, 0, None, p, None) == INVALID
    assert lib.bnn_maxpool_bits(None, 1, 4, 4, 32, 2, 2, 2, None, p, None) == INVALID
    assert lib.bnn_maxpool_bits(p, 0, 4, 4, 32, 2, 2, 2, None, p, None) == 0


# ------------------------------------------------------------------ bnn_bn_fold

def _fold_matches_oracle_everywhere(bn, K, eps=oracle.EPS_DEFAULT):
    g, b, mu, v = bn
    N = len(g)
    thr, flip = bnn.bn_fold(g, b, mu, v, eps, K)
    assert thr.min() >= -K and thr.max() <= K + 1
    s = np.arange(-K, K + 1, dtype=np.int32)[:, None].repeat(N, 1)       # every integer, not only the lattice
    want = oracle.bn_sign(s, g, b, mu, v, eps=eps) == 1
    flipb = ((flip[np.arange(N) // 32] >> (np.arange(N) % 32)) & 1).astype(bool)
    got = (s >= thr[None, :]) ^ flipb[None, :]
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"first mismatch (s index, channel) = {bad[0]}"
    return thr, flipb


@pytest.mark.parametrize("K,N", [(1, 40), (31, 64), (784, 257), (1024, 1024), (4096, 512)])
def test_fold_equals_float_bn_then_sign_for_every_s(K, N):
    """Alg. 4: Sign(BatchNorm(s)) == (s >= thr) ^ flip for all s in [-K, K], each channel,
    including gamma < 0 and gamma == 0 channels."""
    bn = synth.bn_params(np.random.default_rng(K + N), N, K, adversarial=True)
    thr, flipb = _fold_matches_oracle_everywhere(bn, K)
    g = bn[0]
    assert (flipb[g < 0]).mean() > 0.9           # reversed inequality where gamma < 0 (unless constant)
    assert not flipb[g > 0].any()


def test_fold_rounding_boundary_channels():
    """Channels built so that y(s) crosses zero within one float ulp of an integer s:
    an algebraic threshold would be off by one here."""
    rng = np.random.default_rng(3)
    N, K = 2000, 4096
    g = rng.uniform(0.5, 1.5, N).astype(np.float32) * np.where(rng.random(N) < 0.3, -1, 1).astype(np.float32)
    v = (K * rng.uniform(0.5, 1.5, N)).astype(np.float32)
    t = rng.integers(-50, 50, N).astype(np.float32)
    mu = rng.normal(0, 16, N).astype(np.float32)
    inv = (1.0 / np.sqrt(v.astype(np.float64) + 1e-4))
    b = (-(g.astype(np.float64) * (t - mu) * inv)).astype(np.float32)     # y(t) ~ 0 up to rounding
    _fold_matches_oracle_everywhere((g, b, mu, v), K)


def test_fold_constant_channels_and_extremes():
    K = 64
    g = np.array([0.0, 0.0, 1.0, 1.0, -1.0, -1.0, 1e-30, -0.0], np.float32)
    b = np.array([0.5, -0.5, 1e6, -1e6, 1e6, -1e6, 0.0, 0.0], np.float32)
    mu = np.zeros(8, np.float32)
    v = np.ones(8, np.float32)
    thr, flipb = _fold_matches_oracle_everywhere((g, b, mu, v), K)
    # always-true channels answer 1 for every s, always-false 0
    s = np.array([-K, 0, K])[:, None]
    bits = (s >= thr[None, :]) ^ flipb[None, :]
    assert bits[:, [0, 2, 4]].all() and not bits[:, [1, 3, 5]].any()


def test_fold_rejects_bad_parameters():
    one = np.ones(1, np.float32)
    for bad in (np.nan, np.inf):
        with pytest.raises(bnn.BnnError):
            bnn.bn_fold(one * bad, one, one, one, 1e-4, 16)
    with pytest.raises(bnn.BnnError):
        bnn.bn_fold(one, one, one, -one, 1e-4, 16)          # var + eps <= 0
    with pytest.raises(bnn.BnnError):
        bnn.bn_fold(one, one, one, one, 1e-4, 2 ** 31 - 1)  # K too large


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libbnn_hip.so")
    with pytest.raises(ImportError):
        binding.load_library()
