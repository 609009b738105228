"""MI355X-native forward hot path of Binarized Neural Networks.

A thin Python face over ``libbnn_hip.so`` (hand-written HIP for gfx950 behind a
C ABI declared in ``include/bnn.h``).  The functions here only marshal
arguments: device memory and streams come from PyTorch, every step of the path
runs in the library's kernels.  There is no CPU fallback: if the library is not
built or a call fails, an exception is raised.
"""
from .binding import (  # noqa: F401
    BnnError,
    lib_path,
    load_library,
    version,
    words_per_row,
    pack_sign,
    xnor_gemm,
    bn_fold,
    bn_sign_pack,
    xnor_gemm_bn_sign_pack,
    conv_im2col_pack,
    conv_xnor,
    conv_bn_sign_pack,
    conv_pool_bn_sign_pack,
    maxpool_bits,
    pack_bitplanes,
    bitplane_gemm,
    bitplane_gemm_bn_sign_pack,
    gemm_i8_mfma,
    unpack_i8,
    KERNEL_AUTO,
    KERNEL_NAIVE,
    KERNEL_TILED128,
    KERNEL_KSPLIT,
    KERNEL_TILED64,
    KERNEL_MFMA,
    KERNEL_MFMA128,
    KERNEL_MFMA_SHORTK,
    KERNEL_MFMA_PERSIST,
    KERNEL_MFMA_BIG,
    KERNEL_MFMA_SPLITK,
)
from .network import BinaryMLP, BinaryConvLayer, BinaryConvNet  # noqa: F401
