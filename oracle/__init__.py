"""CPU oracle for the binarized-network forward path (test infrastructure only).

Nothing in the product package may import this; only ``tests/``, the smoke
check and the benchmark's ``cpu_baseline`` leg do.  The arithmetic lives in
``bnn_oracle.c`` (plain C, literal +1/-1 integer arithmetic, float32
BatchNorm); this package is a ctypes/numpy wrapper plus the per-network
drivers that chain those steps in the order of Alg. 4 of the paper.
"""
from .bnn_oracle import (  # noqa: F401
    build,
    num_threads,
    sign,
    matmul_pm1,
    bn_float,
    bn_sign,
    pack_bits,
    unpack_bits,
    conv_direct,
    im2col,
    first_layer_bitplanes,
    dense_layer,
    mlp_forward,
    mlp_forward_uint8,
    conv_layer,
    conv_pool_layer,
    maxpool2d,
    EPS_DEFAULT,
)
