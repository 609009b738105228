"""Seeded synthetic inputs for the five workloads (shared by oracle and GPU tests).

This module only draws numbers: it holds none of the method's arithmetic (no
Sign, no packing, no product, no BatchNorm).  Both the CPU oracle and the GPU
path receive the arrays it returns.

The inputs stand in, by shape only, for what the paper runs on: the 784-input,
10-class, 10 000-image MNIST test set with a 3 x 4096 binary MLP (Sec. 2.1),
32 x 32 images (Sec. 2.2, 2.3) through 3 x 3 binary convolutions (Sec. 3.3) and the
8192 x 8192 x 8192 binary matrix product of Sec. 4 / Fig. 3.  No item of any
dataset is used or needed.

Seeds: ``SEED_BASE + 1000 * config_index + tensor_index``.
Distributions:
  * +-1 tensors: i.i.d., P(+1) = p (0.5 unless a case says otherwise), int8;
  * real inputs: N(0, 1) float32;
  * BatchNorm per channel, for a layer with fan-in K:
      gamma ~ N(1, 0.1^2), beta ~ N(0, 0.1^2), running mean ~ N(0, (sqrt(K)/4)^2),
      running var = K * U(0.5, 1.5); ``adversarial=True`` flips the sign of
      gamma on ~10 % of the channels and zeroes it on ~1 %.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 160202830

MLP_SIZES = (784, 4096, 4096, 4096, 10)       # Sec. 2.1 architecture
MLP_BATCH = 10000                             # size of the test set of Sec. 2.1
CONV_LAYERS = (                               # (Cin=Cout, H=W) of a VGG-like binary net
    (128, 32),
    (256, 16),
    (512, 8),
)
CONV_BATCH = 256
GEMM_LARGE = 8192                             # Sec. 4, Fig. 3

RAGGED_MN = (1, 7, 33, 1000)
RAGGED_K = (1, 31, 32, 33, 63, 65, 4097)
RAGGED_P = (0.05, 0.5, 0.95)


def seed_for(config_index: int, tensor_index: int) -> int:
    return SEED_BASE + 1000 * config_index + tensor_index


def rng_for(config_index: int, tensor_index: int) -> np.random.Generator:
    return np.random.default_rng(seed_for(config_index, tensor_index))


def pm1(rng: np.random.Generator, shape, p: float = 0.5) -> np.ndarray:
    """i.i.d. +-1 int8 tensor with P(+1) = p."""
    return np.where(rng.random(shape) < p, 1, -1).astype(np.int8)


def real_input(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(shape, dtype=np.float32)


def uint8_input(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.integers(0, 256, size=shape, dtype=np.uint8)


def bn_params(rng: np.random.Generator, N: int, K: int, adversarial: bool = False):
    """(gamma, beta, mean, var) float32 [N] for a layer of fan-in K."""
    gamma = (1.0 + 0.1 * rng.standard_normal(N)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(N)).astype(np.float32)
    mean = ((np.sqrt(K) / 4.0) * rng.standard_normal(N)).astype(np.float32)
    var = (K * rng.uniform(0.5, 1.5, N)).astype(np.float32)
    if adversarial:
        u = rng.random(N)
        gamma = np.where(u < 0.10, -gamma, gamma).astype(np.float32)
        gamma = np.where(u > 0.99, 0.0, gamma).astype(np.float32)
    return gamma, beta, mean, var


# -- config 0: one binary dense layer ---------------------------------------

def config_dense(M: int = 64, K: int = 1024, N: int = 1024, adversarial: bool = False):
    """A[M][K], Bm[K][N] +-1 and the layer's BatchNorm parameters."""
    A = pm1(rng_for(0, 0), (M, K))
    Bm = pm1(rng_for(0, 1), (K, N))
    bn = bn_params(rng_for(0, 2 + int(adversarial)), N, K, adversarial)
    return A, Bm, bn


# -- config 1: MNIST-shaped MLP ---------------------------------------------

def config_mlp(batch: int = MLP_BATCH, sizes=MLP_SIZES, adversarial: bool = False):
    """Real input x[batch][sizes[0]], +-1 weights Bm_l[K_l][N_l], BN per hidden layer."""
    x = real_input(rng_for(1, 0), (batch, sizes[0]))
    weights = [pm1(rng_for(1, 10 + l), (sizes[l], sizes[l + 1]))
               for l in range(len(sizes) - 1)]
    bns = [bn_params(rng_for(1, 20 + l), sizes[l + 1], sizes[l], adversarial)
           for l in range(len(sizes) - 2)]
    return x, weights, bns


# -- config 2: ragged GEMM shapes -------------------------------------------

def ragged_cases():
    """All (M, N, K, p) of the ragged sweep, in a fixed order."""
    return [(M, N, K, p) for M in RAGGED_MN for N in RAGGED_MN
            for K in RAGGED_K for p in RAGGED_P]


def config_ragged(case_index: int):
    M, N, K, p = ragged_cases()[case_index]
    A = pm1(rng_for(2, 2 * case_index), (M, K), p)
    Bm = pm1(rng_for(2, 2 * case_index + 1), (K, N), p)
    return A, Bm


# -- config 3: binary conv layers -------------------------------------------

def config_conv(layer: int, batch: int = CONV_BATCH, channels: int | None = None,
                size: int | None = None, adversarial: bool = False):
    """x[B][H][W][Cin] +-1, Wt[Cout][3][3][Cin] +-1, BN over Cout with K = 9 Cin."""
    C, HW = CONV_LAYERS[layer]
    C = channels or C
    HW = size or HW
    x = pm1(rng_for(3, 10 * layer), (batch, HW, HW, C))
    Wt = pm1(rng_for(3, 10 * layer + 1), (C, 3, 3, C))
    bn = bn_params(rng_for(3, 10 * layer + 2), C, 9 * C, adversarial)
    return x, Wt, bn


# The binary body of the CIFAR-10 / SVHN ConvNet.  Sec. 2.2 does not print the layer list: it says the
# architecture is that of the BinaryConnect ConvNet it cites.  This build reads that cited architecture
# as: after the first convolution (which sees the real-valued image) come 128C3 - MP2 - 256C3 - 256C3 -
# MP2 - 512C3 - 512C3 - MP2 - 1024FC - 1024FC - 10, all on +-1 activations.  (Cin, Cout, H = W, pooled)
CONVNET_CONVS = ((128, 128, 32, True), (128, 256, 16, False), (256, 256, 16, True),
                 (256, 512, 8, False), (512, 512, 8, True))
CONVNET_FCS = (4 * 4 * 512, 1024, 1024, 10)


def config_convnet(batch: int = CONV_BATCH, adversarial: bool = False):
    """x[B][32][32][128] +-1 (the first layer's output bits), conv filters Wt_l[Cout][3][3][Cin] with
    BN over Cout, dense weights Bm_l[K][N] with BN for the two hidden dense layers."""
    x = pm1(rng_for(5, 0), (batch, 32, 32, 128))
    convs = []
    for l, (cin, cout, _hw, _pool) in enumerate(CONVNET_CONVS):
        Wt = pm1(rng_for(5, 10 + 2 * l), (cout, 3, 3, cin))
        convs.append((Wt, bn_params(rng_for(5, 11 + 2 * l), cout, 9 * cin, adversarial)))
    fcs = [pm1(rng_for(5, 40 + l), (CONVNET_FCS[l], CONVNET_FCS[l + 1])) for l in range(3)]
    fc_bns = [bn_params(rng_for(5, 50 + l), CONVNET_FCS[l + 1], CONVNET_FCS[l], adversarial) for l in range(2)]
    return x, convs, fcs, fc_bns


# -- config 4: large square GEMM --------------------------------------------

def config_gemm_square(n: int = GEMM_LARGE):
    A = pm1(rng_for(4, 0), (n, n))
    Bm = pm1(rng_for(4, 1), (n, n))
    return A, Bm


def hadamard(n: int) -> np.ndarray:
    """Sylvester matrix H[i][j] = (-1)^popcount(i & j), n a power of two, int8."""
    assert n > 0 and n & (n - 1) == 0
    H = np.ones((1, 1), np.int8)
    while H.shape[0] < n:
        H = np.block([[H, H], [H, -H]]).astype(np.int8)
    return H
