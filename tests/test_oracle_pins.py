"""Pins for the CPU oracle: it is checked against what the paper and the
mathematics fix, never against itself and never against the GPU path.

Each test names the passage it leans on and the mistake it is meant to catch.
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from workloads import synth


# ---------------------------------------------------------------- Sign, Eq. (1)

def _read_sign_table(golden_dir):
    bits, want = [], []
    with open(os.path.join(golden_dir, "sign_table.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            h, _name, s = line.split()
            bits.append(int(h, 16))
            want.append(int(s))
    return np.array(bits, np.uint32), np.array(want, np.int8)


def test_sign_table_eq1(golden_dir):
    """Eq. (1): zeros, subnormals, infinities, NaN.  Catches sign-bit shortcuts
    (-0.0 must give +1) and flush-to-zero (negative subnormal must give -1)."""
    bits, want = _read_sign_table(golden_dir)
    got = oracle.sign(bits.view(np.float32))
    assert got.tolist() == want.tolist()


def test_sign_matches_inequality_on_random():
    x = synth.real_input(np.random.default_rng(1), (4096,))
    x[::7] = 0.0
    got = oracle.sign(x)
    want = np.where(x.astype(np.float64) >= 0, 1, -1)
    assert (got == want).all()


# ------------------------------------------------- packing convention, Sec. 4

def test_pack_matches_library_packbits():
    """32 variables per 32-bit word, bit=1 <=> +1, LSB-first: the same thing as
    numpy's little-endian packbits viewed as little-endian uint32."""
    rng = np.random.default_rng(2)
    for cols in (1, 5, 31, 32, 33, 64, 100, 257):
        v = synth.pm1(rng, (7, cols), 0.4)
        words = oracle.pack_bits(v)
        kw = (cols + 31) // 32
        bits01 = np.zeros((7, kw * 32), np.uint8)
        bits01[:, :cols] = (v == 1)
        lib = np.packbits(bits01, axis=1, bitorder="little").view("<u4")
        assert words.shape == (7, kw)
        assert (words == lib).all()
        assert (oracle.unpack_bits(words, cols) == v).all()


def test_pack_pad_bits_zero_and_single_bit_positions():
    v = -np.ones((1, 40), np.int8)
    v[0, 0] = 1
    v[0, 33] = 1
    w = oracle.pack_bits(v)
    assert w.tolist() == [[1, 2]]
    allp = np.ones((1, 40), np.int8)
    assert oracle.pack_bits(allp).tolist() == [[0xFFFFFFFF, 0xFF]]


# ------------------------- XNOR-popcount identity (Sec. 4, Eq. (5)) brute force

def _popcount(x: int) -> int:
    return bin(x).count("1")


def test_identity_all_pairs_small_K():
    """For K <= 8 and every pair of K-bit patterns: the literal +-1 dot product
    of the oracle equals 2*popcount(xnor over the K valid bits) - K, and also
    K - 2*popcount(xor).  Catches a wrong polarity, a wrong affine fix-up and a
    transposed operand (B is not symmetric in the enumeration below)."""
    for K in range(1, 9):
        pats = np.arange(2 ** K)
        V = np.where((pats[:, None] >> np.arange(K)[None, :]) & 1, 1, -1).astype(np.int8)
        C = oracle.matmul_pm1(V, np.ascontiguousarray(V[::-1].T))   # column j = pattern 2^K-1-j
        mask = (1 << K) - 1
        for i in range(2 ** K):
            for j in range(2 ** K):
                b = (2 ** K - 1) - j
                xnor = ~(i ^ b) & mask
                assert C[i, j] == 2 * _popcount(xnor) - K == K - 2 * _popcount(i ^ b)


@pytest.mark.parametrize("K", [31, 32, 33, 63, 64, 65, 127, 130])
def test_identity_random_pairs_via_packed_words(K):
    """Same identity on random rows, with the popcount taken over the oracle's own
    packed words (Python big-int popcount): pins packing + product together."""
    rng = np.random.default_rng(K)
    A = synth.pm1(rng, (300, K), 0.3)
    Bt = synth.pm1(rng, (300, K), 0.6)
    C = oracle.matmul_pm1(A, np.ascontiguousarray(Bt.T))
    pa, pb = oracle.pack_bits(A), oracle.pack_bits(Bt)
    for i, j in itertools.product(range(0, 300, 17), range(0, 300, 13)):
        x = sum(_popcount(int(pa[i, w]) ^ int(pb[j, w])) for w in range(pa.shape[1]))
        assert C[i, j] == K - 2 * x


# ------------------------------------------------------- invariants and closed forms

@pytest.mark.parametrize("K", [1, 2, 31, 64, 257])
def test_invariants_bound_and_parity(K):
    rng = np.random.default_rng(100 + K)
    A = synth.pm1(rng, (33, K), 0.5)
    Bm = synth.pm1(rng, (K, 29), 0.5)
    C = oracle.matmul_pm1(A, Bm)
    assert (np.abs(C) <= K).all()
    assert ((C - K) % 2 == 0).all()


def test_closed_forms():
    rng = np.random.default_rng(5)
    K = 200
    A = synth.pm1(rng, (40, K), 0.5)
    assert (np.diag(oracle.matmul_pm1(A, np.ascontiguousarray(A.T))) == K).all()
    assert (np.diag(oracle.matmul_pm1(A, np.ascontiguousarray(-A.T))) == -K).all()
    ones = np.ones((K, 3), np.int8)
    rows = 2 * (A == 1).sum(1) - K
    assert (oracle.matmul_pm1(A, ones) == rows[:, None]).all()


@pytest.mark.parametrize("n", [1, 2, 64, 1024])
def test_hadamard_orthogonality(n):
    """Sylvester matrix: H H^T = n I exactly.  Any dropped or doubled term breaks it."""
    H = synth.hadamard(n)
    i, j = 5 % n, 3 % n
    assert H[i, j] == (-1) ** _popcount(i & j)
    C = oracle.matmul_pm1(H, np.ascontiguousarray(H.T))
    assert (C == n * np.eye(n, dtype=np.int32)).all()


def test_matmul_equals_library_gemm():
    """Sec. 4: on +-1 inputs the binary product equals the ordinary one.  float32
    BLAS is exact while K < 2^24.  Non-square shapes catch swapped M/N/K."""
    rng = np.random.default_rng(6)
    A = synth.pm1(rng, (37, 301), 0.5)
    Bm = synth.pm1(rng, (301, 53), 0.5)
    C = oracle.matmul_pm1(A, Bm)
    lib = torch.from_numpy(A).float() @ torch.from_numpy(Bm).float()
    assert (C == lib.numpy().astype(np.int64)).all()
    assert (C == A.astype(np.int64) @ Bm.astype(np.int64)).all()


def test_matmul_statistics_of_biased_inputs():
    """i.i.d. P(+1)=p in both operands: E[C] = K (2p-1)^2 (sanity, loose)."""
    rng = np.random.default_rng(7)
    K, p = 1024, 0.95
    C = oracle.matmul_pm1(synth.pm1(rng, (64, K), p), synth.pm1(rng, (K, 64), p))
    assert abs(C.mean() - K * (2 * p - 1) ** 2) < 10


# ------------------------------------------------------------- BatchNorm, Alg. 4

def test_bn_exact_small_numbers():
    """Values chosen so every float32 step is exact: var+eps = 4 -> inv = 0.5.
    y = gamma * (s - mean) * 0.5 + beta.  Catches a dropped beta, swapped
    gamma/beta, var used without sqrt, mean added instead of subtracted."""
    S = np.array([[6, -4, 0]], np.int32)
    gamma = np.array([3.0, -2.0, 0.5], np.float32)
    beta = np.array([-1.0, 0.25, -0.75], np.float32)
    mean = np.array([2.0, -1.0, 1.0], np.float32)
    var = np.array([4.0, 4.0, 4.0], np.float32)
    Y = oracle.bn_float(S, gamma, beta, mean, var, eps=0.0)
    assert Y.tolist() == [[3.0 * 2.0 - 1.0, -2.0 * -1.5 + 0.25, 0.5 * -0.5 - 0.75]]
    # var = 16 -> inv = 0.25 distinguishes sqrt(var) from var.
    Y2 = oracle.bn_float(np.array([[8]], np.int32), [1.0], [0.0], [0.0], [16.0], eps=0.0)
    assert Y2.tolist() == [[2.0]]


def test_bn_epsilon_sits_inside_the_square_root():
    """eps and var both powers of two, so sqrt(var + eps) is exact: a dropped eps, or one added outside
    the root, changes the result.  var = 0, eps = 2^-8 -> inv = 16;  var = 3*2^-8 -> var + eps = 2^-6 -> inv = 8."""
    eps = 2.0 ** -8
    S = np.array([[5, 5]], np.int32)
    Y = oracle.bn_float(S, [0.5, 0.5], [1.0, 1.0], [2.0, 2.0], [0.0, 3.0 * 2.0 ** -8], eps=eps)
    assert Y.tolist() == [[0.5 * (3.0 * 16.0) + 1.0, 0.5 * (3.0 * 8.0) + 1.0]]
    sgn = oracle.bn_sign(np.array([[1]], np.int32), [-1.0], [20.0], [0.0], [0.0], eps=eps)     # -16 + 20 >= 0
    assert sgn.tolist() == [[1]]
    sgn = oracle.bn_sign(np.array([[1]], np.int32), [-1.0], [15.0], [0.0], [0.0], eps=eps)     # -16 + 15 < 0
    assert sgn.tolist() == [[-1]]


def test_bn_matches_library_batch_norm_and_fp64():
    rng = np.random.default_rng(8)
    K, N = 1024, 257
    S = (2 * rng.integers(0, K + 1, (50, N)) - K).astype(np.int32)
    g, b, mu, v = synth.bn_params(rng, N, K, adversarial=True)
    Y = oracle.bn_float(S, g, b, mu, v, eps=1e-4)
    lib = torch.nn.functional.batch_norm(
        torch.from_numpy(S).float(), torch.from_numpy(mu), torch.from_numpy(v),
        torch.from_numpy(g), torch.from_numpy(b), training=False, eps=1e-4).numpy()
    ref64 = (g.astype(np.float64) * (S - mu.astype(np.float64))
             / np.sqrt(v.astype(np.float64) + np.float64(np.float32(1e-4))) + b)
    assert np.allclose(Y, lib, rtol=1e-5, atol=1e-5)
    assert np.allclose(Y, ref64, rtol=1e-5, atol=1e-5)


def test_bn_sign_is_sign_of_bn_and_handles_zero():
    """Sign(BatchNorm(s)) == Eq. (1) applied to the float result; y == 0 -> +1."""
    rng = np.random.default_rng(9)
    K, N = 64, 40
    S = (2 * rng.integers(0, K + 1, (30, N)) - K).astype(np.int32)
    g, b, mu, v = synth.bn_params(rng, N, K, adversarial=True)
    Y = oracle.bn_float(S, g, b, mu, v)
    assert (oracle.bn_sign(S, g, b, mu, v) == np.where(Y >= 0, 1, -1)).all()
    # s == mean, beta == 0  ->  y == 0 exactly -> +1 ; beta == -0.0 as well.
    z = oracle.bn_sign(np.array([[4, 4]], np.int32), [1.0, -1.0], [0.0, -0.0],
                       [4.0, 4.0], [1.0, 1.0])
    assert z.tolist() == [[1, 1]]
    # gamma == 0: output is Sign(beta) whatever s is.
    z = oracle.bn_sign(np.array([[-7, 7], [7, -7]], np.int32), [0.0, 0.0], [0.5, -0.5],
                       [0.0, 0.0], [1.0, 1.0])
    assert z.tolist() == [[1, -1], [1, -1]]


def test_bn_monotone_in_s():
    """The float expression is monotone in s for each channel (what allows an
    integer threshold to replace it)."""
    rng = np.random.default_rng(10)
    K, N = 300, 64
    g, b, mu, v = synth.bn_params(rng, N, K, adversarial=True)
    s = np.arange(-K, K + 1, dtype=np.int32)[:, None].repeat(N, 1)
    bits = oracle.bn_sign(s, g, b, mu, v).astype(np.int32)
    d = np.diff(bits, axis=0)
    assert ((d >= 0).all(0) | (d <= 0).all(0)).all()
    assert ((d >= 0).all(0) == (g >= 0))[g != 0].all()


# ----------------------------------------------------------------- convolution

def _read_conv_corner(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "conv_corner.txt")) as f:
        for line in f:
            if line.startswith(("input:", "output:")):
                k, rest = line.split(":")
                vals[k] = [int(t) for t in rest.split()]
    return vals["input"], vals["output"]


def test_conv_hand_worked_corner(golden_dir):
    inp, out = _read_conv_corner(golden_dir)
    x = np.array(inp, np.int8).reshape(1, 3, 3, 1)
    Wt = np.ones((1, 3, 3, 1), np.int8)
    S = oracle.conv_direct(x, Wt)
    assert S.reshape(-1).tolist() == out


@pytest.mark.parametrize("shape", [
    # B, H, W, Cin, Cout, kh, kw, stride, pad
    (2, 5, 7, 3, 4, 3, 3, 1, 1),
    (1, 8, 8, 32, 5, 3, 3, 1, 1),
    (2, 6, 5, 4, 3, 3, 3, 2, 1),
    (1, 7, 7, 2, 2, 5, 3, 1, 2),
    (1, 4, 4, 8, 2, 1, 1, 1, 0),
])
def test_conv_equals_library_conv2d_on_plus_one_padded_input(shape):
    """Direct conv == torch conv2d on the input explicitly padded with +1.
    Random non-symmetric weights catch swapped ky/kx or channel order."""
    B, H, W, Cin, Cout, kh, kw, stride, pad = shape
    rng = np.random.default_rng(sum(shape))
    x = synth.pm1(rng, (B, H, W, Cin))
    Wt = synth.pm1(rng, (Cout, kh, kw, Cin))
    S = oracle.conv_direct(x, Wt, stride=stride, pad=pad)
    xt = torch.from_numpy(x).float().permute(0, 3, 1, 2)
    xt = torch.nn.functional.pad(xt, (pad, pad, pad, pad), value=1.0)
    wt = torch.from_numpy(Wt).float().permute(0, 3, 1, 2)
    lib = torch.nn.functional.conv2d(xt, wt, stride=stride).permute(0, 2, 3, 1).numpy()
    assert S.shape == lib.shape
    assert (S == lib.astype(np.int64)).all()
    # The lowering: im2col rows times the flattened filters gives the same sums.
    cols = oracle.im2col(x, kh, kw, stride, pad)
    S2 = oracle.matmul_pm1(cols, np.ascontiguousarray(Wt.reshape(Cout, -1).T))
    assert (S2.reshape(S.shape) == S).all()


def test_im2col_matches_library_unfold():
    """im2col against torch's unfold (which orders K as ci*kh*kw + ky*kw + kx);
    the oracle's order is (ky*kw+kx)*Cin + ci."""
    rng = np.random.default_rng(11)
    B, H, W, Cin = 2, 5, 6, 3
    x = synth.pm1(rng, (B, H, W, Cin))
    cols = oracle.im2col(x, 3, 3, 1, 1)
    xt = torch.nn.functional.pad(torch.from_numpy(x).float().permute(0, 3, 1, 2),
                                 (1, 1, 1, 1), value=1.0)
    unf = torch.nn.functional.unfold(xt, (3, 3))            # [B][Cin*9][H*W]
    unf = unf.reshape(B, Cin, 9, H * W).permute(0, 3, 2, 1).reshape(B * H * W, 9 * Cin)
    assert (cols == unf.numpy().astype(np.int8)).all()


@pytest.mark.parametrize("shape", [(2, 8, 8, 5, 2, 2, 2), (1, 7, 9, 3, 3, 2, 1), (2, 6, 6, 4, 3, 3, 3)])
def test_maxpool_equals_library_max_pool2d(shape):
    B, H, W, C, ph, pw, stride = shape
    rng = np.random.default_rng(sum(shape))
    S = rng.integers(-500, 500, (B, H, W, C)).astype(np.int32)
    P = oracle.maxpool2d(S, ph, pw, stride)
    lib = torch.nn.functional.max_pool2d(torch.from_numpy(S).float().permute(0, 3, 1, 2), (ph, pw), stride)
    assert (P == lib.permute(0, 2, 3, 1).numpy().astype(np.int64)).all()


def test_pooling_commutes_with_sign_of_monotone_bn():
    """What lets pooling run on bits: for gamma >= 0 Sign(BN(max s)) is the OR of the window's
    bits, for gamma < 0 the AND (BN is monotone per channel, Sign is monotone)."""
    rng = np.random.default_rng(21)
    x = synth.pm1(rng, (2, 8, 8, 32))
    Wt = synth.pm1(rng, (16, 3, 3, 32))
    bn = synth.bn_params(rng, 16, 9 * 32, adversarial=True)
    _P, a_pool = oracle.conv_pool_layer(x, Wt, bn)
    _S, a = oracle.conv_layer(x, Wt, bn)
    win = a.reshape(2, 4, 2, 4, 2, 16)
    any_plus = (win == 1).any(axis=(2, 4))
    all_plus = (win == 1).all(axis=(2, 4))
    want = np.where(bn[0] < 0, all_plus, any_plus)
    assert ((a_pool == 1) == want).all()


# ------------------------------------------------ first layer, Sec. 1.6 / Alg. 4

def test_first_layer_bitplanes_equals_integer_product():
    """Eq. (4): sum_n 2^(n-1) <x^n, w> == <x, w> for 8-bit x."""
    rng = np.random.default_rng(12)
    X = synth.uint8_input(rng, (9, 100))
    X[0, :4] = (0, 255, 1, 128)
    Wb = synth.pm1(rng, (100, 13))
    S = oracle.first_layer_bitplanes(X, Wb)
    assert (S == X.astype(np.int64) @ Wb.astype(np.int64)).all()


def test_mlp_uint8_driver_first_layer_is_integer_product():
    x8 = synth.uint8_input(np.random.default_rng(13), (10, 40))
    _x, weights, bns = synth.config_mlp(batch=10, sizes=(40, 64, 10))
    tr = oracle.mlp_forward_uint8(x8, weights, bns)
    assert (tr["s"][0] == x8.astype(np.int64) @ weights[0].astype(np.int64)).all()
    a1 = oracle.bn_sign(tr["s"][0], *bns[0])
    assert (tr["s"][1] == a1.astype(np.int64) @ weights[1].astype(np.int64)).all()


# --------------------------------------------------------------- network driver

def test_mlp_driver_chains_the_steps():
    x, weights, bns = synth.config_mlp(batch=12, sizes=(50, 64, 33, 10), adversarial=True)
    tr = oracle.mlp_forward(x, weights, bns)
    a = np.where(x >= 0, 1, -1).astype(np.int64)
    for l, Wb in enumerate(weights):
        s = a @ Wb.astype(np.int64)
        assert (tr["s"][l] == s).all()
        if l < len(bns):
            a = oracle.bn_sign(s.astype(np.int32), *bns[l]).astype(np.int64)
            assert (tr["a"][l + 1] == a).all()
    assert tr["s"][-1].shape == (12, 10)
