"""GPU parity: every entry point of the C ABI against the CPU oracle, bit for bit,
on the same seeded inputs.  All int32 results and all packed words must be
equal; there is no tolerance anywhere."""
import os

import numpy as np
import pytest
import torch

import oracle
import paper_1602_02830_amd as bnn
from workloads import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
EPS = oracle.EPS_DEFAULT
GEMM_KERNELS = {
    "auto": bnn.KERNEL_AUTO,
    "naive": bnn.KERNEL_NAIVE,
    "tiled128": bnn.KERNEL_TILED128,
    "ksplit": bnn.KERNEL_KSPLIT,
    "tiled64": bnn.KERNEL_TILED64,
    "mfma": bnn.KERNEL_MFMA,
    "mfma128": bnn.KERNEL_MFMA128,
}
# Kernel id 8, the persistent form of "mfma", takes only large products (more 256 x 128 tiles than the chip
# holds at once, K a multiple of 512, N a multiple of 128): it has tests of its own and takes part in the
# 8192^3 and full-batch tests through "auto".
# The short-K organisation of the matrix-engine kernel takes only 96 < K <= 1152 and operands that
# allow 16-byte loads, so it has tests of its own instead of a place in the sweeps above.


def words_to_dev(w: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(w).view(np.int32)).to(DEV)


def words_to_host(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().cpu().numpy().view(np.uint32)


def poison_pad_bits(words: np.ndarray, K: int) -> np.ndarray:
    """Sets every pad bit of the last word of each row to 1."""
    out = words.copy()
    r = K % 32
    if r and out.shape[1] > 0:
        out[:, -1] |= np.uint32((0xFFFFFFFF << r) & 0xFFFFFFFF)
    return out


def strided_words(w: np.ndarray, ld: int, fill=0x5A5A5A5A) -> torch.Tensor:
    """Device copy of packed rows with leading dimension ld > row length (pad words = junk)."""
    rows, kw = w.shape
    buf = np.full((rows, ld), fill, np.uint32)
    buf[:, :kw] = w
    return words_to_dev(buf)[:, :kw]


# ------------------------------------------------------------------ pack_sign

def test_pack_sign_table(golden_dir):
    bits, want = [], []
    for line in open(os.path.join(golden_dir, "sign_table.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            h, _n, s = line.split()
            bits.append(int(h, 16))
            want.append(int(s))
    x = np.array(bits, np.uint32).view(np.float32)[None, :]
    got = words_to_host(bnn.pack_sign(torch.from_numpy(x).to(DEV)))
    want_words = oracle.pack_bits(np.array(want, np.int8)[None, :])
    assert (got == want_words).all()
    assert (oracle.pack_bits(oracle.sign(x)) == got).all()


@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 31), (5, 32), (7, 33), (64, 1024), (33, 784),
                                       (2, 4099), (1000, 100), (129, 4096)])
def test_pack_sign_shapes(rows, cols):
    rng = np.random.default_rng(rows * 10007 + cols)
    x = synth.real_input(rng, (rows, cols))
    x[rng.random((rows, cols)) < 0.05] = 0.0
    x[rng.random((rows, cols)) < 0.02] = -0.0
    want = oracle.pack_bits(oracle.sign(x))
    got = words_to_host(bnn.pack_sign(torch.from_numpy(x).to(DEV)))
    assert (got == want).all()


# Rows that are whole numbers of 128 elements take the 4-words-per-group kernels of the Sign packer and of the
# BatchNorm + Sign epilogue: several rows per workgroup (fewer than 32 units per row), several workgroups per
# row, row counts that leave the last workgroup partly empty, strided inputs and outputs with guard words.
UNIT_SHAPES = [(1, 128), (5, 128), (33, 256), (31, 512), (70, 1024), (7, 4096), (3, 8192), (129, 4096), (9, 12288),
               (65, 384), (2, 128 * 33)]          # the last two fit neither split: the general kernels


@pytest.mark.parametrize("rows,cols", UNIT_SHAPES)
def test_pack_sign_rows_of_whole_128_element_units(rows, cols):
    rng = np.random.default_rng(rows * 31 + cols)
    x = synth.real_input(rng, (rows, cols + 8))
    x[rng.random(x.shape) < 0.05] = 0.0
    x[rng.random(x.shape) < 0.02] = -0.0
    xd = torch.from_numpy(x).to(DEV)[:, 4:4 + cols]                 # 16-byte aligned rows, ld_x = cols + 8
    nw = cols // 32
    out = torch.full((rows + 2, nw + 4), 0x0BADBEEF, dtype=torch.int32, device=DEV)
    bnn.pack_sign(xd, out=out[1:rows + 1, :nw])
    host = words_to_host(out)
    assert (host[1:rows + 1, :nw] == oracle.pack_bits(oracle.sign(x[:, 4:4 + cols]))).all()
    host[1:rows + 1, :nw] = 0x0BADBEEF
    assert (host == 0x0BADBEEF).all()


@pytest.mark.parametrize("M,N", UNIT_SHAPES)
def test_bn_sign_pack_rows_of_whole_128_channel_units(M, N):
    rng = np.random.default_rng(M * 37 + N)
    K = 600
    bn = synth.bn_params(rng, N, K, adversarial=True)
    S = np.clip(2 * np.rint(rng.normal(0, np.sqrt(K) / 2, (M, N + 8))) + (K % 2), -K, K).astype(np.int32)
    Sd = torch.from_numpy(S).to(DEV)[:, 4:4 + N]
    thr, flip = _fold_to_dev(bn, K)
    nw = N // 32
    out = torch.full((M + 2, nw + 4), 0x0BADBEEF, dtype=torch.int32, device=DEV)
    bnn.bn_sign_pack(Sd, thr, flip, out=out[1:M + 1, :nw])
    host = words_to_host(out)
    assert (host[1:M + 1, :nw] == oracle.pack_bits(oracle.bn_sign(S[:, 4:4 + N], *bn, eps=EPS))).all()
    host[1:M + 1, :nw] = 0x0BADBEEF
    assert (host == 0x0BADBEEF).all()


def test_pack_sign_unaligned_and_strided():
    rng = np.random.default_rng(77)
    rows, cols = 37, 203
    big = synth.real_input(rng, (rows, cols + 9))
    xd = torch.from_numpy(big).to(DEV)[:, 3:3 + cols]        # ld_x = cols+9, base 12 bytes off
    want = oracle.pack_bits(oracle.sign(big[:, 3:3 + cols]))
    kw = want.shape[1]
    out = torch.full((rows, kw + 3), 0x12345678, dtype=torch.int32, device=DEV)
    bnn.pack_sign(xd, out=out[:, :kw])
    host = words_to_host(out)
    assert (host[:, :kw] == want).all()
    assert (host[:, kw:] == 0x12345678).all()                # words past the row untouched


def test_pack_sign_large_streaming_shape():
    rng = np.random.default_rng(78)
    x = synth.real_input(rng, (4096, 8192))
    want = oracle.pack_bits(oracle.sign(x))
    got = words_to_host(bnn.pack_sign(torch.from_numpy(x).to(DEV)))
    assert (got == want).all()


# ------------------------------------------------------------------ xnor_gemm

def _gemm_case(A, Bm, kernel, poison=False, ld_extra=0):
    M, K = A.shape
    N = Bm.shape[1]
    want = oracle.matmul_pm1(A, Bm)
    pa = oracle.pack_bits(A)
    pb = oracle.pack_bits(np.ascontiguousarray(Bm.T))
    if poison:
        pa, pb = poison_pad_bits(pa, K), poison_pad_bits(pb, K)
    if ld_extra:
        da = strided_words(pa, pa.shape[1] + ld_extra)
        db = strided_words(pb, pb.shape[1] + ld_extra)
    else:
        da, db = words_to_dev(pa), words_to_dev(pb)
    got = bnn.xnor_gemm(da, db, K, kernel=kernel).cpu().numpy()
    assert got.shape == want.shape
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"M={M} N={N} K={K} first mismatch at {bad[0]}: got {got[tuple(bad[0])]} want {want[tuple(bad[0])]}"
    assert (np.abs(got) <= K).all() and ((got - K) % 2 == 0).all()


@pytest.mark.parametrize("kernel", list(GEMM_KERNELS))
def test_xnor_gemm_ragged_sweep(kernel):
    """All 336 ragged cases (M, N in {1,7,33,1000}; K in {1,31,32,33,63,65,4097};
    P(+1) in {.05,.5,.95}), once with zero pad bits and once with poisoned ones."""
    cases = synth.ragged_cases()
    assert len(cases) == 336
    for idx, (M, N, K, p) in enumerate(cases):
        A, Bm = synth.config_ragged(idx)
        _gemm_case(A, Bm, GEMM_KERNELS[kernel], poison=False)
        _gemm_case(A, Bm, GEMM_KERNELS[kernel], poison=True)


@pytest.mark.parametrize("kernel", ["auto", "tiled128", "tiled64", "naive", "ksplit", "mfma", "mfma128"])
def test_xnor_gemm_odd_leading_dimensions(kernel):
    rng = np.random.default_rng(5)
    for (M, N, K) in [(130, 70, 1000), (17, 300, 129), (256, 256, 2048)]:
        A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
        for extra in (1, 3, 4):
            _gemm_case(A, Bm, GEMM_KERNELS[kernel], poison=True, ld_extra=extra)


@pytest.mark.parametrize("kernel", ["auto", "tiled128", "tiled64", "mfma", "mfma128", "ksplit"])
def test_xnor_gemm_multi_tile_shapes(kernel):
    rng = np.random.default_rng(6)
    for (M, N, K) in [(64, 1024, 1024), (300, 520, 784), (1024, 10, 4096), (513, 129, 96), (2, 2048, 640)]:
        _gemm_case(synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N)), GEMM_KERNELS[kernel])


def _offset_words(w: np.ndarray, ld: int, first: int) -> torch.Tensor:
    """Device view of packed rows inside a junk-filled buffer: leading dimension ld, base `first` words
    (4 * first bytes) past an allocation boundary."""
    rows, kw = w.shape
    buf = np.full(first + rows * ld + 4, 0xC3C3C3C3, np.uint32)
    body = buf[first:first + rows * ld].reshape(rows, ld)
    body[:, :kw] = w
    flat = words_to_dev(buf)
    return flat[first:first + rows * ld].view(rows, ld)[:, :kw]


@pytest.mark.parametrize("seed", range(10))
def test_xnor_gemm_randomized_shapes_strides_alignments_and_kernels(seed):
    """Seeded random cases: M, N, K log-uniform, P(+1) anywhere in (0, 1), random leading dimensions and
    base offsets (so both the 16-byte and the word-wise loaders run), poisoned pad bits, every kernel id.
    A kernel either returns the exact product and the exact fused bits, or refuses with UNSUPPORTED."""
    rng = np.random.default_rng(4242 + seed)
    ids = list(GEMM_KERNELS.values()) + [bnn.KERNEL_MFMA_SHORTK, bnn.KERNEL_MFMA_PERSIST, bnn.KERNEL_MFMA_SPLITK]
    fused_ids = {bnn.KERNEL_AUTO, bnn.KERNEL_TILED128, bnn.KERNEL_TILED64, bnn.KERNEL_MFMA, bnn.KERNEL_MFMA128,
                 bnn.KERNEL_MFMA_SHORTK, bnn.KERNEL_MFMA_PERSIST, bnn.KERNEL_MFMA_SPLITK}
    for _case in range(20):
        M, N = (int(np.exp(rng.uniform(0, np.log(600)))) for _ in range(2))
        K = int(np.exp(rng.uniform(0, np.log(5000))))
        p = rng.uniform(0.02, 0.98)
        A, Bm = synth.pm1(rng, (M, K), p), synth.pm1(rng, (K, N), p)
        bn = synth.bn_params(rng, N, K, adversarial=True)
        S, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
        kw = (K + 31) // 32
        pa = poison_pad_bits(oracle.pack_bits(A), K)
        pb = poison_pad_bits(oracle.pack_bits(np.ascontiguousarray(Bm.T)), K)
        if rng.random() < 0.5:          # 16-byte-loadable layout
            ld = (kw + 3) // 4 * 4 + 4 * int(rng.integers(0, 3))
            da, db = _offset_words(pa, ld, 0), _offset_words(pb, ld, 4 * int(rng.integers(0, 3)))
        else:
            da = _offset_words(pa, kw + int(rng.integers(0, 6)), int(rng.integers(0, 4)))
            db = _offset_words(pb, kw + int(rng.integers(0, 6)), int(rng.integers(0, 4)))
        thr, flip = _fold_to_dev(bn, K)
        want_bits = oracle.pack_bits(a_next)
        for kid in ids:
            tag = f"seed {seed} M={M} N={N} K={K} kernel {kid}"
            try:
                got = bnn.xnor_gemm(da, db, K, kernel=kid).cpu().numpy()
            except bnn.BnnError as e:
                assert e.status == 3, tag
                continue
            assert (got == S).all(), tag
            try:
                bits = words_to_host(bnn.xnor_gemm_bn_sign_pack(da, db, K, thr, flip, kernel=kid))
            except bnn.BnnError as e:
                # the naive and the K-split kernel have no fused form: invalid argument, as documented
                assert e.status == (3 if kid in fused_ids else 1), tag
                continue
            assert kid in fused_ids and (bits == want_bits).all(), tag


def _aligned_words(w: np.ndarray) -> torch.Tensor:
    """Device copy with the leading dimension rounded up to 4 words (junk in the extra words)."""
    kw = w.shape[1]
    ld = (kw + 3) // 4 * 4
    return strided_words(w, ld) if ld != kw else words_to_dev(w)


SHORTK_SHAPES = [(128, 128, 128), (300, 200, 97), (130, 200, 1000), (1000, 1000, 1152), (129, 95, 128),
                 (64, 1024, 1024), (777, 333, 513), (500, 260, 640), (300, 4096, 784), (1500, 700, 1151),
                 (257, 129, 1121), (1, 1, 100), (131, 7, 992)]


@pytest.mark.parametrize("M,N,K", SHORTK_SHAPES)
def test_shortk_kernel_int32_and_fused(M, N, K):
    """Kernel 7 on every K-tail length class (whole quads, partial last quad, pad bits in a whole quad),
    ragged M and N, poisoned pad bits; int32 output against the literal product, fused output against
    float BatchNorm + Sign."""
    rng = np.random.default_rng(M * 11 + N * 13 + K * 17)
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    S, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
    pa = _aligned_words(poison_pad_bits(oracle.pack_bits(A), K))
    pb = _aligned_words(poison_pad_bits(oracle.pack_bits(np.ascontiguousarray(Bm.T)), K))
    got = bnn.xnor_gemm(pa, pb, K, kernel=bnn.KERNEL_MFMA_SHORTK).cpu().numpy()
    assert (got == S).all()
    thr, flip = _fold_to_dev(bn, K)
    nw = (N + 31) // 32
    out = torch.full((M, nw + 1), 0x0BADF00D, dtype=torch.int32, device=DEV)
    bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip, out=out[:, :nw], kernel=bnn.KERNEL_MFMA_SHORTK)
    host = words_to_host(out)
    assert (host[:, :nw] == oracle.pack_bits(a_next)).all()
    assert (host[:, nw:] == 0x0BADF00D).all()


def test_shortk_kernel_several_row_tiles_per_workgroup():
    """55 row tiles over 32 column tiles: 24 workgroups per column tile, two or three row tiles each,
    the last one ragged.  Rows sampled from every tile."""
    M, N, K = 7000, 4096, 784
    rng = np.random.default_rng(99)
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    pa = _aligned_words(oracle.pack_bits(A))
    pb = _aligned_words(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    thr, flip = _fold_to_dev(bn, K)
    got = words_to_host(bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip, kernel=bnn.KERNEL_MFMA_SHORTK))
    auto = words_to_host(bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip))      # the default dispatch picks it too
    rows = np.unique(np.concatenate([np.arange(0, M, 37), np.arange(M - 130, M)]))
    _s, a_next = oracle.dense_layer(A[rows], Bm, bn, eps=EPS)
    assert (got[rows] == oracle.pack_bits(a_next)).all()
    assert (auto == got).all()
    c = bnn.xnor_gemm(pa, pb, K, kernel=bnn.KERNEL_MFMA_SHORTK).cpu().numpy()
    assert (c[rows] == oracle.matmul_pm1(A[rows], Bm)).all()


def test_shortk_kernel_rejects_what_it_cannot_take():
    rng = np.random.default_rng(98)
    for K, aligned in ((96, True), (1153, True), (784, False)):
        A, Bm = synth.pm1(rng, (40, K)), synth.pm1(rng, (K, 40))
        pa, pb = oracle.pack_bits(A), oracle.pack_bits(np.ascontiguousarray(Bm.T))
        da, db = (_aligned_words(pa), _aligned_words(pb)) if aligned else (words_to_dev(pa), words_to_dev(pb))
        with pytest.raises(bnn.BnnError) as e:
            bnn.xnor_gemm(da, db, K, kernel=bnn.KERNEL_MFMA_SHORTK)
        assert e.value.status == 3          # BNN_ERR_UNSUPPORTED
        got = bnn.xnor_gemm(da, db, K).cpu().numpy()                                # the default dispatch still serves it
        assert (got == oracle.matmul_pm1(A, Bm)).all()


@pytest.mark.parametrize("kernel", ["mfma", "mfma128", "mfma_splitk"])
def test_mfma_kernels_at_the_exact_accumulation_limit(kernel):
    """K = 2^24 is the largest K the matrix-engine kernels accept: their fp32 sums of 0/1 products reach
    2^24 exactly when every bit of both operands is set.  One K beyond that they refuse, and the default
    dispatch serves the same product on the vector ALU."""
    K = 1 << 24
    kid = bnn.KERNEL_MFMA_SPLITK if kernel == "mfma_splitk" else GEMM_KERNELS[kernel]
    rng = np.random.default_rng(24)
    A = synth.pm1(rng, (4, K))
    Bm = synth.pm1(rng, (K, 3))
    A[0, :] = 1                      # row 0 all +1
    Bm[:, 0] = 1                     # column 0 all +1: C[0][0] = K, the sum of products is 2^24
    A[1, :] = -1                     # row 1 all -1: C[1][0] = -K
    want = oracle.matmul_pm1(A, Bm)
    assert want[0, 0] == K and want[1, 0] == -K
    pa = words_to_dev(oracle.pack_bits(A))
    pb = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    got = bnn.xnor_gemm(pa, pb, K, kernel=kid).cpu().numpy()
    assert (got == want).all()
    # fused form at this K compares in integers (thresholds are folded into fp32 sums only up to K = 2^19)
    thr = torch.tensor([K, 0, -K + 2], dtype=torch.int32, device=DEV)
    flip = torch.tensor([0b100], dtype=torch.int32, device=DEV)
    bits = words_to_host(bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip, kernel=kid))
    want_bits = ((want >= thr.cpu().numpy()[None, :]) != np.array([False, False, True])[None, :])
    assert (bits[:, 0] == (want_bits * (1 << np.arange(3))[None, :]).sum(axis=1)).all()
    # one word more: outside the exact range
    K2 = K + 32
    A2 = np.concatenate([A, np.ones((4, 32), np.int8)], axis=1)
    B2 = np.concatenate([Bm, np.ones((32, 3), np.int8)], axis=0)
    pa2 = words_to_dev(oracle.pack_bits(A2))
    pb2 = words_to_dev(oracle.pack_bits(np.ascontiguousarray(B2.T)))
    with pytest.raises(bnn.BnnError) as e:
        bnn.xnor_gemm(pa2, pb2, K2, kernel=kid)
    assert e.value.status == 3
    assert (bnn.xnor_gemm(pa2, pb2, K2).cpu().numpy() == want + oracle.matmul_pm1(A2[:, K:], B2[K:, :])).all()


@pytest.mark.parametrize("K", [1 << 19, (1 << 19) + 32, 1 << 21])
def test_fused_layer_on_both_sides_of_the_float_compare_limit(K):
    """Up to K = 2^19 the fused epilogue of the matrix-engine kernel folds the threshold into its fp32
    accumulators and reads the output bit off their sign, beyond it compares in integers; both must give
    the folded BatchNorm + Sign bits, also for thresholds at and next to attained values."""
    M, N = 9, 40
    rng = np.random.default_rng(K % 1000)
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    S = oracle.matmul_pm1(A, Bm)
    # thresholds right at, just above and just below attained values, and at the ends of the range
    thr = np.concatenate([S[0, :10], S[1, 10:20] + 1, S[2, 20:30] - 1, [K, K + 1, -K, -K - 1, 0, 1, -1, 2, -2, 3]]).astype(np.int32)
    flip = rng.integers(0, 2, N).astype(bool)
    want = np.where((S >= thr[None, :]) != flip[None, :], 1, -1).astype(np.int8)
    flip_words = oracle.pack_bits(np.where(flip, 1, -1).astype(np.int8)[None, :])[0]
    pa = words_to_dev(oracle.pack_bits(A))
    pb = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    for kernel in ("mfma", "mfma128"):
        got = bnn.xnor_gemm_bn_sign_pack(pa, pb, K, torch.from_numpy(thr).to(DEV), words_to_dev(flip_words[None, :])[0],
                                         kernel=GEMM_KERNELS[kernel])
        assert (words_to_host(got) == oracle.pack_bits(want)).all(), kernel


def test_bitplane_gemm_at_the_exact_accumulation_limit():
    """255 * K < 2^24 bounds the 8-bit first layer on the matrix engine: K = 65792 with every input 255 and
    every weight +1 gives 16776960, the largest sum it must represent."""
    K = 65792
    rng = np.random.default_rng(65)
    X = synth.uint8_input(rng, (3, K))
    X[0, :] = 255
    Wb = synth.pm1(rng, (K, 2))
    Wb[:, 0] = 1
    S = oracle.first_layer_bitplanes(X, Wb)
    assert S[0, 0] == 255 * K
    planes = bnn.pack_bitplanes(torch.from_numpy(X).to(DEV))
    wb = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Wb.T)))
    assert (bnn.bitplane_gemm(planes, wb, K).cpu().numpy() == S).all()


@pytest.mark.parametrize("K", [65794, 65824, 70001])
def test_bitplane_gemm_past_the_matrix_engine_limit(K):
    """One step past 255 * K < 2^24 (and a ragged K further out): the product leaves the matrix engine for the
    and/popcount kernel; int32 sums and fused bits against the oracle, pad bits of both operands poisoned."""
    rng = np.random.default_rng(K)
    M, N = 5, 37
    X = synth.uint8_input(rng, (M, K))
    X[0, :] = 255
    Wb = synth.pm1(rng, (K, N))
    Wb[:, 0] = 1
    S = oracle.first_layer_bitplanes(X, Wb)
    assert S[0, 0] == 255 * K and S[0, 0] >= 1 << 24
    planes = bnn.pack_bitplanes(torch.from_numpy(X).to(DEV))
    w_words = poison_pad_bits(oracle.pack_bits(np.ascontiguousarray(Wb.T)), K)
    if K % 32:
        planes[:, -8:] |= torch.tensor(np.int32(np.uint32((0xFFFFFFFF << (K % 32)) & 0xFFFFFFFF).view(np.int32)), device=DEV)
    wb = words_to_dev(w_words)
    assert (bnn.bitplane_gemm(planes, wb, K).cpu().numpy() == S).all()
    bn = synth.bn_params(rng, N, 255 * K, adversarial=True)
    thr, flip = _fold_to_dev(bn, 255 * K)
    got = bnn.bitplane_gemm_bn_sign_pack(planes, wb, K, thr, flip)
    assert (words_to_host(got) == oracle.pack_bits(oracle.bn_sign(S, *bn, eps=EPS))).all()


def test_xnor_gemm_ldc_and_canary():
    rng = np.random.default_rng(7)
    M, N, K = 100, 77, 500
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    out = torch.full((M, N + 5), -12345, dtype=torch.int32, device=DEV)
    bnn.xnor_gemm(words_to_dev(oracle.pack_bits(A)), words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T))),
                  K, out=out[:, :N])
    host = out.cpu().numpy()
    assert (host[:, :N] == oracle.matmul_pm1(A, Bm)).all()
    assert (host[:, N:] == -12345).all()


def test_xnor_gemm_empty_and_k_zero():
    a = torch.zeros((0, 4), dtype=torch.int32, device=DEV)
    b = torch.zeros((5, 4), dtype=torch.int32, device=DEV)
    assert bnn.xnor_gemm(a, b, 100).shape == (0, 5)
    a1 = torch.zeros((3, 1), dtype=torch.int32, device=DEV)
    c = bnn.xnor_gemm(a1, b[:, :1], 0)
    assert (c.cpu().numpy() == 0).all()


@pytest.mark.parametrize("kernel", ["auto", "tiled128", "mfma"])
def test_xnor_gemm_dense_layer_config(kernel):
    """Config: A 64x1024, B 1024x1024, K = 1024."""
    A, Bm, _ = synth.config_dense()
    _gemm_case(A, Bm, GEMM_KERNELS[kernel])


@pytest.mark.parametrize("adversarial", [False, True])
def test_dense_layer_config_chained_as_specified(adversarial):
    """The single binary dense layer as the workload states it: A 64 x 1024 and B 1024 x 1024 of +-1 from the
    seed, packed on the device; int32 output 64 x 1024; then BatchNorm-then-Sign with the workload's own
    per-channel parameters (and the copy with negative / zero gammas) folded to integer thresholds; output
    packed.  Chained GEMM -> epilogue as two launches and as the fused launch, every element."""
    A, Bm, bn = synth.config_dense(adversarial=adversarial)
    S_want, a_want = oracle.dense_layer(A, Bm, bn, eps=EPS)
    a_bits = bnn.pack_sign(torch.from_numpy(A.astype(np.float32)).to(DEV))
    b_bits = bnn.pack_sign(torch.from_numpy(np.ascontiguousarray(Bm.T).astype(np.float32)).to(DEV))
    assert (words_to_host(a_bits) == oracle.pack_bits(A)).all()
    thr, flip = _fold_to_dev(bn, 1024)
    S = bnn.xnor_gemm(a_bits, b_bits, 1024)
    assert (S.cpu().numpy() == S_want).all()
    out = bnn.bn_sign_pack(S, thr, flip)
    assert (words_to_host(out) == oracle.pack_bits(a_want)).all()
    fused = bnn.xnor_gemm_bn_sign_pack(a_bits, b_bits, 1024, thr, flip)
    assert (words_to_host(fused) == oracle.pack_bits(a_want)).all()


@pytest.mark.parametrize("M,N,K", [
    (10241, 4096, 1024),     # 41 x 32 tiles on 512 slots; last row tile shifted by 255 rows; 2 K-tiles (the minimum)
    (10000, 4096, 1536),     # odd number of K-tiles: the LDS buffer parity differs from tile to tile
    (256 * 33, 2048, 2560),  # whole row tiles, 528 tiles: most workgroups walk one tile, 16 walk two
    (9000, 8192, 1024),      # 36 x 64 tiles: up to five tiles per workgroup
])
def test_persistent_tile_walk_of_the_large_product_kernel(M, N, K):
    """Products with more 256 x 128 tiles than the chip holds at once take the persistent form of the
    matrix-engine kernel (a workgroup walks over several tiles, the next tile's first K-tile fetched
    during the current tile's last): every int32 result and every fused output bit against the oracle."""
    rng = np.random.default_rng(M + N + K)
    A, Bm = synth.pm1(rng, (M, K), 0.6), synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    S, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
    pa = words_to_dev(oracle.pack_bits(A))
    pb = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    for kernel in (bnn.KERNEL_MFMA_PERSIST, bnn.KERNEL_AUTO):
        got = bnn.xnor_gemm(pa, pb, K, kernel=kernel).cpu().numpy()
        bad = np.argwhere(got != S)
        assert bad.size == 0, f"kernel {kernel}: first mismatch at {bad[0]}"
    thr, flip = _fold_to_dev(bn, K)
    want = oracle.pack_bits(a_next)
    for kernel in (bnn.KERNEL_MFMA_PERSIST, bnn.KERNEL_AUTO):
        out = torch.full((M, N // 32), 0x55AA55AA, dtype=torch.int32, device=DEV)
        bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip, out=out, kernel=kernel)
        assert (words_to_host(out) == want).all(), f"kernel {kernel}"


def test_persistent_kernel_refuses_what_it_does_not_take():
    """Kernel id 8 answers BNN_ERR_UNSUPPORTED, launching nothing, outside its shapes: K not a multiple of 512,
    N not a multiple of 128, fewer tiles than resident slots, operands that do not allow 16-byte loads."""
    def refused(M, N, K, ld_extra=0):
        kw = (K + 31) // 32
        a = torch.zeros((M, kw + ld_extra), dtype=torch.int32, device=DEV)[:, :kw]
        b = torch.zeros((N, kw + ld_extra), dtype=torch.int32, device=DEV)[:, :kw]
        with pytest.raises(bnn.BnnError) as e:
            bnn.xnor_gemm(a, b, K, kernel=bnn.KERNEL_MFMA_PERSIST)
        return e.value.status == 3
    assert refused(10000, 4096, 4000)
    assert refused(10000, 4096, 512)
    assert refused(10000, 4000, 1024)
    assert refused(4096, 4096, 1024)             # 16 x 32 = 512 tiles: no more than the slots
    assert refused(10000, 4096, 1024, ld_extra=1)


@pytest.mark.parametrize("M,N,K,ld_extra", [
    (10000, 4096, 4096, 0),    # the MLP's hidden layer: 16 strips of 625 rows = two 256-row tiles and a 128-row tile
    (10007, 4096, 2048, 4),    # strips of 625 and 626 rows; padded operand rows
    (13001, 2048, 2048, 0),    # 32 strips of 406 / 407 rows: one tile and a second one shifted up over it
    (12000, 2048, 2560, 8),    # 375 rows: one tile and a 128-row tile; 5 K-tiles
    (65536, 256, 2048, 0),     # one column tile, 256 strips of exactly one tile; 4 K-tiles (the minimum)
    (8192, 8192, 3072, 0),     # 8 strips of four whole tiles
])
def test_one_wavefront_per_simd_kernel_of_the_fused_layer(M, N, K, ld_extra):
    """The 256 x 256-tile kernel of the fused hidden layer (one workgroup per compute unit, row strips of
    256-row tiles plus a 128-row tile, K-tile stream running on across a workgroup's tiles): every output
    bit against the oracle, as the explicit kernel and as the library's own choice, with adversarial
    thresholds, pad words between the rows and an output buffer whose pad words must stay untouched."""
    rng = np.random.default_rng(M + 3 * N + K)
    A, Bm = synth.pm1(rng, (M, K), 0.55), synth.pm1(rng, (K, N), 0.45)
    bn = synth.bn_params(rng, N, K, adversarial=True)
    _, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
    want = oracle.pack_bits(a_next)
    kw, nw = K // 32, N // 32
    pa = torch.full((M, kw + ld_extra), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
    pb = torch.full((N, kw + ld_extra), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
    pa[:, :kw] = words_to_dev(oracle.pack_bits(A))
    pb[:, :kw] = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    thr, flip = _fold_to_dev(bn, K)
    for kernel in (bnn.KERNEL_MFMA_BIG, bnn.KERNEL_AUTO):
        out = torch.full((M, nw + 2), 0x55AA55AA, dtype=torch.int32, device=DEV)
        bnn.xnor_gemm_bn_sign_pack(pa[:, :kw], pb[:, :kw], K, thr, flip, out=out[:, :nw], kernel=kernel)
        got = out.cpu().numpy().view(np.uint32)
        bad = np.argwhere(got[:, :nw] != want)
        assert bad.size == 0, f"kernel {kernel}: first mismatch at {bad[0]}"
        assert (got[:, nw:] == 0x55AA55AA).all(), f"kernel {kernel}: pad words of the output written"


def test_one_wavefront_per_simd_kernel_at_its_largest_k():
    """K = 2^19 is the largest K whose threshold the fused epilogue folds exactly into fp32 sums, and the
    largest the 256 x 256-tile kernel takes: 1024 K-tiles per output tile, sums up to 2^19 and thresholds at,
    just above and just below attained values.  The oracle computes sampled rows x sampled columns
    (the operands are drawn as packed words; 640 MB on the device); one K-tile more is refused."""
    M, N, K = 2048, 8192, 1 << 19
    kw = K // 32
    rng = np.random.default_rng(19)
    aw = rng.integers(0, 1 << 32, (M, kw + 16), dtype=np.uint64).astype(np.uint32)
    bw = rng.integers(0, 1 << 32, (N, kw + 16), dtype=np.uint64).astype(np.uint32)
    aw[5, :kw] = 0xFFFFFFFF                                  # a row and a column of all +1: the sum K itself
    bw[7, :kw] = 0xFFFFFFFF
    rows = np.array([0, 5, 255, 256, 1000, 1023, 1024, 2047])
    cols = np.concatenate([np.arange(0, 40), [7, 255, 256, 4095, 4096, 8191]])
    S = oracle.matmul_pm1(oracle.unpack_bits(aw[rows, :kw], K), np.ascontiguousarray(oracle.unpack_bits(bw[cols, :kw], K).T))
    assert S[1, 40] == K
    thr = np.zeros(N, dtype=np.int32)
    thr[cols[:10]] = S[0, :10]
    thr[cols[10:20]] = S[2, 10:20] + 1
    thr[cols[20:30]] = S[3, 20:30] - 1
    thr[cols[30:40]] = [K, K + 1, -K, -K - 1, 0, 1, -1, 2, -2, 3]
    thr[7] = K
    flip = rng.integers(0, 2, N).astype(bool)
    want = (S >= thr[cols][None, :]) != flip[cols][None, :]
    flip_words = oracle.pack_bits(np.where(flip, 1, -1).astype(np.int8)[None, :])[0]
    pa, pb = words_to_dev(aw), words_to_dev(bw)
    thr_d, flip_d = torch.from_numpy(thr).to(DEV), words_to_dev(flip_words[None, :])[0]
    out = bnn.xnor_gemm_bn_sign_pack(pa[:, :kw], pb[:, :kw], K, thr_d, flip_d, kernel=bnn.KERNEL_MFMA_BIG)
    got = oracle.unpack_bits(words_to_host(out)[rows], N)[:, cols] > 0
    bad = np.argwhere(got != want)
    assert bad.size == 0, f"first mismatch at sampled (row, column) {bad[0]}"
    with pytest.raises(bnn.BnnError) as e:
        bnn.xnor_gemm_bn_sign_pack(pa[:, :kw + 16], pb[:, :kw + 16], K + 512, thr_d, flip_d, kernel=bnn.KERNEL_MFMA_BIG)
    assert e.value.status == 3


@pytest.mark.parametrize("M,N,K,ld_extra", [
    (256, 1024, 8192, 0),      # first fully connected layer of the ConvNet at batch 256: 256 tiles, 8 quads per lane
    (33, 65, 128, 4),          # one quad per row: seven of the eight lane groups multiply zeros; ragged M and N
    (1, 1, 128, 0),
    (100, 1000, 4096, 0),      # ragged last row tile and last column word
    (31, 33, 256, 8),
    (512, 512, 2048, 0),
    (64, 40, 1152, 0),         # 9 quads per row: a second, mostly empty pass of the lanes
    (7, 300, 16384, 0),        # 128 quads per row: four batches per lane
    (256, 256, 8576, 12),      # 67 quads per row: the last batch is ragged across the wavefronts
    (1024, 1024, 4096, 0),     # 1024 tiles, the most the automatic choice gives this kernel
])
def test_k_split_matrix_engine_kernel_int32_and_fused(M, N, K, ld_extra):
    """Kernel id 10 (32 x 32 output tiles, K split over the wavefronts of a workgroup), by explicit id and
    through the automatic choice (which takes it for these small outputs once K >= 512), on padded operand rows
    filled with junk: every int32 result and every fused output bit against the oracle; words of the output
    beyond ceil(N / 32) untouched."""
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    A, Bm = synth.pm1(rng, (M, K), 0.55), synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    S, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
    kw = K // 32
    pa = _offset_words(oracle.pack_bits(A), kw + ld_extra, 0)
    pb = _offset_words(oracle.pack_bits(np.ascontiguousarray(Bm.T)), kw + ld_extra, 4)
    thr, flip = _fold_to_dev(bn, K)
    want = oracle.pack_bits(a_next)
    nw = (N + 31) // 32
    for kernel in (bnn.KERNEL_MFMA_SPLITK, bnn.KERNEL_AUTO):
        got = bnn.xnor_gemm(pa, pb, K, kernel=kernel).cpu().numpy()
        bad = np.argwhere(got != S)
        assert bad.size == 0, f"kernel {kernel}: first mismatch at {bad[0]}"
        out = torch.full((M, nw + 1), 0x55AA55AA, dtype=torch.int32, device=DEV)
        bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip, out=out[:, :nw], kernel=kernel)
        host = words_to_host(out)
        assert (host[:, :nw] == want).all(), f"kernel {kernel}"
        assert (host[:, nw] == 0x55AA55AA).all(), f"kernel {kernel}: wrote past the row's words"


@pytest.mark.parametrize("M,N", [(256, 1024), (257, 1024), (512, 1024), (513, 1024), (1024, 1024), (1025, 1024),
                                 (10000, 10), (16385, 16), (3, 16384), (4, 2048)])
@pytest.mark.parametrize("K", [384, 512, 1920, 2048, 4096])
def test_automatic_choice_on_both_sides_of_the_small_output_limits(M, N, K):
    """The automatic choice hands small outputs to kernel 10 up to 256 tiles of 32 x 32 (K >= 512), 512 tiles
    (K >= 2048) and 1024 tiles (K >= 4096), skinny int32 outputs included, and everything else to the other
    kernels: on both sides of each limit the int32 product and the fused bits equal the oracle's."""
    rng = np.random.default_rng(M * 31 + N * 17 + K)
    A, Bm = synth.pm1(rng, (M, K), 0.45), synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    S, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
    pa = words_to_dev(oracle.pack_bits(A))
    pb = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    got = bnn.xnor_gemm(pa, pb, K).cpu().numpy()
    bad = np.argwhere(got != S)
    assert bad.size == 0, f"first mismatch at {bad[0]}"
    thr, flip = _fold_to_dev(bn, K)
    bits = words_to_host(bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip))
    assert (bits == oracle.pack_bits(a_next)).all()


@pytest.mark.parametrize("seed", range(6))
def test_k_split_matrix_engine_kernel_randomized(seed):
    """Seeded random cases for kernel 10: M, N log-uniform up to 700, K a random multiple of 128 up to 10240, P(+1)
    anywhere in (0, 1), operand rows padded by a random multiple of 4 words and based a random multiple of 16 bytes
    into a junk-filled buffer: the exact product and the exact fused bits."""
    rng = np.random.default_rng(9090 + seed)
    for _case in range(15):
        M, N = (int(np.exp(rng.uniform(0, np.log(700)))) for _ in range(2))
        K = 128 * int(rng.integers(1, 81))
        p = rng.uniform(0.02, 0.98)
        A, Bm = synth.pm1(rng, (M, K), p), synth.pm1(rng, (K, N), p)
        bn = synth.bn_params(rng, N, K, adversarial=True)
        S, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
        kw = K // 32
        da = _offset_words(oracle.pack_bits(A), kw + 4 * int(rng.integers(0, 4)), 4 * int(rng.integers(0, 3)))
        db = _offset_words(oracle.pack_bits(np.ascontiguousarray(Bm.T)), kw + 4 * int(rng.integers(0, 4)), 4 * int(rng.integers(0, 3)))
        thr, flip = _fold_to_dev(bn, K)
        tag = f"seed {seed} M={M} N={N} K={K}"
        assert (bnn.xnor_gemm(da, db, K, kernel=bnn.KERNEL_MFMA_SPLITK).cpu().numpy() == S).all(), tag
        bits = words_to_host(bnn.xnor_gemm_bn_sign_pack(da, db, K, thr, flip, kernel=bnn.KERNEL_MFMA_SPLITK))
        assert (bits == oracle.pack_bits(a_next)).all(), tag


def test_k_split_matrix_engine_kernel_refuses_what_it_does_not_take():
    """Kernel id 10 answers BNN_ERR_UNSUPPORTED, launching nothing, outside its shapes: K not a multiple of
    128 (or zero), operands that do not allow 16-byte loads."""
    def refused(M, N, K, ld_extra=0, first=0, fused=False):
        kw = (K + 31) // 32
        a = torch.zeros(first + M * (kw + ld_extra), dtype=torch.int32, device=DEV)[first:].view(M, kw + ld_extra)[:, :kw]
        b = torch.zeros((N, kw + ld_extra), dtype=torch.int32, device=DEV)[:, :kw]
        with pytest.raises(bnn.BnnError) as e:
            if fused:
                thr = torch.zeros(N, dtype=torch.int32, device=DEV)
                flip = torch.zeros((N + 31) // 32, dtype=torch.int32, device=DEV)
                bnn.xnor_gemm_bn_sign_pack(a, b, K, thr, flip, kernel=bnn.KERNEL_MFMA_SPLITK)
            else:
                bnn.xnor_gemm(a, b, K, kernel=bnn.KERNEL_MFMA_SPLITK)
        return e.value.status == 3
    for fused in (False, True):
        assert refused(64, 64, 1000, fused=fused)
        assert refused(64, 64, 96, fused=fused)
        assert refused(64, 64, 1024 + 64, fused=fused)
        assert refused(64, 64, 1024, ld_extra=2, fused=fused)
        assert refused(64, 64, 1024, first=1, fused=fused)


def test_one_wavefront_per_simd_kernel_refuses_what_it_does_not_take():
    """Kernel id 9 answers BNN_ERR_UNSUPPORTED, launching nothing, outside its shapes: the int32 product,
    K not a multiple of 512 or below 2048, N not a multiple of 256 or with a tile count that does not divide
    the compute units, strips of fewer than 256 rows, operands that do not allow 16-byte loads, output rows
    that do not allow 8-byte stores."""
    def refused(M, N, K, ld_extra=0, out_extra=0, int32=False):
        kw = (K + 31) // 32
        a = torch.zeros((M, kw + ld_extra), dtype=torch.int32, device=DEV)[:, :kw]
        b = torch.zeros((N, kw + ld_extra), dtype=torch.int32, device=DEV)[:, :kw]
        thr = torch.zeros(N, dtype=torch.int32, device=DEV)
        flip = torch.zeros((N + 31) // 32, dtype=torch.int32, device=DEV)
        out = torch.zeros((M, (N + 31) // 32 + out_extra), dtype=torch.int32, device=DEV)[:, :(N + 31) // 32]
        with pytest.raises(bnn.BnnError) as e:
            if int32:
                bnn.xnor_gemm(a, b, K, kernel=bnn.KERNEL_MFMA_BIG)
            else:
                bnn.xnor_gemm_bn_sign_pack(a, b, K, thr, flip, out=out, kernel=bnn.KERNEL_MFMA_BIG)
        return e.value.status == 3
    assert refused(10000, 4096, 4096, int32=True)
    assert refused(10000, 4096, 4000)
    assert refused(10000, 4096, 1536)
    assert refused(10000, 4000, 4096)
    assert refused(10000, 768, 4096)             # 3 column tiles do not divide 256 compute units
    assert refused(4000, 4096, 4096)             # 16 strips of 250 rows
    assert refused(10000, 4096, 4096, ld_extra=1)
    assert refused(10000, 4096, 4096, out_extra=1)


_LARGE_SQUARE = {}


def _large_square_oracle():
    """The 8192^3 workload and the oracle's full product (a few seconds on the host cores), computed once
    for all the tests that check a kernel's 8192 x 8192 result on every element."""
    if not _LARGE_SQUARE:
        A, Bm = synth.config_gemm_square(synth.GEMM_LARGE)
        _LARGE_SQUARE.update(A=A, Bm=Bm, C=oracle.matmul_pm1(A, Bm))
    return _LARGE_SQUARE["A"], _LARGE_SQUARE["Bm"], _LARGE_SQUARE["C"]


@pytest.mark.parametrize("kernel", ["auto", "tiled128", "mfma", "mfma128"])
def test_xnor_gemm_large_square_hadamard_and_every_element(kernel):
    """8192^3 in the launch configuration the benchmark times.  (i) Sylvester-Hadamard
    operands: the full 8192 x 8192 result must be 8192 * I (closed form, checked on
    every element).  (ii) random +-1 operands: every element against the oracle's
    full product."""
    n = synth.GEMM_LARGE
    H = synth.hadamard(n)
    hb = words_to_dev(oracle.pack_bits(H))
    C = bnn.xnor_gemm(hb, hb, n, kernel=GEMM_KERNELS[kernel])
    assert torch.equal(C, n * torch.eye(n, dtype=torch.int32, device=DEV))
    del C
    A, Bm, want = _large_square_oracle()
    da = words_to_dev(oracle.pack_bits(A))
    db = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    C = bnn.xnor_gemm(da, db, n, kernel=GEMM_KERNELS[kernel]).cpu().numpy()
    bad = np.argwhere(C != want)
    assert bad.size == 0, f"first mismatch at {bad[0]}"
    assert (np.abs(C) <= n).all() and (C % 2 == 0).all()


def test_fused_layer_large_square_every_element():
    """bnn_xnor_gemm_bn_sign_pack at 8192^3 (the fused launch the benchmark also times): every output bit
    against the oracle's float BatchNorm + Sign of its full product."""
    n = synth.GEMM_LARGE
    A, Bm, S = _large_square_oracle()
    bn = synth.bn_params(synth.rng_for(4, 2), n, n, adversarial=True)
    want = oracle.pack_bits(oracle.bn_sign(S, *bn, eps=EPS))
    thr, flip = _fold_to_dev(bn, n)
    got = bnn.xnor_gemm_bn_sign_pack(words_to_dev(oracle.pack_bits(A)),
                                     words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T))), n, thr, flip)
    assert (words_to_host(got) == want).all()


def test_matrices_of_more_than_2_31_elements():
    """Maximum sizes: an int32 result of 2.16e9 elements (8.6 GB, element offsets beyond 2^31), the
    streaming epilogue and the Sign packer on matrices of that size, and the fused layer writing the
    same rows.  Rows are sampled at the start, around element 2^31 and at the ragged end."""
    M, N, K = 65536 + 130, 32768 + 70, 64
    rng = np.random.default_rng(231)
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    da = words_to_dev(oracle.pack_bits(A))
    db = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    thr, flip = _fold_to_dev(bn, K)
    first_past = (1 << 31) // N                         # the row that holds element 2^31
    rows = np.unique(np.concatenate([np.arange(3), np.arange(first_past - 2, first_past + 3), np.arange(M - 140, M)]))
    rows_t = torch.from_numpy(rows).to(DEV)
    S_want, a_want = oracle.dense_layer(A[rows], Bm, bn, eps=EPS)
    bits_want = oracle.pack_bits(a_want)
    C = torch.empty((M, N), dtype=torch.int32, device=DEV)
    for kernel in ("auto", "naive", "tiled128", "tiled64", "mfma", "mfma128"):
        C.fill_(0x5EED5EED)
        bnn.xnor_gemm(da, db, K, out=C, kernel=GEMM_KERNELS[kernel])
        assert (C[rows_t].cpu().numpy() == S_want).all(), kernel
        assert int(C.max()) <= K and int(C.min()) >= -K, kernel         # every element was written
    bits = bnn.bn_sign_pack(C, thr, flip)
    assert (words_to_host(bits[rows_t]) == bits_want).all()
    for kernel in ("auto", "tiled128", "mfma", "mfma128"):
        fused = bnn.xnor_gemm_bn_sign_pack(da, db, K, thr, flip, kernel=GEMM_KERNELS[kernel])
        assert torch.equal(fused, bits), kernel
    del bits, fused
    g = torch.Generator(device=DEV)
    g.manual_seed(231)
    x = C.view(torch.float32)                            # reuse the 8.6 GB: overwritten with N(0,1) draws
    x.normal_(generator=g)
    x[rows_t[0], :5] = torch.tensor([0.0, -0.0, float("nan"), 1e-45, -1e-45], device=DEV)
    packed = bnn.pack_sign(x)
    assert (words_to_host(packed[rows_t]) == oracle.pack_bits(oracle.sign(x[rows_t].cpu().numpy()))).all()


def test_packed_operand_of_more_than_4_GiB():
    """A packed A of 65666 x 2^19 bits (4.3 GB: byte offsets beyond 2^32) against a small B; the operand is
    drawn on the device from a seeded generator and the oracle multiplies sampled rows of it."""
    M, N, K = 65536 + 130, 40, 1 << 19
    kw = K // 32
    g = torch.Generator(device=DEV)
    g.manual_seed(232)
    da = torch.randint(-2 ** 31, 2 ** 31 - 1, (M, kw), dtype=torch.int32, device=DEV, generator=g)
    rng = np.random.default_rng(232)
    Bm = synth.pm1(rng, (K, N))
    db = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    rows = np.unique(np.concatenate([np.arange(2), [32767, 32768, 32769], np.arange(M - 6, M)]))
    rows_t = torch.from_numpy(rows).to(DEV)
    A_rows = oracle.unpack_bits(words_to_host(da[rows_t]), K)
    want = oracle.matmul_pm1(A_rows, Bm)
    for kernel in ("auto", "tiled64", "mfma128"):
        got = bnn.xnor_gemm(da, db, K, kernel=GEMM_KERNELS[kernel])
        assert (got[rows_t].cpu().numpy() == want).all(), kernel


# ------------------------------------------------------------------ bn_sign_pack

def _fold_to_dev(bn, K):
    thr, flip = bnn.bn_fold(*bn, EPS, K)
    return torch.from_numpy(thr).to(DEV), torch.from_numpy(flip.view(np.int32)).to(DEV)


@pytest.mark.parametrize("M,N,K,adv", [(64, 1024, 1024, False), (64, 1024, 1024, True), (5, 1, 40, True),
                                       (33, 31, 64, True), (100, 33, 784, True), (7, 1000, 4096, True),
                                       (300, 4096, 4096, False)])
def test_bn_sign_pack_matches_float_bn_then_sign(M, N, K, adv):
    rng = np.random.default_rng(M + N + K)
    bn = synth.bn_params(rng, N, K, adversarial=adv)
    # pre-activations on the lattice {-K, -K+2, ..., K}, concentrated near the thresholds
    S = np.clip(2 * np.rint(rng.normal(0, np.sqrt(K) / 2, (M, N))) + (K % 2), -K, K).astype(np.int32)
    want = oracle.pack_bits(oracle.bn_sign(S, *bn, eps=EPS))
    thr, flip = _fold_to_dev(bn, K)
    got = words_to_host(bnn.bn_sign_pack(torch.from_numpy(S).to(DEV), thr, flip))
    assert (got == want).all()


def test_bn_sign_pack_strided_unaligned_and_canary():
    rng = np.random.default_rng(9)
    M, N, K = 50, 77, 300
    bn = synth.bn_params(rng, N, K, adversarial=True)
    S = (2 * rng.integers(0, K + 1, (M, N)) - K).astype(np.int32)
    big = torch.zeros((M, N + 3), dtype=torch.int32, device=DEV)
    big[:, 1:N + 1] = torch.from_numpy(S).to(DEV)
    thr, flip = _fold_to_dev(bn, K)
    nw = (N + 31) // 32
    out = torch.full((M, nw + 2), 0x0BADBEEF, dtype=torch.int32, device=DEV)
    bnn.bn_sign_pack(big[:, 1:N + 1], thr, flip, out=out[:, :nw])
    host = words_to_host(out)
    assert (host[:, :nw] == oracle.pack_bits(oracle.bn_sign(S, *bn, eps=EPS))).all()
    assert (host[:, nw:] == 0x0BADBEEF).all()


# ------------------------------------------------------------------ fused GEMM + BN + Sign

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (7, 33, 31), (33, 7, 65), (64, 1024, 1024), (130, 200, 1000),
                                   (1000, 1000, 4097), (300, 4096, 784), (2000, 4096, 4096), (129, 95, 96)])
@pytest.mark.parametrize("kernel", ["auto", "tiled128", "tiled64", "mfma", "mfma128"])
def test_fused_layer_matches_float_bn_then_sign(M, N, K, kernel):
    """Alg. 4 hidden layer in one launch == oracle product, float BatchNorm, Sign, pack."""
    rng = np.random.default_rng(M * 3 + N * 5 + K * 7)
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    _s, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
    want = oracle.pack_bits(a_next)
    thr, flip = _fold_to_dev(bn, K)
    pa = words_to_dev(poison_pad_bits(oracle.pack_bits(A), K))
    pb = words_to_dev(poison_pad_bits(oracle.pack_bits(np.ascontiguousarray(Bm.T)), K))
    nw = (N + 31) // 32
    out = torch.full((M, nw + 1), 0x0BADF00D, dtype=torch.int32, device=DEV)
    bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip, out=out[:, :nw], kernel=GEMM_KERNELS[kernel])
    host = words_to_host(out)
    assert (host[:, :nw] == want).all()
    assert (host[:, nw:] == 0x0BADF00D).all()
    # and bit-identical to the two-call sequence
    two = bnn.bn_sign_pack(bnn.xnor_gemm(pa, pb, K), thr, flip)
    assert torch.equal(two, out[:, :nw])


@pytest.mark.parametrize("kernel", ["auto", "tiled128", "tiled64", "mfma", "mfma128"])
def test_fused_layer_with_thresholds_outside_the_result_range(kernel):
    """Thresholds need not come from the fold: any int32 is a valid threshold, including values far
    outside [-K, K] (constant channels).  Expected bits: (dot >= thr) XOR flip on the oracle's product."""
    M, N, K = 150, 130, 700
    rng = np.random.default_rng(77)
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    S = oracle.matmul_pm1(A, Bm)
    extremes = np.array([-2 ** 31, -2 ** 31 + 1, -2 ** 30, -K - 1, -K, -1, 0, 1, K, K + 1, 2 ** 30, 2 ** 31 - 1], np.int64)
    thr = extremes[rng.integers(0, len(extremes), N)].astype(np.int32)
    flip = rng.integers(0, 2, N).astype(bool)
    want_pm1 = np.where((S >= thr[None, :].astype(np.int64)) != flip[None, :], 1, -1).astype(np.int8)
    flip_words = oracle.pack_bits(np.where(flip, 1, -1).astype(np.int8)[None, :])[0]
    pa = words_to_dev(oracle.pack_bits(A))
    pb = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    got = bnn.xnor_gemm_bn_sign_pack(pa, pb, K, torch.from_numpy(thr).to(DEV), words_to_dev(flip_words[None, :])[0],
                                     kernel=GEMM_KERNELS[kernel])
    assert (words_to_host(got) == oracle.pack_bits(want_pm1)).all()


@pytest.mark.parametrize("adversarial", [False, True])
def test_fused_mlp_full_batch_every_row(adversarial):
    """Batch 10000 through the fused layers, as the benchmark runs it (adversarial=False is the benchmark's
    own workload): every row of every layer's packed activations and of the scores against the oracle."""
    x, weights, bns = synth.config_mlp(adversarial=adversarial)
    wr = [torch.from_numpy(np.ascontiguousarray(w.T).astype(np.float32)).to(DEV) for w in weights]
    net = bnn.BinaryMLP(wr, bns, EPS, synth.MLP_BATCH, fused=True)
    scores = net.forward(torch.from_numpy(x).to(DEV)).cpu().numpy()
    tr = oracle.mlp_forward(x, weights, bns, eps=EPS)
    for l in range(len(weights)):
        assert (words_to_host(net.a_bits[l]) == oracle.pack_bits(tr["a"][l])).all(), f"a^b_{l}"
    assert (scores == tr["s"][-1]).all()


# ------------------------------------------------------------------ conv_im2col_pack

def _pack_nhwc(x: np.ndarray) -> np.ndarray:
    B, H, W, C = x.shape
    return oracle.pack_bits(x.reshape(-1, C)).reshape(B, H, W, -1)


@pytest.mark.parametrize("shape", [
    # B, H, W, Cin, kh, kw, stride, pad
    (2, 8, 8, 128, 3, 3, 1, 1),
    (3, 5, 7, 32, 3, 3, 1, 1),
    (2, 6, 6, 64, 3, 3, 2, 1),
    (1, 9, 4, 96, 1, 1, 1, 0),
    (2, 5, 5, 3, 3, 3, 1, 1),
    (1, 7, 6, 40, 3, 3, 1, 1),
    (2, 4, 4, 33, 5, 3, 1, 2),
    (1, 32, 32, 128, 3, 3, 1, 1),
])
def test_im2col_pack_matches_oracle_lowering(shape):
    B, H, W, Cin, kh, kw, stride, pad = shape
    rng = np.random.default_rng(sum(shape))
    x = synth.pm1(rng, (B, H, W, Cin))
    want = oracle.pack_bits(oracle.im2col(x, kh, kw, stride, pad))
    xb = _pack_nhwc(x)
    if Cin % 32:
        xb[..., -1] |= np.uint32((0xFFFFFFFF << (Cin % 32)) & 0xFFFFFFFF)    # poisoned channel pad bits
    got = words_to_host(bnn.conv_im2col_pack(words_to_dev(xb.reshape(-1, xb.shape[-1])).view(B, H, W, -1),
                                             Cin, kh, kw, stride, pad))
    assert got.shape == want.shape
    assert (got == want).all()


def test_conv_layers_end_to_end_small_batch():
    """The three conv layer shapes (128@32x32, 256@16x16, 512@8x8), batch 2:
    im2col -> XNOR GEMM -> BN+Sign against direct convolution + float BN + Sign."""
    for layer in range(3):
        x, Wt, bn = synth.config_conv(layer, batch=2, adversarial=(layer == 1))
        S_want, a_want = oracle.conv_layer(x, Wt, bn, eps=EPS)
        B, H, W, C = x.shape
        conv = bnn.BinaryConvLayer(torch.from_numpy(Wt.astype(np.float32)).to(DEV), bn, EPS, B, H, W)
        xb = words_to_dev(_pack_nhwc(x).reshape(-1, C // 32)).view(B, H, W, C // 32)
        out = conv.forward(xb)
        assert (conv.s.cpu().numpy().reshape(S_want.shape) == S_want).all()
        assert (words_to_host(out.reshape(-1, out.shape[-1])) == oracle.pack_bits(a_want.reshape(-1, C))).all()


@pytest.mark.parametrize("implicit", [False, True])
@pytest.mark.parametrize("fused", [False, True])
def test_conv_layers_full_batch_every_image(fused, implicit):
    """Batch 256 as benchmarked, through the im2col matrix and without it: every pre-activation and every
    output bit of all 256 images against the oracle's direct convolution + float BatchNorm + Sign."""
    for layer in range(3):
        x, Wt, bn = synth.config_conv(layer, adversarial=fused)
        B, H, W, C = x.shape
        conv = bnn.BinaryConvLayer(torch.from_numpy(Wt.astype(np.float32)).to(DEV), bn, EPS, B, H, W, fused=fused,
                                   implicit=implicit)
        xb = words_to_dev(_pack_nhwc(x).reshape(-1, C // 32)).view(B, H, W, C // 32)
        out = words_to_host(conv.forward(xb).reshape(B * H * W, -1))
        assert conv.implicit == implicit
        S_want, a_want = oracle.conv_layer(x, Wt, bn, eps=EPS)
        if not fused:
            assert (conv.s.cpu().numpy().reshape(B, H, W, C) == S_want).all(), f"layer {layer}: pre-activations"
        assert (out == oracle.pack_bits(a_want.reshape(-1, C))).all(), f"layer {layer}: output bits"


@pytest.mark.parametrize("shape", [
    # B, H, W, Cin, Cout, kh, kw, stride, pad
    (2, 8, 8, 128, 64, 3, 3, 1, 1),
    (3, 5, 7, 128, 33, 3, 3, 1, 1),
    (2, 9, 6, 256, 130, 3, 3, 2, 1),
    (1, 6, 6, 128, 40, 5, 3, 1, 2),
    (2, 4, 4, 384, 16, 1, 1, 1, 0),
    (1, 32, 32, 128, 128, 3, 3, 1, 1),
    (40, 8, 8, 512, 512, 3, 3, 1, 1),
    # short receptive fields (K <= 1152): the conv mode of the short-K kernel
    (5, 13, 11, 128, 200, 3, 3, 2, 1),
    (3, 9, 9, 256, 64, 2, 2, 1, 0),
    (2, 5, 5, 1152, 32, 1, 1, 1, 0),
    (7, 3, 50, 128, 130, 3, 3, 1, 2),
    # "same" convolutions whose tiles are whole image rows or whole images: the LDS-patch kernel
    (3, 16, 16, 256, 130, 3, 3, 1, 1),      # 8 image rows per tile
    (5, 8, 8, 128, 40, 3, 3, 1, 1),         # 2 images per tile, the last tile holds one
    (2, 4, 4, 128, 33, 3, 3, 1, 1),         # 8 images per tile, 2 exist
    (1, 64, 64, 128, 64, 5, 5, 1, 2),       # 5 x 5 window, 2 image rows per tile
    (2, 32, 32, 128, 70, 1, 1, 1, 0),       # 1 x 1 window, no halo
    (3, 6, 128, 128, 20, 3, 3, 1, 1),       # one image row per tile
    (9, 16, 16, 384, 200, 3, 3, 1, 1),      # 3 channel quads per pixel, K-tiles that straddle taps
    # channel counts that are multiples of 32 but not of 128 (the half-width net's 64-channel block): the
    # LDS-patch kernel with single-word planes
    (6, 32, 32, 64, 64, 3, 3, 1, 1),        # 2 words per tap: 18 K-words, the last quad half empty
    (5, 16, 16, 32, 40, 3, 3, 1, 1),        # 1 word per tap: a step spans two taps, 9 K-words (odd)
    (3, 8, 8, 96, 130, 3, 3, 1, 1),         # 3 words per tap, two images per tile
    (2, 16, 16, 160, 33, 3, 3, 1, 1),       # 5 words per tap: 45 K-words
    (2, 4, 4, 64, 20, 5, 5, 1, 2),          # 5 x 5 window, 50 K-words, 8 images per tile of which 2 exist
    (40, 32, 32, 64, 64, 3, 3, 1, 1),       # 320 tiles of 128 pixels
    (520, 16, 16, 64, 128, 3, 3, 1, 1),     # 520 tiles of 256 pixels: the grid that takes the larger tile
])
def test_implicit_conv_matches_direct_convolution(shape):
    """Implicit-GEMM conv (no im2col matrix) == the oracle's direct convolution; fused form ==
    direct convolution, float BatchNorm, Sign."""
    B, H, W, Cin, Cout, kh, kw, stride, pad = shape
    rng = np.random.default_rng(sum(shape))
    x = synth.pm1(rng, (B, H, W, Cin))
    Wt = synth.pm1(rng, (Cout, kh, kw, Cin))
    bn = synth.bn_params(rng, Cout, kh * kw * Cin, adversarial=True)
    S = oracle.conv_direct(x, Wt, stride=stride, pad=pad)
    xb = words_to_dev(_pack_nhwc(x).reshape(-1, Cin // 32)).view(B, H, W, Cin // 32)
    wb = _aligned_words(oracle.pack_bits(Wt.reshape(Cout, -1)))     # junk behind filters that are not whole quads
    got = bnn.conv_xnor(xb, Cin, wb, kh, kw, stride, pad).cpu().numpy()
    assert (got.reshape(S.shape) == S).all()
    thr, flip = _fold_to_dev(bn, kh * kw * Cin)
    bits = words_to_host(bnn.conv_bn_sign_pack(xb, Cin, wb, thr, flip, kh, kw, stride, pad))
    want = oracle.pack_bits(oracle.bn_sign(S.reshape(-1, Cout), *bn, eps=EPS))
    assert (bits == want).all()


@pytest.mark.parametrize("seed", range(4))
def test_implicit_conv_randomized_geometries(seed):
    """Seeded random geometries (batch, image size, channels, filter size, stride, padding, filters):
    int32 sums against the oracle's direct convolution, fused bits against float BatchNorm + Sign."""
    rng = np.random.default_rng(777 + seed)
    for _case in range(12):
        kh, kw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        pad, stride = int(rng.integers(0, 3)), int(rng.integers(1, 3))
        H = int(rng.integers(max(1, kh - 2 * pad), 14))
        W = int(rng.integers(max(1, kw - 2 * pad), 14))
        B, Cin, Cout = int(rng.integers(1, 5)), 128 * int(rng.integers(1, 4)), int(rng.integers(1, 200))
        tag = f"seed {seed} B={B} H={H} W={W} Cin={Cin} Cout={Cout} k={kh}x{kw} stride={stride} pad={pad}"
        x = synth.pm1(rng, (B, H, W, Cin), rng.uniform(0.1, 0.9))
        Wt = synth.pm1(rng, (Cout, kh, kw, Cin))
        bn = synth.bn_params(rng, Cout, kh * kw * Cin, adversarial=True)
        S = oracle.conv_direct(x, Wt, stride=stride, pad=pad)
        xb = words_to_dev(_pack_nhwc(x).reshape(-1, Cin // 32)).view(B, H, W, Cin // 32)
        wb = words_to_dev(oracle.pack_bits(Wt.reshape(Cout, -1)))
        got = bnn.conv_xnor(xb, Cin, wb, kh, kw, stride, pad).cpu().numpy()
        assert (got.reshape(S.shape) == S).all(), tag
        thr, flip = _fold_to_dev(bn, kh * kw * Cin)
        bits = words_to_host(bnn.conv_bn_sign_pack(xb, Cin, wb, thr, flip, kh, kw, stride, pad))
        assert (bits == oracle.pack_bits(oracle.bn_sign(S.reshape(-1, Cout), *bn, eps=EPS))).all(), tag


@pytest.mark.parametrize("shape", [
    # B, H, W, Cin, Cout, k, stride, pad: receptive fields of just over 2^24 bits
    (1, 2, 2, (1 << 24) + 128, 3, 1, 1, 0),
    (1, 3, 3, 1864192, 2, 3, 1, 1),
    (1, 4, 3, 1864192 + 32, 5, 3, 2, 1),
])
def test_implicit_conv_past_the_matrix_engine_limit(shape):
    """K = kh*kw*Cin > 2^24 is beyond the exact range of the matrix engine's accumulation: bnn_conv_xnor and
    bnn_conv_bn_sign_pack take the xor/popcount kernel instead of refusing."""
    B, H, W, Cin, Cout, k, stride, pad = shape
    assert k * k * Cin > 1 << 24
    rng = np.random.default_rng(Cin % 100003)
    x = synth.pm1(rng, (B, H, W, Cin), 0.7)
    Wt = synth.pm1(rng, (Cout, k, k, Cin))
    bn = synth.bn_params(rng, Cout, k * k * Cin, adversarial=True)
    S = oracle.conv_direct(x, Wt, stride=stride, pad=pad)
    xb = words_to_dev(_pack_nhwc(x).reshape(-1, Cin // 32)).view(B, H, W, Cin // 32)
    wb = words_to_dev(oracle.pack_bits(Wt.reshape(Cout, -1)))
    got = bnn.conv_xnor(xb, Cin, wb, k, k, stride, pad).cpu().numpy()
    assert (got.reshape(S.shape) == S).all()
    thr, flip = _fold_to_dev(bn, k * k * Cin)
    bits = words_to_host(bnn.conv_bn_sign_pack(xb, Cin, wb, thr, flip, k, k, stride, pad))
    assert (bits == oracle.pack_bits(oracle.bn_sign(S.reshape(-1, Cout), *bn, eps=EPS))).all()


@pytest.mark.parametrize("seed", range(3))
def test_implicit_conv_randomized_same_size_layers_with_any_whole_word_channel_count(seed):
    """Seeded random same-size stride-1 layers whose rows tile 128 pixels, Cin any multiple of 32 up to 256
    (single-word planes unless Cin % 128 == 0): int32 sums, fused bits and the pooled layer."""
    rng = np.random.default_rng(4242 + seed)
    for _case in range(10):
        W = int(rng.choice([2, 4, 8, 16, 32, 64]))
        rows_per_tile = 128 // W
        H = int(rng.choice([h for h in (1, 2, 4, 6, 8, 12, 16, 32) if h % rows_per_tile == 0 or rows_per_tile % h == 0]))
        k = int(rng.choice([1, 3])) if W >= 2 else 1
        B, Cin, Cout = int(rng.integers(1, 6)), 32 * int(rng.integers(1, 9)), int(rng.integers(1, 200))
        if k * k * Cin > 2560 and Cin % 128:
            Cin = 64
        tag = f"seed {seed} B={B} H={H} W={W} Cin={Cin} Cout={Cout} k={k}"
        x = synth.pm1(rng, (B, H, W, Cin), rng.uniform(0.1, 0.9))
        Wt = synth.pm1(rng, (Cout, k, k, Cin))
        bn = synth.bn_params(rng, Cout, k * k * Cin, adversarial=True)
        pad = k // 2
        S = oracle.conv_direct(x, Wt, stride=1, pad=pad)
        xb = words_to_dev(_pack_nhwc(x).reshape(-1, Cin // 32)).view(B, H, W, Cin // 32)
        wb = _aligned_words(oracle.pack_bits(Wt.reshape(Cout, -1)))
        got = bnn.conv_xnor(xb, Cin, wb, k, k, 1, pad).cpu().numpy()
        assert (got.reshape(S.shape) == S).all(), tag
        thr, flip = _fold_to_dev(bn, k * k * Cin)
        bits = words_to_host(bnn.conv_bn_sign_pack(xb, Cin, wb, thr, flip, k, k, 1, pad))
        assert (bits == oracle.pack_bits(oracle.bn_sign(S.reshape(-1, Cout), *bn, eps=EPS))).all(), tag
        if H % 2 == 0 and W % 2 == 0 and W <= 32:
            try:
                pooled = bnn.conv_pool_bn_sign_pack(xb, Cin, wb, thr, flip, k, k, 1, pad)
            except bnn.BnnError as e:
                assert e.status == 3, tag            # a geometry whose pooling windows do not fit the tiles
                continue
            _P, a_want = oracle.conv_pool_layer(x, Wt, bn, pool=2, pad=pad, eps=EPS)
            assert (words_to_host(pooled) == oracle.pack_bits(a_want.reshape(-1, Cout))).all(), tag + " pooled"


def test_implicit_conv_rejects_what_only_the_im2col_path_takes():
    """BNN_ERR_UNSUPPORTED before any launch: channel counts that are not whole words, and channel counts
    that are not multiples of 128 on anything but a same-size stride-1 layer with a short receptive field."""
    def refused(x_shape, Cin, Cout, kh, kw, stride, pad):
        xb = torch.zeros(x_shape, dtype=torch.int32, device=DEV)
        wb = torch.zeros((Cout, (kh * kw * Cin + 31) // 32 + 3 & ~3), dtype=torch.int32, device=DEV)
        with pytest.raises(bnn.BnnError) as e:
            bnn.conv_xnor(xb, Cin, wb, kh, kw, stride, pad)
        return e.value.status == 3
    assert refused((1, 4, 4, 2), 40, 8, 3, 3, 1, 1)            # Cin % 32 != 0
    assert refused((1, 8, 8, 2), 64, 8, 3, 3, 2, 1)            # stride 2
    assert refused((1, 8, 8, 2), 64, 8, 3, 3, 1, 0)            # output smaller than the input
    assert refused((1, 5, 7, 2), 64, 8, 3, 3, 1, 1)            # image rows do not tile 128 pixels
    assert refused((1, 8, 8, 11), 352, 8, 3, 3, 1, 1)          # 99 K-words: filters not resident


def test_conv_layer_class_falls_back_to_im2col_for_other_channel_counts():
    """BinaryConvLayer(implicit=True) on a layer the implicit form refuses (40 channels: taps that are not
    whole words; 64 channels at stride 2) lowers through bnn_conv_im2col_pack instead, same result."""
    for (B, H, W, Cin, Cout, stride) in [(2, 6, 6, 40, 33, 1), (3, 9, 9, 64, 20, 2)]:
        rng = np.random.default_rng(B + Cin)
        x = synth.pm1(rng, (B, H, W, Cin))
        Wt = synth.pm1(rng, (Cout, 3, 3, Cin))
        bn = synth.bn_params(rng, Cout, 9 * Cin, adversarial=True)
        S_want, a_want = oracle.conv_layer(x, Wt, bn, stride=stride, eps=EPS)
        for fused in (False, True):
            conv = bnn.BinaryConvLayer(torch.from_numpy(Wt.astype(np.float32)).to(DEV), bn, EPS, B, H, W, stride=stride,
                                       fused=fused, implicit=True)
            xb = words_to_dev(_pack_nhwc(x).reshape(-1, (Cin + 31) // 32)).view(B, H, W, -1)
            out = words_to_host(conv.forward(xb).reshape(-1, (Cout + 31) // 32))
            assert not conv.implicit
            if not fused:
                assert (conv.s.cpu().numpy().reshape(S_want.shape) == S_want).all()
            assert (out == oracle.pack_bits(a_want.reshape(-1, Cout))).all()


@pytest.mark.parametrize("shape", [(2, 8, 8, 128, 2, 2), (3, 7, 9, 40, 2, 2), (1, 6, 6, 33, 3, 3), (2, 5, 5, 64, 2, 1)])
def test_maxpool_bits_matches_pooling_of_preactivations(shape):
    """Pooling on output bits == the oracle's max pooling of int32 pre-activations, then float
    BatchNorm, then Sign (the paper's order), including gamma < 0 and gamma == 0 channels."""
    B, H, W, C, pool, stride = shape
    rng = np.random.default_rng(sum(shape))
    K = 300
    S = (2 * rng.integers(0, K + 1, (B, H, W, C)) - K).astype(np.int32)
    S = np.clip(np.rint(S / 8), -K, K).astype(np.int32)           # concentrate near the thresholds
    bn = synth.bn_params(rng, C, K, adversarial=True)
    want = oracle.bn_sign(oracle.maxpool2d(S, pool, pool, stride).reshape(-1, C), *bn, eps=EPS)
    thr, flip = _fold_to_dev(bn, K)
    bits = bnn.bn_sign_pack(torch.from_numpy(S.reshape(-1, C)).to(DEV), thr, flip)
    pooled = bnn.maxpool_bits(bits.view(B, H, W, -1), C, flip, pool, pool, stride)
    assert (words_to_host(pooled.reshape(-1, pooled.shape[-1])) == oracle.pack_bits(want)).all()


@pytest.mark.parametrize("shape", [
    # B, H, W, Cin, Cout
    (3, 32, 32, 128, 130),      # row pairs in neighbouring accumulator blocks
    (5, 16, 16, 256, 64),       # vertical neighbour 16 lanes away
    (6, 8, 8, 128, 40),         # two images per tile
    (3, 4, 4, 128, 33),
    (70, 2, 2, 128, 20),        # 32 images per tile, the last tile partly empty
    (2, 64, 64, 128, 40),       # 64-pixel rows: row pairs two blocks apart (256-pixel tiles)
    (300, 32, 32, 128, 128),    # enough tiles for the 256-pixel form
])
def test_conv_pool_layer_in_one_launch(shape):
    """conv -> 2x2 max pool of the pre-activations -> BatchNorm -> Sign in one launch against the oracle's
    layer in that order, and against the two-call sequence (conv_bn_sign_pack, maxpool_bits)."""
    B, H, W, Cin, Cout = shape
    rng = np.random.default_rng(sum(shape))
    x = synth.pm1(rng, (B, H, W, Cin))
    Wt = synth.pm1(rng, (Cout, 3, 3, Cin))
    bn = synth.bn_params(rng, Cout, 9 * Cin, adversarial=True)
    xb = words_to_dev(_pack_nhwc(x).reshape(-1, Cin // 32)).view(B, H, W, Cin // 32)
    wb = words_to_dev(oracle.pack_bits(Wt.reshape(Cout, -1)))
    thr, flip = _fold_to_dev(bn, 9 * Cin)
    got = bnn.conv_pool_bn_sign_pack(xb, Cin, wb, thr, flip)
    bits = bnn.conv_bn_sign_pack(xb, Cin, wb, thr, flip)
    two_calls = bnn.maxpool_bits(bits.view(B, H, W, -1), Cout, flip, 2, 2, 2)
    assert torch.equal(got, two_calls.reshape(got.shape))
    imgs = list(range(B)) if B <= 8 else [0, B // 2, B - 1]
    for img in imgs:
        _P, a_want = oracle.conv_pool_layer(x[img:img + 1], Wt, bn, pool=2, eps=EPS)
        per = (H // 2) * (W // 2)
        assert (words_to_host(got[img * per:(img + 1) * per]) == oracle.pack_bits(a_want.reshape(-1, Cout))).all(), img


def test_conv_pool_layer_refuses_what_does_not_fit_its_tiles():
    for (H, W, stride, pool) in ((6, 6, 1, 2), (32, 32, 2, 2), (32, 32, 1, 3), (16, 128, 1, 2)):
        xb = torch.zeros((2, H, W, 4), dtype=torch.int32, device=DEV)
        wb = torch.zeros((8, 36), dtype=torch.int32, device=DEV)
        thr = torch.zeros(8, dtype=torch.int32, device=DEV)
        flip = torch.zeros(1, dtype=torch.int32, device=DEV)
        with pytest.raises(bnn.BnnError) as e:
            bnn.conv_pool_bn_sign_pack(xb, 128, wb, thr, flip, 3, 3, stride, 1, pool)
        assert e.value.status == 3, (H, W, stride, pool)
    # the layer class falls back to the two-call sequence on such a geometry
    x, Wt, bn = synth.config_conv(0, batch=2, size=6)
    conv = bnn.BinaryConvLayer(torch.from_numpy(Wt.astype(np.float32)).to(DEV), bn, EPS, 2, 6, 6, fused=True,
                               implicit=True, pool=2)
    xb = words_to_dev(_pack_nhwc(x).reshape(-1, 4)).view(2, 6, 6, 4)
    out = words_to_host(conv.forward(xb).reshape(2 * 9, -1))
    _P, a_want = oracle.conv_pool_layer(x, Wt, bn, pool=2, eps=EPS)
    assert (out == oracle.pack_bits(a_want.reshape(-1, 128))).all() and not conv.pool_in_conv


def test_conv_pool_layers_full_batch_every_image():
    """conv -> max pool -> BatchNorm -> Sign at batch 256 with the implicit, fused layer and the pooling
    inside the launch: every output bit of all 256 images."""
    for layer in range(3):
        x, Wt, bn = synth.config_conv(layer, adversarial=True)
        B, H, W, C = x.shape
        conv = bnn.BinaryConvLayer(torch.from_numpy(Wt.astype(np.float32)).to(DEV), bn, EPS, B, H, W, fused=True,
                                   implicit=True, pool=2)
        xb = words_to_dev(_pack_nhwc(x).reshape(-1, C // 32)).view(B, H, W, C // 32)
        out = words_to_host(conv.forward(xb).reshape(B * (H // 2) * (W // 2), -1))
        assert conv.pool_in_conv
        _P, a_want = oracle.conv_pool_layer(x, Wt, bn, pool=2, eps=EPS)
        assert (out == oracle.pack_bits(a_want.reshape(-1, C))).all(), f"layer {layer}"


def _convnet_oracle(x, convs, fcs, fc_bns):
    """The ConvNet body in the paper's order, from the oracle's layer functions: per convolution
    conv -> (max pool of the pre-activations) -> BatchNorm -> Sign; then the dense layers."""
    acts = []
    a = x
    for (Wt, bn), (_cin, _cout, _hw, pooled) in zip(convs, synth.CONVNET_CONVS):
        a = oracle.conv_pool_layer(a, Wt, bn, pool=2, eps=EPS)[1] if pooled else oracle.conv_layer(a, Wt, bn, eps=EPS)[1]
        acts.append(a)
    v = a.reshape(a.shape[0], -1)
    for Bm, bn in zip(fcs[:-1], fc_bns):
        v = oracle.dense_layer(v, Bm, bn, eps=EPS)[1]
        acts.append(v)
    return acts, oracle.matmul_pm1(v, fcs[-1])


def _convnet_on_gpu(x, convs, fcs, fc_bns):
    B = x.shape[0]
    dev_convs = [(torch.from_numpy(Wt.astype(np.float32)).to(DEV), bn, pooled)
                 for (Wt, bn), (_ci, _co, _hw, pooled) in zip(convs, synth.CONVNET_CONVS)]
    dev_fcs = [torch.from_numpy(np.ascontiguousarray(Bm.T).astype(np.float32)).to(DEV) for Bm in fcs]
    net = bnn.BinaryConvNet(dev_convs, dev_fcs, fc_bns, EPS, B, 32, 32)
    xb = words_to_dev(_pack_nhwc(x).reshape(-1, 4)).view(B, 32, 32, 4)
    scores = net.forward(xb).cpu().numpy()
    return net, scores


def test_convnet_body_every_intermediate_small_batch():
    """128C3-MP2-256C3-256C3-MP2-512C3-512C3-MP2-1024FC-1024FC-10 on 3 images: every layer's packed output
    and the scores against the oracle's chain (pooling of pre-activations before BatchNorm + Sign)."""
    x, convs, fcs, fc_bns = synth.config_convnet(batch=3, adversarial=True)
    acts, scores_want = _convnet_oracle(x, convs, fcs, fc_bns)
    net, scores = _convnet_on_gpu(x, convs, fcs, fc_bns)
    for l, layer in enumerate(net.convs):
        got = layer.pooled if layer.pool else layer.out_bits
        C = acts[l].shape[-1]
        assert (words_to_host(got.reshape(-1, C // 32)) == oracle.pack_bits(acts[l].reshape(-1, C))).all(), f"conv {l}"
    for l, a in enumerate(net.a_bits):
        assert (words_to_host(a) == oracle.pack_bits(acts[len(net.convs) + l])).all(), f"dense {l}"
    assert (scores == scores_want).all()


def test_convnet_body_full_batch_every_image():
    """Batch 256 as benchmarked: every layer's packed output and the scores of all 256 images against the
    oracle's chain."""
    x, convs, fcs, fc_bns = synth.config_convnet()
    acts, scores_want = _convnet_oracle(x, convs, fcs, fc_bns)
    net, scores = _convnet_on_gpu(x, convs, fcs, fc_bns)
    for l, layer in enumerate(net.convs):
        got = layer.pooled if layer.pool else layer.out_bits
        C = acts[l].shape[-1]
        assert (words_to_host(got.reshape(-1, C // 32)) == oracle.pack_bits(acts[l].reshape(-1, C))).all(), f"conv {l}"
    for l, a in enumerate(net.a_bits):
        assert (words_to_host(a) == oracle.pack_bits(acts[len(net.convs) + l])).all(), f"dense {l}"
    assert (scores == scores_want).all()


# ------------------------------------------------------------------ MLP chain

def _mlp_on_gpu(x, weights, bns, batch):
    wr = [torch.from_numpy(np.ascontiguousarray(w.T).astype(np.float32)).to(DEV) for w in weights]
    net = bnn.BinaryMLP(wr, bns, EPS, batch)
    net.forward(torch.from_numpy(x).to(DEV))
    torch.cuda.synchronize()
    return net


def test_mlp_chain_every_intermediate_small_batch():
    x, weights, bns = synth.config_mlp(batch=200, adversarial=True)
    tr = oracle.mlp_forward(x, weights, bns, eps=EPS)
    net = _mlp_on_gpu(x, weights, bns, 200)
    for l in range(len(weights)):
        assert (words_to_host(net.a_bits[l]) == oracle.pack_bits(tr["a"][l])).all(), f"a^b_{l}"
        assert (net.s[l].cpu().numpy() == tr["s"][l]).all(), f"s_{l}"


def test_mlp_forward_captured_in_a_hip_graph_replays_bit_exact():
    """The library allocates nothing and never synchronises, so a forward pass can be captured in a HIP
    graph.  Every replay, on fresh inputs written into the captured input buffer and with eager work and
    synchronisations in between, must give the oracle's scores and activations."""
    batch = 600
    x0, weights, bns = synth.config_mlp(batch=batch, adversarial=True)
    wr = [torch.from_numpy(np.ascontiguousarray(w.T).astype(np.float32)).to(DEV) for w in weights]
    net = bnn.BinaryMLP(wr, bns, EPS, batch)
    x_static = torch.from_numpy(x0).to(DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                        # warm-up outside the capture, as torch asks
        net.forward(x_static)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        net.forward(x_static)
    rng = np.random.default_rng(600)
    for replay in range(4):
        x = synth.real_input(rng, x0.shape)
        tr = oracle.mlp_forward(x, weights, bns, eps=EPS)
        x_static.copy_(torch.from_numpy(x))
        for buf in net.s + net.a_bits:
            if buf is not None:
                buf.fill_(0x3C3C3C3C)                        # nothing may survive from the previous replay
        graph.replay()
        torch.cuda.synchronize()
        assert (net.s[-1].cpu().numpy() == tr["s"][-1]).all(), f"scores, replay {replay}"
        for l in range(1, len(weights)):
            assert (words_to_host(net.a_bits[l]) == oracle.pack_bits(tr["a"][l])).all(), f"a^b_{l}, replay {replay}"
        # eager work of the same library between the replays
        net.forward(torch.from_numpy(x0).to(DEV))
        torch.cuda.synchronize()
        assert (net.s[-1].cpu().numpy() == oracle.mlp_forward(x0, weights, bns, eps=EPS)["s"][-1]).all()


@pytest.mark.parametrize("kernel,K", [(bnn.KERNEL_MFMA_PERSIST, 1024), (bnn.KERNEL_MFMA_BIG, 2048)])
def test_tile_walk_kernel_captured_in_a_hip_graph_replays_bit_exact(kernel, K):
    """The kernels in which a workgroup takes several output tiles keep no state between launches (no
    counters, no scratch memory): captured in a HIP graph, every replay on new inputs, with eager launches
    of the same kernel in between, gives the oracle's bits."""
    M, N = 10000, 4096
    rng = np.random.default_rng(31)
    Bm = synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    pb = words_to_dev(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    thr, flip = _fold_to_dev(bn, K)
    a_static = torch.zeros((M, K // 32), dtype=torch.int32, device=DEV)
    out = torch.zeros((M, N // 32), dtype=torch.int32, device=DEV)
    launch = lambda: bnn.xnor_gemm_bn_sign_pack(a_static, pb, K, thr, flip, out=out, kernel=kernel)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        launch()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        launch()
    for replay in range(3):
        A = synth.pm1(rng, (M, K), 0.3 + 0.2 * replay)
        want = oracle.pack_bits(oracle.dense_layer(A, Bm, bn, eps=EPS)[1])
        a_static.copy_(words_to_dev(oracle.pack_bits(A)))
        out.fill_(0x3C3C3C3C)
        graph.replay()
        torch.cuda.synchronize()
        assert (words_to_host(out) == want).all(), f"replay {replay}"
        out.fill_(0)
        launch()                                     # eager, between the replays
        torch.cuda.synchronize()
        assert (words_to_host(out) == want).all(), f"eager launch after replay {replay}"


def test_mlp_full_batch_every_row():
    """Batch 10000 with separate GEMM and BN+Sign launches: every int32 pre-activation and every packed
    activation of all 10000 rows against the oracle."""
    x, weights, bns = synth.config_mlp()
    net = _mlp_on_gpu(x, weights, bns, synth.MLP_BATCH)
    tr = oracle.mlp_forward(x, weights, bns, eps=EPS)
    for l in range(len(weights)):
        assert (words_to_host(net.a_bits[l]) == oracle.pack_bits(tr["a"][l])).all(), f"a^b_{l}"
        assert (net.s[l].cpu().numpy() == tr["s"][l]).all(), f"s_{l}"


# ------------------------------------------------------------------ first layer on 8-bit inputs

@pytest.mark.parametrize("rows,cols", [(1, 1), (3, 31), (5, 32), (7, 33), (33, 784), (130, 100), (2, 4099)])
def test_pack_bitplanes(rows, cols):
    """Plane p of the packed output == the oracle's packing of bit p of every input byte."""
    rng = np.random.default_rng(rows * 131 + cols)
    X = synth.uint8_input(rng, (rows, cols))
    X.flat[:4] = (0, 255, 1, 128)[:min(4, X.size)]
    got = words_to_host(bnn.pack_bitplanes(torch.from_numpy(X).to(DEV)))
    kw = (cols + 31) // 32
    assert got.shape == (rows, 8 * kw)
    for p in range(8):
        plane = np.where((X >> p) & 1, 1, -1).astype(np.int8)
        assert (got[:, p::8] == oracle.pack_bits(plane)).all(), f"plane {p}"


def test_pack_bitplanes_unaligned_input():
    rng = np.random.default_rng(5)
    big = synth.uint8_input(rng, (9, 77))
    xd = torch.from_numpy(big).to(DEV)[:, 1:71]             # base 1 byte off, ld 77
    got = words_to_host(bnn.pack_bitplanes(xd))
    for p in range(8):
        plane = np.where((big[:, 1:71] >> p) & 1, 1, -1).astype(np.int8)
        assert (got[:, p::8] == oracle.pack_bits(plane)).all()


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (7, 33, 31), (33, 7, 65), (130, 200, 1000), (300, 4096, 784),
                                   (513, 129, 96), (64, 1024, 1024), (1000, 10, 784)])
def test_bitplane_gemm_first_layer(M, N, K):
    """Alg. 4 step 1 / Sec. 1.6: sum_n 2^(n-1) <x^n, w> on 8-bit inputs, and its fused BN+Sign form."""
    rng = np.random.default_rng(M * 17 + N * 3 + K)
    X = synth.uint8_input(rng, (M, K))
    Wb = synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, 255 * K, adversarial=True)
    bn = (bn[0], bn[1], (bn[2] * 4).astype(np.float32), bn[3])        # spread the thresholds over the wider range
    S = oracle.first_layer_bitplanes(X, Wb)
    planes = bnn.pack_bitplanes(torch.from_numpy(X).to(DEV))
    wb = words_to_dev(poison_pad_bits(oracle.pack_bits(np.ascontiguousarray(Wb.T)), K))
    got = bnn.bitplane_gemm(planes, wb, K).cpu().numpy()
    assert (got == S).all()
    thr, flip = bnn.bn_fold(*bn, EPS, 255 * K)
    fused = bnn.bitplane_gemm_bn_sign_pack(planes, wb, K, torch.from_numpy(thr).to(DEV),
                                           torch.from_numpy(flip.view(np.int32)).to(DEV))
    assert (words_to_host(fused) == oracle.pack_bits(oracle.bn_sign(S, *bn, eps=EPS))).all()


def test_bitplane_gemm_ignores_pad_bits_of_the_planes():
    rng = np.random.default_rng(8)
    M, N, K = 40, 50, 70
    X = synth.uint8_input(rng, (M, K))
    Wb = synth.pm1(rng, (K, N))
    planes = words_to_host(bnn.pack_bitplanes(torch.from_numpy(X).to(DEV))).copy()
    planes[:, -8:] |= np.uint32((0xFFFFFFFF << (K % 32)) & 0xFFFFFFFF)      # poison the last K-word of every plane
    got = bnn.bitplane_gemm(words_to_dev(planes), words_to_dev(oracle.pack_bits(np.ascontiguousarray(Wb.T))), K)
    assert (got.cpu().numpy() == oracle.first_layer_bitplanes(X, Wb)).all()


@pytest.mark.parametrize("fused", [False, True])
def test_mlp_uint8_first_layer_full_batch_every_row(fused):
    """Alg. 4 as printed (8-bit inputs through bit planes), batch 10000, MNIST-shaped MLP: every row."""
    _x, weights, bns = synth.config_mlp()
    x8 = synth.uint8_input(synth.rng_for(1, 1), (synth.MLP_BATCH, synth.MLP_SIZES[0]))
    bn0 = synth.bn_params(synth.rng_for(1, 30), synth.MLP_SIZES[1], 255 * synth.MLP_SIZES[0])
    bns = [bn0] + list(bns[1:])
    wr = [torch.from_numpy(np.ascontiguousarray(w.T).astype(np.float32)).to(DEV) for w in weights]
    net = bnn.BinaryMLP(wr, bns, EPS, synth.MLP_BATCH, fused=fused, input_uint8=True)
    scores = net.forward(torch.from_numpy(x8).to(DEV)).cpu().numpy()
    tr = oracle.mlp_forward_uint8(x8, weights, bns, eps=EPS)
    for l in range(1, len(weights)):
        assert (words_to_host(net.a_bits[l]) == oracle.pack_bits(tr["a"][l])).all(), f"a^b_{l}"
    if not fused:
        assert (net.s[0].cpu().numpy() == tr["s"][0]).all()
    assert (scores == tr["s"][-1]).all()


# ------------------------------------------------------------------ int8 MFMA variant

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (7, 33, 31), (33, 7, 65), (128, 128, 64), (130, 200, 1000),
                                   (1000, 1000, 4097), (64, 1024, 1024), (513, 129, 96)])
def test_gemm_i8_mfma_matches_oracle(M, N, K):
    rng = np.random.default_rng(M * 31 + N * 7 + K)
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    want = oracle.matmul_pm1(A, Bm)
    ld = (K + 15) // 16 * 16
    a = torch.full((M, ld), 77, dtype=torch.int8, device=DEV)       # junk in the row padding
    b = torch.full((N, ld), 77, dtype=torch.int8, device=DEV)
    a[:, :K] = torch.from_numpy(A).to(DEV)
    b[:, :K] = torch.from_numpy(np.ascontiguousarray(Bm.T)).to(DEV)
    got = bnn.gemm_i8_mfma(a[:, :K], b[:, :K]).cpu().numpy()
    assert (got == want).all()


def test_unpack_i8_then_mfma_equals_xnor_path():
    rng = np.random.default_rng(11)
    M, N, K = 300, 260, 1000
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    pa = words_to_dev(poison_pad_bits(oracle.pack_bits(A), K))
    pb = words_to_dev(poison_pad_bits(oracle.pack_bits(np.ascontiguousarray(Bm.T)), K))
    a8, b8 = bnn.unpack_i8(pa, K), bnn.unpack_i8(pb, K)
    assert (a8.cpu().numpy() == A).all()
    assert (b8.cpu().numpy() == Bm.T).all()
    assert (bnn.gemm_i8_mfma(a8, b8).cpu().numpy() == oracle.matmul_pm1(A, Bm)).all()


def test_gemm_i8_mfma_large_square_every_element():
    n = synth.GEMM_LARGE
    A, Bm, want = _large_square_oracle()
    a = torch.from_numpy(A).to(DEV)
    b = torch.from_numpy(np.ascontiguousarray(Bm.T)).to(DEV)
    C = bnn.gemm_i8_mfma(a, b).cpu().numpy()
    assert (C == want).all()
    H = torch.from_numpy(synth.hadamard(n)).to(DEV)
    assert torch.equal(bnn.gemm_i8_mfma(H, H), n * torch.eye(n, dtype=torch.int32, device=DEV))


# ------------------------------------------------------------------ the C ABI from a non-Python caller

def test_c_abi_from_a_plain_hip_program():
    """tests/c_abi/hidden_layer.cpp (built by __graft_entry__.build()) links against libbnn_hip.so, allocates
    with the HIP runtime and runs one hidden layer through include/bnn.h; it checks the results itself."""
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "hidden_layer")
    assert os.path.exists(exe), "tests/c_abi/hidden_layer is not built: run __graft_entry__.build()"
    proc = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert proc.returncode == 0 and "c_abi ok" in proc.stdout, proc.stdout

