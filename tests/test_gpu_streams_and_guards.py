"""Every entry point of the C ABI once on the default stream and once on a second stream, writing into an
output that lies inside a larger allocation with guard words BEFORE its first row, AFTER its last row and
between the rows: the result must equal the oracle's on both streams and no guard word may change.
(The parity tests proper are in test_gpu_parity.py; this file is about where a kernel writes and which
stream it runs on.)"""
import numpy as np
import pytest
import torch

import oracle
import paper_1602_02830_amd as bnn
from workloads import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
EPS = oracle.EPS_DEFAULT
GUARD32 = 0x6B6B6B6B
GUARD8 = 0x6B


class Guarded:
    """A [rows][cols] output view with leading dimension cols + pad_cols inside a flat allocation that has
    `lead` guard elements in front of the first row and `tail` behind the last one.  lead keeps the view
    16-byte aligned, so the kernels' fast paths are the ones under test."""

    def __init__(self, rows, cols, dtype=torch.int32, pad_cols=3, lead=64, tail=64):
        self.rows, self.cols, self.ld, self.lead = rows, cols, cols + pad_cols, lead
        self.guard = GUARD8 if dtype == torch.int8 else GUARD32
        self.flat = torch.full((lead + rows * self.ld + tail,), self.guard, dtype=dtype, device=DEV)
        self.view = self.flat[lead:lead + rows * self.ld].view(rows, self.ld)[:, :cols]

    def result_and_check(self):
        host = self.flat.cpu().numpy()
        body = host[self.lead:self.lead + self.rows * self.ld].reshape(self.rows, self.ld)
        assert (host[:self.lead] == self.guard).all(), "guard words before the output were overwritten"
        assert (host[self.lead + self.rows * self.ld:] == self.guard).all(), "guard words after the output were overwritten"
        assert (body[:, self.cols:] == self.guard).all(), "guard words between the rows were overwritten"
        return body[:, :self.cols].copy()


def _dev_words(w):
    return torch.from_numpy(np.ascontiguousarray(w).view(np.int32)).to(DEV)


def _fold(bn, K):
    thr, flip = bnn.bn_fold(*bn, EPS, K)
    return torch.from_numpy(thr).to(DEV), torch.from_numpy(flip.view(np.int32)).to(DEV)


def _pack_nhwc(x):
    B, H, W, C = x.shape
    return oracle.pack_bits(x.reshape(-1, C)).reshape(B, H, W, -1)


def _cases():
    """(name, make_output, launch(out_view), expected numpy) per entry point; inputs live on the device."""
    rng = np.random.default_rng(20260)
    cases = []

    # bnn_pack_sign
    x = synth.real_input(rng, (37, 100))
    xd = torch.from_numpy(x).to(DEV)
    cases.append(("pack_sign", lambda: Guarded(37, 4), lambda o: bnn.pack_sign(xd, out=o),
                  oracle.pack_bits(oracle.sign(x)).view(np.int32)))

    # bnn_xnor_gemm(_kernel) and bnn_xnor_gemm_bn_sign_pack(_kernel), every kernel id
    M, N, K = 130, 200, 1000
    A, Bm = synth.pm1(rng, (M, K)), synth.pm1(rng, (K, N))
    bn = synth.bn_params(rng, N, K, adversarial=True)
    S, a_next = oracle.dense_layer(A, Bm, bn, eps=EPS)
    pa, pb = _dev_words(oracle.pack_bits(A)), _dev_words(oracle.pack_bits(np.ascontiguousarray(Bm.T)))
    thr, flip = _fold(bn, K)
    for name, kid in [("auto", bnn.KERNEL_AUTO), ("naive", bnn.KERNEL_NAIVE), ("tiled128", bnn.KERNEL_TILED128),
                      ("ksplit", bnn.KERNEL_KSPLIT), ("tiled64", bnn.KERNEL_TILED64), ("mfma", bnn.KERNEL_MFMA),
                      ("mfma128", bnn.KERNEL_MFMA128), ("mfma_shortk", bnn.KERNEL_MFMA_SHORTK)]:
        cases.append((f"xnor_gemm[{name}]", lambda: Guarded(M, N),
                      lambda o, kid=kid: bnn.xnor_gemm(pa, pb, K, out=o, kernel=kid), S))
        if name not in ("naive", "ksplit"):
            cases.append((f"xnor_gemm_bn_sign_pack[{name}]", lambda: Guarded(M, (N + 31) // 32),
                          lambda o, kid=kid: bnn.xnor_gemm_bn_sign_pack(pa, pb, K, thr, flip, out=o, kernel=kid),
                          oracle.pack_bits(a_next).view(np.int32)))

    # the whole-tile 256 x 128 kernel as a tile walk (kernel id 8) needs more tiles than the chip holds at once
    Mw, Nw, Kw = 10241, 4096, 1024
    Aw, Bw = synth.pm1(rng, (Mw, Kw)), synth.pm1(rng, (Kw, Nw))
    bnw = synth.bn_params(rng, Nw, Kw, adversarial=True)
    Sw, aw_next = oracle.dense_layer(Aw, Bw, bnw, eps=EPS)
    paw, pbw = _dev_words(oracle.pack_bits(Aw)), _dev_words(oracle.pack_bits(np.ascontiguousarray(Bw.T)))
    thrw, flipw = _fold(bnw, Kw)
    cases.append(("xnor_gemm[mfma_walk]", lambda: Guarded(Mw, Nw),
                  lambda o: bnn.xnor_gemm(paw, pbw, Kw, out=o, kernel=bnn.KERNEL_MFMA_PERSIST), Sw))
    cases.append(("xnor_gemm[mfma_whole_tiles]", lambda: Guarded(Mw, Nw),
                  lambda o: bnn.xnor_gemm(paw, pbw, Kw, out=o, kernel=bnn.KERNEL_MFMA), Sw))
    cases.append(("xnor_gemm_bn_sign_pack[mfma_walk]", lambda: Guarded(Mw, Nw // 32),
                  lambda o: bnn.xnor_gemm_bn_sign_pack(paw, pbw, Kw, thrw, flipw, out=o, kernel=bnn.KERNEL_MFMA_PERSIST),
                  oracle.pack_bits(aw_next).view(np.int32)))

    # the 256 x 256-tile kernel of the fused layer (kernel id 9): strips of two tiles and a 128-row tile
    Mg, Ng, Kg = 5000, 2048, 2048
    Ag, Bg = synth.pm1(rng, (Mg, Kg)), synth.pm1(rng, (Kg, Ng))
    bng = synth.bn_params(rng, Ng, Kg, adversarial=True)
    _, ag_next = oracle.dense_layer(Ag, Bg, bng, eps=EPS)
    pag, pbg = _dev_words(oracle.pack_bits(Ag)), _dev_words(oracle.pack_bits(np.ascontiguousarray(Bg.T)))
    thrg, flipg = _fold(bng, Kg)
    cases.append(("xnor_gemm_bn_sign_pack[mfma_big]", lambda: Guarded(Mg, Ng // 32, pad_cols=2),   # rows of 8-byte stores
                  lambda o: bnn.xnor_gemm_bn_sign_pack(pag, pbg, Kg, thrg, flipg, out=o, kernel=bnn.KERNEL_MFMA_BIG),
                  oracle.pack_bits(ag_next).view(np.int32)))

    # 32 x 32 tiles with K split inside the workgroup (kernel id 10): ragged last row tile and last column word
    Ms, Ns, Ks = 70, 150, 1152
    As, Bs = synth.pm1(rng, (Ms, Ks)), synth.pm1(rng, (Ks, Ns))
    bns = synth.bn_params(rng, Ns, Ks, adversarial=True)
    Ss, as_next = oracle.dense_layer(As, Bs, bns, eps=EPS)
    pas, pbs = _dev_words(oracle.pack_bits(As)), _dev_words(oracle.pack_bits(np.ascontiguousarray(Bs.T)))
    thrs, flips = _fold(bns, Ks)
    cases.append(("xnor_gemm[mfma_splitk]", lambda: Guarded(Ms, Ns),
                  lambda o: bnn.xnor_gemm(pas, pbs, Ks, out=o, kernel=bnn.KERNEL_MFMA_SPLITK), Ss))
    cases.append(("xnor_gemm_bn_sign_pack[mfma_splitk]", lambda: Guarded(Ms, (Ns + 31) // 32),
                  lambda o: bnn.xnor_gemm_bn_sign_pack(pas, pbs, Ks, thrs, flips, out=o, kernel=bnn.KERNEL_MFMA_SPLITK),
                  oracle.pack_bits(as_next).view(np.int32)))

    # bnn_bn_sign_pack
    Sd = torch.from_numpy(S).to(DEV)
    cases.append(("bn_sign_pack", lambda: Guarded(M, (N + 31) // 32), lambda o: bnn.bn_sign_pack(Sd, thr, flip, out=o),
                  oracle.pack_bits(a_next).view(np.int32)))

    # first layer on 8-bit inputs: bnn_pack_bitplanes, bnn_bitplane_gemm, bnn_bitplane_gemm_bn_sign_pack
    Mp, Kp, Np = 70, 300, 150
    x8 = synth.uint8_input(rng, (Mp, Kp))
    Wp = synth.pm1(rng, (Kp, Np))
    bnp = synth.bn_params(rng, Np, 255 * Kp, adversarial=True)
    Sp = oracle.first_layer_bitplanes(x8, Wp)
    x8d = torch.from_numpy(x8).to(DEV)
    kwp = (Kp + 31) // 32
    planes = np.zeros((Mp, 8 * kwp), np.uint32)
    padded = np.zeros((Mp, 32 * kwp), np.uint8)
    padded[:, :Kp] = x8
    for w in range(kwp):
        for p in range(8):
            bits = ((padded[:, 32 * w:32 * w + 32] >> p) & 1).astype(np.int8) * 2 - 1
            planes[:, 8 * w + p] = oracle.pack_bits(bits)[:, 0]
    xp = bnn.pack_bitplanes(x8d)
    pwp = _dev_words(oracle.pack_bits(np.ascontiguousarray(Wp.T)))
    thrp, flipp = _fold(bnp, 255 * Kp)
    cases.append(("pack_bitplanes", lambda: Guarded(Mp, 8 * kwp, pad_cols=4), lambda o: bnn.pack_bitplanes(x8d, out=o),
                  planes.view(np.int32)))
    cases.append(("bitplane_gemm", lambda: Guarded(Mp, Np), lambda o: bnn.bitplane_gemm(xp, pwp, Kp, out=o), Sp))
    cases.append(("bitplane_gemm_bn_sign_pack", lambda: Guarded(Mp, (Np + 31) // 32),
                  lambda o: bnn.bitplane_gemm_bn_sign_pack(xp, pwp, Kp, thrp, flipp, out=o),
                  oracle.pack_bits(oracle.bn_sign(Sp, *bnp, eps=EPS)).view(np.int32)))

    # convolutions: bnn_conv_im2col_pack, bnn_conv_xnor, bnn_conv_bn_sign_pack, bnn_conv_pool_bn_sign_pack,
    # bnn_maxpool_bits
    Bc, Hc, Wc, Cc, Co = 3, 8, 8, 128, 96
    xc = synth.pm1(rng, (Bc, Hc, Wc, Cc))
    Wt = synth.pm1(rng, (Co, 3, 3, Cc))
    bnc = synth.bn_params(rng, Co, 9 * Cc, adversarial=True)
    Sc, ac = oracle.conv_layer(xc, Wt, bnc, eps=EPS)
    _Pc, apc = oracle.conv_pool_layer(xc, Wt, bnc, pool=2, eps=EPS)
    xcb = _dev_words(_pack_nhwc(xc).reshape(-1, Cc // 32)).view(Bc, Hc, Wc, Cc // 32)
    wtb = _dev_words(oracle.pack_bits(Wt.reshape(Co, -1)))
    thrc, flipc = _fold(bnc, 9 * Cc)
    Mc = Bc * Hc * Wc
    cases.append(("conv_im2col_pack", lambda: Guarded(Mc, 9 * Cc // 32, pad_cols=4),
                  lambda o: bnn.conv_im2col_pack(xcb, Cc, out=o), oracle.pack_bits(oracle.im2col(xc)).view(np.int32)))
    cases.append(("conv_xnor", lambda: Guarded(Mc, Co), lambda o: bnn.conv_xnor(xcb, Cc, wtb, out=o),
                  Sc.reshape(Mc, Co)))
    cases.append(("conv_bn_sign_pack", lambda: Guarded(Mc, Co // 32),
                  lambda o: bnn.conv_bn_sign_pack(xcb, Cc, wtb, thrc, flipc, out=o),
                  oracle.pack_bits(ac.reshape(Mc, Co)).view(np.int32)))
    cases.append(("conv_pool_bn_sign_pack", lambda: Guarded(Mc // 4, Co // 32),
                  lambda o: bnn.conv_pool_bn_sign_pack(xcb, Cc, wtb, thrc, flipc, out=o),
                  oracle.pack_bits(apc.reshape(Mc // 4, Co)).view(np.int32)))
    acb = _dev_words(oracle.pack_bits(ac.reshape(Mc, Co))).view(Bc, Hc, Wc, Co // 32)
    # the pooled map is a contiguous [B][Hp][Wp][Cw] array: guards before and after only
    cases.append(("maxpool_bits", lambda: Guarded(Mc // 4, Co // 32, pad_cols=0),
                  lambda o: bnn.maxpool_bits(acb, Co, flipc, out=o.view(Bc, Hc // 2, Wc // 2, Co // 32)),
                  oracle.pack_bits(apc.reshape(Mc // 4, Co)).view(np.int32)))

    # the int8 variant: bnn_unpack_i8 through its own output view, bnn_gemm_i8_mfma
    a8 = torch.from_numpy(A).to(DEV)
    b8 = torch.from_numpy(np.ascontiguousarray(Bm.T)).to(DEV)
    ld8 = (K + 15) // 16 * 16
    a8p = torch.zeros((M, ld8), dtype=torch.int8, device=DEV)
    b8p = torch.zeros((N, ld8), dtype=torch.int8, device=DEV)
    a8p[:, :K], b8p[:, :K] = a8, b8
    cases.append(("gemm_i8_mfma", lambda: Guarded(M, N), lambda o: bnn.gemm_i8_mfma(a8p[:, :K], b8p[:, :K], out=o), S))
    return cases


@pytest.fixture(scope="module")
def cases():
    return {name: (make, launch, want) for name, make, launch, want in _cases()}


CASE_NAMES = ["pack_sign"] + \
    [f"xnor_gemm[{k}]" for k in ("auto", "naive", "tiled128", "ksplit", "tiled64", "mfma", "mfma128", "mfma_shortk")] + \
    [f"xnor_gemm_bn_sign_pack[{k}]" for k in ("auto", "tiled128", "tiled64", "mfma", "mfma128", "mfma_shortk")] + \
    ["xnor_gemm[mfma_walk]", "xnor_gemm[mfma_whole_tiles]", "xnor_gemm_bn_sign_pack[mfma_walk]"] + \
    ["bn_sign_pack", "pack_bitplanes", "bitplane_gemm", "bitplane_gemm_bn_sign_pack", "conv_im2col_pack", "conv_xnor",
     "conv_bn_sign_pack", "conv_pool_bn_sign_pack", "maxpool_bits", "gemm_i8_mfma"]


@pytest.mark.parametrize("name", CASE_NAMES)
def test_entry_point_on_two_streams_with_guards_around_the_output(cases, name):
    make, launch, want = cases[name]
    # default stream
    g = make()
    launch(g.view)
    torch.cuda.synchronize()
    got = g.result_and_check()
    assert got.shape == want.shape and (got == want).all(), f"{name}: default stream"
    # a second stream of the same priority; the inputs were produced on the default stream
    side = torch.cuda.Stream()
    g2 = make()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        assert torch.cuda.current_stream() == side
        launch(g2.view)
    side.synchronize()
    got2 = g2.result_and_check()
    assert (got2 == want).all(), f"{name}: second stream"


def test_unpack_i8_with_guards_on_two_streams():
    """bnn_unpack_i8 allocates its int8 output itself in the binding, so it is called through the C ABI here:
    rows of K = 1000 values inside a guarded int8 array with ld_out = 1008."""
    rng = np.random.default_rng(77)
    rows, K, ld = 33, 1000, 1008
    V = synth.pm1(rng, (rows, K))
    bits = _dev_words(oracle.pack_bits(V))
    lib = bnn.load_library()
    want = np.zeros((rows, ld), np.int8)
    want[:, :K] = V
    for stream in (None, torch.cuda.Stream()):
        g = Guarded(rows, ld, dtype=torch.int8, pad_cols=0, lead=64, tail=64)
        handle = None if stream is None else stream.cuda_stream
        if stream is not None:
            stream.wait_stream(torch.cuda.current_stream())
        st = lib.bnn_unpack_i8(bits.data_ptr(), bits.stride(0), rows, K, g.view.data_ptr(), ld, handle)
        assert st == 0
        torch.cuda.synchronize()
        got = g.result_and_check()
        assert (got == want).all()        # +-1 for k < K, 0 for K <= k < ld_out
