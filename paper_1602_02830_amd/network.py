"""Layer chaining for the forward path of Alg. 4 ("Running a BNN").

These classes own device buffers and call the library in the order the
algorithm states; they do no arithmetic themselves.  Packed words are held in
int32 tensors.  Leading dimensions of packed buffers are rounded up to 4 words
so that every row is 16-byte aligned (the fast-path requirement of the GEMM).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def _round_up(x: int, m: int) -> int:
    return (x + m - 1) // m * m


def _packed_buffer(rows: int, K: int, device) -> torch.Tensor:
    kw = B.words_per_row(K)
    ld = _round_up(kw, 4)
    buf = torch.zeros((rows, ld), dtype=torch.int32, device=device)
    return buf[:, :kw] if ld != kw else buf


class BinaryMLP:
    """Fully binarized MLP: Sign+pack the real input, then per hidden layer
    XnorDotProduct -> Sign(BatchNorm) (Alg. 4, step 2); the last layer emits the
    int32 pre-activations.

    weights_real: list of float32 device tensors W_l [N_l][K_l] (row n = output unit n);
        they are binarized with Eq. (1) and packed once, on the device.
    bns: per hidden layer (gamma, beta, mean, var) as numpy float32 [N_l]; folded once on the host.
    """

    def __init__(self, weights_real, bns, eps: float, batch: int, keep_preacts: bool = True,
                 fused: bool = False, kernel: int = B.KERNEL_AUTO, input_uint8: bool = False):
        assert len(bns) == len(weights_real) - 1
        dev = weights_real[0].device
        self.device = dev
        self.batch = batch
        self.fused = fused          # hidden layers as one launch each; their int32 pre-activations are not produced
        self.kernel = kernel        # GEMM kernel of the hidden layers (KERNEL_AUTO = the library's choice)
        # input_uint8: the first layer takes 8-bit inputs as eight bit planes (Alg. 4 step 1, Sec. 1.6)
        # instead of Sign-binarizing a real input.
        self.input_uint8 = input_uint8
        self.K = [int(w.shape[1]) for w in weights_real]
        self.N = [int(w.shape[0]) for w in weights_real]
        self.w_bits = []
        for w in weights_real:
            buf = _packed_buffer(w.shape[0], w.shape[1], dev)
            B.pack_sign(w, out=buf)
            self.w_bits.append(buf)
        self.thr, self.flip = [], []
        for l, bn in enumerate(bns):
            # The first layer's pre-activations on 8-bit inputs range over [-255 K, 255 K].
            thr, flip = B.bn_fold(*bn, eps, self.K[l] * (255 if (input_uint8 and l == 0) else 1))
            self.thr.append(torch.from_numpy(thr).to(dev))
            self.flip.append(torch.from_numpy(flip.view(np.int32)).to(dev))
        # Activations a^b_l (packed) and pre-activations s_l (int32), allocated once.
        if input_uint8:
            self.a_bits = [torch.empty((batch, 8 * B.words_per_row(self.K[0])), dtype=torch.int32, device=dev)]
        else:
            self.a_bits = [_packed_buffer(batch, self.K[0], dev)]
        for l in range(len(bns)):
            self.a_bits.append(_packed_buffer(batch, self.N[l], dev))
        self.keep_preacts = keep_preacts
        if fused:
            self.s = [None] * (len(weights_real) - 1)
            self.s.append(torch.empty((batch, self.N[-1]), dtype=torch.int32, device=dev))
        elif keep_preacts:
            self.s = [torch.empty((batch, n), dtype=torch.int32, device=dev) for n in self.N]
        else:
            # One scratch buffer reused by every hidden layer, plus the score buffer.
            scratch = torch.empty((batch, max(self.N[:-1])), dtype=torch.int32, device=dev)
            self.s = [scratch[:, :n] if n != scratch.shape[1] else scratch for n in self.N[:-1]]
            self.s.append(torch.empty((batch, self.N[-1]), dtype=torch.int32, device=dev))

    def forward(self, x: torch.Tensor, span_events=None) -> torch.Tensor:
        """x: float32 device tensor [batch][K_0].  Returns the int32 scores [batch][N_last].

        span_events: optional (first_layer, last_layer, dict); one event is recorded on the current
        stream before the GEMM launch of first_layer and one right after that of last_layer:
        dict["start"], dict["end"] (created here unless the caller put events there already).
        """
        if self.input_uint8:
            B.pack_bitplanes(x, out=self.a_bits[0])
        else:
            B.pack_sign(x, out=self.a_bits[0])
        n_layers = len(self.w_bits)
        for l in range(n_layers):
            if span_events is not None and l == span_events[0]:
                if "start" not in span_events[2]:
                    span_events[2]["start"] = torch.cuda.Event(enable_timing=True)
                span_events[2]["start"].record()
            hidden = l + 1 < n_layers
            if self.input_uint8 and l == 0:
                if self.fused and hidden:
                    B.bitplane_gemm_bn_sign_pack(self.a_bits[0], self.w_bits[0], self.K[0], self.thr[0],
                                                 self.flip[0], out=self.a_bits[1])
                else:
                    B.bitplane_gemm(self.a_bits[0], self.w_bits[0], self.K[0], out=self.s[0])
            elif self.fused and hidden:
                B.xnor_gemm_bn_sign_pack(self.a_bits[l], self.w_bits[l], self.K[l], self.thr[l], self.flip[l],
                                         out=self.a_bits[l + 1], kernel=self.kernel)
            else:
                B.xnor_gemm(self.a_bits[l], self.w_bits[l], self.K[l], out=self.s[l],
                            kernel=self.kernel if hidden else B.KERNEL_AUTO)
            if span_events is not None and l == span_events[1]:
                if "end" not in span_events[2]:
                    span_events[2]["end"] = torch.cuda.Event(enable_timing=True)
                span_events[2]["end"].record()
            if hidden and not self.fused:
                B.bn_sign_pack(self.s[l], self.thr[l], self.flip[l], out=self.a_bits[l + 1])
        return self.s[-1]


class BinaryConvLayer:
    """One binary 3x3 (or kh x kw) convolution layer lowered to the binary GEMM:
    im2col on packed NHWC bits -> XnorDotProduct -> Sign(BatchNorm) -> packed NHWC bits.

    weight_real: float32 device tensor [Cout][kh][kw][Cin], binarized by Eq. (1) on the device.
    Any Cin is taken: a filter flattened as (ky, kx, ci) has exactly the bit order of the rows that
    bnn_conv_im2col_pack writes, whether or not a tap fills whole words.

    implicit=True asks for the layer without the im2col matrix (bnn_conv_xnor / bnn_conv_bn_sign_pack).
    The library takes that form for Cin % 32 == 0 on same-size stride-1 layers and for Cin % 128 == 0
    on any geometry; for everything else it answers "unsupported" before launching anything, and the
    layer then keeps to bnn_conv_im2col_pack followed by the GEMM (self.implicit turns False).
    """

    def __init__(self, weight_real, bn, eps: float, batch: int, H: int, W: int, stride: int = 1, pad: int = 1,
                 fused: bool = False, implicit: bool = False, pool: int = 0):
        dev = weight_real.device
        self.fused = fused      # GEMM and BN+Sign in one launch; the int32 pre-activations are not produced
        self.implicit = implicit  # receptive fields gathered inside the GEMM (no im2col matrix); Cin % 128 == 0
        self.pool = pool        # pool x pool max pooling (stride pool) of the pre-activations, done on the output bits
        self.Cout, self.kh, self.kw, self.Cin = (int(d) for d in weight_real.shape)
        self.stride, self.pad = stride, pad
        self.B, self.H, self.W = batch, H, W
        self.Ho = (H + 2 * pad - self.kh) // stride + 1
        self.Wo = (W + 2 * pad - self.kw) // stride + 1
        self.K = self.kh * self.kw * self.Cin
        self.M = batch * self.Ho * self.Wo
        self.w_bits = _packed_buffer(self.Cout, self.K, dev)
        B.pack_sign(weight_real.reshape(self.Cout, self.K), out=self.w_bits)
        thr, flip = B.bn_fold(*bn, eps, self.K)
        self.thr = torch.from_numpy(thr).to(dev)
        self.flip = torch.from_numpy(flip.view(np.int32)).to(dev)
        self.cols = None if implicit else _packed_buffer(self.M, self.K, dev)     # the im2col matrix
        self.s = None if fused else torch.empty((self.M, self.Cout), dtype=torch.int32, device=dev)
        self.out_bits = torch.empty((self.M, B.words_per_row(self.Cout)), dtype=torch.int32, device=dev)
        if pool:
            self.Hp, self.Wp = (self.Ho - pool) // pool + 1, (self.Wo - pool) // pool + 1
            self.pooled = torch.empty((batch, self.Hp, self.Wp, B.words_per_row(self.Cout)), dtype=torch.int32,
                                      device=dev)
        # Pooled, fused, implicit layers try the one-launch form first; the library refuses geometries whose
        # pooling windows do not fit its tiles (before launching anything), and the layer then keeps to
        # conv -> bnn_maxpool_bits.
        self.pool_in_conv = bool(pool) and fused and implicit and self.Ho % pool == 0 and self.Wo % pool == 0

    def forward(self, x_bits: torch.Tensor) -> torch.Tensor:
        """x_bits: packed NHWC int32 [B][H][W][Cin/32].  Returns packed NHWC [B][Ho][Wo][ceil(Cout/32)]."""
        if self.pool_in_conv:
            try:
                B.conv_pool_bn_sign_pack(x_bits, self.Cin, self.w_bits, self.thr, self.flip, self.kh, self.kw,
                                         self.stride, self.pad, self.pool,
                                         out=self.pooled.view(self.B * self.Hp * self.Wp, -1))
                return self.pooled
            except B.BnnError as e:
                if e.status != 3:
                    raise
                self.pool_in_conv = False
        if self.implicit:
            try:
                if self.fused:
                    B.conv_bn_sign_pack(x_bits, self.Cin, self.w_bits, self.thr, self.flip, self.kh, self.kw,
                                        self.stride, self.pad, out=self.out_bits)
                else:
                    B.conv_xnor(x_bits, self.Cin, self.w_bits, self.kh, self.kw, self.stride, self.pad, out=self.s)
                    B.bn_sign_pack(self.s, self.thr, self.flip, out=self.out_bits)
            except B.BnnError as e:
                if e.status != 3:
                    raise
                # Refused before any launch (channel count or geometry): lower through the im2col matrix from now on.
                self.implicit = False
                self.cols = _packed_buffer(self.M, self.K, x_bits.device)
        if not self.implicit:
            B.conv_im2col_pack(x_bits, self.Cin, self.kh, self.kw, self.stride, self.pad, out=self.cols)
            if self.fused:
                B.xnor_gemm_bn_sign_pack(self.cols, self.w_bits, self.K, self.thr, self.flip, out=self.out_bits)
            else:
                B.xnor_gemm(self.cols, self.w_bits, self.K, out=self.s)
                B.bn_sign_pack(self.s, self.thr, self.flip, out=self.out_bits)
        out = self.out_bits.view(self.B, self.Ho, self.Wo, -1)
        if self.pool:
            B.maxpool_bits(out, self.Cout, self.flip, self.pool, self.pool, self.pool, out=self.pooled)
            return self.pooled
        return out


class BinaryConvNet:
    """The binary body of the CIFAR-10 / SVHN ConvNet, from the first layer's output bits to the class
    scores.  Sec. 2.2 only says the network has the architecture of the BinaryConnect ConvNet it cites;
    the layer list used here (128C3-MP2-256C3-256C3-MP2-512C3-512C3-MP2-1024FC-1024FC-10 after the first
    convolution) and the position of the pooling (before BatchNorm) are this build's reading of that
    cited architecture.  Layers: 3x3 binary convolutions (fused with Sign(BatchNorm), max pooling on
    the output bits where the architecture pools), then binary dense layers.  Every layer's packed NHWC
    output is the next layer's input as it stands; the pooled bits of the last convolution, read row by
    row, are the (y, x, channel)-ordered input of the first dense layer.

    convs: list of (float32 device filters [Cout][3][3][Cin], bn, pooled) per convolution;
    fcs:   list of float32 device weights [N][K]; fc_bns: bn per hidden dense layer.
    """

    def __init__(self, convs, fcs, fc_bns, eps: float, batch: int, H: int, W: int):
        assert len(fc_bns) == len(fcs) - 1
        self.batch = batch
        self.convs = []
        for w, bn, pooled in convs:
            layer = BinaryConvLayer(w, bn, eps, batch, H, W, fused=True, implicit=True, pool=2 if pooled else 0)
            self.convs.append(layer)
            if pooled:
                H, W = layer.Hp, layer.Wp
        dev = fcs[0].device
        self.K = [int(w.shape[1]) for w in fcs]
        self.N = [int(w.shape[0]) for w in fcs]
        if self.K[0] != H * W * self.convs[-1].Cout:
            raise ValueError("first dense layer does not match the last feature map")
        self.w_bits, self.thr, self.flip = [], [], []
        for w in fcs:
            buf = _packed_buffer(w.shape[0], w.shape[1], dev)
            B.pack_sign(w, out=buf)
            self.w_bits.append(buf)
        for l, bn in enumerate(fc_bns):
            thr, flip = B.bn_fold(*bn, eps, self.K[l])
            self.thr.append(torch.from_numpy(thr).to(dev))
            self.flip.append(torch.from_numpy(flip.view(np.int32)).to(dev))
        self.a_bits = [_packed_buffer(batch, n, dev) for n in self.N[:-1]]
        self.scores = torch.empty((batch, self.N[-1]), dtype=torch.int32, device=dev)

    def forward(self, x_bits: torch.Tensor) -> torch.Tensor:
        """x_bits: packed NHWC int32 [B][H][W][Cin/32].  Returns the int32 scores [B][classes]."""
        a = x_bits
        for layer in self.convs:
            a = layer.forward(a)
        a = a.reshape(self.batch, -1)                    # (y, x, channel words) of one image = one packed row
        for l in range(len(self.w_bits) - 1):
            B.xnor_gemm_bn_sign_pack(a, self.w_bits[l], self.K[l], self.thr[l], self.flip[l], out=self.a_bits[l])
            a = self.a_bits[l]
        B.xnor_gemm(a, self.w_bits[-1], self.K[-1], out=self.scores)
        return self.scores

