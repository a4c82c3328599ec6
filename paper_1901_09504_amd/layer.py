"""Buffer ownership and call order for one OCS-expanded quantized layer.

A convenience over `binding`: it allocates the device buffers (PyTorch is the allocator),
keeps the split lists and scales on the device, and issues the C-ABI calls in order.  No
arithmetic happens here.

  weight OCS (Sec. 3.2 Eq. 3, the variant the paper finds effective, Sec. 5.2):
      prepare_weights(W)           off-line: select on W, halve, quantize        (W1-W3)
      prepare_weights(W, qa=True)  the same with the quantization-aware members of Sec. 3.3
      forward(X[, threshold])      per batch: duplicate channels + quantize, GEMM (X1/X2, G1, G2)
  activation OCS (Eq. 4) with the channels chosen on the batch itself (Sec. 5.3):
      forward_act_ocs(W, X)        select on X, duplicate weights, halve + quantize X, GEMM
"""
import torch

from . import binding as B


class ExpandedLayer:
    def __init__(self, N, C, g, r, bits_w=8, bits_x=8, clip_ratio_w=1.0, clip_ratio_x=1.0,
                 max_rows=None, device="cuda"):
        self.N, self.C, self.g = int(N), int(C), int(g)
        self.K = self.C * self.g
        self.s = B.ocs_num_splits(self.C, r)
        self.Ke = (self.C + self.s) * self.g
        self.ldq = B.ocs_padded_cols(self.Ke)
        self.bits_w, self.bits_x = int(bits_w), int(bits_x)
        self.clip_ratio_w, self.clip_ratio_x = float(clip_ratio_w), float(clip_ratio_x)
        self.device = device
        E = self.C + self.s
        i32 = dict(dtype=torch.int32, device=device)
        self.split_src = torch.empty(max(self.s, 1), **i32)
        self.chan_src = torch.empty(E, **i32)
        self.chan_depth = torch.empty(E, **i32)
        self.chan_path = None      # uint32 bits, allocated by the first QA preparation
        self._dup_base = None      # weight tensor whose codes sit in Wq's first C*g columns (Eq. 4)
        self.Wq = torch.empty((self.N, self.ldq), dtype=torch.int8, device=device)
        self.scale_w = torch.empty(2, dtype=torch.float32, device=device)
        self.scale_x = torch.empty(2, dtype=torch.float32, device=device)
        self.wmax = torch.empty(1, dtype=torch.float32, device=device)
        self.ws_w = B.alloc_workspace(self.N, self.K, device)
        self._rows = 0
        self.Xq = self.Y = self.ws_x = None
        if max_rows:
            self._ensure_rows(max_rows)

    def _ensure_rows(self, M):
        if M > self._rows:
            self.Xq = torch.empty((M, self.ldq), dtype=torch.int8, device=self.device)
            self.Y = torch.empty((M, self.N), dtype=torch.float32, device=self.device)
            self.ws_x = B.alloc_workspace(M, self.K, self.device)
            self._rows = M

    # ---- off-line ---------------------------------------------------------------------------
    def prepare_weights(self, W, W_out=None, clip_ratio_w=None, stream=None, qa=False):
        """W fp32 [N, C*g] on the device -> split lists, Wq, scale_w (and W' if W_out given).
        qa: quantization-aware split members and floor(x + 1/2) weight codes (Sec. 3.3) instead
        of plain halves (Eq. 3); the activation side is the same either way."""
        assert W.dtype == torch.float32 and W.shape == (self.N, self.K)
        clip = self.clip_ratio_w if clip_ratio_w is None else float(clip_ratio_w)
        self._dup_base = None
        if qa:
            if self.chan_path is None:
                self.chan_path = torch.empty(self.C + self.s, dtype=torch.int32, device=self.device)
            B.ocs_split_weights_qa(W, self.N, self.C, self.g, W.stride(0), self.s, self.split_src,
                                   self.chan_src, self.chan_depth, self.chan_path, W_out,
                                   0 if W_out is None else W_out.stride(0), self.bits_w, clip,
                                   self.Wq, self.ldq, self.scale_w, self.ws_w, stream)
            return
        B.ocs_split_weights(W, self.N, self.C, self.g, W.stride(0), self.s, B.MODE_HALVE,
                            self.split_src, self.chan_src, self.chan_depth, W_out,
                            0 if W_out is None else W_out.stride(0), self.wmax, self.bits_w, clip,
                            self.Wq, self.ldq, self.scale_w, self.ws_w, stream)

    def fold_weights(self, stream=None):
        """After prepare_weights: fold the expanded weight codes back onto the C original channels
        (sum over a channel's copies).  Returns a device int32 holding the largest |folded code|;
        the folded path is valid when it is <= 127 (any weight width below 8 bits, in practice)."""
        self.ldf = B.ocs_padded_cols(self.K)
        if getattr(self, "Wf", None) is None:
            self.Wf = torch.empty((self.N, self.ldf), dtype=torch.int8, device=self.device)
            self.fold_max = torch.zeros(1, dtype=torch.int32, device=self.device)
        B.ocs_fold_weights(self.Wq, self.ldq, self.N, self.C, self.g, self.s, self.chan_src, self.Wf,
                           self.ldf, self.fold_max, stream)
        return self.fold_max

    def forward_folded(self, X, threshold=None, acc_out=None, stream=None):
        """The same outputs as forward(), bit for bit, with no expansion at run time: plain
        quantization of X and a GEMM over the original K against the folded weight codes."""
        M = X.shape[0]
        self._ensure_rows(M)
        if getattr(self, "Xf", None) is None or self.Xf.shape[0] < M:
            self.Xf = torch.empty((M, self.ldf), dtype=torch.int8, device=self.device)
        B.ocs_quantize(X, M, self.K, X.stride(0), self.bits_x, threshold, self.clip_ratio_x, self.Xf,
                       self.ldf, self.scale_x, self.ws_x, stream)
        B.ocs_qgemm(self.Xf, self.ldf, self.Wf, self.ldf, M, self.N, self.K, self.bits_x, 8,
                    self.scale_x, self.scale_w, acc_out, 0 if acc_out is None else acc_out.stride(0),
                    self.Y, self.N, None, stream)
        return self.Y[:M]

    # ---- per batch --------------------------------------------------------------------------
    def split_act(self, X, threshold=None, stream=None):
        M = X.shape[0]
        self._ensure_rows(M)
        B.ocs_split_act(X, M, self.C, self.g, X.stride(0), self.chan_src, None, self.s, self.bits_x,
                        threshold, self.clip_ratio_x, self.Xq, self.ldq, self.scale_x, self.ws_x,
                        stream)

    def qgemm(self, M, acc_out=None, stream=None):
        B.ocs_qgemm(self.Xq, self.ldq, self.Wq, self.ldq, M, self.N, self.Ke, self.bits_x,
                    self.bits_w, self.scale_x, self.scale_w, acc_out,
                    0 if acc_out is None else acc_out.stride(0), self.Y, self.N, None, stream)

    def fused_fits(self, X):
        """Whether forward_fused serves this layer (one tile of output columns, whole K-steps of X)."""
        return B.ocs_split_act_qgemm_fits(X.shape[0], self.C, self.g, self.s, self.N, X.stride(0))

    def fused_pays(self, X):
        """Whether the library expects forward_fused to be ahead of forward on this layer."""
        return B.ocs_split_act_qgemm_pays(X.shape[0], self.C, self.g, self.s, self.N, X.stride(0))

    def forward_fused(self, X, threshold, acc_out=None, stream=None):
        """forward() on a static grid as one launch: the GEMM quantizes and duplicates X's channels
        itself and the code tensor is never written.  Same outputs, bit for bit."""
        M = X.shape[0]
        self._ensure_rows(M)
        B.ocs_split_act_qgemm(X, M, self.C, self.g, X.stride(0), self.chan_src, self.s, self.bits_x, threshold,
                              self.Wq, self.ldq, self.N, self.bits_w, self.scale_w, self.scale_x, acc_out,
                              0 if acc_out is None else acc_out.stride(0), self.Y, self.N, stream)
        return self.Y[:M]

    def forward(self, X, threshold=None, acc_out=None, stream=None):
        """X fp32 [M, C*g] -> Y fp32 [M, N].  threshold: device float tensor for a static
        activation grid (Sec. 5: fixed from profiling), None for a per-batch dynamic one."""
        M = X.shape[0]
        self.split_act(X, threshold, stream)
        self.qgemm(M, acc_out, stream)
        return self.Y[:M]

    def forward_act_ocs(self, W, X, acc_out=None, stream=None, qa=False):
        """Activation OCS with the channel choice made on this batch (Eq. 4, Sec. 5.3).
        qa: quantization-aware members on the activations (Sec. 3.3) instead of plain halves.
        W's own codes are computed on the first call with a given tensor object and kept (an
        in-place change of W needs prepare_weights() or a new tensor to be seen)."""
        M = X.shape[0]
        self._ensure_rows(M)
        xmax = torch.empty(1, dtype=torch.float32, device=self.device)
        B.ocs_select_channels(X, M, self.C, self.g, X.stride(0), self.s, self.split_src,
                              self.chan_src, self.chan_depth, xmax, self.ws_x, stream)
        if self._dup_base is not W:
            # once per weight tensor: its own codes in the first C*g columns (they do not depend
            # on the batch's choice); afterwards only the appended columns are rewritten per batch
            B.ocs_quantize(W, self.N, self.K, W.stride(0), self.bits_w, None, self.clip_ratio_w,
                           self.Wq, self.ldq, self.scale_w, self.ws_w, stream)
            self._dup_base = W
        B.ocs_duplicate_weight_codes(self.Wq, self.ldq, self.N, self.C, self.g, self.s, self.chan_src,
                                     stream)
        if qa:
            if self.chan_path is None:
                self.chan_path = torch.empty(self.C + self.s, dtype=torch.int32, device=self.device)
            B.ocs_split_act_qa(X, M, self.C, self.g, X.stride(0), self.split_src, self.chan_src,
                               self.chan_depth, self.chan_path, self.s, self.bits_x, xmax, self.Xq,
                               self.ldq, self.scale_x, stream)
            self.qgemm(M, acc_out, stream)
            return self.Y[:M]
        # the selector already returned the largest magnitude of the halved activations: with no
        # clipping that is the threshold, and the pass over X that would recompute it is skipped
        thr = xmax if self.clip_ratio_x == 1.0 else None
        B.ocs_split_act(X, M, self.C, self.g, X.stride(0), self.chan_src, self.chan_depth, self.s,
                        self.bits_x, thr, self.clip_ratio_x, self.Xq, self.ldq, self.scale_x,
                        self.ws_x, stream)
        self.qgemm(M, acc_out, stream)
        return self.Y[:M]


class ExpandedConv:
    """The same layer for a convolution given un-lowered: activations A [B, H, W, C] fp32 (NHWC),
    weights [N, C*kh*kw] (channel c owns kh*kw columns).  The activation is split and quantized
    once on its [B*H*W, C] view and the lowering happens inside the GEMM kernel's loader
    (ocs_qconv), so the kh*kw-times larger lowered matrix never exists.  Weight OCS only."""

    def __init__(self, N, C, kh, kw, stride, pad, r, bits_w=8, bits_x=8, clip_ratio_w=1.0,
                 device="cuda"):
        self.kh, self.kw, self.stride, self.pad = int(kh), int(kw), int(stride), int(pad)
        self.g = self.kh * self.kw
        self.w = ExpandedLayer(N, C, self.g, r, bits_w, bits_x, clip_ratio_w=clip_ratio_w, device=device)
        self.N, self.C, self.s = self.w.N, self.w.C, self.w.s
        self.E = self.C + self.s
        self.ldc = B.ocs_padded_channels(self.E)
        self.ldt = B.ocs_conv_weight_cols(self.g, self.ldc)
        self.Wt = torch.empty((self.N + 1, self.ldt), dtype=torch.int8, device=device)
        self.scale_x = torch.empty(2, dtype=torch.float32, device=device)
        self.device = device
        self._pixels = 0
        self.Aq = self.Y = self.ws_a = None

    def prepare_weights(self, W, stream=None):
        self.w.prepare_weights(W, stream=stream)
        B.ocs_conv_weights_tap_major(self.w.Wq, self.N, self.E, self.g, self.w.ldq, self.Wt, self.ldc,
                                     stream)

    def out_size(self, H, W):
        return ((H + 2 * self.pad - self.kh) // self.stride + 1,
                (W + 2 * self.pad - self.kw) // self.stride + 1)

    def ensure_input(self, P):
        """Room for the codes of P input pixels."""
        if P > self._pixels:
            self.Aq = torch.empty((P, self.ldc), dtype=torch.int8, device=self.device)
            self.ws_a = B.alloc_workspace(P, self.C, self.device)
            self._pixels = P

    def ensure_output(self, M):
        if self.Y is None or self.Y.shape[0] < M:
            self.Y = torch.empty((M, self.N), dtype=torch.float32, device=self.device)

    def split_act(self, A, threshold=None, stream=None):
        """A fp32 [B, H, W, C] contiguous -> codes of the un-lowered activation in self.Aq."""
        Bn, H, W, C = A.shape
        assert C == self.C and A.is_contiguous()
        P = Bn * H * W
        self.ensure_input(P)
        B.ocs_split_act(A, P, self.C, 1, self.C, self.w.chan_src, None, self.s, self.w.bits_x, threshold,
                        1.0, self.Aq, self.ldc, self.scale_x, self.ws_a, stream)

    def conv(self, Bn, H, W, acc_out=None, stream=None):
        """The convolution on the codes in self.Aq -> Y fp32 [B*Ho*Wo, N]."""
        Ho, Wo = self.out_size(H, W)
        M = Bn * Ho * Wo
        self.ensure_output(M)
        B.ocs_qconv(self.Aq, self.ldc, Bn, H, W, self.E, self.kh, self.kw, self.stride, self.pad, self.Wt,
                    self.N, self.w.bits_x, self.w.bits_w, self.scale_x, self.w.scale_w, acc_out,
                    0 if acc_out is None else acc_out.stride(0), self.Y, self.N, stream)
        return self.Y[:M]

    def conv_to_codes(self, Bn, H, W, nxt, next_threshold, relu=True, acc_out=None, stream=None):
        """The convolution on the codes in self.Aq, its output handed to the layer `nxt` as that
        layer's input codes (nxt.Aq, nxt.scale_x): the next layer's static grid after an optional
        ReLU, with the channels the next layer splits duplicated."""
        Ho, Wo = self.out_size(H, W)
        M = Bn * Ho * Wo
        assert nxt.C == self.N
        nxt.ensure_input(M)
        B.ocs_qconv_requant(self.Aq, self.ldc, Bn, H, W, self.E, self.kh, self.kw, self.stride, self.pad,
                            self.Wt, self.N, self.w.bits_x, self.w.bits_w, self.scale_x, self.w.scale_w, relu,
                            next_threshold, nxt.w.bits_x, nxt.w.chan_src, nxt.s, nxt.Aq, nxt.ldc, nxt.scale_x,
                            acc_out, 0 if acc_out is None else acc_out.stride(0), stream)
        return Ho, Wo

    def forward(self, A, threshold=None, acc_out=None, stream=None):
        """A fp32 [B, H, W, C] contiguous -> Y fp32 [B*Ho*Wo, N]."""
        Bn, H, W, _ = A.shape
        self.split_act(A, threshold, stream)
        return self.conv(Bn, H, W, acc_out, stream)


class ConvChain:
    """A run of convolutions whose activations travel from layer to layer as codes: weight OCS on
    every layer, static activation grids (Sec. 5: fixed from profiling), ReLU between the layers.
    The first layer's input is split and quantized once, un-lowered; every layer but the last hands
    its output to the next one through the re-quantizing epilogue; the last writes fp32.
    specs: [(N, k, stride, pad), ...]."""

    def __init__(self, C_in, specs, r, bits_w=8, bits_x=8, clip_ratio_w=1.0, device="cuda"):
        self.layers = []
        c = C_in
        for (N, k, stride, pad) in specs:
            self.layers.append(ExpandedConv(N, c, k, k, stride, pad, r, bits_w, bits_x,
                                            clip_ratio_w=clip_ratio_w, device=device))
            c = N

    def prepare_weights(self, weights, stream=None):
        for L, W in zip(self.layers, weights):
            L.prepare_weights(W, stream)

    def forward(self, A, thresholds, acc_out=None, stream=None):
        """A fp32 [B, H, W, C]; thresholds: one device float per layer (its input grid's range).
        Returns Y fp32 [B*Ho*Wo, N_last]; acc_out (optional) receives the last layer's accumulators."""
        Bn, H, W, _ = A.shape
        self.layers[0].split_act(A, thresholds[0], stream)
        for i, L in enumerate(self.layers[:-1]):
            H, W = L.conv_to_codes(Bn, H, W, self.layers[i + 1], thresholds[i + 1], True, None, stream)
        return self.layers[-1].conv(Bn, H, W, acc_out, stream)
