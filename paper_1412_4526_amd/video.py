"""Whole-video forward / backward of a cube classifier (3-D convolution and pooling, the extension the
paper's closing section proposes): chains the libdsk video calls in the order of Algorithm 1 and Sec. 4,
with Algorithm 1 run once on the temporal kernel sizes / strides and once on the spatial ones.  This file
only sequences library calls on preallocated device buffers.
"""
from types import SimpleNamespace

import torch

from . import binding as B
from .net import GraphReplay


class WholeVideoNet(GraphReplay):
    """net: object with C0, patch_t, patch, layers (each: kind, K, k, s, kt, st, act) -- the ORIGINAL strided
    cube CNN.  Maps are [N, T, C, H, W] (frame-major); weights [kt, K, C, k, k]."""

    def __init__(self, net, N, T, H, W, dtype="f32", device="cuda:0", train=True):
        self.net, self.N, self.T, self.H, self.W = net, N, T, H, W
        self.device = dev = torch.device(device)
        self.act_dtype = torch.float32 if dtype == "f32" else torch.bfloat16
        self.code = B.DSK_F32 if dtype == "f32" else B.DSK_BF16
        self.train = train
        # Algorithm 1 on each axis: spacing = product of the earlier strides along that axis
        sp = [SimpleNamespace(kind=L.kind, K=L.K, k=L.k, s=L.s, act=L.act) for L in net.layers]
        tp = [SimpleNamespace(kind=L.kind, K=L.K, k=L.kt, s=L.st, act=L.act) for L in net.layers]
        self.plan, self.rf, self.pad_lo, self.pad_hi = B.dsk_plan(sp, net.C0, H, W, net.patch)
        self.tplan, self.rf_t, self.tpad_lo, self.tpad_hi = B.dsk_plan(tp, net.C0, T, T, net.patch_t)
        L = len(self.plan)
        if (self.plan[-1].Ho, self.plan[-1].Wo, self.tplan[-1].Ho) != (H, W, T):
            raise ValueError("plan does not end at the video size")
        Tp, Hp, Wp = T + self.rf_t - 1, H + self.rf - 1, W + self.rf - 1
        self.xpad = torch.empty((N, Tp, net.C0, Hp, Wp), dtype=self.act_dtype, device=dev)
        self.maps = [self.xpad]
        self.argmax = [None] * L
        ws_bytes = 0
        for l, (p, q) in enumerate(zip(self.plan, self.tplan)):
            out_dtype = torch.float32 if l == L - 1 else self.act_dtype
            self.maps.append(torch.empty((N, q.Ho, p.K, p.Ho, p.Wo), dtype=out_dtype, device=dev))
            if p.kind == B.DSK_MAXPOOL and train:
                self.argmax[l] = torch.empty((N, q.Ho, p.K, p.Ho, p.Wo), dtype=torch.uint8, device=dev)
            if p.kind == B.DSK_CONV:
                shape = (N, q.H, p.C, p.H, p.W, p.K, q.k, p.k, p.k, q.d, p.d)
                whiches = (B.DSK_WS_CONV_FWD, B.DSK_WS_CONV_BWD_DATA, B.DSK_WS_CONV_BWD_WEIGHT) if train \
                    else (B.DSK_WS_CONV_FWD,)
                for which in whiches:
                    ws_bytes = max(ws_bytes, B.dsk_conv3d_workspace_bytes(which, *shape, self.code))
        self.scores = self.maps[-1]
        self.weights, self.biases = [], []
        for p, q in zip(self.plan, self.tplan):
            if p.kind == B.DSK_CONV:
                self.weights.append(torch.zeros((q.k, p.K, p.C, p.k, p.k), dtype=torch.float32, device=dev))
                self.biases.append(torch.zeros((p.K,), dtype=torch.float32, device=dev))
        if train:
            ws_bytes = max(ws_bytes, B.dsk_softmax_xent_workspace_bytes(N * T, self.plan[-1].K, H, W))
            ws_bytes = max([ws_bytes] + [B.dsk_act_bwd_bias_workspace_bytes(p.K) for p in self.plan])
            ws_bytes = max([ws_bytes] + [B.dsk_conv_bwd_data_act_bias_workspace_bytes(N * q.H, p.C, p.H, p.W, p.K, 1, 1, p.d,
                                                                                      self.code, self.code)
                                         for l, (p, q) in enumerate(zip(self.plan, self.tplan)) if self._pointwise_pair(l)])
            self.loss = torch.zeros((1,), dtype=torch.float32, device=dev)
            self.dw = [torch.empty_like(w) for w in self.weights]
            self.db = [torch.empty_like(b) for b in self.biases]
            biggest = max(m.numel() for m in self.maps[1:])
            self._g = [torch.empty(biggest, dtype=self.act_dtype, device=dev) for _ in range(2)]
        self.ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        self.timeline = None

    def _pointwise_pair(self, l):
        """Layer l is a 1x1x1 convolution directly on top of another convolution."""
        p, q = self.plan[l], self.tplan[l]
        return (l > 0 and p.kind == B.DSK_CONV and self.plan[l - 1].kind == B.DSK_CONV and p.k == 1 and q.k == 1)

    def _timed(self, tag, layer, fn, *a, **kw):
        if self.timeline is None:
            return fn(*a, **kw)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn(*a, **kw)
        e1.record()
        self.timeline.append((tag, layer, e0, e1))
        return out

    def load_params(self, weights, biases):
        """weights: one [K, C, kt, k, k] array per conv layer (the cube CNN's own layout); biases [K]."""
        for dst, src in zip(self.weights, weights):
            dst.copy_(torch.as_tensor(src, dtype=torch.float32).permute(2, 0, 1, 3, 4).reshape(dst.shape))
        for dst, src in zip(self.biases, biases):
            dst.copy_(torch.as_tensor(src, dtype=torch.float32).reshape(dst.shape))

    def forward(self, video):
        """video: fp32 GPU tensor [N, T, C0, H, W] (unpadded).  Returns scores [N, T, Cls, H, W] fp32."""
        self._timed("pad", -1, B.dsk_pad_video, video, self.tpad_lo, self.tpad_hi, self.pad_lo, self.pad_hi, xpad=self.xpad)
        ci = 0
        for l, (p, q) in enumerate(zip(self.plan, self.tplan)):
            x, y = self.maps[l], self.maps[l + 1]
            if p.kind == B.DSK_CONV:
                self._timed("conv3d_fwd", l, B.dsk_conv3d_fwd, x, self.weights[ci], self.biases[ci], q.d, p.d, p.act,
                            y=y, ws=self.ws)
                ci += 1
            elif p.kind == B.DSK_MAXPOOL:
                self._timed("maxpool3d_fwd", l, B.dsk_maxpool3d_fwd, x, q.k, p.k, q.d, p.d, y=y, argmax=self.argmax[l],
                            want_argmax=self.train)
            else:
                self._timed("avgpool3d_fwd", l, B.dsk_avgpool3d_fwd, x, q.k, p.k, q.d, p.d, y=y)
        return self.scores

    def loss_backward(self, labels, mask):
        """labels int32 [N, T, H, W], mask uint8 [N, T, H, W] on the GPU; forward() must have run.
        Returns (loss [1], dw list ([kt, K, C, k, k] each), db list)."""
        assert self.train
        L = len(self.plan)
        NT = self.N * self.T
        cur = 0
        sc = self.scores.view(NT, *self.scores.shape[2:])
        g = self._g[cur][:sc.numel()].view(sc.shape)
        self._timed("softmax_xent", L, B.dsk_masked_softmax_xent, sc, labels.view(NT, self.H, self.W),
                    mask.view(NT, self.H, self.W), loss=self.loss, dscores=g, ws=self.ws)
        g = g.view(self.scores.shape)
        ci = len(self.weights) - 1
        act_done = False      # the error map in g already went through the non-linearity of the layer it belongs to
        for l in range(L - 1, -1, -1):
            p, q = self.plan[l], self.tplan[l]
            x, y = self.maps[l], self.maps[l + 1]
            gin = self._g[1 - cur][:x.numel()].view(x.shape) if l > 0 else None
            if p.kind == B.DSK_CONV:
                flat = (y.shape[0] * y.shape[1],) + tuple(y.shape[2:])      # frames as a batch of images
                if not act_done:
                    self._timed("act_bwd", l, B.dsk_act_bwd_bias, y.view(flat), g.view(flat), p.act, db=self.db[ci], ws=self.ws)
                act_done = False
                self._timed("conv3d_bwd_weight", l, B.dsk_conv3d_bwd_weight, x, g, q.k, p.k, p.k, q.d, p.d,
                            dw=self.dw[ci], want_db=False, ws=self.ws)
                if self._pointwise_pair(l):
                    # a 1x1x1 layer on top of a convolution: the frames are a batch of images, and the 2-D call writes
                    # the error map behind the non-linearity of the layer below, and that layer's bias gradient, in one pass
                    flatx = (x.shape[0] * x.shape[1],) + tuple(x.shape[2:])
                    self._timed("conv_bwd_data_act", l, B.dsk_conv_bwd_data_act_bias, g.view(flat), self.weights[ci][0],
                                x.view(flatx), p.d, self.plan[l - 1].act, dx=gin.view(flatx), db=self.db[ci - 1], ws=self.ws)
                    act_done = True
                elif l > 0:
                    self._timed("conv3d_bwd_data", l, B.dsk_conv3d_bwd_data, g, self.weights[ci], q.d, p.d,
                                q.H, p.H, p.W, dx=gin, ws=self.ws)
                ci -= 1
            elif p.kind == B.DSK_MAXPOOL:
                self._timed("maxpool3d_bwd", l, B.dsk_maxpool3d_bwd, g, self.argmax[l], q.k, p.k, q.d, p.d,
                            q.H, p.H, p.W, dx=gin)
            else:
                self._timed("avgpool3d_bwd", l, B.dsk_avgpool3d_bwd, g, q.k, p.k, q.d, p.d, q.H, p.H, p.W, dx=gin)
            if l > 0:
                g = gin
                cur = 1 - cur
        return self.loss, self.dw, self.db

    def conv_flops(self):
        """Algorithmic FLOPs (non-zero taps only) of one forward pass over all conv layers."""
        return sum(2.0 * self.N * q.Ho * p.C * p.K * q.k * p.k * p.k * p.Ho * p.Wo
                   for p, q in zip(self.plan, self.tplan) if p.kind == B.DSK_CONV)
