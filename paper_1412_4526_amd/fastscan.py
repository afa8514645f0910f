"""Fast scanning (the paper's comparison method: Sec. 2; Sec. 3.6, last paragraph; Table 1), forward only,
as a chain of library calls on preallocated buffers: every layer keeps its ORIGINAL stride; a strided layer
runs once per starting offset and multiplies the number of fragments by s*s; the fragments of the last layer
are re-organised into the label map.  All arithmetic runs in the library's kernels."""
import torch

from . import binding as B


def _ceil_div(a, b):
    return -(-a // b)


class FastScanNet:
    """net: the ORIGINAL strided patch CNN (C0, patch, layers with kind, K, k, s, act)."""

    def __init__(self, net, N, H, W, dtype="f32", device="cuda:0"):
        self.net, self.N, self.H, self.W = net, N, H, W
        self.device = torch.device(device)
        self.act_dtype = torch.float32 if dtype == "f32" else torch.bfloat16
        # whole-image map sizes per layer (Algorithm 1's bookkeeping): fragment (fy, fx) at spacing D of a map with
        # Hl rows has ceil((Hl - fy) / D) rows
        self.plan, self.rf, self.pad_lo, self.pad_hi = B.dsk_plan(net.layers, net.C0, H, W, net.patch)
        dev = self.device
        Hp, Wp = H + self.pad_lo + self.pad_hi, W + self.pad_lo + self.pad_hi
        self.xpad = torch.empty((N, net.C0, Hp, Wp), dtype=self.act_dtype, device=dev)
        self.frags = [self.xpad]
        self.spacing = [1]
        D, ws_bytes = 1, 0
        L = len(self.plan)
        for l, (p, layer) in enumerate(zip(self.plan, net.layers)):
            Do = D * layer.s
            ho, wo = _ceil_div(p.Ho, Do), _ceil_div(p.Wo, Do)
            out_dtype = torch.float32 if l == L - 1 else self.act_dtype
            self.frags.append(torch.empty((N * Do * Do, p.K, ho, wo), dtype=out_dtype, device=dev))
            if p.kind == B.DSK_CONV and layer.s == 1:
                hi, wi = self.frags[l].shape[2:]
                assert (ho, wo) == (hi - p.k + 1, wi - p.k + 1)
                ws_bytes = max(ws_bytes, B.dsk_conv_workspace_bytes(B.DSK_WS_CONV_FWD, N * D * D, p.C, hi, wi, p.K, p.k, p.k, 1,
                                                                    B.DSK_F32 if self.act_dtype == torch.float32 else B.DSK_BF16))
            D = Do
            self.spacing.append(D)
        self.scores = torch.empty((N, self.plan[-1].K, H, W), dtype=torch.float32, device=dev)
        self.weights, self.biases = [], []
        for p in self.plan:
            if p.kind == B.DSK_CONV:
                self.weights.append(torch.zeros((p.K, p.C, p.k, p.k), dtype=torch.float32, device=dev))
                self.biases.append(torch.zeros((p.K,), dtype=torch.float32, device=dev))
        self.ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        self.timeline = None

    def load_params(self, weights, biases):
        for dst, src in zip(self.weights, weights):
            dst.copy_(torch.as_tensor(src, dtype=torch.float32).reshape(dst.shape))
        for dst, src in zip(self.biases, biases):
            dst.copy_(torch.as_tensor(src, dtype=torch.float32).reshape(dst.shape))

    def _timed(self, tag, layer, fn, *a, **kw):
        if self.timeline is None:
            return fn(*a, **kw)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn(*a, **kw)
        e1.record()
        self.timeline.append((tag, layer, e0, e1))
        return out

    def fragments(self):
        """Number of fragments per image after each layer."""
        return [d * d for d in self.spacing[1:]]

    def forward(self, image):
        """image: fp32 GPU tensor [N, C0, H, W] (unpadded).  Returns scores [N, Cls, H, W] fp32."""
        self._timed("pad", -1, B.dsk_pad_image, image, self.pad_lo, self.pad_hi, xpad=self.xpad)
        ci = 0
        for l, (p, layer) in enumerate(zip(self.plan, self.net.layers)):
            x, y, D = self.frags[l], self.frags[l + 1], self.spacing[l]
            ho, wo = y.shape[2:]
            if p.kind == B.DSK_CONV:
                if layer.s == 1:      # a dense layer on the batch of fragments
                    self._timed("conv_fwd", l, B.dsk_conv_fwd, x, self.weights[ci], self.biases[ci], 1, p.act, y=y, ws=self.ws)
                else:
                    self._timed("fs_conv_fwd", l, B.dsk_fs_conv_fwd, x, self.weights[ci], self.biases[ci], D, layer.s, ho, wo,
                                p.act, out=y)
                ci += 1
            else:
                self._timed("fs_pool_fwd", l, B.dsk_fs_pool_fwd, p.kind, x, D, p.k, layer.s, ho, wo, out=y)
        self._timed("fs_assemble", len(self.plan), B.dsk_fs_assemble, self.frags[-1], self.spacing[-1], self.H, self.W,
                    out=self.scores)
        return self.scores
