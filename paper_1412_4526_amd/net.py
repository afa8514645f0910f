"""Whole-image forward / backward of a patch CNN: chains the libdsk calls in the
order Algorithm 1 (forward) and Sec. 4 (backward) of the paper prescribe.  This
file only sequences library calls on preallocated device buffers; all arithmetic
runs in the library's kernels.
"""
import torch

from . import binding as B


class GraphReplay:
    """Capture of one step (forward, and loss + backward when labels and a mask are given) into a HIP graph,
    for runners whose step is `forward(x)` then `loss_backward(labels, mask)` on preallocated buffers."""

    def capture(self, image, labels=None, mask=None):
        """Record one step (forward, and loss + backward when labels and mask are given) into a
        HIP graph.  Every call of a step is a kernel launch of libdsk on preallocated buffers, so
        the step replays as a whole; small networks are launch-bound otherwise.  `replay` copies
        new inputs into the captured input tensors."""
        assert self.timeline is None, "events of a timeline cannot be recorded into a graph"
        self._in = [image.clone(), None if labels is None else labels.clone(), None if mask is None else mask.clone()]
        side = torch.cuda.Stream(device=self.device)
        side.wait_stream(torch.cuda.current_stream(self.device))
        with torch.cuda.stream(side):          # warm-up off the capture, as torch asks for
            self._step_eager()
        torch.cuda.current_stream(self.device).wait_stream(side)
        torch.cuda.synchronize(self.device)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self._step_eager()
        return self

    def _step_eager(self):
        self.forward(self._in[0])
        if self._in[1] is not None:
            self.loss_backward(self._in[1], self._in[2])

    def replay(self, image=None, labels=None, mask=None):
        """Run the captured step; results are in scores / loss / dw / db as after the eager calls."""
        for dst, src in zip(self._in, (image, labels, mask)):
            if src is not None and dst is not None and src.data_ptr() != dst.data_ptr():
                dst.copy_(src)
        self.graph.replay()
        return self.scores


class WholeImageNet(GraphReplay):
    """The stride-1, d-regularly-sparse version of an original strided patch CNN,
    bound to one image batch shape.

    net: object with C0, patch, layers (each: kind, K, k, s, act) -- the ORIGINAL CNN.
    dtype: "f32", or "bf16" (activations and error maps stored in bfloat16, fp32
    accumulation; scores, loss, weights and their gradients stay fp32).
    fuse=False keeps every backward step a call of its own (pool gradient, then
    non-linearity backward + bias gradient).
    """

    def __init__(self, net, N, H, W, dtype="f32", device="cuda:0", train=True, fuse=True):
        self.net, self.N, self.H, self.W = net, N, H, W
        self.fuse = fuse      # backward: pool gradient + non-linearity backward + bias gradient as one call
        self.device = torch.device(device)
        self.act_dtype = torch.float32 if dtype == "f32" else torch.bfloat16
        self.code = B.DSK_F32 if dtype == "f32" else B.DSK_BF16
        self.train = train
        self.plan, self.rf, self.pad_lo, self.pad_hi = B.dsk_plan(net.layers, net.C0, H, W, net.patch)
        L = len(self.plan)
        last = self.plan[-1]
        if (last.Ho, last.Wo) != (H, W):
            raise ValueError("plan does not end at the image size")
        dev = self.device
        Hp, Wp = H + self.pad_lo + self.pad_hi, W + self.pad_lo + self.pad_hi
        self.xpad = torch.empty((N, net.C0, Hp, Wp), dtype=self.act_dtype, device=dev)
        self.maps = [self.xpad]          # maps[l] = input of layer l; maps[L] = scores
        self.argmax = [None] * L
        ws_bytes = 0
        for l, p in enumerate(self.plan):
            out_dtype = torch.float32 if l == L - 1 else self.act_dtype
            self.maps.append(torch.empty((N, p.K, p.Ho, p.Wo), dtype=out_dtype, device=dev))
            if p.kind == B.DSK_MAXPOOL and train:
                self.argmax[l] = torch.empty((N, p.K, p.Ho, p.Wo), dtype=torch.uint8, device=dev)
            if p.kind == B.DSK_CONV:
                shape = (N, p.C, p.H, p.W, p.K, p.k, p.k, p.d)
                whiches = (B.DSK_WS_CONV_FWD, B.DSK_WS_CONV_BWD_DATA, B.DSK_WS_CONV_BWD_WEIGHT) if train \
                    else (B.DSK_WS_CONV_FWD,)
                for which in whiches:
                    ws_bytes = max(ws_bytes, B.dsk_conv_workspace_bytes(which, *shape, self.code))
        self.scores = self.maps[-1]
        self.weights, self.biases = [], []
        for p in self.plan:
            if p.kind == B.DSK_CONV:
                self.weights.append(torch.zeros((p.K, p.C, p.k, p.k), dtype=torch.float32, device=dev))
                self.biases.append(torch.zeros((p.K,), dtype=torch.float32, device=dev))
        if train:
            ws_bytes = max(ws_bytes, B.dsk_softmax_xent_workspace_bytes(N, last.K, H, W))
            ws_bytes = max([ws_bytes] + [B.dsk_act_bwd_bias_workspace_bytes(p.K) for p in self.plan])
            ws_bytes = max([ws_bytes] + [B.dsk_pool_bwd_act_bias_workspace_bytes(p.kind, N, p.C, p.H, p.W, p.k, p.d, self.code)
                                         for p in self.plan if p.kind != B.DSK_CONV])
            ws_bytes = max([ws_bytes] + [B.dsk_conv_bwd_data_act_bias_workspace_bytes(N, p.C, p.H, p.W, p.K, p.k, p.k, p.d,
                                                                                      self.code, self.code)
                                         for l, p in enumerate(self.plan)
                                         if l > 0 and p.kind == B.DSK_CONV and self.plan[l - 1].kind == B.DSK_CONV])
            self.loss = torch.zeros((1,), dtype=torch.float32, device=dev)
            self.dw = [torch.empty_like(w) for w in self.weights]
            self.db = [torch.empty_like(b) for b in self.biases]
            # error maps: the one arriving at layer l's output and the one leaving at its input
            # alternate between two flat buffers sized for the largest map
            biggest = max(m.numel() for m in self.maps[1:])
            self._g = [torch.empty(biggest, dtype=self.act_dtype, device=dev) for _ in range(2)]
        self.ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
        self.timeline = None     # set to a list to collect (tag, layer, start_event, end_event) per call

    def _timed(self, tag, layer, fn, *a, **kw):
        """Run one library call; when a timeline is attached, bracket it with events on
        the current stream (the stream the library launches on)."""
        if self.timeline is None:
            return fn(*a, **kw)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn(*a, **kw)
        e1.record()
        self.timeline.append((tag, layer, e0, e1))
        return out

    # ------------------------------------------------------------------ parameters
    def load_params(self, weights, biases):
        """weights / biases: sequences of arrays or tensors, one per conv layer."""
        for dst, src in zip(self.weights, weights):
            dst.copy_(torch.as_tensor(src, dtype=torch.float32).reshape(dst.shape))
        for dst, src in zip(self.biases, biases):
            dst.copy_(torch.as_tensor(src, dtype=torch.float32).reshape(dst.shape))

    # ------------------------------------------------------------------ Algorithm 1
    def forward(self, image):
        """image: fp32 GPU tensor [N, C0, H, W] (unpadded).  Returns scores [N, Cls, H, W] fp32."""
        self._timed("pad", -1, B.dsk_pad_image, image, self.pad_lo, self.pad_hi, xpad=self.xpad)
        ci = 0
        for l, p in enumerate(self.plan):
            x, y = self.maps[l], self.maps[l + 1]
            if p.kind == B.DSK_CONV:
                self._timed("conv_fwd", l, B.dsk_conv_fwd, x, self.weights[ci], self.biases[ci], p.d, p.act,
                            y=y, ws=self.ws)
                ci += 1
            elif p.kind == B.DSK_MAXPOOL:
                self._timed("maxpool_fwd", l, B.dsk_maxpool_fwd, x, p.k, p.d, y=y, argmax=self.argmax[l],
                            want_argmax=self.train)
            else:
                self._timed("avgpool_fwd", l, B.dsk_avgpool_fwd, x, p.k, p.d, y=y)
        return self.scores

    # ------------------------------------------------------------------ Sec. 4
    def _gbuf(self, which, like):
        return self._g[which][:like.numel()].view(like.shape)

    def loss_backward(self, labels, mask):
        """labels int32 [N,H,W], mask uint8 [N,H,W] on the GPU; forward() must have run.
        Returns (loss tensor [1], dw list, db list)."""
        assert self.train
        L = len(self.plan)
        cur = 0
        g = self._gbuf(cur, self.scores)
        self._timed("softmax_xent", L, B.dsk_masked_softmax_xent, self.scores, labels, mask, loss=self.loss,
                    dscores=g, ws=self.ws)
        ci = len(self.weights) - 1
        act_done = False      # the error map in g already went through the non-linearity of the conv layer it belongs to
        for l in range(L - 1, -1, -1):
            p = self.plan[l]
            x, y = self.maps[l], self.maps[l + 1]
            gin = self._g[1 - cur][:x.numel()].view(x.shape) if l > 0 else None
            if p.kind == B.DSK_CONV:
                if not act_done:
                    # non-linearity backward and bias gradient in one pass over the error map
                    self._timed("act_bwd", l, B.dsk_act_bwd_bias, y, g, p.act, db=self.db[ci], ws=self.ws)
                act_done = False
                self._timed("conv_bwd_weight", l, B.dsk_conv_bwd_weight, x, g, p.k, p.k, p.d, dw=self.dw[ci],
                            want_db=False, ws=self.ws)
                if l > 0 and self.plan[l - 1].kind == B.DSK_CONV and self.fuse:
                    # the error map of the conv layer below, through that layer's non-linearity, and its bias
                    # gradient (x is that layer's output)
                    self._timed("conv_bwd_data_act", l, B.dsk_conv_bwd_data_act_bias, g, self.weights[ci], x, p.d,
                                self.plan[l - 1].act, dx=gin, db=self.db[ci - 1], ws=self.ws)
                    act_done = True
                elif l > 0:      # nobody needs the error map of the image itself
                    self._timed("conv_bwd_data", l, B.dsk_conv_bwd_data, g, self.weights[ci], p.d, p.H, p.W,
                                dx=gin, ws=self.ws)
                ci -= 1
            elif l > 0 and self.plan[l - 1].kind == B.DSK_CONV and self.fuse:
                # the pool's gradient, the non-linearity backward of the conv layer in front of it and that
                # layer's bias gradient: one pass (x is that layer's output)
                q = self.plan[l - 1]
                self._timed("pool_bwd_act", l, B.dsk_pool_bwd_act_bias, p.kind, g, self.argmax[l], x, p.k, p.d,
                            p.H, p.W, q.act, dx=gin, db=self.db[ci], ws=self.ws)
                act_done = True
            elif p.kind == B.DSK_MAXPOOL:
                self._timed("maxpool_bwd", l, B.dsk_maxpool_bwd, g, self.argmax[l], p.k, p.d, p.H, p.W, dx=gin)
            else:
                self._timed("avgpool_bwd", l, B.dsk_avgpool_bwd, g, p.k, p.d, p.H, p.W, dx=gin)
            if l > 0:
                g = gin
                cur = 1 - cur
        return self.loss, self.dw, self.db

    # ------------------------------------------------------------------ bookkeeping for benchmarks
    def conv_flops(self):
        """Algorithmic FLOPs (non-zero taps only) of one forward pass over all conv layers."""
        return sum(2.0 * self.N * p.C * p.K * p.k * p.k * p.Ho * p.Wo
                   for p in self.plan if p.kind == B.DSK_CONV)
