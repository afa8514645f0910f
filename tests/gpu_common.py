"""Shared helpers of the GPU parity tests: tolerances and oracle adapters.

Tolerances (per tensor, max-norm):
  fp32 path:  max|gpu - ref| <= 1e-4 * max|ref| + 1e-5
  bf16 path:  max|gpu - ref| <= 2e-2 * max|ref|   (+ 1e-6 absolute floor)
Integer results (argmax) are compared bit-exactly.

A single stride-1 layer with spacing d is checked against the oracle through a
two-layer ORIGINAL network the oracle can scan patch by patch without knowing
about spacing: a 1x1 pool with stride d (pure sub-sampling) followed by the
layer itself.  Algorithm 1 turns exactly that network into "identity, then the
layer with spacing d".
"""
import numpy as np
import torch

import oracle
from workloads import Net, conv, maxpool, avgpool
from workloads.nets import Layer, MAXPOOL

F32_REL, F32_ABS = 1e-4, 1e-5
BF16_REL, BF16_ABS = 2e-2, 1e-6


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def assert_close(got, want, what, bf16=False):
    got = to_np(got) if isinstance(got, torch.Tensor) else np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if want.size == 0:
        return
    scale = np.abs(want).max()
    tol = (BF16_REL * scale + BF16_ABS) if bf16 else (F32_REL * scale + F32_ABS)
    err = np.abs(got - want).max()
    assert np.isfinite(got).all(), "%s: non-finite values" % what
    assert err <= tol, "%s: max|err| %.4g > tol %.4g (max|ref| %.4g)" % (what, err, tol, scale)


def all_pixels(N, H, W):
    n, i, j = np.meshgrid(np.arange(N), np.arange(H), np.arange(W), indexing="ij")
    return np.stack([n.ravel(), i.ravel(), j.ravel()], 1).astype(np.int32)


def single_layer_net(C, layer, k, d):
    """Original network whose whole-image form is [identity, layer with spacing d]."""
    layers = ((maxpool(1, d),) if d > 1 else ()) + (layer,)
    return Net("single", C, 1 + (k - 1) * d, layers)


def bf16_round(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).float().numpy()


def oracle_conv_fwd(x, w, b, d, act):
    """x [N,C,H,W], w [K,C,k,k] -> y [N,K,Ho,Wo] by patch scanning."""
    N, C, H, W = x.shape
    K, _, k, _ = w.shape
    net = single_layer_net(C, conv(K, k, 1, act), k, d)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    s = oracle.scan_forward(net, oracle.pack_params([w], [b]), x, all_pixels(N, Ho, Wo))
    return s.reshape(N, Ho, Wo, K).transpose(0, 3, 1, 2)


def oracle_conv_bwd(x, w, b, d, act, dy):
    """Returns (dw, db, dx) for the output error dy [N,K,Ho,Wo] (error w.r.t. the
    activated output when act != none)."""
    N, C, H, W = x.shape
    K, _, k, _ = w.shape
    net = single_layer_net(C, conv(K, k, 1, act), k, d)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    delta = np.asarray(dy, np.float64).transpose(0, 2, 3, 1).reshape(-1, K)
    g, dx = oracle.scan_backward(net, oracle.pack_params([w], [b]), x, all_pixels(N, Ho, Wo), delta,
                                 want_dx=True)
    dws, dbs = oracle.unpack_params(net, g)
    return dws[0], dbs[0], dx


def oracle_pool_fwd(x, k, d, is_max):
    N, C, H, W = x.shape
    net = single_layer_net(C, maxpool(k, k) if is_max else avgpool(k, k), k, d)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    pix = all_pixels(N, Ho, Wo)
    if is_max:
        s, am = oracle.scan_forward(net, np.zeros(0), x, pix, want_argmax=True)
        return (s.reshape(N, Ho, Wo, C).transpose(0, 3, 1, 2),
                am.reshape(N, Ho, Wo, C).transpose(0, 3, 1, 2))
    s = oracle.scan_forward(net, np.zeros(0), x, pix)
    return s.reshape(N, Ho, Wo, C).transpose(0, 3, 1, 2), None


def oracle_pool_bwd(x, k, d, is_max, dy):
    N, C, H, W = x.shape
    net = single_layer_net(C, maxpool(k, k) if is_max else avgpool(k, k), k, d)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    delta = np.asarray(dy, np.float64).transpose(0, 2, 3, 1).reshape(-1, C)
    _, dx = oracle.scan_backward(net, np.zeros(0), x, all_pixels(N, Ho, Wo), delta, want_dx=True)
    return dx
