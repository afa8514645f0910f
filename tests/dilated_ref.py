"""Test-only whole-image reference (numpy, fp64): Algorithm 1 written out with
naive dilated loops.  It exists to pin the oracle to the paper's exact-
equivalence claim (abstract; Sec. 3.1 last paragraph; Sec. 4.3): the oracle's
patch-by-patch result must equal this at EVERY pixel.  It is neither the oracle
nor the product and is used on tiny inputs only.
"""
import numpy as np


def dilations(net):
    """Algorithm 1: d starts at 1 and is multiplied by each layer's stride after it."""
    d, out = 1, []
    for L in net.layers:
        out.append(d)
        d *= L.s
    return out


def forward(net, weights, biases, xpad):
    """xpad [C0, Hp, Wp] -> (maps list incl. input, argmax list) with every stride 1."""
    x = np.asarray(xpad, np.float64)
    maps, ams = [x], [None]
    wi = 0
    for L, d in zip(net.layers, dilations(net)):
        C, H, W = x.shape
        Ho, Wo = H - (L.k - 1) * d, W - (L.k - 1) * d
        if L.kind == 0:
            w = np.asarray(weights[wi], np.float64)
            b = np.asarray(biases[wi], np.float64)
            wi += 1
            y = np.zeros((L.K, Ho, Wo)) + b[:, None, None]
            for a in range(L.k):
                for bb in range(L.k):
                    y += np.einsum("kc,chw->khw", w[:, :, a, bb],
                                   x[:, a * d:a * d + Ho, bb * d:bb * d + Wo])
            if L.act == 1:
                y = np.maximum(y, 0.0)
            elif L.act == 2:
                y = np.tanh(y)
            am = None
        elif L.kind == 1:
            y = x[:, 0:Ho, 0:Wo].copy()
            am = np.zeros((C, Ho, Wo), np.int32)
            for a in range(L.k):
                for bb in range(L.k):
                    t = x[:, a * d:a * d + Ho, bb * d:bb * d + Wo]
                    better = t > y
                    y = np.where(better, t, y)
                    am = np.where(better, a * L.k + bb, am)
        else:
            y = np.zeros((C, Ho, Wo))
            for a in range(L.k):
                for bb in range(L.k):
                    y += x[:, a * d:a * d + Ho, bb * d:bb * d + Wo]
            y /= L.k * L.k
            am = None
        maps.append(y)
        ams.append(am)
        x = y
    return maps, ams


def backward(net, weights, maps, ams, dlast):
    """Gradients of the stride-1 dilated network: returns (dws, dbs, dx_input)."""
    dy = np.asarray(dlast, np.float64)
    convs = [i for i, L in enumerate(net.layers) if L.kind == 0]
    dws, dbs = [None] * len(convs), [None] * len(convs)
    ds = dilations(net)
    for li in range(len(net.layers) - 1, -1, -1):
        L, d = net.layers[li], ds[li]
        x, y = maps[li], maps[li + 1]
        C, H, W = x.shape
        _, Ho, Wo = y.shape
        dx = np.zeros_like(x)
        if L.kind == 0:
            wi = convs.index(li)
            w = np.asarray(weights[wi], np.float64)
            if L.act == 1:
                dy = dy * (y > 0)
            elif L.act == 2:
                dy = dy * (1 - y * y)
            dbs[wi] = dy.sum(axis=(1, 2))
            dw = np.zeros_like(w)
            for a in range(L.k):
                for bb in range(L.k):
                    xs = x[:, a * d:a * d + Ho, bb * d:bb * d + Wo]
                    dw[:, :, a, bb] = np.einsum("khw,chw->kc", dy, xs)
                    dx[:, a * d:a * d + Ho, bb * d:bb * d + Wo] += np.einsum(
                        "kc,khw->chw", w[:, :, a, bb], dy)
            dws[wi] = dw
        elif L.kind == 1:
            for a in range(L.k):
                for bb in range(L.k):
                    dx[:, a * d:a * d + Ho, bb * d:bb * d + Wo] += dy * (ams[li + 1] == a * L.k + bb)
        else:
            for a in range(L.k):
                for bb in range(L.k):
                    dx[:, a * d:a * d + Ho, bb * d:bb * d + Wo] += dy / (L.k * L.k)
        dy = dx
    return dws, dbs, dy
