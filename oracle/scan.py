"""TEST INFRASTRUCTURE -- ctypes binding of patchscan.c plus the padding rule.

A `net` argument is any object with attributes C0, patch and layers, each layer
with kind (0 conv, 1 maxpool, 2 avgpool), K, k, s, act (0 none, 1 relu, 2 tanh):
the ORIGINAL strided CNN.  Nothing here knows about dilation.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "patchscan.c")
_LIB = os.path.join(_HERE, "libpatchscan.so")
_lib = None


class _CLayer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("K", ctypes.c_int), ("k", ctypes.c_int),
                ("s", ctypes.c_int), ("act", ctypes.c_int)]


def build(force=False):
    """Compile patchscan.c with gcc (OpenMP over patches)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lp = ctypes.POINTER(ctypes.c_long)
        Lp = ctypes.POINTER(_CLayer)
        ci, cl = ctypes.c_int, ctypes.c_long
        lib.orc_sizes.argtypes = [Lp, ci, ci, ci, lp, lp, ip, ip]
        lib.orc_geometry.argtypes = [Lp, ci, ci, ci, ip, ip, lp, lp]
        lib.orc_patch_forward.argtypes = [Lp, ci, ci, ci, dp, dp, dp, ip, dp, ci]
        lib.orc_scan_forward.argtypes = [Lp, ci, ci, ci, dp, dp, ci, ci, ci, ip, cl, dp, ip, ci]
        lib.orc_scan_forward_maps.argtypes = [Lp, ci, ci, ci, dp, dp, ci, ci, ci, ip, cl, dp, ip, dp, ci]
        lib.orc_scan_backward.argtypes = [Lp, ci, ci, ci, dp, dp, ci, ci, ci, ip, cl, dp, dp, dp, ci]
        lib.orc_num_threads.restype = ci
        _lib = lib
    return _lib


def num_threads():
    return int(_load().orc_num_threads())


def _clayers(net):
    arr = (_CLayer * len(net.layers))()
    for i, L in enumerate(net.layers):
        arr[i] = _CLayer(int(L.kind), int(L.K), int(L.k), int(L.s), int(L.act))
    return arr, len(net.layers)


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _iptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def geometry(net):
    """Per-map channels C[l], sizes m[l], activation offsets (l = 0..L) and
    per-layer parameter offsets of the patch CNN, plus totals."""
    lib = _load()
    arr, nL = _clayers(net)
    C = np.zeros(nL + 1, np.int32)
    m = np.zeros(nL + 1, np.int32)
    ao = np.zeros(nL + 1, np.int64)
    po = np.zeros(nL, np.int64)
    if lib.orc_geometry(arr, nL, net.C0, net.patch, _iptr(C), _iptr(m),
                        ao.ctypes.data_as(ctypes.POINTER(ctypes.c_long)),
                        po.ctypes.data_as(ctypes.POINTER(ctypes.c_long))):
        raise ValueError("malformed net")
    tot, npar = ctypes.c_long(), ctypes.c_long()
    cls, ml = ctypes.c_int(), ctypes.c_int()
    lib.orc_sizes(arr, nL, net.C0, net.patch, ctypes.byref(tot), ctypes.byref(npar),
                  ctypes.byref(cls), ctypes.byref(ml))
    return dict(C=C, m=m, act_off=ao, par_off=po, act_total=tot.value,
                n_params=npar.value, classes=cls.value, m_last=ml.value)


def pad_image(image, n):
    """Zero-pad [N, C, H, W] so that every pixel has an n x n patch (Sec. 3.3).

    floor(n/2) rows/columns go on the top/left and n-1-floor(n/2) on the
    bottom/right, so the padded size is H+n-1: for odd n this is the paper's
    h + 2*floor(n/2); for even n it is the paper's padding without its last row
    and column, which would produce an (H+1) x (W+1) output.  Pixel (i, j)'s
    patch is padded rows i..i+n-1 and columns j..j+n-1."""
    x = np.asarray(image, np.float64)
    N, C, H, W = x.shape
    lo = n // 2
    out = np.zeros((N, C, H + n - 1, W + n - 1), np.float64)
    out[:, :, lo:lo + H, lo:lo + W] = x
    return out


def pack_params(weights, biases):
    """Flat fp64 vector: for every conv layer its weights [K,C,k,k] then its bias [K]."""
    parts = []
    for w, b in zip(weights, biases):
        parts.append(np.asarray(w, np.float64).ravel())
        parts.append(np.asarray(b, np.float64).ravel())
    return np.ascontiguousarray(np.concatenate(parts)) if parts else np.zeros(0)


def unpack_params(net, flat):
    """Inverse of pack_params: lists of [K,C,k,k] and [K] arrays."""
    ws, bs, c, o = [], [], net.C0, 0
    for L in net.layers:
        if L.kind == 0:
            nw = L.K * c * L.k * L.k
            ws.append(flat[o:o + nw].reshape(L.K, c, L.k, L.k).copy())
            o += nw
            bs.append(flat[o:o + L.K].copy())
            o += L.K
            c = L.K
    assert o == flat.size
    return ws, bs


STORE_EXACT, STORE_BF16 = 0, 1


def _split_maps(g, flat, nL):
    out = []
    for l in range(nL + 1):
        o, C, m = int(g["act_off"][l]), int(g["C"][l]), int(g["m"][l])
        out.append(flat[..., o:o + C * m * m].reshape(flat.shape[:-1] + (C, m, m)))
    return out


def patch_forward(net, params, patch, storage=STORE_EXACT, want_pre=False):
    """Original CNN on one patch [C0, n, n].  Returns (maps, argmax): lists over
    l = 0..L of fp64 [C_l, m_l, m_l] maps (map 0 is the patch) and int32 arrays of
    the same shapes holding the winning tap index a*k+b of max-pool outputs
    (-1 elsewhere).  With want_pre a third list: the values of conv outputs before
    the non-linearity (0 elsewhere)."""
    lib = _load()
    g = geometry(net)
    arr, nL = _clayers(net)
    params = np.ascontiguousarray(params, np.float64)
    patch = np.ascontiguousarray(patch, np.float64)
    assert patch.shape == (net.C0, net.patch, net.patch)
    assert params.size == g["n_params"]
    acts = np.zeros(g["act_total"], np.float64)
    amax = np.zeros(g["act_total"], np.int32)
    pre = np.zeros(g["act_total"], np.float64) if want_pre else None
    if lib.orc_patch_forward(arr, nL, net.C0, net.patch, _dptr(params), _dptr(patch),
                             _dptr(acts), _iptr(amax), _dptr(pre) if want_pre else None, storage):
        raise ValueError("malformed net")
    res = ([m.copy() for m in _split_maps(g, acts, nL)], [m.copy() for m in _split_maps(g, amax, nL)])
    if want_pre:
        res += ([m.copy() for m in _split_maps(g, pre, nL)],)
    return res


def scan_forward_maps(net, params, xpad, pix, storage=STORE_EXACT):
    """Every map of every listed patch.  Returns (maps, argmax, pre): lists over l = 0..L of
    arrays [P, C_l, m_l, m_l] -- fp64 maps (map 0 = the patches), int32 winning tap indices of
    max-pool outputs (-1 elsewhere), fp64 conv outputs before the non-linearity (0 elsewhere).
    Entry (u, v) of map l of the patch at (i, j) is the whole-image map l at (i + D*u, j + D*v),
    D = product of the strides of layers 1..l (Fig. 3)."""
    lib = _load()
    g = geometry(net)
    arr, nL = _clayers(net)
    params = np.ascontiguousarray(params, np.float64)
    xpad = np.ascontiguousarray(xpad, np.float64)
    pix = np.ascontiguousarray(pix, np.int32).reshape(-1, 3)
    assert params.size == g["n_params"]
    N, C0, Hp, Wp = xpad.shape
    assert C0 == net.C0
    P = pix.shape[0]
    acts = np.zeros((P, g["act_total"]), np.float64)
    amax = np.zeros((P, g["act_total"]), np.int32)
    pre = np.zeros((P, g["act_total"]), np.float64)
    rc = lib.orc_scan_forward_maps(arr, nL, net.C0, net.patch, _dptr(params), _dptr(xpad),
                                   N, Hp, Wp, _iptr(pix), P, _dptr(acts), _iptr(amax), _dptr(pre), storage)
    if rc:
        raise ValueError("orc_scan_forward_maps failed: %d" % rc)
    return _split_maps(g, acts, nL), _split_maps(g, amax, nL), _split_maps(g, pre, nL)


def scan_forward(net, params, xpad, pix, want_argmax=False, storage=STORE_EXACT):
    """Scores [P, classes] of the patches at pix [P, 3] = (image, i, j).  With
    want_argmax (last layer a max pool) also the winning tap indices [P, classes].
    storage=STORE_BF16 rounds the patch and every layer output but the last to bfloat16."""
    lib = _load()
    g = geometry(net)
    if g["m_last"] != 1:
        raise ValueError("net does not reduce the patch to 1x1")
    arr, nL = _clayers(net)
    params = np.ascontiguousarray(params, np.float64)
    xpad = np.ascontiguousarray(xpad, np.float64)
    pix = np.ascontiguousarray(pix, np.int32).reshape(-1, 3)
    assert params.size == g["n_params"]
    N, C0, Hp, Wp = xpad.shape
    assert C0 == net.C0
    out = np.zeros((pix.shape[0], g["classes"]), np.float64)
    am = np.zeros((pix.shape[0], g["classes"]), np.int32) if want_argmax else None
    rc = lib.orc_scan_forward(arr, nL, net.C0, net.patch, _dptr(params), _dptr(xpad),
                              N, Hp, Wp, _iptr(pix), pix.shape[0], _dptr(out),
                              _iptr(am) if want_argmax else None, storage)
    if rc:
        raise ValueError("orc_scan_forward failed: %d" % rc)
    return (out, am) if want_argmax else out


def scan_backward(net, params, xpad, pix, delta, want_dx=False, storage=STORE_EXACT):
    """Sum over the listed patches of the parameter gradients for output errors
    delta [P, classes].  Returns (dparams flat, dxpad or None)."""
    lib = _load()
    g = geometry(net)
    if g["m_last"] != 1:
        raise ValueError("net does not reduce the patch to 1x1")
    arr, nL = _clayers(net)
    params = np.ascontiguousarray(params, np.float64)
    xpad = np.ascontiguousarray(xpad, np.float64)
    pix = np.ascontiguousarray(pix, np.int32).reshape(-1, 3)
    delta = np.ascontiguousarray(delta, np.float64).reshape(pix.shape[0], g["classes"])
    N, C0, Hp, Wp = xpad.shape
    assert C0 == net.C0
    dpar = np.zeros(max(g["n_params"], 1), np.float64)
    dx = np.zeros_like(xpad) if want_dx else None
    rc = lib.orc_scan_backward(arr, nL, net.C0, net.patch, _dptr(params), _dptr(xpad),
                               N, Hp, Wp, _iptr(pix), pix.shape[0], _dptr(delta), _dptr(dpar),
                               _dptr(dx) if want_dx else None, storage)
    if rc:
        raise ValueError("orc_scan_backward failed: %d" % rc)
    return dpar[:g["n_params"]], dx
