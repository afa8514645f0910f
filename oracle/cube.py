"""TEST INFRASTRUCTURE -- ctypes binding of cubescan.c (cube-by-cube scanning of a
video through the original strided 3-D CNN, fp64) plus the padding rule in 3-D.

A `net` argument is any object with attributes C0, patch_t, patch and layers, each
layer with kind (0 conv, 1 maxpool, 2 avgpool), K, k, s, kt, st, act.  Videos are
[N, C, T, H, W], conv weights [K, C, kt, k, k].  Nothing here knows about dilation.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cubescan.c")
_LIB = os.path.join(_HERE, "libcubescan.so")
_lib = None


class _CLayer3(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("K", ctypes.c_int), ("k", ctypes.c_int), ("s", ctypes.c_int),
                ("kt", ctypes.c_int), ("st", ctypes.c_int), ("act", ctypes.c_int)]


def build3d(force=False):
    """Compile cubescan.c with gcc (OpenMP over cubes)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build3d()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int)
        lp = ctypes.POINTER(ctypes.c_long)
        Lp = ctypes.POINTER(_CLayer3)
        ci, cl = ctypes.c_int, ctypes.c_long
        lib.orc3_geometry.argtypes = [Lp, ci, ci, ci, ci, ip, ip, ip, lp, lp, lp]
        lib.orc3_scan_forward_maps.argtypes = [Lp, ci, ci, ci, ci, dp, dp, ci, ci, ci, ci, ip, cl, dp, ip]
        lib.orc3_scan_forward.argtypes = [Lp, ci, ci, ci, ci, dp, dp, ci, ci, ci, ci, ip, cl, dp]
        lib.orc3_scan_backward.argtypes = [Lp, ci, ci, ci, ci, dp, dp, ci, ci, ci, ci, ip, cl, dp, dp, dp]
        _lib = lib
    return _lib


def _clayers(net):
    arr = (_CLayer3 * len(net.layers))()
    for i, L in enumerate(net.layers):
        arr[i] = _CLayer3(int(L.kind), int(L.K), int(L.k), int(L.s), int(L.kt), int(L.st), int(L.act))
    return arr, len(net.layers)


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _iptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def _lptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_long))


def geometry3d(net):
    """Channels C[l], temporal / spatial sizes mt[l], m[l] and activation offsets of the maps l = 0..L of the
    cube CNN, parameter offsets per layer, totals."""
    lib = _load()
    arr, nL = _clayers(net)
    C = np.zeros(nL + 1, np.int32)
    mt = np.zeros(nL + 1, np.int32)
    m = np.zeros(nL + 1, np.int32)
    ao = np.zeros(nL + 2, np.int64)
    po = np.zeros(nL, np.int64)
    npar = ctypes.c_long()
    if lib.orc3_geometry(arr, nL, net.C0, net.patch_t, net.patch, _iptr(C), _iptr(mt), _iptr(m), _lptr(ao), _lptr(po),
                         ctypes.byref(npar)):
        raise ValueError("malformed net")
    return dict(C=C, mt=mt, m=m, act_off=ao, par_off=po, act_total=int(ao[nL + 1]), n_params=npar.value,
                classes=int(C[nL]))


def pad_video(video, nt, n):
    """Zero-pad [N, C, T, H, W] so that every voxel has an nt x n x n cube: the rule of Sec. 3.3 on each of the
    three axes (floor(size/2) in front, size-1-floor(size/2) behind).  Voxel (t, i, j)'s cube is padded frames
    t..t+nt-1, rows i..i+n-1, columns j..j+n-1."""
    x = np.asarray(video, np.float64)
    N, C, T, H, W = x.shape
    lt, lo = nt // 2, n // 2
    out = np.zeros((N, C, T + nt - 1, H + n - 1, W + n - 1), np.float64)
    out[:, :, lt:lt + T, lo:lo + H, lo:lo + W] = x
    return out


def pack_params3d(weights, biases):
    """Flat fp64 vector: for every conv layer its weights [K,C,kt,k,k] then its bias [K]."""
    parts = []
    for w, b in zip(weights, biases):
        parts.append(np.asarray(w, np.float64).ravel())
        parts.append(np.asarray(b, np.float64).ravel())
    return np.ascontiguousarray(np.concatenate(parts))


def unpack_params3d(net, flat):
    ws, bs, c, o = [], [], net.C0, 0
    for L in net.layers:
        if L.kind == 0:
            nw = L.K * c * L.kt * L.k * L.k
            ws.append(flat[o:o + nw].reshape(L.K, c, L.kt, L.k, L.k).copy())
            o += nw
            bs.append(flat[o:o + L.K].copy())
            o += L.K
            c = L.K
    assert o == flat.size
    return ws, bs


def _prep(net, params, xpad, vox):
    g = geometry3d(net)
    params = np.ascontiguousarray(params, np.float64)
    xpad = np.ascontiguousarray(xpad, np.float64)
    vox = np.ascontiguousarray(vox, np.int32).reshape(-1, 4)
    assert params.size == g["n_params"] and xpad.shape[1] == net.C0
    return g, params, xpad, vox


def cube_forward_maps(net, params, xpad, vox):
    """Every map of every listed cube.  Returns (maps, argmax): lists over l = 0..L of [P, C_l, mt_l, m_l, m_l]
    arrays -- fp64 maps (map 0 = the cubes) and int32 winning tap indices (e*k + a)*k + b of max-pool outputs
    (-1 elsewhere).  Entry (q, u, v) of map l of the cube at (t, i, j) is the whole-video map l at
    (t + Dt*q, i + D*u, j + D*v), Dt / D = products of the temporal / spatial strides of layers 1..l."""
    lib = _load()
    g, params, xpad, vox = _prep(net, params, xpad, vox)
    arr, nL = _clayers(net)
    N, _, Tp, Hp, Wp = xpad.shape
    P = vox.shape[0]
    acts = np.zeros((P, g["act_total"]), np.float64)
    amax = np.zeros((P, g["act_total"]), np.int32)
    rc = lib.orc3_scan_forward_maps(arr, nL, net.C0, net.patch_t, net.patch, _dptr(params), _dptr(xpad),
                                    N, Tp, Hp, Wp, _iptr(vox), P, _dptr(acts), _iptr(amax))
    if rc:
        raise ValueError("orc3_scan_forward_maps failed: %d" % rc)

    def split(flat):
        out = []
        for l in range(nL + 1):
            o, C, mt, m = int(g["act_off"][l]), int(g["C"][l]), int(g["mt"][l]), int(g["m"][l])
            out.append(flat[:, o:o + C * mt * m * m].reshape(P, C, mt, m, m))
        return out
    return split(acts), split(amax)


def cube_scan_forward(net, params, xpad, vox):
    """Scores [P, classes] of the cubes at vox [P, 4] = (video, t, i, j)."""
    lib = _load()
    g, params, xpad, vox = _prep(net, params, xpad, vox)
    arr, nL = _clayers(net)
    N, _, Tp, Hp, Wp = xpad.shape
    out = np.zeros((vox.shape[0], g["classes"]), np.float64)
    rc = lib.orc3_scan_forward(arr, nL, net.C0, net.patch_t, net.patch, _dptr(params), _dptr(xpad),
                               N, Tp, Hp, Wp, _iptr(vox), vox.shape[0], _dptr(out))
    if rc:
        raise ValueError("orc3_scan_forward failed: %d" % rc)
    return out


def cube_scan_backward(net, params, xpad, vox, delta, want_dx=False):
    """Sum over the listed cubes of the parameter gradients for output errors delta [P, classes].
    Returns (dparams flat, dxpad or None)."""
    lib = _load()
    g, params, xpad, vox = _prep(net, params, xpad, vox)
    arr, nL = _clayers(net)
    N, _, Tp, Hp, Wp = xpad.shape
    delta = np.ascontiguousarray(delta, np.float64).reshape(vox.shape[0], g["classes"])
    dpar = np.zeros(max(g["n_params"], 1), np.float64)
    dx = np.zeros_like(xpad) if want_dx else None
    rc = lib.orc3_scan_backward(arr, nL, net.C0, net.patch_t, net.patch, _dptr(params), _dptr(xpad),
                                N, Tp, Hp, Wp, _iptr(vox), vox.shape[0], _dptr(delta), _dptr(dpar),
                                _dptr(dx) if want_dx else None)
    if rc:
        raise ValueError("orc3_scan_backward failed: %d" % rc)
    return dpar[:g["n_params"]], dx
