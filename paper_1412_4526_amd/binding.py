"""ctypes binding of libdsk.so: the same names as include/dsk.h, argument
marshalling only.  Tensors are torch tensors on the GPU (torch is used for device
memory and streams); every step of the computation runs in the library's kernels.

The library is loaded from this directory; if it has not been built the import
fails loudly -- there is no fallback path.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libdsk.so")

DSK_OK, DSK_EINVAL, DSK_ESHAPE, DSK_EDTYPE, DSK_EWORKSPACE, DSK_ELAUNCH = 0, -1, -2, -3, -4, -5
DSK_F32, DSK_BF16 = 0, 1
DSK_ACT_NONE, DSK_ACT_RELU, DSK_ACT_TANH = 0, 1, 2
DSK_CONV, DSK_MAXPOOL, DSK_AVGPOOL = 0, 1, 2
DSK_WS_CONV_FWD, DSK_WS_CONV_BWD_DATA, DSK_WS_CONV_BWD_WEIGHT = 0, 1, 2

# every symbol include/dsk.h declares
SYMBOLS = ("dsk_plan", "dsk_status_string", "dsk_pad_image", "dsk_conv_workspace_bytes",
           "dsk_conv_fwd", "dsk_conv_bwd_data", "dsk_conv_bwd_weight",
           "dsk_maxpool_fwd", "dsk_maxpool_bwd", "dsk_avgpool_fwd", "dsk_avgpool_bwd",
           "dsk_act_bwd", "dsk_act_bwd_bias_workspace_bytes", "dsk_act_bwd_bias",
           "dsk_pool_bwd_act_bias_workspace_bytes", "dsk_pool_bwd_act_bias",
           "dsk_conv_bwd_data_act_bias_workspace_bytes", "dsk_conv_bwd_data_act_bias",
           "dsk_softmax_xent_workspace_bytes", "dsk_masked_softmax_xent", "dsk_masked_softmax_xent_static",
           "dsk_fs_pool_fwd", "dsk_fs_conv_fwd", "dsk_fs_assemble",
           "dsk_pad_video", "dsk_conv3d_workspace_bytes", "dsk_conv3d_fwd", "dsk_conv3d_bwd_data", "dsk_conv3d_bwd_weight",
           "dsk_maxpool3d_fwd", "dsk_maxpool3d_bwd", "dsk_avgpool3d_fwd", "dsk_avgpool3d_bwd",
           "dsk_set_conv_algo")


class DskError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_string(status)))


class dsk_layer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("K", ctypes.c_int), ("k", ctypes.c_int),
                ("s", ctypes.c_int), ("act", ctypes.c_int)]


class dsk_layer_plan(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("act", ctypes.c_int), ("C", ctypes.c_int), ("K", ctypes.c_int),
                ("k", ctypes.c_int), ("d", ctypes.c_int), ("H", ctypes.c_int), ("W", ctypes.c_int),
                ("Ho", ctypes.c_int), ("Wo", ctypes.c_int)]

    def __repr__(self):
        return "plan(kind=%d C=%d K=%d k=%d d=%d %dx%d->%dx%d act=%d)" % (
            self.kind, self.C, self.K, self.k, self.d, self.H, self.W, self.Ho, self.Wo, self.act)


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libdsk.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_1412_4526_amd/build.py) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    ip = ctypes.POINTER(ctypes.c_int)
    lib.dsk_plan.argtypes = [ctypes.POINTER(dsk_layer), ci, ci, ci, ci, ci,
                             ctypes.POINTER(dsk_layer_plan), ip, ip, ip]
    lib.dsk_status_string.argtypes = [ci]
    lib.dsk_status_string.restype = ctypes.c_char_p
    lib.dsk_pad_image.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.dsk_conv_workspace_bytes.argtypes = [ci] * 10
    lib.dsk_conv_workspace_bytes.restype = sz
    lib.dsk_conv_fwd.argtypes = [vp, vp, vp, vp] + [ci] * 8 + [ci, ci, ci, vp, sz, vp]
    lib.dsk_conv_bwd_data.argtypes = [vp, vp, vp] + [ci] * 8 + [ci, ci, vp, sz, vp]
    lib.dsk_conv_bwd_weight.argtypes = [vp, vp, vp, vp] + [ci] * 8 + [ci, vp, sz, vp]
    lib.dsk_maxpool_fwd.argtypes = [vp, vp, vp] + [ci] * 6 + [ci, vp]
    lib.dsk_maxpool_bwd.argtypes = [vp, vp, vp] + [ci] * 6 + [ci, vp]
    lib.dsk_avgpool_fwd.argtypes = [vp, vp] + [ci] * 6 + [ci, vp]
    lib.dsk_avgpool_bwd.argtypes = [vp, vp] + [ci] * 6 + [ci, vp]
    lib.dsk_act_bwd.argtypes = [vp, vp, sz, ci, ci, vp]
    lib.dsk_act_bwd_bias_workspace_bytes.argtypes = [ci]
    lib.dsk_act_bwd_bias_workspace_bytes.restype = sz
    lib.dsk_act_bwd_bias.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.dsk_pool_bwd_act_bias_workspace_bytes.argtypes = [ci] * 8
    lib.dsk_pool_bwd_act_bias_workspace_bytes.restype = sz
    lib.dsk_pool_bwd_act_bias.argtypes = [ci, vp, vp, vp, vp, vp] + [ci] * 6 + [ci, ci, vp, sz, vp]
    lib.dsk_conv_bwd_data_act_bias_workspace_bytes.argtypes = [ci] * 10
    lib.dsk_conv_bwd_data_act_bias_workspace_bytes.restype = sz
    lib.dsk_conv_bwd_data_act_bias.argtypes = [vp] * 5 + [ci] * 8 + [ci, ci, ci, vp, sz, vp]
    lib.dsk_softmax_xent_workspace_bytes.argtypes = [ci] * 4
    lib.dsk_softmax_xent_workspace_bytes.restype = sz
    lib.dsk_masked_softmax_xent.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
    lib.dsk_masked_softmax_xent_static.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
    lib.dsk_fs_pool_fwd.argtypes = [ci, vp, vp] + [ci] * 9 + [ci, vp]
    lib.dsk_fs_conv_fwd.argtypes = [vp, vp, vp, vp] + [ci] * 10 + [ci, ci, vp]
    lib.dsk_fs_assemble.argtypes = [vp, vp] + [ci] * 7 + [ci, ci, vp]
    lib.dsk_pad_video.argtypes = [vp, vp] + [ci] * 9 + [ci, vp]
    lib.dsk_conv3d_workspace_bytes.argtypes = [ci] * 13
    lib.dsk_conv3d_workspace_bytes.restype = sz
    lib.dsk_conv3d_fwd.argtypes = [vp, vp, vp, vp] + [ci] * 11 + [ci, ci, ci, vp, sz, vp]
    lib.dsk_conv3d_bwd_data.argtypes = [vp, vp, vp] + [ci] * 11 + [ci, ci, vp, sz, vp]
    lib.dsk_conv3d_bwd_weight.argtypes = [vp, vp, vp, vp] + [ci] * 11 + [ci, vp, sz, vp]
    lib.dsk_maxpool3d_fwd.argtypes = [vp, vp, vp] + [ci] * 9 + [ci, vp]
    lib.dsk_maxpool3d_bwd.argtypes = [vp, vp, vp] + [ci] * 9 + [ci, vp]
    lib.dsk_avgpool3d_fwd.argtypes = [vp, vp] + [ci] * 9 + [ci, vp]
    lib.dsk_avgpool3d_bwd.argtypes = [vp, vp] + [ci] * 9 + [ci, vp]
    lib.dsk_set_conv_algo.argtypes = [ci]
    for name in SYMBOLS:
        getattr(lib, name)      # AttributeError here = header and library disagree
    return lib


lib = _load()


def status_string(status):
    return lib.dsk_status_string(int(status)).decode()


def _check(rc, where):
    if rc != DSK_OK:
        raise DskError(rc, where)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return DSK_F32
    if t.dtype == torch.bfloat16:
        return DSK_BF16
    raise TypeError("libdsk tensors are float32 or bfloat16, got %s" % t.dtype)


def torch_dtype(code):
    return torch.float32 if code == DSK_F32 else torch.bfloat16


def _dev(t, dtype=None):
    """Device pointer of a contiguous GPU tensor."""
    if not t.is_cuda:
        raise ValueError("libdsk needs GPU tensors")
    if not t.is_contiguous():
        raise ValueError("libdsk needs contiguous tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    return _dev(ws), ws.numel() * ws.element_size()


# --------------------------------------------------------------------------- planner (host only)
def dsk_plan(layers, C0, H, W, n=0):
    """layers: iterable of objects with kind, K, k, s, act (the original strided CNN).
    Returns (list of dsk_layer_plan, rf, pad_lo, pad_hi)."""
    layers = list(layers)
    arr = (dsk_layer * max(len(layers), 1))()
    for i, L in enumerate(layers):
        arr[i] = dsk_layer(int(L.kind), int(L.K), int(L.k), int(L.s), int(L.act))
    out = (dsk_layer_plan * max(len(layers), 1))()
    rf, lo, hi = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(lib.dsk_plan(arr, len(layers), C0, H, W, n, out, ctypes.byref(rf), ctypes.byref(lo),
                        ctypes.byref(hi)), "dsk_plan")
    return [out[i] for i in range(len(layers))], rf.value, lo.value, hi.value


def dsk_set_conv_algo(algo):
    return lib.dsk_set_conv_algo(int(algo))


# --------------------------------------------------------------------------- device entry points
def dsk_pad_image(x, lo, hi, out_dtype=torch.float32, xpad=None):
    N, C, H, W = x.shape
    if xpad is None:
        xpad = torch.empty((N, C, H + lo + hi, W + lo + hi), dtype=out_dtype, device=x.device)
    _check(lib.dsk_pad_image(_dev(x, torch.float32), _dev(xpad), N, C, H, W, lo, hi, _dtype_code(xpad),
                             _stream()), "dsk_pad_image")
    return xpad


def dsk_conv_workspace_bytes(which, N, C, H, W, K, kh, kw, d, in_code):
    return int(lib.dsk_conv_workspace_bytes(which, N, C, H, W, K, kh, kw, d, in_code))


def _conv_ws(which, shape, in_code, ws, device):
    need = dsk_conv_workspace_bytes(which, *shape, in_code)
    if need and (ws is None or ws.numel() * ws.element_size() < need):
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws


def dsk_conv_fwd(x, w, b, d, act=DSK_ACT_NONE, out_dtype=None, y=None, ws=None):
    N, C, H, W = x.shape
    K, Cw, kh, kw = w.shape
    assert Cw == C
    if y is None:
        Ho, Wo = H - (kh - 1) * d, W - (kw - 1) * d
        if Ho < 1 or Wo < 1:
            raise DskError(DSK_ESHAPE, "dsk_conv_fwd")
        y = torch.empty((N, K, Ho, Wo), dtype=out_dtype or x.dtype, device=x.device)
    ws = _conv_ws(DSK_WS_CONV_FWD, (N, C, H, W, K, kh, kw, d), _dtype_code(x), ws, x.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_conv_fwd(_dev(x), _dev(w, torch.float32), None if b is None else _dev(b, torch.float32),
                            _dev(y), N, C, H, W, K, kh, kw, d, _dtype_code(x), _dtype_code(y), act,
                            wsp, wsb, _stream()), "dsk_conv_fwd")
    return y


def dsk_conv_bwd_data(dy, w, d, H, W, out_dtype=None, dx=None, ws=None):
    N, K, Ho, Wo = dy.shape
    Kw, C, kh, kw = w.shape
    assert Kw == K and Ho == H - (kh - 1) * d and Wo == W - (kw - 1) * d
    if dx is None:
        dx = torch.empty((N, C, H, W), dtype=out_dtype or dy.dtype, device=dy.device)
    ws = _conv_ws(DSK_WS_CONV_BWD_DATA, (N, C, H, W, K, kh, kw, d), _dtype_code(dy), ws, dy.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_conv_bwd_data(_dev(dy), _dev(w, torch.float32), _dev(dx), N, C, H, W, K, kh, kw, d,
                                 _dtype_code(dy), _dtype_code(dx), wsp, wsb, _stream()), "dsk_conv_bwd_data")
    return dx


def dsk_conv_bwd_weight(x, dy, kh, kw, d, dw=None, db=None, want_db=True, ws=None):
    N, C, H, W = x.shape
    N2, K, Ho, Wo = dy.shape
    assert N2 == N and Ho == H - (kh - 1) * d and Wo == W - (kw - 1) * d and x.dtype == dy.dtype
    if dw is None:
        dw = torch.empty((K, C, kh, kw), dtype=torch.float32, device=x.device)
    if db is None and want_db:
        db = torch.empty((K,), dtype=torch.float32, device=x.device)
    ws = _conv_ws(DSK_WS_CONV_BWD_WEIGHT, (N, C, H, W, K, kh, kw, d), _dtype_code(x), ws, x.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_conv_bwd_weight(_dev(x), _dev(dy), _dev(dw, torch.float32),
                                   None if db is None else _dev(db, torch.float32),
                                   N, C, H, W, K, kh, kw, d, _dtype_code(x), wsp, wsb, _stream()),
           "dsk_conv_bwd_weight")
    return dw, db


def dsk_maxpool_fwd(x, k, d, y=None, argmax=None, want_argmax=True):
    N, C, H, W = x.shape
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    if Ho < 1 or Wo < 1:
        raise DskError(DSK_ESHAPE, "dsk_maxpool_fwd")
    if y is None:
        y = torch.empty((N, C, Ho, Wo), dtype=x.dtype, device=x.device)
    if argmax is None and want_argmax:
        argmax = torch.empty((N, C, Ho, Wo), dtype=torch.uint8, device=x.device)
    _check(lib.dsk_maxpool_fwd(_dev(x), _dev(y), None if argmax is None else _dev(argmax, torch.uint8),
                               N, C, H, W, k, d, _dtype_code(x), _stream()), "dsk_maxpool_fwd")
    return y, argmax


def dsk_maxpool_bwd(dy, argmax, k, d, H, W, dx=None):
    N, C, Ho, Wo = dy.shape
    assert Ho == H - (k - 1) * d and Wo == W - (k - 1) * d and argmax.shape == dy.shape
    if dx is None:
        dx = torch.empty((N, C, H, W), dtype=dy.dtype, device=dy.device)
    _check(lib.dsk_maxpool_bwd(_dev(dy), _dev(argmax, torch.uint8), _dev(dx), N, C, H, W, k, d,
                               _dtype_code(dy), _stream()), "dsk_maxpool_bwd")
    return dx


def dsk_avgpool_fwd(x, k, d, y=None):
    N, C, H, W = x.shape
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    if Ho < 1 or Wo < 1:
        raise DskError(DSK_ESHAPE, "dsk_avgpool_fwd")
    if y is None:
        y = torch.empty((N, C, Ho, Wo), dtype=x.dtype, device=x.device)
    _check(lib.dsk_avgpool_fwd(_dev(x), _dev(y), N, C, H, W, k, d, _dtype_code(x), _stream()),
           "dsk_avgpool_fwd")
    return y


def dsk_avgpool_bwd(dy, k, d, H, W, dx=None):
    N, C, Ho, Wo = dy.shape
    assert Ho == H - (k - 1) * d and Wo == W - (k - 1) * d
    if dx is None:
        dx = torch.empty((N, C, H, W), dtype=dy.dtype, device=dy.device)
    _check(lib.dsk_avgpool_bwd(_dev(dy), _dev(dx), N, C, H, W, k, d, _dtype_code(dy), _stream()),
           "dsk_avgpool_bwd")
    return dx


def dsk_act_bwd(y, dy, act):
    """In place on dy."""
    assert y.shape == dy.shape and y.dtype == dy.dtype
    _check(lib.dsk_act_bwd(_dev(y), _dev(dy), y.numel(), act, _dtype_code(y), _stream()), "dsk_act_bwd")
    return dy


def dsk_act_bwd_bias_workspace_bytes(K):
    return int(lib.dsk_act_bwd_bias_workspace_bytes(K))


def dsk_act_bwd_bias(y, dy, act, db=None, ws=None):
    """In place on dy; returns db [K] (fp32)."""
    N, K, Ho, Wo = dy.shape
    assert act == DSK_ACT_NONE or (y.shape == dy.shape and y.dtype == dy.dtype)
    if db is None:
        db = torch.empty((K,), dtype=torch.float32, device=dy.device)
    need = dsk_act_bwd_bias_workspace_bytes(K)
    if ws is None or ws.numel() * ws.element_size() < need:
        ws = torch.empty(need, dtype=torch.uint8, device=dy.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_act_bwd_bias(None if act == DSK_ACT_NONE else _dev(y), _dev(dy), _dev(db, torch.float32),
                                N, K, Ho, Wo, act, _dtype_code(dy), wsp, wsb, _stream()), "dsk_act_bwd_bias")
    return db


def dsk_pool_bwd_act_bias_workspace_bytes(kind, N, C, H, W, k, d, code):
    return int(lib.dsk_pool_bwd_act_bias_workspace_bytes(kind, N, C, H, W, k, d, code))


def dsk_pool_bwd_act_bias(kind, dy, argmax, y, k, d, H, W, act, dx=None, db=None, ws=None):
    """Pool gradient, non-linearity backward of the conv layer in front of the pool and that layer's bias
    gradient in one pass.  Returns (dx, db)."""
    N, C, Ho, Wo = dy.shape
    assert Ho == H - (k - 1) * d and Wo == W - (k - 1) * d
    if dx is None:
        dx = torch.empty((N, C, H, W), dtype=dy.dtype, device=dy.device)
    if db is None:
        db = torch.empty((C,), dtype=torch.float32, device=dy.device)
    need = dsk_pool_bwd_act_bias_workspace_bytes(kind, N, C, H, W, k, d, _dtype_code(dy))
    if ws is None or ws.numel() * ws.element_size() < need:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dy.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_pool_bwd_act_bias(kind, _dev(dy), None if argmax is None else _dev(argmax, torch.uint8),
                                     None if act == DSK_ACT_NONE else _dev(y), _dev(dx), _dev(db, torch.float32),
                                     N, C, H, W, k, d, act, _dtype_code(dy), wsp, wsb, _stream()),
           "dsk_pool_bwd_act_bias")
    return dx, db


def dsk_conv_bwd_data_act_bias_workspace_bytes(N, C, H, W, K, kh, kw, d, in_code, out_code):
    return int(lib.dsk_conv_bwd_data_act_bias_workspace_bytes(N, C, H, W, K, kh, kw, d, in_code, out_code))


def dsk_conv_bwd_data_act_bias(dy, w, x, d, act, dx=None, db=None, ws=None):
    """Backward-data of a conv layer, non-linearity backward of the conv layer below it (whose stored
    output x is this layer's input) and that layer's bias gradient.  Returns (dx, db)."""
    N, K, Ho, Wo = dy.shape
    Kw, C, kh, kw = w.shape
    _, Cx, H, W = x.shape
    assert Kw == K and Cx == C and Ho == H - (kh - 1) * d and Wo == W - (kw - 1) * d
    if dx is None:
        dx = torch.empty((N, C, H, W), dtype=x.dtype, device=dy.device)
    assert dx.dtype == x.dtype
    if db is None:
        db = torch.empty((C,), dtype=torch.float32, device=dy.device)
    need = dsk_conv_bwd_data_act_bias_workspace_bytes(N, C, H, W, K, kh, kw, d, _dtype_code(dy), _dtype_code(dx))
    if ws is None or ws.numel() * ws.element_size() < need:
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dy.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_conv_bwd_data_act_bias(_dev(dy), _dev(w, torch.float32), None if act == DSK_ACT_NONE else _dev(x),
                                          _dev(dx), _dev(db, torch.float32), N, C, H, W, K, kh, kw, d,
                                          _dtype_code(dy), _dtype_code(dx), act, wsp, wsb, _stream()),
           "dsk_conv_bwd_data_act_bias")
    return dx, db


def dsk_softmax_xent_workspace_bytes(N, Cls, H, W):
    return int(lib.dsk_softmax_xent_workspace_bytes(N, Cls, H, W))


def dsk_masked_softmax_xent(scores, labels, mask, dscores_dtype=torch.float32, loss=None, dscores=None,
                            ws=None):
    N, Cls, H, W = scores.shape
    assert labels.shape == (N, H, W) and mask.shape == (N, H, W)
    if loss is None:
        loss = torch.empty((1,), dtype=torch.float32, device=scores.device)
    if dscores is None:
        dscores = torch.empty((N, Cls, H, W), dtype=dscores_dtype, device=scores.device)
    need = dsk_softmax_xent_workspace_bytes(N, Cls, H, W)
    if ws is None or ws.numel() * ws.element_size() < need:
        ws = torch.empty(need, dtype=torch.uint8, device=scores.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_masked_softmax_xent(_dev(scores, torch.float32), _dev(labels, torch.int32),
                                       _dev(mask, torch.uint8), _dev(loss, torch.float32), _dev(dscores),
                                       _dtype_code(dscores), N, Cls, H, W, wsp, wsb, _stream()),
           "dsk_masked_softmax_xent")
    return loss, dscores


def dsk_masked_softmax_xent_static(scores, labels, mask, loss, dscores):
    """The allocation-free form: every buffer is the caller's, the scratch memory is the library's own."""
    N, Cls, H, W = scores.shape
    assert labels.shape == (N, H, W) and mask.shape == (N, H, W) and dscores.shape == scores.shape
    _check(lib.dsk_masked_softmax_xent_static(_dev(scores, torch.float32), _dev(labels, torch.int32),
                                              _dev(mask, torch.uint8), _dev(loss, torch.float32), _dev(dscores),
                                              _dtype_code(dscores), N, Cls, H, W, _stream()),
           "dsk_masked_softmax_xent_static")
    return loss, dscores


# --------------------------------------------------------------------------- fast scanning (comparison method)
def dsk_fs_pool_fwd(kind, x, D, k, s, ho, wo, out=None):
    """x [N*D*D, C, hi, wi] -> [N*D*s*D*s, C, ho, wo]: a strided pool run once per starting offset."""
    F, C, hi, wi = x.shape
    N = F // (D * D)
    if out is None:
        out = torch.empty((F * s * s, C, ho, wo), dtype=x.dtype, device=x.device)
    _check(lib.dsk_fs_pool_fwd(kind, _dev(x), _dev(out), N, D, C, hi, wi, k, s, ho, wo, _dtype_code(x), _stream()),
           "dsk_fs_pool_fwd")
    return out


def dsk_fs_conv_fwd(x, w, b, D, s, ho, wo, act=DSK_ACT_NONE, out=None):
    F, C, hi, wi = x.shape
    K, Cw, k, _ = w.shape
    assert Cw == C
    N = F // (D * D)
    if out is None:
        out = torch.empty((F * s * s, K, ho, wo), dtype=x.dtype, device=x.device)
    _check(lib.dsk_fs_conv_fwd(_dev(x), _dev(w, torch.float32), None if b is None else _dev(b, torch.float32), _dev(out),
                               N, D, C, hi, wi, K, k, s, ho, wo, act, _dtype_code(x), _stream()), "dsk_fs_conv_fwd")
    return out


def dsk_fs_assemble(frag, D, H, W, out=None, out_dtype=None):
    F, C, hf, wf = frag.shape
    N = F // (D * D)
    if out is None:
        out = torch.empty((N, C, H, W), dtype=out_dtype or frag.dtype, device=frag.device)
    _check(lib.dsk_fs_assemble(_dev(frag), _dev(out), N, D, C, hf, wf, H, W, _dtype_code(frag), _dtype_code(out),
                               _stream()), "dsk_fs_assemble")
    return out


# --------------------------------------------------------------------------- video (3-D) layers
# maps [N, T, C, H, W]; weights [kt, K, C, kh, kw]
def dsk_pad_video(x, tlo, thi, lo, hi, out_dtype=torch.float32, xpad=None):
    N, T, C, H, W = x.shape
    if xpad is None:
        xpad = torch.empty((N, T + tlo + thi, C, H + lo + hi, W + lo + hi), dtype=out_dtype, device=x.device)
    _check(lib.dsk_pad_video(_dev(x, torch.float32), _dev(xpad), N, T, C, H, W, tlo, thi, lo, hi, _dtype_code(xpad),
                             _stream()), "dsk_pad_video")
    return xpad


def dsk_conv3d_workspace_bytes(which, N, T, C, H, W, K, kt, kh, kw, dt, d, in_code):
    return int(lib.dsk_conv3d_workspace_bytes(which, N, T, C, H, W, K, kt, kh, kw, dt, d, in_code))


def _conv3d_ws(which, shape, in_code, ws, device):
    need = dsk_conv3d_workspace_bytes(which, *shape, in_code)
    if need and (ws is None or ws.numel() * ws.element_size() < need):
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws


def dsk_conv3d_fwd(x, w, b, dt, d, act=DSK_ACT_NONE, out_dtype=None, y=None, ws=None):
    N, T, C, H, W = x.shape
    kt, K, Cw, kh, kw = w.shape
    assert Cw == C
    if y is None:
        To, Ho, Wo = T - (kt - 1) * dt, H - (kh - 1) * d, W - (kw - 1) * d
        if To < 1 or Ho < 1 or Wo < 1:
            raise DskError(DSK_ESHAPE, "dsk_conv3d_fwd")
        y = torch.empty((N, To, K, Ho, Wo), dtype=out_dtype or x.dtype, device=x.device)
    shape = (N, T, C, H, W, K, kt, kh, kw, dt, d)
    ws = _conv3d_ws(DSK_WS_CONV_FWD, shape, _dtype_code(x), ws, x.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_conv3d_fwd(_dev(x), _dev(w, torch.float32), None if b is None else _dev(b, torch.float32), _dev(y),
                              *shape, _dtype_code(x), _dtype_code(y), act, wsp, wsb, _stream()), "dsk_conv3d_fwd")
    return y


def dsk_conv3d_bwd_data(dy, w, dt, d, T, H, W, out_dtype=None, dx=None, ws=None):
    N, To, K, Ho, Wo = dy.shape
    kt, Kw, C, kh, kw = w.shape
    assert Kw == K and To == T - (kt - 1) * dt and Ho == H - (kh - 1) * d and Wo == W - (kw - 1) * d
    if dx is None:
        dx = torch.empty((N, T, C, H, W), dtype=out_dtype or dy.dtype, device=dy.device)
    shape = (N, T, C, H, W, K, kt, kh, kw, dt, d)
    ws = _conv3d_ws(DSK_WS_CONV_BWD_DATA, shape, _dtype_code(dy), ws, dy.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_conv3d_bwd_data(_dev(dy), _dev(w, torch.float32), _dev(dx), *shape, _dtype_code(dy), _dtype_code(dx),
                                   wsp, wsb, _stream()), "dsk_conv3d_bwd_data")
    return dx


def dsk_conv3d_bwd_weight(x, dy, kt, kh, kw, dt, d, dw=None, db=None, want_db=True, ws=None):
    N, T, C, H, W = x.shape
    N2, To, K, Ho, Wo = dy.shape
    assert N2 == N and To == T - (kt - 1) * dt and Ho == H - (kh - 1) * d and Wo == W - (kw - 1) * d and x.dtype == dy.dtype
    if dw is None:
        dw = torch.empty((kt, K, C, kh, kw), dtype=torch.float32, device=x.device)
    if db is None and want_db:
        db = torch.empty((K,), dtype=torch.float32, device=x.device)
    shape = (N, T, C, H, W, K, kt, kh, kw, dt, d)
    ws = _conv3d_ws(DSK_WS_CONV_BWD_WEIGHT, shape, _dtype_code(x), ws, x.device)
    wsp, wsb = _ws(ws)
    _check(lib.dsk_conv3d_bwd_weight(_dev(x), _dev(dy), _dev(dw, torch.float32), None if db is None else _dev(db, torch.float32),
                                     *shape, _dtype_code(x), wsp, wsb, _stream()), "dsk_conv3d_bwd_weight")
    return dw, db


def _pool3d_out(x, kt, k, dt, d, where):
    N, T, C, H, W = x.shape
    To, Ho, Wo = T - (kt - 1) * dt, H - (k - 1) * d, W - (k - 1) * d
    if To < 1 or Ho < 1 or Wo < 1:
        raise DskError(DSK_ESHAPE, where)
    return (N, To, C, Ho, Wo)


def dsk_maxpool3d_fwd(x, kt, k, dt, d, y=None, argmax=None, want_argmax=True):
    N, T, C, H, W = x.shape
    shp = _pool3d_out(x, kt, k, dt, d, "dsk_maxpool3d_fwd")
    if y is None:
        y = torch.empty(shp, dtype=x.dtype, device=x.device)
    if argmax is None and want_argmax:
        argmax = torch.empty(shp, dtype=torch.uint8, device=x.device)
    _check(lib.dsk_maxpool3d_fwd(_dev(x), _dev(y), None if argmax is None else _dev(argmax, torch.uint8),
                                 N, T, C, H, W, kt, k, dt, d, _dtype_code(x), _stream()), "dsk_maxpool3d_fwd")
    return y, argmax


def dsk_maxpool3d_bwd(dy, argmax, kt, k, dt, d, T, H, W, dx=None):
    N, To, C, Ho, Wo = dy.shape
    assert To == T - (kt - 1) * dt and Ho == H - (k - 1) * d and Wo == W - (k - 1) * d and argmax.shape == dy.shape
    if dx is None:
        dx = torch.empty((N, T, C, H, W), dtype=dy.dtype, device=dy.device)
    _check(lib.dsk_maxpool3d_bwd(_dev(dy), _dev(argmax, torch.uint8), _dev(dx), N, T, C, H, W, kt, k, dt, d,
                                 _dtype_code(dy), _stream()), "dsk_maxpool3d_bwd")
    return dx


def dsk_avgpool3d_fwd(x, kt, k, dt, d, y=None):
    N, T, C, H, W = x.shape
    shp = _pool3d_out(x, kt, k, dt, d, "dsk_avgpool3d_fwd")
    if y is None:
        y = torch.empty(shp, dtype=x.dtype, device=x.device)
    _check(lib.dsk_avgpool3d_fwd(_dev(x), _dev(y), N, T, C, H, W, kt, k, dt, d, _dtype_code(x), _stream()),
           "dsk_avgpool3d_fwd")
    return y


def dsk_avgpool3d_bwd(dy, kt, k, dt, d, T, H, W, dx=None):
    N, To, C, Ho, Wo = dy.shape
    assert To == T - (kt - 1) * dt and Ho == H - (k - 1) * d and Wo == W - (k - 1) * d
    if dx is None:
        dx = torch.empty((N, T, C, H, W), dtype=dy.dtype, device=dy.device)
    _check(lib.dsk_avgpool3d_bwd(_dev(dy), _dev(dx), N, T, C, H, W, kt, k, dt, d, _dtype_code(dy), _stream()),
           "dsk_avgpool3d_bwd")
    return dx
