"""Host-side logic of libdsk, no GPU: the library loads and exports every symbol
the header declares, Algorithm 1's planner reproduces the geometry the paper
prints, and every argument error is reported before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_1412_4526_amd as dsk
from workloads import Net, conv, maxpool, avgpool, CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _golden():
    out = {}
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_geometry.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = [int(t) for t in v.split()]
    return out


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dsk.h")).read()
    declared = set(re.findall(r"\b(dsk_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(dsk.SYMBOLS)
    raw = ctypes.CDLL(dsk.LIB_PATH)
    for name in declared:
        assert getattr(raw, name) is not None


def test_plan_reproduces_paper_example():
    g = _golden()
    net = Net("example", 1, 15, (conv(1, 2), maxpool(2, 2), conv(1, 2), maxpool(3, 3), conv(1, 2)))
    plan, rf, lo, hi = dsk.dsk_plan(net.layers, 1, g["example_image"][0], g["example_image"][0], 0)
    assert rf == g["example_patch"][0]
    assert g["example_image"][0] + lo + hi == g["example_padded"][0]
    assert [p.d for p in plan] == g["example_spacings"]
    sizes = [plan[0].H] + [p.Ho for p in plan]
    assert sizes == g["example_whole_image_sizes"]
    assert all(p.H == p.W and p.Ho == p.Wo for p in plan)
    assert net.patch_sizes() == g["example_patch_sizes"][1:]


def test_plan_reproduces_padded_sizes_of_paper_models():
    g = _golden()
    out = g["plaincnn1_output"][0]
    # Plain CNN_1 (Table 1): conv 6x6, pool 8x8/8, conv 3x3, pool 2x2 (/2), conv 7x7
    plain = (conv(50, 6), maxpool(8, 8), conv(50, 3), maxpool(2, 2), conv(32, 7))
    plan, rf, lo, hi = dsk.dsk_plan(plain, 3, out, out, 0)
    assert out + lo + hi == g["plaincnn1_padded"][0] and rf == 133
    assert [p.d for p in plan] == [1, 1, 8, 8, 16]
    # RCNN_3 (Table 2): three instances of conv 8x8, pool 2/2, conv 8x8, conv 1x1 chained
    inst = (conv(25, 8), maxpool(2, 2), conv(50, 8), conv(32, 1))
    plan, rf, lo, hi = dsk.dsk_plan(inst * 3, 3, out, out, 0)
    assert out + lo + hi == g["rcnn3_padded"][0] and rf == 155
    assert [p.d for p in plan] == [1, 1, 2, 2, 2, 2, 4, 4, 4, 4, 8, 8]


def test_plan_of_the_five_benchmark_networks():
    expect_d = {0: [1, 1, 2, 2, 4], 1: [1, 1, 2, 2, 4, 4, 8, 8], 3: [1, 1, 2, 2, 4, 4, 8, 8, 16, 16],
                4: [1, 2, 4, 4, 8, 8], 5: [1, 1, 8, 8, 16], 6: [1, 1, 4, 4, 8], 7: [1, 1, 2, 2, 4]}      # Algorithm 1; the strided net has receptive field 67
    for i, c in enumerate(CONFIGS):
        plan, rf, lo, hi = dsk.dsk_plan(c.net.layers, c.net.C0, c.H, c.W, c.net.patch)
        assert rf == c.net.patch and lo == c.net.patch // 2 and lo + hi == c.net.patch - 1
        assert (plan[-1].Ho, plan[-1].Wo, plan[-1].K) == (c.H, c.W, c.net.classes)
        if i in expect_d:
            assert [p.d for p in plan] == expect_d[i]
        for a, b in zip(plan[:-1], plan[1:]):
            assert (a.Ho, a.Wo, a.K) == (b.H, b.W, b.C)


def test_plan_uneven_strides_and_errors():
    # 8 -> pool 3/2 -> floor((8-3)/2)+1 = 3 (last row/col of the patch unused) -> conv 3 -> 1
    layers = (maxpool(3, 2), conv(2, 3))
    plan, rf, lo, hi = dsk.dsk_plan(layers, 1, 6, 6, 8)
    assert rf == 7 and lo == 4 and hi == 2 and plan[-1].Ho == 6
    with pytest.raises(dsk.DskError) as e:
        dsk.dsk_plan(layers, 1, 6, 6, 5)           # declared patch smaller than the receptive field
    assert e.value.status == dsk.DSK_ESHAPE
    with pytest.raises(dsk.DskError) as e:
        dsk.dsk_plan((maxpool(16, 16),), 1, 6, 6, 0)   # k*k > 255
    assert e.value.status == dsk.DSK_ESHAPE
    for bad in [(conv(0, 3),), (conv(2, 0),), (Net("x", 1, 1, ()).layers)]:
        with pytest.raises(dsk.DskError) as e:
            dsk.dsk_plan(bad, 1, 6, 6, 0)
        assert e.value.status == dsk.DSK_EINVAL


# ---- argument validation happens before any launch, so it is testable without a GPU.
# 0x1000 stands in for a 16-byte aligned device pointer that is never dereferenced.
P = 0x1000


def test_conv_argument_errors():
    L = dsk.lib
    ok_dims = (1, 3, 16, 16, 4, 3, 3, 2)
    f = lambda *a: L.dsk_conv_fwd(*a)
    assert f(None, P, P, P, *ok_dims, 0, 0, 0, None, 0, None) == dsk.DSK_EINVAL
    assert f(P, P, P, P + 4, *ok_dims, 0, 0, 0, None, 0, None) == dsk.DSK_EINVAL          # misaligned
    assert f(P, P, P, P, 1, 3, 16, 16, 4, 3, 3, 0, 0, 0, 0, None, 0, None) == dsk.DSK_EINVAL  # d < 1
    assert f(P, P, P, P, 0, 3, 16, 16, 4, 3, 3, 1, 0, 0, 0, None, 0, None) == dsk.DSK_EINVAL
    assert f(P, P, P, P, *ok_dims, 7, 0, 0, None, 0, None) == dsk.DSK_EINVAL              # bad dtype
    assert f(P, P, P, P, *ok_dims, 0, 0, 9, None, 0, None) == dsk.DSK_EINVAL              # bad act
    assert f(P, P, P, P, 1, 3, 16, 16, 4, 3, 3, 8, 0, 0, 0, None, 0, None) == dsk.DSK_ESHAPE  # 16-2*8 = 0
    assert f(P, P, P, P, 1, 3, 4, 40, 4, 3, 3, 2, 0, 0, 0, None, 0, None) == dsk.DSK_ESHAPE
    assert f(P, P, P, P, 64, 64, 1024, 1024, 4, 1, 1, 1, 0, 0, 0, None, 0, None) == dsk.DSK_ESHAPE  # 2^32 elems
    g = lambda *a: L.dsk_conv_bwd_data(*a)
    assert g(P, None, P, *ok_dims, 0, 0, None, 0, None) == dsk.DSK_EINVAL
    assert g(P, P, P, 1, 3, 16, 16, 4, 9, 3, 2, 0, 0, None, 0, None) == dsk.DSK_ESHAPE
    h = lambda *a: L.dsk_conv_bwd_weight(*a)
    assert h(P, P, None, P, *ok_dims, 0, None, 0, None) == dsk.DSK_EINVAL
    assert h(P, P, P, P, 1, 3, 16, 16, 4, 3, 3, -1, 0, None, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_conv_workspace_bytes(0, 1, 3, 16, 16, 4, 3, 3, 8, 0) == 0               # invalid -> 0


def test_conv_workspace_errors():
    L = dsk.lib
    big = (1, 64, 128, 128, 64, 3, 3, 2)
    for which, call in ((0, lambda ws, n: L.dsk_conv_fwd(P, P, P, P, *big, 0, 0, 0, ws, n, None)),
                        (1, lambda ws, n: L.dsk_conv_bwd_data(P, P, P, *big, 0, 0, ws, n, None)),
                        (2, lambda ws, n: L.dsk_conv_bwd_weight(P, P, P, P, *big, 0, ws, n, None))):
        need = L.dsk_conv_workspace_bytes(which, *big, 0)
        if need:
            assert call(None, 0) == dsk.DSK_EWORKSPACE
            assert call(P, need - 1) == dsk.DSK_EWORKSPACE


def test_pool_act_loss_argument_errors():
    L = dsk.lib
    assert L.dsk_maxpool_fwd(None, P, P, 1, 2, 8, 8, 2, 1, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_maxpool_fwd(P, P, P, 1, 2, 8, 8, 2, 0, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_maxpool_fwd(P, P, P, 1, 2, 8, 8, 2, 8, 0, None) == dsk.DSK_ESHAPE       # 8-1*8 = 0
    assert L.dsk_maxpool_fwd(P, P, P, 1, 2, 80, 80, 16, 1, 0, None) == dsk.DSK_ESHAPE    # 256 taps
    assert L.dsk_maxpool_bwd(P, None, P, 1, 2, 8, 8, 2, 1, 0, None) == dsk.DSK_EINVAL    # argmax required
    assert L.dsk_avgpool_fwd(P, P + 2, 1, 2, 8, 8, 2, 1, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_avgpool_bwd(P, P, 1, 2, 8, 8, 2, 1, 5, None) == dsk.DSK_EINVAL
    assert L.dsk_act_bwd(P, None, 10, 1, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_act_bwd(P, P, 10, 4, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_pad_image(P, P, 1, 3, 8, 8, -1, 0, 0, None) == dsk.DSK_EINVAL
    nb = L.dsk_act_bwd_bias_workspace_bytes(7)
    assert nb > 0
    assert L.dsk_act_bwd_bias(P, P, P, 1, 7, 8, 8, 1, 0, None, 0, None) == dsk.DSK_EWORKSPACE
    assert L.dsk_act_bwd_bias(None, P, P, 1, 7, 8, 8, 1, 0, P, nb, None) == dsk.DSK_EINVAL   # y needed for ReLU
    assert L.dsk_act_bwd_bias(P, P, None, 1, 7, 8, 8, 0, 0, P, nb, None) == dsk.DSK_EINVAL
    # backward-data with the backward of the conv layer below: 1 x 1 (one pass) and 3 x 3 (two passes)
    for dims in ((1, 40, 16, 16, 7, 1, 1, 1), (1, 3, 16, 16, 4, 3, 3, 2)):
        nw = L.dsk_conv_bwd_data_act_bias_workspace_bytes(*dims, 0, 0)
        assert nw >= max(L.dsk_conv_workspace_bytes(1, *dims, 0), L.dsk_act_bwd_bias_workspace_bytes(dims[1])) > 0
        q = lambda *a: L.dsk_conv_bwd_data_act_bias(*a)
        assert q(P, P, P, P, P, *dims, 0, 0, 1, None, 0, None) == dsk.DSK_EWORKSPACE
        assert q(P, P, P, P, P, *dims, 0, 0, 1, P, nw - 1, None) == dsk.DSK_EWORKSPACE
        assert q(P, P, None, P, P, *dims, 0, 0, 1, P, nw, None) == dsk.DSK_EINVAL        # x needed for ReLU
        assert q(P, P, P, P, None, *dims, 0, 0, 0, P, nw, None) == dsk.DSK_EINVAL        # db required
        assert q(P, P, P, P, P, *dims, 0, 0, 5, P, nw, None) == dsk.DSK_EINVAL           # bad act
        assert q(P, P, P, P, P, *dims, 0, 3, 1, P, nw, None) == dsk.DSK_EINVAL           # bad dtype
    assert L.dsk_conv_bwd_data_act_bias(P, P, P, P, P, 1, 3, 16, 16, 4, 9, 3, 2, 0, 0, 1, P, 1 << 20, None) == dsk.DSK_ESHAPE
    assert L.dsk_conv_bwd_data_act_bias_workspace_bytes(1, 3, 16, 16, 4, 3, 3, 8, 0, 0) == 0      # invalid -> 0
    need = L.dsk_softmax_xent_workspace_bytes(1, 5, 8, 8)
    assert need > 0
    assert L.dsk_masked_softmax_xent(P, P, P, P, P, 0, 1, 5, 8, 8, None, 0, None) == dsk.DSK_EWORKSPACE
    assert L.dsk_masked_softmax_xent(P, P, P, P, P, 0, 1, 5, 8, 8, P, need - 1, None) == dsk.DSK_EWORKSPACE
    assert L.dsk_masked_softmax_xent(P, P, None, P, P, 0, 1, 5, 8, 8, P, need, None) == dsk.DSK_EINVAL
    assert L.dsk_masked_softmax_xent(P, P, P, P, P, 0, 1, 0, 8, 8, P, need, None) == dsk.DSK_EINVAL
    assert "DSK_EWORKSPACE" in dsk.status_string(dsk.DSK_EWORKSPACE)
    assert dsk.status_string(0) == "DSK_OK"


def test_video_argument_errors():
    L = dsk.lib
    ok = (1, 6, 4, 16, 16, 8, 2, 3, 3, 2, 2)        # N T C H W K kt kh kw dt d
    f = lambda *a: L.dsk_conv3d_fwd(*a)
    assert f(None, P, P, P, *ok, 0, 0, 0, None, 0, None) == dsk.DSK_EINVAL
    assert f(P, P, P + 8, P, *ok, 0, 0, 0, None, 0, None) == dsk.DSK_EINVAL                       # misaligned bias
    assert f(P, P, P, P, 1, 6, 4, 16, 16, 8, 2, 3, 3, 0, 2, 0, 0, 0, None, 0, None) == dsk.DSK_EINVAL   # dt < 1
    assert f(P, P, P, P, 1, 6, 4, 16, 16, 8, 4, 3, 3, 2, 2, 0, 0, 0, None, 0, None) == dsk.DSK_ESHAPE   # 6-3*2 = 0 frames
    assert f(P, P, P, P, 1, 6, 4, 16, 16, 8, 2, 9, 3, 2, 2, 0, 0, 0, None, 0, None) == dsk.DSK_ESHAPE
    assert f(P, P, P, P, *ok, 0, 3, 0, None, 0, None) == dsk.DSK_EINVAL                          # bad dtype
    assert L.dsk_conv3d_bwd_data(P, None, P, *ok, 0, 0, None, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_conv3d_bwd_weight(P, P, None, P, *ok, 0, None, 0, None) == dsk.DSK_EINVAL
    big = (1, 8, 64, 64, 64, 64, 3, 3, 3, 2, 2)
    for which, call in ((0, lambda ws, n: L.dsk_conv3d_fwd(P, P, P, P, *big, 0, 0, 0, ws, n, None)),
                        (1, lambda ws, n: L.dsk_conv3d_bwd_data(P, P, P, *big, 0, 0, ws, n, None)),
                        (2, lambda ws, n: L.dsk_conv3d_bwd_weight(P, P, P, P, *big, 0, ws, n, None))):
        need = L.dsk_conv3d_workspace_bytes(which, *big, 0)
        assert need > 0
        assert call(None, 0) == dsk.DSK_EWORKSPACE
        assert call(P, need - 1) == dsk.DSK_EWORKSPACE
    assert L.dsk_conv3d_workspace_bytes(0, 1, 2, 4, 16, 16, 8, 3, 3, 3, 1, 1, 0) == 0             # invalid -> 0
    pool = (1, 4, 2, 8, 8)
    assert L.dsk_maxpool3d_fwd(None, P, P, *pool, 2, 2, 1, 1, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_maxpool3d_fwd(P, P, P, *pool, 2, 2, 4, 1, 0, None) == dsk.DSK_ESHAPE              # 4-1*4 = 0 frames
    assert L.dsk_maxpool3d_fwd(P, P, P, *pool, 4, 8, 1, 1, 0, None) == dsk.DSK_ESHAPE              # 256 taps
    assert L.dsk_maxpool3d_bwd(P, None, P, *pool, 2, 2, 1, 1, 0, None) == dsk.DSK_EINVAL           # argmax required
    assert L.dsk_avgpool3d_fwd(P, P, *pool, 2, 2, 1, 0, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_avgpool3d_bwd(P, P + 4, *pool, 2, 2, 1, 1, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_pad_video(P, P, 1, 4, 3, 8, 8, -1, 0, 0, 0, 0, None) == dsk.DSK_EINVAL
    assert L.dsk_pad_video(P, None, 1, 4, 3, 8, 8, 1, 1, 2, 2, 0, None) == dsk.DSK_EINVAL


def test_product_does_not_touch_the_oracle():
    """The HIP path and the oracle share no code: nothing under the package mentions it."""
    pkg = os.path.join(ROOT, "paper_1412_4526_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() and "patchscan" not in text, f
