"""Pins of the CPU oracle against things other than itself (no GPU).

  * library special cases: torch CPU fp64 conv2d / max_pool2d / avg_pool2d and
    autograd on single patches and patch mini-batches;
  * hand-computed values and the max-pool tie rule;
  * the paper's exact-equivalence claim (abstract, Sec. 3.1, Sec. 4.3): an
    independent whole-image dilated implementation of Algorithm 1 must equal
    patch scanning at every pixel, forward and backward;
  * central finite differences of the masked loss;
  * closed forms of softmax cross-entropy; mask linearity; empty mask.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from workloads import Net, conv, maxpool, avgpool, make_params, CONFIGS
from workloads.nets import ACT_RELU, ACT_TANH, ACT_NONE, CONV, MAXPOOL, AVGPOOL

import dilated_ref

# the paper's worked example (Sec. 3.4): conv2, pool2/2, conv2, pool3/3, conv2; patch 15
EXAMPLE = Net("example15", 1, 15, (conv(1, 2), maxpool(2, 2), conv(1, 2), maxpool(3, 3), conv(1, 2)))
EXAMPLE_MC = Net("example15mc", 2, 15, (conv(3, 2, 1, ACT_TANH), maxpool(2, 2), conv(4, 2, 1, ACT_RELU),
                                        maxpool(3, 3), conv(5, 2)))
STRIDED = Net("s2", 2, 23, (conv(4, 3, 2, ACT_TANH), maxpool(3, 2), conv(5, 2, 1, ACT_RELU),
                            avgpool(2, 2), conv(3, 2)))
STRIDE3 = Net("s3", 2, 16, (conv(3, 4, 3, ACT_TANH), maxpool(2, 1), avgpool(2, 2), conv(4, 2)))
SMOOTH = Net("smooth", 2, 11, (conv(3, 3, 2, ACT_TANH), avgpool(2, 1), conv(4, 2, 1, ACT_TANH),
                               avgpool(3, 1), conv(3, 1)))
NETS = [EXAMPLE, EXAMPLE_MC, STRIDED, STRIDE3, SMOOTH, CONFIGS[0].net]


def _params(net, seed, bias_std=0.3):
    rng = np.random.default_rng(seed)
    ws, bs = make_params(net, rng, bias_std=bias_std)
    ws = [w.astype(np.float64) * 2.0 for w in ws]
    bs = [b.astype(np.float64) for b in bs]
    return ws, bs


def _torch_patch_forward(net, ws, bs, patches):
    """patches: torch fp64 [B, C0, n, n] -> list of maps (incl. input) and pool indices."""
    x = patches
    maps, idxs = [x], [None]
    wi = 0
    for L in net.layers:
        if L.kind == CONV:
            x = F.conv2d(x, ws[wi], bs[wi], stride=L.s)
            wi += 1
            if L.act == ACT_RELU:
                x = torch.relu(x)
            elif L.act == ACT_TANH:
                x = torch.tanh(x)
            idxs.append(None)
        elif L.kind == MAXPOOL:
            x, idx = F.max_pool2d(x, L.k, L.s, return_indices=True)
            idxs.append(idx)
        else:
            x = F.avg_pool2d(x, L.k, L.s)
            idxs.append(None)
        maps.append(x)
    return maps, idxs


@pytest.mark.parametrize("net", NETS, ids=lambda n: n.name)
def test_patch_forward_matches_torch_layers(net):
    ws, bs = _params(net, 3)
    rng = np.random.default_rng(4)
    patch = rng.uniform(-1, 1, (net.C0, net.patch, net.patch))
    maps, ams = oracle.patch_forward(net, oracle.pack_params(ws, bs), patch)
    tmaps, tidx = _torch_patch_forward(net, [torch.from_numpy(w) for w in ws],
                                       [torch.from_numpy(b) for b in bs],
                                       torch.from_numpy(patch)[None])
    assert [m.shape[1] for m in maps] == [net.patch] + net.patch_sizes()
    for l, (m, t) in enumerate(zip(maps, tmaps)):
        np.testing.assert_allclose(m, t[0].numpy(), rtol=1e-12, atol=1e-13, err_msg="map %d" % l)
    # winning tap index: torch reports the flat index inside the input plane
    for l, L in enumerate(net.layers):
        if L.kind != MAXPOOL:
            continue
        idx = tidx[l + 1][0].numpy()
        mi = maps[l].shape[1]
        C, mo, _ = idx.shape
        u = np.arange(mo)[None, :, None]
        v = np.arange(mo)[None, None, :]
        a = idx // mi - u * L.s
        b = idx % mi - v * L.s
        np.testing.assert_array_equal(ams[l + 1], a * L.k + b)


@pytest.mark.parametrize("net", NETS, ids=lambda n: n.name)
def test_scan_backward_matches_torch_autograd(net):
    ws, bs = _params(net, 5)
    rng = np.random.default_rng(6)
    N, H, W = 2, 5, 4
    img = rng.uniform(-1, 1, (N, net.C0, H, W))
    xpad = oracle.pad_image(img, net.patch)
    pix = np.array([(n, i, j) for n in range(N) for i in range(H) for j in range(W)], np.int32)
    pix = pix[rng.permutation(len(pix))[:17]]
    delta = rng.standard_normal((len(pix), net.classes))
    params = oracle.pack_params(ws, bs)
    dpar, dx = oracle.scan_backward(net, params, xpad, pix, delta, want_dx=True)
    scores = oracle.scan_forward(net, params, xpad, pix)

    tw = [torch.from_numpy(w).requires_grad_() for w in ws]
    tb = [torch.from_numpy(b).requires_grad_() for b in bs]
    txp = torch.from_numpy(xpad).requires_grad_()
    n = net.patch
    patches = torch.stack([txp[p[0], :, p[1]:p[1] + n, p[2]:p[2] + n] for p in pix])
    out = _torch_patch_forward(net, tw, tb, patches)[0][-1][:, :, 0, 0]
    np.testing.assert_allclose(scores, out.detach().numpy(), rtol=1e-11, atol=1e-12)
    (out * torch.from_numpy(delta)).sum().backward()
    dws, dbs = oracle.unpack_params(net, dpar)
    for i in range(len(ws)):
        np.testing.assert_allclose(dws[i], tw[i].grad.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dbs[i], tb[i].grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dx, txp.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_hand_values_conv_ones_and_delta():
    # all-ones image and weights: every output is C*k*k + b
    net = Net("ones", 3, 4, (conv(2, 4),))
    w = np.ones((2, 3, 4, 4))
    b = np.array([0.5, -2.0])
    img = np.ones((1, 3, 3, 3))
    # interior pixel (1,1) of a 3x3 image padded for n=4: pad 2 top/left, 1 bottom/right
    xpad = oracle.pad_image(img, 4)
    assert xpad.shape == (1, 3, 6, 6)
    s = oracle.scan_forward(net, oracle.pack_params([w], [b]), xpad, [(0, 1, 1)])
    # patch rows 1..4 of the padded image hold image rows -1..2 -> 3 rows inside, same for columns
    np.testing.assert_allclose(s[0], 3 * 3 * 3 + b)
    # a delta kernel picks exactly one input entry: tap (a, b) of channel c
    net1 = Net("delta", 2, 3, (conv(1, 3),))
    rng = np.random.default_rng(0)
    img = rng.uniform(-1, 1, (1, 2, 6, 7))
    xpad = oracle.pad_image(img, 3)
    for (c, a, bb) in [(0, 0, 0), (1, 2, 1), (0, 1, 2)]:
        w = np.zeros((1, 2, 3, 3))
        w[0, c, a, bb] = 1.0
        pix = [(0, i, j) for i in range(6) for j in range(7)]
        s = oracle.scan_forward(net1, oracle.pack_params([w], [np.zeros(1)]), xpad, pix)
        np.testing.assert_array_equal(s[:, 0].reshape(6, 7), xpad[0, c, a:a + 6, bb:bb + 7])


def test_hand_values_1x1_conv_is_per_pixel_matmul():
    net = Net("pw", 4, 1, (conv(3, 1),))
    rng = np.random.default_rng(1)
    w = rng.standard_normal((3, 4, 1, 1))
    b = rng.standard_normal(3)
    img = rng.uniform(-1, 1, (2, 4, 3, 5))
    pix = [(n, i, j) for n in range(2) for i in range(3) for j in range(5)]
    s = oracle.scan_forward(net, oracle.pack_params([w], [b]), oracle.pad_image(img, 1), pix)
    ref = np.einsum("kc,nchw->nhwk", w[:, :, 0, 0], img).reshape(-1, 3) + b
    np.testing.assert_allclose(s, ref, rtol=1e-13, atol=1e-14)


def test_hand_values_pool_ramp_constant_and_ties():
    net = Net("p", 1, 3, (maxpool(3, 3),))
    ramp = np.arange(9.0).reshape(1, 3, 3)
    maps, ams = oracle.patch_forward(net, np.zeros(0), ramp)
    assert maps[1][0, 0, 0] == 8.0 and ams[1][0, 0, 0] == 8          # last tap of a rising ramp
    maps, ams = oracle.patch_forward(net, np.zeros(0), np.full((1, 3, 3), 2.5))
    assert maps[1][0, 0, 0] == 2.5 and ams[1][0, 0, 0] == 0          # constant: lowest index wins
    t = np.array([[[0.0, 7.0, 1.0], [7.0, -1.0, 7.0], [2.0, 7.0, 0.0]]])
    maps, ams = oracle.patch_forward(net, np.zeros(0), t)
    assert maps[1][0, 0, 0] == 7.0 and ams[1][0, 0, 0] == 1          # first of several equal maxima
    z = np.array([[[-0.0, 0.0, 0.0], [0.0, 0.0, 0.0], [0.0, 0.0, 0.0]]])
    maps, ams = oracle.patch_forward(net, np.zeros(0), z)
    assert ams[1][0, 0, 0] == 0                                      # -0.0 == +0.0, first wins
    # average pool: mean of the window, stride respected
    neta = Net("a", 1, 4, (avgpool(2, 2),))
    maps, _ = oracle.patch_forward(neta, np.zeros(0), np.arange(16.0).reshape(1, 4, 4))
    np.testing.assert_allclose(maps[1][0], [[2.5, 4.5], [10.5, 12.5]])
    # max-pool backward routes the error to the recorded tap only
    net2 = Net("p2", 1, 2, (maxpool(2, 2),))
    img = np.array([[[[1.0, 5.0], [3.0, 2.0]]]])          # 2x2 image; patch of pixel (1,1) covers it all
    xpad = oracle.pad_image(img, 2)
    dpar, dx = oracle.scan_backward(net2, np.zeros(0), xpad, [(0, 1, 1)], [[2.0]], want_dx=True)
    expect = np.zeros_like(xpad)
    expect[0, 0, 1, 2] = 2.0                              # padded position of the value 5
    np.testing.assert_array_equal(dx, expect)


def test_padding_rule():
    img = np.arange(2 * 3 * 4, dtype=np.float64).reshape(1, 2, 3, 4) + 1
    for n in (1, 2, 5, 6):
        xp = oracle.pad_image(img, n)
        assert xp.shape == (1, 2, 3 + n - 1, 4 + n - 1)
        lo = n // 2
        np.testing.assert_array_equal(xp[:, :, lo:lo + 3, lo:lo + 4], img)
        assert xp.sum() == img.sum()
    # odd n: the paper's size h + 2*floor(n/2) (Sec. 3.3); the worked example pads 5x5 to 19x19 for n=15
    assert oracle.pad_image(np.zeros((1, 1, 5, 5)), 15).shape[-2:] == (19, 19)


@pytest.mark.parametrize("net", NETS, ids=lambda n: n.name)
def test_equivalence_with_whole_image_dilated_forward_backward(net):
    """Exact-equivalence claim: one stride-1 pass with d-regularly sparse kernels
    gives, at every pixel, the patch CNN's output, its per-layer intermediates at
    the positions (i + D*u, j + D*v) (Fig. 3), and -- with any error map -- the
    summed per-patch gradients."""
    ws, bs = _params(net, 11)
    rng = np.random.default_rng(12)
    H, W = (7, 6) if net.patch < 20 else (4, 5)
    img = rng.uniform(-1, 1, (1, net.C0, H, W))
    xpad = oracle.pad_image(img, net.patch)
    params = oracle.pack_params(ws, bs)
    pix = np.array([(0, i, j) for i in range(H) for j in range(W)], np.int32)
    scores = oracle.scan_forward(net, params, xpad, pix)
    maps, ams = dilated_ref.forward(net, ws, bs, xpad[0])
    assert maps[-1].shape == (net.classes, H, W)
    np.testing.assert_allclose(scores.T.reshape(net.classes, H, W), maps[-1], rtol=1e-11, atol=1e-12)

    # per-layer correspondence for three pixels
    D = np.cumprod([L.s for L in net.layers])
    for (i, j) in [(0, 0), (H - 1, W - 1), (H // 2, W // 3)]:
        pm, pam = oracle.patch_forward(net, params, xpad[0, :, i:i + net.patch, j:j + net.patch])
        for l in range(1, len(net.layers) + 1):
            m = pm[l].shape[1]
            sub = maps[l][:, i:i + D[l - 1] * m:D[l - 1], j:j + D[l - 1] * m:D[l - 1]]
            np.testing.assert_allclose(pm[l], sub, rtol=1e-11, atol=1e-12)
            if net.layers[l - 1].kind == MAXPOOL:
                suba = ams[l][:, i:i + D[l - 1] * m:D[l - 1], j:j + D[l - 1] * m:D[l - 1]]
                np.testing.assert_array_equal(pam[l], suba)

    # backward with a sparse (masked) error map and with a dense one
    for frac in (0.3, 1.0):
        keep = rng.random(len(pix)) < frac
        delta = rng.standard_normal((len(pix), net.classes)) * keep[:, None]
        dpar, dx = oracle.scan_backward(net, params, xpad, pix[keep], delta[keep], want_dx=True)
        dlast = delta.T.reshape(net.classes, H, W)
        dws, dbs, dx0 = dilated_ref.backward(net, ws, maps, ams, dlast)
        ows, obs = oracle.unpack_params(net, dpar)
        for i in range(len(ws)):
            np.testing.assert_allclose(ows[i], dws[i], rtol=1e-9, atol=1e-11)
            np.testing.assert_allclose(obs[i], dbs[i], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(dx[0], dx0, rtol=1e-9, atol=1e-11)


def test_finite_differences_of_masked_loss():
    net = SMOOTH                      # tanh + average pools: no kinks
    ws, bs = _params(net, 21)
    rng = np.random.default_rng(22)
    N, H, W = 2, 4, 3
    img = rng.uniform(-1, 1, (N, net.C0, H, W))
    labels = rng.integers(0, net.classes, (N, H, W))
    mask = (rng.random((N, H, W)) < 0.5).astype(np.uint8)
    mask[0, 0, 0] = 1
    xpad = oracle.pad_image(img, net.patch)
    allpix = np.array([(n, i, j) for n in range(N) for i in range(H) for j in range(W)], np.int32)

    def loss_of(params):
        s = oracle.scan_forward(net, params, xpad, allpix)
        smap = s.reshape(N, H, W, net.classes).transpose(0, 3, 1, 2)
        return oracle.masked_softmax_xent(smap, labels, mask)

    params = oracle.pack_params(ws, bs)
    loss, delta, count = loss_of(params)
    assert count == int(mask.sum())
    mpix = allpix[mask.ravel() != 0]
    dm = delta.transpose(0, 2, 3, 1).reshape(-1, net.classes)[mask.ravel() != 0]
    dpar, _ = oracle.scan_backward(net, params, xpad, mpix, dm)
    h = 1e-5
    idx = rng.permutation(params.size)[:60]
    for t in idx:
        p1, p2 = params.copy(), params.copy()
        p1[t] += h
        p2[t] -= h
        fd = (loss_of(p1)[0] - loss_of(p2)[0]) / (2 * h)
        assert abs(fd - dpar[t]) <= 1e-7 * max(1.0, abs(fd)), (t, fd, dpar[t])


def test_softmax_xent_closed_forms():
    N, Cls, H, W = 2, 7, 3, 4
    rng = np.random.default_rng(5)
    labels = rng.integers(0, Cls, (N, H, W))
    mask = (rng.random((N, H, W)) < 0.4).astype(np.uint8)
    mask[1, 2, 3] = 1
    M = int(mask.sum())
    # all-equal scores: loss = log(Cls), delta = (1/Cls - onehot)/|M| on masked pixels
    loss, delta, count = oracle.masked_softmax_xent(np.full((N, Cls, H, W), 3.25), labels, mask)
    assert count == M
    assert abs(loss - np.log(Cls)) < 1e-14
    onehot = np.eye(Cls)[labels].transpose(0, 3, 1, 2)
    np.testing.assert_allclose(delta, (1.0 / Cls - onehot) * mask[:, None] / M, atol=1e-15)
    # general scores: errors sum to zero over classes, unmasked pixels are exactly zero
    s = rng.standard_normal((N, Cls, H, W)) * 30
    loss, delta, _ = oracle.masked_softmax_xent(s, labels, mask)
    np.testing.assert_allclose(delta.sum(axis=1), 0.0, atol=1e-15)
    assert np.all(delta * (1 - mask[:, None]) == 0)
    ref = F.cross_entropy(torch.from_numpy(s).permute(0, 2, 3, 1)[torch.from_numpy(mask) != 0],
                          torch.from_numpy(labels)[torch.from_numpy(mask) != 0], reduction="mean")
    assert abs(loss - ref.item()) < 1e-12
    # a hugely confident correct prediction: loss -> 0, no overflow
    big = np.zeros((1, 3, 1, 1))
    big[0, 1] = 1e4
    loss, delta, _ = oracle.masked_softmax_xent(big, np.array([[[1]]]), np.ones((1, 1, 1)))
    assert loss == 0.0 and np.all(np.isfinite(delta))
    # empty mask
    loss, delta, count = oracle.masked_softmax_xent(s, labels, np.zeros((N, H, W)))
    assert loss == 0.0 and count == 0 and not delta.any()


def test_mask_linearity_and_empty_mask():
    net = CONFIGS[0].net
    ws, bs = _params(net, 31)
    rng = np.random.default_rng(32)
    img = rng.uniform(-1, 1, (1, 3, 6, 6))
    xpad = oracle.pad_image(img, net.patch)
    params = oracle.pack_params(ws, bs)
    pix = np.array([(0, i, j) for i in range(6) for j in range(6)], np.int32)
    delta = rng.standard_normal((36, net.classes))
    a, b = np.arange(36) % 3 == 0, np.arange(36) % 3 == 1
    ga, _ = oracle.scan_backward(net, params, xpad, pix[a], delta[a])
    gb, _ = oracle.scan_backward(net, params, xpad, pix[b], delta[b])
    gab, _ = oracle.scan_backward(net, params, xpad, pix[a | b], delta[a | b])
    np.testing.assert_allclose(gab, ga + gb, rtol=1e-10, atol=1e-13)
    g0, dx0 = oracle.scan_backward(net, params, xpad, pix[:0], delta[:0], want_dx=True)
    assert not g0.any() and not dx0.any()


def test_patch_geometry_of_paper_models():
    """Patch sizes implied by the padded sizes the paper prints (Sec. 5.1): Plain CNN_1 pads
    256 to 388 (patch 133), and its layers (Table 1) reduce a 133 patch to 1x1."""
    plain = Net("plaincnn1", 3, 133, (conv(50, 6), maxpool(8, 8), conv(50, 3), maxpool(2, 2), conv(32, 7)))
    g = oracle.geometry(plain)
    assert list(g["m"]) == [133, 128, 16, 14, 7, 1]
    assert 256 + 133 - 1 == 388
    g = oracle.geometry(EXAMPLE)
    assert list(g["m"]) == [15, 14, 7, 6, 2, 1]        # Fig. 3 (c2)-(f2)


# ---------------------------------------------------------------------------
# The bf16-storage mode, the pre-activation output and the all-maps scan: options of the
# oracle that the end-to-end GPU checks rely on, pinned here to torch's bfloat16 conversion,
# to hand-rounded values and to the plain scan.
# ---------------------------------------------------------------------------
def _torch_bf16(a):
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


def test_bf16_storage_rounds_like_torch_and_ties_to_even():
    net = Net("id", 1, 8, (conv(1, 8),))          # map 0 (the patch) is what gets rounded
    e = 2.0 ** -8                                   # half a bf16 step at 1.0 (8 significant bits)
    hand = [
        (1.0 + e, 1.0),                  # exact tie, kept mantissa even -> down
        (1.0 + 3 * e, 1.0 + 4 * e),      # exact tie, kept mantissa odd -> up to the even one
        (1.0 + 5 * e, 1.0 + 4 * e),      # exact tie -> down to the even one
        (1.0 + e + 2.0 ** -20, 1.0 + 2 * e),   # just above a tie -> up
        (1.0 + e - 2.0 ** -20, 1.0),           # just below a tie -> down
        (-1.0 - 3 * e, -1.0 - 4 * e),    # sign does not matter
        (-1.0 - e, -1.0),
        (3.0 + 3.0 / 128, 3.03125),      # 11.0000011b: tie, odd -> 11.000010b
        (0.0, 0.0), (255.0, 255.0), (257.0, 256.0), (259.0, 260.0),
        (2.0 ** -126, 2.0 ** -126), (1e-3, float(_torch_bf16([1e-3])[0])),
    ]
    rng = np.random.default_rng(0)
    vals = [h[0] for h in hand]
    vals += list(rng.standard_normal(64 - len(vals)).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 64 - len(vals)))
    patch = np.asarray(vals, np.float64).reshape(1, 8, 8)
    maps, _ = oracle.patch_forward(net, np.zeros(65), patch, storage=oracle.STORE_BF16)
    got = maps[0].ravel()
    for t, (v, want) in enumerate(hand):
        assert got[t] == want, (v, got[t], want)
    np.testing.assert_array_equal(got, _torch_bf16(patch).ravel())
    # truncation instead of nearest-even would fail here
    assert got[1] != np.float64(np.float32(1.0 + 2 * e)) and got[3] == 1.0 + 2 * e
    # exact mode leaves the patch alone
    maps, _ = oracle.patch_forward(net, np.zeros(65), patch)
    np.testing.assert_array_equal(maps[0], patch)


def test_bf16_storage_rounds_every_map_but_the_last():
    """Three 1x1 layers on a 1x1 patch: every value is known by hand.
    patch 1 + 2^-8 + 2^-20 -> stored 1 + 2^-7; layer 1 (w = 3): 3 + 3/128 is a tie, stored
    3.03125; layer 2 (w = 0.5, ReLU): 1.515625 = 1.1000010b is representable; the last layer
    (w = 0.3) is not rounded."""
    net = Net("chain", 1, 1, (conv(1, 1), conv(1, 1, 1, ACT_RELU), conv(1, 1)))
    params = oracle.pack_params([np.full((1, 1, 1, 1), 3.0), np.full((1, 1, 1, 1), 0.5), np.full((1, 1, 1, 1), 0.3)],
                                [np.zeros(1), np.zeros(1), np.zeros(1)])
    x = 1.0 + 2.0 ** -8 + 2.0 ** -20
    maps, _ = oracle.patch_forward(net, params, np.full((1, 1, 1), x), storage=oracle.STORE_BF16)
    assert maps[0].item() == 1.0 + 2.0 ** -7
    assert maps[1].item() == 3.03125
    assert maps[2].item() == 1.515625
    assert maps[3].item() == 0.3 * 1.515625
    exact, _ = oracle.patch_forward(net, params, np.full((1, 1, 1), x))
    assert exact[3].item() == 0.3 * (0.5 * (3.0 * x))
    # the scans use the same storage rule: scores and the gradient of the stored chain
    xpad = np.full((1, 1, 1, 1), x)
    s = oracle.scan_forward(net, params, xpad, [(0, 0, 0)], storage=oracle.STORE_BF16)
    assert s.item() == 0.3 * 1.515625
    g, dx = oracle.scan_backward(net, params, xpad, [(0, 0, 0)], [[1.0]], want_dx=True, storage=oracle.STORE_BF16)
    dws, dbs = oracle.unpack_params(net, g)
    # d out / d w3 = stored map 2; d out / d w2 = 0.3 * stored map 1; d out / d w1 = 0.3 * 0.5 * stored patch
    assert dws[2].item() == 1.515625 and dws[1].item() == 0.3 * 3.03125
    np.testing.assert_allclose(dws[0].item(), 0.3 * 0.5 * (1.0 + 2.0 ** -7), rtol=1e-15)


def test_bf16_storage_decides_gates_and_winners_on_stored_values():
    # a pool window whose largest value rounds down onto its neighbour: a tie in storage precision, lowest index wins
    net = Net("p", 1, 2, (maxpool(2, 2),))
    w = np.array([[[1.0, 1.0 + 2.0 ** -9], [0.5, 0.25]]])
    _, ams = oracle.patch_forward(net, np.zeros(0), w)
    assert ams[1].item() == 1
    maps, ams = oracle.patch_forward(net, np.zeros(0), w, storage=oracle.STORE_BF16)
    assert ams[1].item() == 0 and maps[1].item() == 1.0
    # against torch on a random network: layer by layer with torch's own bfloat16 conversions
    net = EXAMPLE_MC
    ws, bs = _params(net, 41)
    ws = [_torch_bf16(w) for w in ws]
    rng = np.random.default_rng(42)
    patch = rng.uniform(-1, 1, (net.C0, net.patch, net.patch))
    maps, ams = oracle.patch_forward(net, oracle.pack_params(ws, bs), patch, storage=oracle.STORE_BF16)
    x = torch.from_numpy(_torch_bf16(patch))[None]
    wi = 0
    for l, L in enumerate(net.layers):
        if L.kind == CONV:
            x = F.conv2d(x, torch.from_numpy(ws[wi]), torch.from_numpy(bs[wi]), stride=L.s)
            wi += 1
            x = torch.relu(x) if L.act == ACT_RELU else torch.tanh(x) if L.act == ACT_TANH else x
        elif L.kind == MAXPOOL:
            x = F.max_pool2d(x, L.k, L.s)
        else:
            x = F.avg_pool2d(x, L.k, L.s)
        if l + 1 < len(net.layers):
            # fp64 -> fp32 -> bf16 as the oracle does (a value within 1e-12 of a rounding boundary could differ; none here)
            x = x.to(torch.float32).to(torch.bfloat16).to(torch.float64)
        np.testing.assert_allclose(maps[l + 1], x[0].numpy(), rtol=1e-12, atol=1e-13, err_msg="map %d" % (l + 1))


@pytest.mark.parametrize("net", NETS, ids=lambda n: n.name)
def test_pre_activation_output_and_all_maps_scan(net):
    ws, bs = _params(net, 51)
    rng = np.random.default_rng(52)
    N, H, W = 2, 4, 5
    img = rng.uniform(-1, 1, (N, net.C0, H, W))
    xpad = oracle.pad_image(img, net.patch)
    params = oracle.pack_params(ws, bs)
    pix = np.array([(1, 3, 4), (0, 0, 0), (1, 2, 1), (0, 3, 2), (0, 1, 4)], np.int32)
    maps, ams, pre = oracle.scan_forward_maps(net, params, xpad, pix)
    np.testing.assert_array_equal(maps[-1][:, :, 0, 0], oracle.scan_forward(net, params, xpad, pix))
    n = net.patch
    tw, tb = [torch.from_numpy(w) for w in ws], [torch.from_numpy(b) for b in bs]
    for t, (im, i, j) in enumerate(pix):
        pm, pam, ppre = oracle.patch_forward(net, params, xpad[im, :, i:i + n, j:j + n], want_pre=True)
        x = torch.from_numpy(xpad[im, :, i:i + n, j:j + n])[None]
        wi = 0
        for l, L in enumerate(net.layers):
            np.testing.assert_array_equal(maps[l + 1][t], pm[l + 1])
            np.testing.assert_array_equal(ams[l + 1][t], pam[l + 1])
            np.testing.assert_array_equal(pre[l + 1][t], ppre[l + 1])
            if L.kind == CONV:
                # pinned to torch: the convolution WITHOUT its non-linearity, computed on the oracle's own input map
                z = F.conv2d(torch.from_numpy(pm[l])[None], tw[wi], tb[wi], stride=L.s)[0].numpy()
                wi += 1
                np.testing.assert_allclose(ppre[l + 1], z, rtol=1e-12, atol=1e-13)
                want = np.maximum(z, 0) if L.act == ACT_RELU else np.tanh(z) if L.act == ACT_TANH else z
                np.testing.assert_allclose(pm[l + 1], want, rtol=1e-12, atol=1e-13)
                assert np.array_equal(pm[l + 1] > 0, ppre[l + 1] > 0) or L.act != ACT_RELU
                assert (pam[l + 1] == -1).all()
            else:
                assert not ppre[l + 1].any()
                assert ((pam[l + 1] >= 0).all() and (pam[l + 1] < L.k * L.k).all()) if L.kind == MAXPOOL else (pam[l + 1] == -1).all()
