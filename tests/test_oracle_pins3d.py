"""Pins of the video (3-D) oracle against things other than itself (no GPU).

  * library special cases: torch CPU fp64 conv3d / max_pool3d / avg_pool3d layer by layer
    (values and winners) and autograd (parameter and input gradients) on mini-batches of cubes;
  * hand-computed values that tell the temporal axis from the spatial ones: one-hot kernels
    that pick a shifted voxel, window counts, ramps and the tie rule of max pooling;
  * a network without temporal extent (kt = 1) must give, frame by frame, what the 2-D oracle
    gives (itself pinned in test_oracle_pins.py);
  * central finite differences through the scan; the padding rule.
"""
import numpy as np
import torch
import torch.nn.functional as F

import oracle
from workloads import (VideoNet, conv3, maxpool3, avgpool3, make_video_params, TINY_VIDEO, STRIDED_VIDEO,
                       Net, conv, maxpool)
from workloads.nets import ACT_RELU, ACT_TANH, CONV, MAXPOOL

NETS = [TINY_VIDEO, STRIDED_VIDEO]


def _params(net, seed, bias_std=0.3):
    rng = np.random.default_rng(seed)
    ws, bs = make_video_params(net, rng, bias_std=bias_std)
    return [w.astype(np.float64) * 2.0 for w in ws], [b.astype(np.float64) for b in bs]


def _torch_forward(net, ws, bs, cubes):
    """cubes: torch fp64 [B, C0, nt, n, n] -> maps (incl. input) and pool winner tap indices."""
    x = cubes
    maps, taps = [x], [None]
    wi = 0
    for L in net.layers:
        if L.kind == CONV:
            x = F.conv3d(x, ws[wi], bs[wi], stride=(L.st, L.s, L.s))
            wi += 1
            x = torch.relu(x) if L.act == ACT_RELU else torch.tanh(x) if L.act == ACT_TANH else x
            taps.append(None)
        elif L.kind == MAXPOOL:
            xin = x
            x, idx = F.max_pool3d(xin, (L.kt, L.k, L.k), (L.st, L.s, L.s), return_indices=True)
            # flat index into the input volume -> tap index (e*k + a)*k + b within the window
            Ti, Hi, Wi = xin.shape[2:]
            it, ih, iw = idx // (Hi * Wi), (idx // Wi) % Hi, idx % Wi
            q = torch.arange(x.shape[2]).view(1, 1, -1, 1, 1) * L.st
            u = torch.arange(x.shape[3]).view(1, 1, 1, -1, 1) * L.s
            v = torch.arange(x.shape[4]).view(1, 1, 1, 1, -1) * L.s
            taps.append(((it - q) * L.k + (ih - u)) * L.k + (iw - v))
        else:
            x = F.avg_pool3d(x, (L.kt, L.k, L.k), (L.st, L.s, L.s))
            taps.append(None)
        maps.append(x)
    return maps, taps


def _video(net, N, T, H, W, seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(-1, 1, size=(N, net.C0, T, H, W))


def _all_voxels(N, T, H, W):
    g = np.stack(np.meshgrid(np.arange(N), np.arange(T), np.arange(H), np.arange(W), indexing="ij"), -1)
    return g.reshape(-1, 4).astype(np.int32)


def _crop(xpad, net, vox):
    return np.stack([xpad[v[0], :, v[1]:v[1] + net.patch_t, v[2]:v[2] + net.patch, v[3]:v[3] + net.patch] for v in vox])


def test_every_layer_matches_torch_conv3d_and_pool3d():
    for si, net in enumerate(NETS):
        ws, bs = _params(net, 10 + si)
        params = oracle.pack_params3d(ws, bs)
        xpad = oracle.pad_video(_video(net, 2, 3, 4, 5, 20 + si), net.patch_t, net.patch)
        vox = _all_voxels(2, 3, 4, 5)[::7]
        maps, amax = oracle.cube_forward_maps(net, params, xpad, vox)
        tm, tt = _torch_forward(net, [torch.from_numpy(w) for w in ws], [torch.from_numpy(b) for b in bs],
                                torch.from_numpy(_crop(xpad, net, vox)))
        for l in range(len(net.layers) + 1):
            assert maps[l].shape == tuple(tm[l].shape)
            np.testing.assert_allclose(maps[l], tm[l].numpy(), rtol=1e-12, atol=1e-13)
            if tt[l] is not None:
                assert np.array_equal(amax[l], tt[l].numpy())
            else:
                assert (amax[l] == -1).all()
        scores = oracle.cube_scan_forward(net, params, xpad, vox)
        np.testing.assert_allclose(scores, tm[-1].numpy().reshape(len(vox), -1), rtol=1e-12, atol=1e-13)


def test_backward_matches_autograd():
    for si, net in enumerate(NETS):
        ws, bs = _params(net, 30 + si)
        params = oracle.pack_params3d(ws, bs)
        xpad = oracle.pad_video(_video(net, 1, 3, 4, 4, 40 + si), net.patch_t, net.patch)
        vox = _all_voxels(1, 3, 4, 4)[::5]
        rng = np.random.default_rng(50 + si)
        g = oracle.geometry3d(net)
        delta = rng.standard_normal((len(vox), g["classes"]))
        dpar, dx = oracle.cube_scan_backward(net, params, xpad, vox, delta, want_dx=True)
        tw = [torch.from_numpy(w).requires_grad_() for w in ws]
        tb = [torch.from_numpy(b).requires_grad_() for b in bs]
        txp = torch.from_numpy(xpad).requires_grad_()
        cubes = torch.stack([txp[v[0], :, v[1]:v[1] + net.patch_t, v[2]:v[2] + net.patch, v[3]:v[3] + net.patch]
                             for v in vox])
        out = _torch_forward(net, tw, tb, cubes)[0][-1].reshape(len(vox), -1)
        (out * torch.from_numpy(delta)).sum().backward()
        dws, dbs = oracle.unpack_params3d(net, dpar)
        for a, b in zip(dws, tw):
            np.testing.assert_allclose(a, b.grad.numpy(), rtol=1e-10, atol=1e-12)
        for a, b in zip(dbs, tb):
            np.testing.assert_allclose(a, b.grad.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(dx, txp.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_one_hot_kernels_pick_the_shifted_voxel():
    """w = 1 at (c, e, a, b) only: the output is the input voxel (t+e, i+a, j+b) of channel c.  A swapped or
    transposed axis, or a flipped kernel, picks another voxel."""
    net = VideoNet("pick", 2, 3, 4, (conv3(1, 4, 3),))
    rng = np.random.default_rng(3)
    video = rng.uniform(-1, 1, size=(1, 2, 4, 5, 6))
    xpad = oracle.pad_video(video, 3, 4)
    vox = _all_voxels(1, 4, 5, 6)
    for (c, e, a, b) in [(0, 0, 0, 0), (1, 2, 0, 3), (0, 1, 3, 0), (1, 0, 2, 1), (0, 2, 3, 3)]:
        w = np.zeros((1, 2, 3, 4, 4))
        w[0, c, e, a, b] = 1.0
        got = oracle.cube_scan_forward(net, oracle.pack_params3d([w], [np.array([0.25])]), xpad, vox)
        want = np.array([xpad[0, c, v[1] + e, v[2] + a, v[3] + b] for v in vox]) + 0.25
        np.testing.assert_array_equal(got[:, 0], want)


def test_window_counts_ramps_and_ties():
    # all-ones input and weights: every output is the number of taps (+ bias)
    net = VideoNet("ones", 3, 4, 5, (conv3(2, 3, 2), avgpool3(3, 3, s=1, st=1)))
    xp = np.ones((1, 3, 4, 5, 5))
    w = np.ones((2, 3, 2, 3, 3))
    got = oracle.cube_scan_forward(net, oracle.pack_params3d([w], [np.array([0.5, -1.0])]), xp, [[0, 0, 0, 0]])
    np.testing.assert_allclose(got, [[3 * 2 * 9 + 0.5, 3 * 2 * 9 - 1.0]], rtol=0, atol=1e-12)
    # max pool over a 2 x 2 x 2 window of a cube that holds t*100 + i*10 + j: the winner is the last tap in
    # every axis; with the time axis negated the first temporal tap wins: index (e*k + a)*k + b
    pool = VideoNet("pool", 1, 2, 2, (maxpool3(2, 2),))
    cube = np.fromfunction(lambda n, c, t, i, j: t * 100 + i * 10 + j, (1, 1, 2, 2, 2))
    maps, amax = oracle.cube_forward_maps(pool, np.zeros(0), cube, [[0, 0, 0, 0]])
    assert maps[1].ravel()[0] == 111.0 and amax[1].ravel()[0] == 7
    cube2 = np.fromfunction(lambda n, c, t, i, j: -t * 100 + i * 10 + j, (1, 1, 2, 2, 2))
    maps, amax = oracle.cube_forward_maps(pool, np.zeros(0), cube2, [[0, 0, 0, 0]])
    assert maps[1].ravel()[0] == 11.0 and amax[1].ravel()[0] == 3
    cube3 = np.fromfunction(lambda n, c, t, i, j: t * 100 - i * 10 + j, (1, 1, 2, 2, 2))
    maps, amax = oracle.cube_forward_maps(pool, np.zeros(0), cube3, [[0, 0, 0, 0]])
    assert maps[1].ravel()[0] == 101.0 and amax[1].ravel()[0] == 5
    # ties: the lowest index wins, also between +0.0 and -0.0
    const = np.full((1, 1, 2, 2, 2), 0.0)
    const[0, 0, 1, 1, 1] = -0.0
    maps, amax = oracle.cube_forward_maps(pool, np.zeros(0), const, [[0, 0, 0, 0]])
    assert amax[1].ravel()[0] == 0
    two = np.zeros((1, 1, 2, 2, 2))
    two[0, 0, 0, 1, 0] = two[0, 0, 1, 0, 1] = 3.0
    maps, amax = oracle.cube_forward_maps(pool, np.zeros(0), two, [[0, 0, 0, 0]])
    assert amax[1].ravel()[0] == 2
    # backward routes the whole error to the recorded winner; the average pool spreads it evenly
    dpar, dx = oracle.cube_scan_backward(VideoNet("p", 1, 2, 2, (maxpool3(2, 2), conv3(1, 1, 1))),
                                         np.array([2.0, 0.0]), two, [[0, 0, 0, 0]], [[1.5]], want_dx=True)
    want = np.zeros_like(two)
    want[0, 0, 0, 1, 0] = 3.0
    np.testing.assert_array_equal(dx, want)
    dpar, dx = oracle.cube_scan_backward(VideoNet("a", 1, 2, 2, (avgpool3(2, 2), conv3(1, 1, 1))),
                                         np.array([2.0, 0.0]), two, [[0, 0, 0, 0]], [[1.5]], want_dx=True)
    np.testing.assert_allclose(dx, np.full_like(two, 3.0 / 8.0), rtol=0, atol=1e-15)
    np.testing.assert_allclose(dpar, [1.5 * 6.0 / 8.0, 1.5], rtol=0, atol=1e-15)


def test_no_temporal_extent_is_the_2d_oracle_frame_by_frame():
    net3 = VideoNet("flat", 2, 1, 9, (conv3(4, 3, 1, act=ACT_RELU), maxpool3(2, 1, s=2, st=1), conv3(3, 3, 1)))
    net2 = Net("flat2d", 2, 9, (conv(4, 3, 1, ACT_RELU), maxpool(2, 2), conv(3, 3)))
    ws, bs = _params(net3, 7)
    video = _video(net3, 1, 3, 5, 6, 8)
    xpad3 = oracle.pad_video(video, 1, 9)
    vox = _all_voxels(1, 3, 5, 6)
    s3 = oracle.cube_scan_forward(net3, oracle.pack_params3d(ws, bs), xpad3, vox)
    frames = np.ascontiguousarray(video[0].transpose(1, 0, 2, 3))          # [T, C, H, W]: frames as a batch
    xpad2 = oracle.pad_image(frames, 9)
    pix = vox[:, 1:]
    s2 = oracle.scan_forward(net2, oracle.pack_params([w[:, :, 0] for w in ws], bs), xpad2, pix)
    np.testing.assert_allclose(s3, s2, rtol=1e-13, atol=1e-14)
    rng = np.random.default_rng(9)
    delta = rng.standard_normal(s3.shape)
    d3, _ = oracle.cube_scan_backward(net3, oracle.pack_params3d(ws, bs), xpad3, vox, delta)
    d2, _ = oracle.scan_backward(net2, oracle.pack_params([w[:, :, 0] for w in ws], bs), xpad2, pix, delta)
    np.testing.assert_allclose(d3, d2, rtol=1e-11, atol=1e-13)


def test_finite_differences_through_the_scan():
    net = VideoNet("smooth", 2, 4, 5, (conv3(3, 2, 2, act=ACT_TANH), avgpool3(2, 2, s=1, st=1), conv3(2, 3, 2, act=ACT_TANH),
                                       conv3(3, 1, 1)))
    ws, bs = _params(net, 11)
    params = oracle.pack_params3d(ws, bs)
    xpad = oracle.pad_video(_video(net, 1, 2, 3, 3, 12), 4, 5)
    vox = _all_voxels(1, 2, 3, 3)
    rng = np.random.default_rng(13)
    g = oracle.geometry3d(net)
    delta = rng.standard_normal((len(vox), g["classes"]))

    def loss(p):
        return float((oracle.cube_scan_forward(net, p, xpad, vox) * delta).sum())
    dpar, _ = oracle.cube_scan_backward(net, params, xpad, vox, delta)
    for i in rng.permutation(params.size)[:40]:
        h = 1e-6
        pp, pm = params.copy(), params.copy()
        pp[i] += h
        pm[i] -= h
        fd = (loss(pp) - loss(pm)) / (2 * h)
        assert abs(fd - dpar[i]) <= 1e-6 * max(1.0, abs(dpar[i])), (i, fd, dpar[i])


def test_pad_video_rule():
    v = np.arange(2 * 1 * 2 * 3 * 3, dtype=np.float64).reshape(2, 1, 2, 3, 3) + 1
    p = oracle.pad_video(v, 4, 5)       # 2 frames in front, 1 behind; 2 rows / columns before, 2 after
    assert p.shape == (2, 1, 5, 7, 7)
    assert np.array_equal(p[:, :, 2:4, 2:5, 2:5], v)
    assert p.sum() == v.sum()
    p = oracle.pad_video(v, 3, 4)       # even spatial size: 2 before, 1 after
    assert p.shape == (2, 1, 4, 6, 6)
    assert np.array_equal(p[:, :, 1:3, 2:5, 2:5], v)
