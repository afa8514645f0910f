"""Parity of the video (3-D) entry points with the cube-scanning oracle, through the C ABI.

Single layers are checked against the oracle through a two-layer ORIGINAL cube network it can scan without
knowing about spacing: a 1 x 1 x 1 pool with strides (dt, d) -- pure sub-sampling -- followed by the layer
itself; Algorithm 1 on each axis turns exactly that network into "identity, then the layer with spacings
(dt, d)".  Whole networks are checked at every voxel (small nets) and at sampled voxels (the clip workload).
Layouts differ on purpose: the oracle takes [N, C, T, H, W] videos and [K, C, kt, k, k] weights, the library
[N, T, C, H, W] and [kt, K, C, k, k].
"""
import sys

import numpy as np
import pytest
import torch

import oracle
from workloads import (VideoNet, conv3, maxpool3, avgpool3, make_video_workload, TINY_VIDEO, STRIDED_VIDEO,
                       VIDEO_CONFIGS, video_workload)
from workloads.nets import ACT_NONE, ACT_RELU, ACT_TANH
from gpu_common import assert_close, to_np, bf16_round

pytestmark = pytest.mark.gpu
dsk = pytest.importorskip("paper_1412_4526_amd") if torch.cuda.is_available() else None
DEV = "cuda:0"


def _say(*a):
    print(*a, file=sys.stderr, flush=True)


def _all_voxels(N, T, H, W):
    g = np.stack(np.meshgrid(np.arange(N), np.arange(T), np.arange(H), np.arange(W), indexing="ij"), -1)
    return g.reshape(-1, 4).astype(np.int32)


def _single(C, layer, kt, k, dt, d):
    layers = ((maxpool3(1, 1, s=d, st=dt),) if (d > 1 or dt > 1) else ()) + (layer,)
    return VideoNet("single", C, 1 + (kt - 1) * dt, 1 + (k - 1) * d, layers)


def _lib_video(x):      # [N, C, T, H, W] -> the library's [N, T, C, H, W]
    return np.ascontiguousarray(np.transpose(x, (0, 2, 1, 3, 4)))


def _gpu(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV).to(dtype)


# (N, T, C, H, W, K, kt, k, dt, d, act)
CONV_CASES = [
    (1, 5, 3, 12, 14, 8, 3, 3, 1, 1, ACT_RELU),       # 3 channels: chunks straddle the temporal taps
    (1, 7, 4, 13, 70, 40, 2, 3, 2, 2, ACT_NONE),      # two column tiles, two filter groups
    (2, 6, 8, 20, 21, 33, 3, 2, 2, 3, ACT_TANH),      # two videos: frames of the second start after a gap
    (1, 9, 16, 11, 12, 16, 2, 4, 4, 1, ACT_RELU),     # fewer output frames than the temporal reach
    (2, 3, 5, 9, 10, 6, 1, 3, 1, 2, ACT_RELU),        # no temporal extent: the 2-D layer on every frame
    (1, 4, 6, 8, 9, 7, 2, 1, 3, 1, ACT_NONE),         # 1 x 1 spatial kernel with temporal taps
    (1, 8, 32, 24, 40, 64, 3, 3, 2, 2, ACT_RELU),     # whole chunks per tap, several row tiles
]


@pytest.mark.parametrize("algo", [0, 1])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "N%dT%dC%d_%dx%d_K%d_kt%dk%d_dt%dd%d" % c[:10])
def test_conv3d(case, dtype, algo):
    N, T, C, H, W, K, kt, k, dt, d, act = case
    if algo == 1 and dtype == "bf16":
        pytest.skip("the plain kernels are covered in fp32")
    _say("conv3d", case, dtype, "algo", algo)
    bf = dtype == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    rng = np.random.default_rng(hash(case) % 2**31)
    x = rng.uniform(-1, 1, size=(N, C, T, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, kt, k, k)) / np.sqrt(C * kt * k * k)).astype(np.float32)
    b = (rng.standard_normal(K) * 0.1).astype(np.float32)
    To, Ho, Wo = T - (kt - 1) * dt, H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, K, To, Ho, Wo)).astype(np.float32)
    if bf:      # the kernels see bf16 maps and weights rounded to bf16: give the oracle the same numbers
        x, w, dy = bf16_round(x), bf16_round(w), bf16_round(dy)
    net = _single(C, conv3(K, k, kt, act=act), kt, k, dt, d)
    vox = _all_voxels(N, To, Ho, Wo)
    params = oracle.pack_params3d([w], [b])
    ref = oracle.cube_scan_forward(net, params, x, vox).reshape(N, To, Ho, Wo, K).transpose(0, 4, 1, 2, 3)
    # backward: the oracle differentiates through the non-linearity; the library's conv calls take the error
    # map after dsk_act_bwd, so feed both the error w.r.t. the activated output
    delta = dy.transpose(0, 2, 3, 4, 1).reshape(-1, K)
    rg, rdx = oracle.cube_scan_backward(net, params, x, vox, delta, want_dx=True)
    rdw, rdb = oracle.unpack_params3d(net, rg)
    prev = dsk.dsk_set_conv_algo(algo)
    try:
        xg = _gpu(_lib_video(x), td)
        wg = _gpu(np.transpose(w, (2, 0, 1, 3, 4)))
        y = dsk.dsk_conv3d_fwd(xg, wg, _gpu(b), dt, d, act)
        g = _gpu(_lib_video(dy), td)
        flat = (N * To, K, Ho, Wo)
        db = dsk.dsk_act_bwd_bias(y.view(flat), g.view(flat), act)
        dw, _ = dsk.dsk_conv3d_bwd_weight(xg, g, kt, k, k, dt, d, want_db=False)
        dx = dsk.dsk_conv3d_bwd_data(g, wg, dt, d, T, H, W)
        torch.cuda.synchronize()
    finally:
        dsk.dsk_set_conv_algo(prev)
    assert_close(y.permute(0, 2, 1, 3, 4), ref, "y", bf16=bf)
    if bf and act != ACT_NONE:
        return      # act'(y) is taken on the rounded output: covered by the whole-network tests
    assert_close(dw.permute(1, 2, 0, 3, 4), rdw[0], "dw", bf16=bf)
    assert_close(db, rdb[0], "db", bf16=bf)
    assert_close(dx.permute(0, 2, 1, 3, 4), rdx, "dx", bf16=bf)


# (N, T, C, H, W, kt, k, dt, d)
POOL_CASES = [
    (1, 4, 3, 9, 10, 2, 2, 1, 1),
    (2, 7, 5, 12, 17, 2, 3, 2, 2),
    (1, 9, 2, 20, 70, 3, 2, 3, 4),
    (1, 3, 4, 8, 9, 1, 2, 1, 2),
    (1, 6, 6, 13, 8, 2, 1, 2, 1),
    (1, 5, 33, 31, 130, 2, 2, 2, 2),
]


@pytest.mark.parametrize("ties", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("is_max", [True, False])
@pytest.mark.parametrize("case", POOL_CASES, ids=lambda c: "N%dT%dC%d_%dx%d_kt%dk%d_dt%dd%d" % c)
def test_pool3d(case, is_max, dtype, ties):
    N, T, C, H, W, kt, k, dt, d = case
    if ties and not is_max:
        pytest.skip("ties matter to max pooling only")
    _say("pool3d", case, is_max, dtype, ties)
    bf = dtype == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    rng = np.random.default_rng(hash(case) % 2**31)
    x = rng.uniform(-1, 1, size=(N, C, T, H, W)).astype(np.float32)
    if ties:
        x = np.round(x * 2) / 2          # five distinct values: ties in most windows, -0.0 among them
    if bf:
        x = bf16_round(x)
    To, Ho, Wo = T - (kt - 1) * dt, H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, C, To, Ho, Wo)).astype(np.float32)
    if bf:
        dy = bf16_round(dy)
    net = _single(C, maxpool3(k, kt) if is_max else avgpool3(k, kt), kt, k, dt, d)
    vox = _all_voxels(N, To, Ho, Wo)
    maps, amax = oracle.cube_forward_maps(net, np.zeros(0), x, vox)
    ref = maps[-1].reshape(N, To, Ho, Wo, C).transpose(0, 4, 1, 2, 3)
    ram = amax[-1].reshape(N, To, Ho, Wo, C).transpose(0, 4, 1, 2, 3)
    _, rdx = oracle.cube_scan_backward(net, np.zeros(0), x, vox, dy.transpose(0, 2, 3, 4, 1).reshape(-1, C), want_dx=True)
    xg, g = _gpu(_lib_video(x), td), _gpu(_lib_video(dy), td)
    if is_max:
        y, am = dsk.dsk_maxpool3d_fwd(xg, kt, k, dt, d)
        dx = dsk.dsk_maxpool3d_bwd(g, am, kt, k, dt, d, T, H, W)
        torch.cuda.synchronize()
        assert np.array_equal(to_np(y.permute(0, 2, 1, 3, 4)), ref), "max-pool values must be exact"
        assert np.array_equal(am.permute(0, 2, 1, 3, 4).cpu().numpy().astype(np.int32), ram), "winners must be bit-exact"
    else:
        y = dsk.dsk_avgpool3d_fwd(xg, kt, k, dt, d)
        dx = dsk.dsk_avgpool3d_bwd(g, kt, k, dt, d, T, H, W)
        torch.cuda.synchronize()
        assert_close(y.permute(0, 2, 1, 3, 4), ref, "y", bf16=bf)
    assert_close(dx.permute(0, 2, 1, 3, 4), rdx, "dx", bf16=bf)


def _oracle_full(net, wl, vox=None):
    """Scores at every voxel (or the listed ones), loss and gradients with the workload's mask."""
    N, _, T, H, W = wl.video.shape
    xpad = oracle.pad_video(wl.video, net.patch_t, net.patch)
    params = oracle.pack_params3d(wl.weights, wl.biases)
    allv = _all_voxels(N, T, H, W)
    scores = oracle.cube_scan_forward(net, params, xpad, allv if vox is None else vox)
    return xpad, params, scores


# a 1x1x1 classifier on top of a fully connected layer (3 frames of 5 x 5 pixels): backward-data of the classifier
# takes the 2-D call that also does the non-linearity backward and bias gradient of the layer below
FC_VIDEO = VideoNet("fccube", 2, 3, 5, (
    conv3(6, 3, 2, act=ACT_RELU),               # -> 2 x 3 x 3
    conv3(40, 3, 2, act=ACT_TANH),              # -> 1 x 1 x 1
    conv3(4, 1, 1)), init="n0.05")

NET_CASES = [(TINY_VIDEO, 1, 5, 12, 14, 0.10), (TINY_VIDEO, 2, 3, 9, 70, 0.05), (STRIDED_VIDEO, 1, 4, 10, 9, 0.2),
             (STRIDED_VIDEO, 2, 7, 6, 11, 0.1), (FC_VIDEO, 2, 4, 9, 13, 0.2)]


@pytest.mark.parametrize("algo", [0, 1])
@pytest.mark.parametrize("case", NET_CASES, ids=lambda c: "%s_N%d_%dx%dx%d" % (c[0].name, c[1], c[2], c[3], c[4]))
def test_small_video_nets_in_full(case, algo):
    net, N, T, H, W, frac = case
    _say("video net", net.name, N, T, H, W, "algo", algo)
    wl = make_video_workload(net, N, T, H, W, frac, seed=1, bias_std=0.1)
    xpad, params, rs = _oracle_full(net, wl)
    cls = net.classes
    rscores = rs.reshape(N, T, H, W, cls).transpose(0, 1, 4, 2, 3)          # [N, T, Cls, H, W]
    rloss, rdelta, cnt = oracle.masked_softmax_xent(rscores.reshape(N * T, cls, H, W), wl.labels.reshape(N * T, H, W),
                                                    wl.mask.reshape(N * T, H, W))
    assert cnt > 0
    vox = _all_voxels(N, T, H, W)
    delta = rdelta.reshape(N, T, cls, H, W).transpose(0, 1, 3, 4, 2).reshape(-1, cls)
    keep = np.abs(delta).sum(1) > 0
    rg, _ = oracle.cube_scan_backward(net, params, xpad, vox[keep], delta[keep])
    rdws, rdbs = oracle.unpack_params3d(net, rg)
    prev = dsk.dsk_set_conv_algo(algo)
    try:
        m = dsk.WholeVideoNet(net, N, T, H, W, "f32", DEV)
        m.load_params(wl.weights, wl.biases)
        scores = m.forward(_gpu(_lib_video(wl.video)))
        loss, dws, dbs = m.loss_backward(torch.from_numpy(wl.labels).to(DEV), torch.from_numpy(wl.mask).to(DEV))
        torch.cuda.synchronize()
        # a second pass gives bit-identical results (fixed summation orders, no atomics)
        first = [scores.clone(), loss.clone()] + [t.clone() for t in dws + dbs]
        m.forward(_gpu(_lib_video(wl.video)))
        m.loss_backward(torch.from_numpy(wl.labels).to(DEV), torch.from_numpy(wl.mask).to(DEV))
        torch.cuda.synchronize()
        for a, b in zip(first, [m.scores, m.loss] + m.dw + m.db):
            assert torch.equal(a, b)
    finally:
        dsk.dsk_set_conv_algo(prev)
    assert_close(scores, rscores, "scores")
    assert_close(loss, np.array([rloss]), "loss")
    for i in range(len(rdws)):
        assert_close(dws[i].permute(1, 2, 0, 3, 4), rdws[i], "dw%d" % i)
        assert_close(dbs[i], rdbs[i], "db%d" % i)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_clip_workload_sampled(dtype):
    """The measured video workload at its real size: scores at sampled voxels (the corners of the clip among
    them), and the gradients of a test mask of sampled voxels against the sum of the oracle's per-cube gradients."""
    cfg = VIDEO_CONFIGS[1]
    net, N, T, H, W = cfg.net, cfg.N, cfg.T, cfg.H, cfg.W
    _say("clip workload", dtype)
    bf = dtype == "bf16"
    wl = video_workload(1, bias_std=0.1)
    rng = np.random.default_rng(5)
    fixed = [(0, t, i, j) for t in (0, T - 1) for i in (0, H - 1) for j in (0, W - 1)]
    rnd = [(0, int(rng.integers(T)), int(rng.integers(H)), int(rng.integers(W))) for _ in range(88)]
    vox = np.asarray(sorted(set(fixed + rnd)), np.int32)
    video, weights = (bf16_round(wl.video), [bf16_round(w) for w in wl.weights]) if bf else (wl.video, wl.weights)
    xpad = oracle.pad_video(video, net.patch_t, net.patch)
    params = oracle.pack_params3d(weights, wl.biases)
    rs = oracle.cube_scan_forward(net, params, xpad, vox)
    mask = np.zeros((N, T, H, W), np.uint8)
    mask[vox[:, 0], vox[:, 1], vox[:, 2], vox[:, 3]] = 1
    m = dsk.WholeVideoNet(net, N, T, H, W, dtype, DEV)
    m.load_params(wl.weights, wl.biases)
    scores = m.forward(_gpu(_lib_video(wl.video)))
    loss, dws, dbs = m.loss_backward(torch.from_numpy(wl.labels).to(DEV), torch.from_numpy(mask).to(DEV))
    torch.cuda.synchronize()
    got = to_np(scores)[vox[:, 0], vox[:, 1], :, vox[:, 2], vox[:, 3]]
    assert_close(got, rs, "scores at sampled voxels", bf16=bf)
    if bf:
        return      # gradients in bf16 storage differ from the exact ones by the storage format itself (see the 2-D tests)

    # Every stored map of every sampled cube against the oracle's per-cube maps: entry (q, u, v) of map l of the cube
    # at (t, i, j) is the whole-video map l at (t + Dt*q, i + D*u, j + D*v).  Parity of the maps at the fp32 bar implies
    # that a ReLU gate or pool winner the two sides decide differently is a near-tie: a gate differs only where both
    # values are within the tolerance of zero, a winner only where the two taps are within twice the tolerance of each
    # other in the pool's input map.  The gradient is discontinuous at such units (the whole error goes to the
    # recorded winner), so gradients are compared on the cubes whose decisions are all identical.
    maps, amax = oracle.cube_forward_maps(net, params, xpad, vox)
    flipped = np.zeros(len(vox), bool)
    decisions = 0
    Dt = D = 1
    for l, L in enumerate(net.layers):
        Dt, D = Dt * L.st, D * L.s
        ref = maps[l + 1]                                  # [P, C, mt, m, m]
        mt, mm = ref.shape[2], ref.shape[3]
        gm = m.maps[l + 1]
        got = torch.stack([gm[v[0], v[1]:v[1] + Dt * mt:Dt, :, v[2]:v[2] + D * mm:D, v[3]:v[3] + D * mm:D] for v in vox])
        got = to_np(got.permute(0, 2, 1, 3, 4))
        assert_close(got, ref, "map %d of the sampled cubes" % (l + 1))
        if L.kind == 1:      # max pool: recorded winners
            ga = torch.stack([m.argmax[l][v[0], v[1]:v[1] + Dt * mt:Dt, :, v[2]:v[2] + D * mm:D, v[3]:v[3] + D * mm:D] for v in vox])
            diff = ga.permute(0, 2, 1, 3, 4).cpu().numpy().astype(np.int32) != amax[l + 1]
        elif L.act == ACT_RELU:
            diff = (got > 0) != (ref > 0)
        else:
            continue
        decisions += diff.size
        flipped |= diff.reshape(len(vox), -1).any(1)
    _say("clip workload: %d of %d sampled cubes hold a decision that differs (of %d decisions)" % (flipped.sum(), len(vox), decisions))
    assert flipped.sum() <= len(vox) // 8
    keep = vox[~flipped]
    rk = rs[~flipped]
    mask = np.zeros((N, T, H, W), np.uint8)
    mask[keep[:, 0], keep[:, 1], keep[:, 2], keep[:, 3]] = 1
    loss, dws, dbs = m.loss_backward(torch.from_numpy(wl.labels).to(DEV), torch.from_numpy(mask).to(DEV))
    torch.cuda.synchronize()
    # per-voxel error from the oracle's own scores
    cls = net.classes
    lab = wl.labels[keep[:, 0], keep[:, 1], keep[:, 2], keep[:, 3]]
    z = rk - rk.max(1, keepdims=True)
    p = np.exp(z) / np.exp(z).sum(1, keepdims=True)
    delta = (p - np.eye(cls)[lab]) / len(keep)
    rloss = -np.log(p[np.arange(len(keep)), lab]).mean()
    rg, _ = oracle.cube_scan_backward(net, params, xpad, keep, delta)
    rdws, rdbs = oracle.unpack_params3d(net, rg)
    assert_close(loss, np.array([rloss]), "loss")
    for i in range(len(rdws)):
        assert_close(dws[i].permute(1, 2, 0, 3, 4), rdws[i], "dw%d" % i)
        assert_close(dbs[i], rdbs[i], "db%d" % i)


@pytest.mark.parametrize("case", CONV_CASES + [(1, 6, 32, 70, 200, 64, 3, 3, 2, 2, ACT_RELU), (2, 5, 64, 40, 130, 128, 2, 4, 1, 8, ACT_RELU)],
                         ids=lambda c: "N%dT%dC%d_%dx%d_K%d_kt%dk%d_dt%dd%d" % c[:10])
def test_conv3d_workspace_is_enough_and_respected(case):
    """The three video convolution calls stay inside the workspace size the library asks for: a guard band behind
    it keeps its pattern (results are covered by the parity tests)."""
    N, T, C, H, W, K, kt, k, dt, d, act = case
    _say("conv3d workspace", case)
    x = torch.rand((N, T, C, H, W), device=DEV) - 0.5
    w = torch.randn((kt, K, C, k, k), device=DEV) * 0.1
    To, Ho, Wo = T - (kt - 1) * dt, H - (k - 1) * d, W - (k - 1) * d
    dy = torch.randn((N, To, K, Ho, Wo), device=DEV)
    guard = 1 << 16
    for which in (dsk.DSK_WS_CONV_FWD, dsk.DSK_WS_CONV_BWD_DATA, dsk.DSK_WS_CONV_BWD_WEIGHT):
        need = dsk.dsk_conv3d_workspace_bytes(which, N, T, C, H, W, K, kt, k, k, dt, d, dsk.DSK_F32)
        need16 = (need + 15) // 16 * 16
        buf = torch.full((need16 + guard,), 0xA5, dtype=torch.uint8, device=DEV)
        ws = buf[:max(need16, 16)]
        if which == dsk.DSK_WS_CONV_FWD:
            dsk.dsk_conv3d_fwd(x, w, None, dt, d, act, ws=ws)
        elif which == dsk.DSK_WS_CONV_BWD_DATA:
            dsk.dsk_conv3d_bwd_data(dy, w, dt, d, T, H, W, ws=ws)
        else:
            dsk.dsk_conv3d_bwd_weight(x, dy, kt, k, k, dt, d, ws=ws)
        torch.cuda.synchronize()
        assert bool((buf[need16:] == 0xA5).all()), "write beyond the workspace (call %d)" % which


def test_video_graph_replay_matches_eager():
    """A video step captured in a HIP graph gives bit-identical results on every replay, also with new inputs and
    with eager work and synchronisations between the replays."""
    net, N, T, H, W = TINY_VIDEO, 1, 4, 20, 70
    wls = [make_video_workload(net, N, T, H, W, 0.1, seed=s, bias_std=0.1) for s in (21, 22)]
    m = dsk.WholeVideoNet(net, N, T, H, W, "f32", DEV)
    m.load_params(wls[0].weights, wls[0].biases)
    dev = [(_gpu(_lib_video(wl.video)), torch.from_numpy(wl.labels).to(DEV), torch.from_numpy(wl.mask).to(DEV)) for wl in wls]
    eager = []
    for video, labels, mask in dev:
        scores = m.forward(video).clone()
        loss, dws, dbs = m.loss_backward(labels, mask)
        torch.cuda.synchronize()
        eager.append([scores, loss.clone()] + [t.clone() for t in dws + dbs])
    m.capture(*dev[0])
    for rnd in range(3):
        for i, (video, labels, mask) in enumerate(dev):
            m.replay(video, labels, mask)
            torch.cuda.synchronize()
            for a, b in zip(eager[i], [m.scores, m.loss] + m.dw + m.db):
                assert torch.equal(a, b), "replay %d of input %d differs from the eager pass" % (rnd, i)
            # the program's own eager work between replays
            junk = torch.rand((257, 129), device=DEV)
            (junk @ junk.t()).sum().item()


def test_video_argument_errors():
    x = torch.zeros((1, 4, 2, 8, 8), device=DEV)
    w = torch.zeros((3, 4, 2, 3, 3), device=DEV)
    with pytest.raises(dsk.DskError):
        dsk.dsk_conv3d_fwd(x, w, None, 2, 1)            # temporal reach 5 > 4 frames
    with pytest.raises(dsk.DskError):
        dsk.dsk_maxpool3d_fwd(x, 2, 9, 1, 1)            # window larger than the map
    with pytest.raises(dsk.DskError):
        dsk.dsk_maxpool3d_fwd(x, 4, 8, 1, 1)            # tap index would not fit a byte
