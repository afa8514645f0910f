"""End-to-end parity: whole-image forward + masked backward on the GPU against
literal patch-by-patch scanning by the oracle.

Small networks and benchmark configuration 0 are scanned in full (every pixel,
every gradient).  The large benchmark configurations are checked on sampled
patches: forward scores and every intermediate map of every sampled patch (a
patch-CNN entry (u, v) after layer l sits at whole-image position
(i + D_l*u, j + D_l*v), D_l = product of the original strides through layer l;
Fig. 3 of the paper), every ReLU gate and max-pool winner, gradients through a
test mask of the sampled pixels, and -- at the configuration's real mask
density -- linearity of the gradients in the mask (Sec. 4.3)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1412_4526_amd as dsk
from workloads import Net, conv, maxpool, avgpool, CONFIGS, make_workload, sample_pixels
from workloads.nets import ACT_RELU, ACT_TANH, MAXPOOL, CONV
from gpu_common import assert_close, to_np, all_pixels, bf16_round, F32_REL, F32_ABS, BF16_REL, BF16_ABS

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(*a):
    print(*a, flush=True)


SMALL_NETS = [
    (CONFIGS[0].net, 1, 40, 40, 0.10),                      # benchmark configuration 0, in full
    (Net("example15", 2, 15, (conv(3, 2, 1, ACT_TANH), maxpool(2, 2), conv(4, 2, 1, ACT_RELU),
                              maxpool(3, 3), conv(5, 2))), 2, 9, 13, 0.3),
    (Net("s2", 2, 23, (conv(4, 3, 2, ACT_TANH), maxpool(3, 2), conv(5, 2, 1, ACT_RELU),
                       avgpool(2, 2), conv(3, 2))), 1, 21, 17, 0.5),
    (Net("s3", 2, 16, (conv(3, 4, 3, ACT_TANH), maxpool(2, 1), avgpool(2, 2), conv(4, 2))), 2, 11, 10, 1.0),
    (Net("uneven", 2, 8, (maxpool(3, 2), conv(3, 3))), 1, 12, 9, 0.4),   # patch larger than the receptive field
]


def _oracle_full(net, wl):
    N, _, H, W = wl.image.shape
    params = oracle.pack_params(wl.weights, wl.biases)
    xpad = oracle.pad_image(wl.image, net.patch)
    pix = all_pixels(N, H, W)
    scores = oracle.scan_forward(net, params, xpad, pix).reshape(N, H, W, -1).transpose(0, 3, 1, 2)
    loss, delta, count = oracle.masked_softmax_xent(scores, wl.labels, wl.mask)
    keep = wl.mask.ravel() != 0
    d = delta.transpose(0, 2, 3, 1).reshape(-1, scores.shape[1])[keep]
    g, _ = oracle.scan_backward(net, params, xpad, pix[keep], d)
    dws, dbs = oracle.unpack_params(net, g)
    return scores, loss, dws, dbs


@pytest.mark.parametrize("case", SMALL_NETS, ids=lambda c: c[0].name)
@pytest.mark.parametrize("algo", [0, 1], ids=["auto", "direct"])
def test_small_nets_in_full(case, algo):
    net, N, H, W, frac = case
    _say("small net", net.name, "algo", algo)
    wl = make_workload(net, N, H, W, frac, seed=0, bias_std=0.1 if net.name != "tiny16" else 0.0)
    rscores, rloss, rdws, rdbs = _oracle_full(net, wl)
    prev = dsk.dsk_set_conv_algo(algo)
    try:
        m = dsk.WholeImageNet(net, N, H, W, "f32", DEV)
        m.load_params(wl.weights, wl.biases)
        scores = m.forward(torch.from_numpy(wl.image).to(DEV))
        loss, dws, dbs = m.loss_backward(torch.from_numpy(wl.labels).to(DEV), torch.from_numpy(wl.mask).to(DEV))
        torch.cuda.synchronize()
    finally:
        dsk.dsk_set_conv_algo(prev)
    assert_close(scores, rscores, "scores")
    assert_close(loss, np.array([rloss]), "loss")
    for i in range(len(rdws)):
        assert_close(dws[i], rdws[i], "dw%d" % i)
        assert_close(dbs[i], rdbs[i], "db%d" % i)


def test_empty_mask_gives_zero_loss_and_gradients():
    net = CONFIGS[0].net
    wl = make_workload(net, 1, 12, 12, 0.0, seed=3)
    m = dsk.WholeImageNet(net, 1, 12, 12, "f32", DEV)
    m.load_params(wl.weights, wl.biases)
    m.forward(torch.from_numpy(wl.image).to(DEV))
    loss, dws, dbs = m.loss_backward(torch.from_numpy(wl.labels).to(DEV), torch.from_numpy(wl.mask).to(DEV))
    torch.cuda.synchronize()
    assert loss.item() == 0.0
    assert all(not t.any().item() for t in dws + dbs)


def test_whole_net_is_run_to_run_deterministic():
    """No atomics anywhere on the path: two passes over the same input give bit-identical
    scores, loss and gradients (split-K partial sums and split tiles are added in a fixed order)."""
    cfg = CONFIGS[1]
    net = cfg.net
    N, H, W = 2, 150, 210
    wl = make_workload(net, N, H, W, 0.05, seed=5, bias_std=0.1)
    m = dsk.WholeImageNet(net, N, H, W, "f32", DEV)
    m.load_params(wl.weights, wl.biases)
    image = torch.from_numpy(wl.image).to(DEV)
    labels = torch.from_numpy(wl.labels).to(DEV)
    mask = torch.from_numpy(wl.mask).to(DEV)
    runs = []
    for _ in range(2):
        scores = m.forward(image).clone()
        loss, dws, dbs = m.loss_backward(labels, mask)
        torch.cuda.synchronize()
        runs.append([scores, loss.clone()] + [t.clone() for t in dws + dbs])
    for a, b in zip(*runs):
        assert torch.equal(a, b)


def test_graph_replay_matches_eager():
    """A step captured in a HIP graph gives bit-identical results on every replay, also with new
    inputs and with eager work and synchronisations between the replays."""
    cfg = CONFIGS[0]
    net = cfg.net
    N, H, W = 1, 70, 90
    wls = [make_workload(net, N, H, W, 0.1, seed=s, bias_std=0.1) for s in (11, 12)]
    m = dsk.WholeImageNet(net, N, H, W, "f32", DEV)
    m.load_params(wls[0].weights, wls[0].biases)
    dev = [tuple(torch.from_numpy(a).to(DEV) for a in (wl.image, wl.labels, wl.mask)) for wl in wls]
    eager = []
    for image, labels, mask in dev:
        scores = m.forward(image).clone()
        loss, dws, dbs = m.loss_backward(labels, mask)
        torch.cuda.synchronize()
        eager.append([scores, loss.clone()] + [t.clone() for t in dws + dbs])
    m.capture(*dev[0])
    for which in (0, 1, 1, 0, 1):
        m.replay(*dev[which])
        torch.cuda.synchronize()
        got = [m.scores, m.loss] + m.dw + m.db
        for a, b in zip(got, eager[which]):
            assert torch.equal(a, b), "replay with input set %d differs from the eager step" % which
        # eager work between the replays, on the same buffers
        m.forward(dev[1 - which][0])
        torch.cuda.synchronize()


@pytest.mark.parametrize("case", SMALL_NETS, ids=lambda c: c[0].name)
def test_fast_scanning_comparator_small_nets(case):
    """The comparison method (fast scanning: strided layers run once per starting offset, fragments re-organised at
    the end) gives the same label map: against the oracle at every pixel."""
    net, N, H, W, frac = case
    _say("fast scanning", net.name)
    wl = make_workload(net, N, H, W, frac, seed=0, bias_std=0.1)
    params = oracle.pack_params(wl.weights, wl.biases)
    xpad = oracle.pad_image(wl.image, net.patch)
    ref = oracle.scan_forward(net, params, xpad, all_pixels(N, H, W)).reshape(N, H, W, -1).transpose(0, 3, 1, 2)
    fs = dsk.FastScanNet(net, N, H, W, "f32", DEV)
    fs.load_params(wl.weights, wl.biases)
    scores = fs.forward(torch.from_numpy(wl.image).to(DEV))
    torch.cuda.synchronize()
    assert_close(scores, ref, "fast scanning scores")
    strides = int(np.prod([L.s for L in net.layers]))
    assert fs.fragments()[-1] == strides * strides


def test_fast_scanning_comparator_plain_cnn1():
    """Plain CNN_1 of the paper's Table 1 at full size (256 x 256 labelled pixels): 64, then 256 fragments per image."""
    cfg = CONFIGS[5]
    net = cfg.net
    wl = make_workload(net, cfg.N, cfg.H, cfg.W, cfg.mask_frac, cfg.seed)
    params = oracle.pack_params(wl.weights, wl.biases)
    xpad = oracle.pad_image(wl.image, net.patch)
    pix = sample_pixels(cfg.N, cfg.H, cfg.W, 256, seed=4)
    ref = oracle.scan_forward(net, params, xpad, pix)
    fs = dsk.FastScanNet(net, cfg.N, cfg.H, cfg.W, "f32", DEV)
    fs.load_params(wl.weights, wl.biases)
    scores = fs.forward(torch.from_numpy(wl.image).to(DEV))
    torch.cuda.synchronize()
    assert fs.fragments() == [1, 64, 64, 256, 256]
    assert_close(to_np(scores[pix[:, 0], :, pix[:, 1], pix[:, 2]]), ref, "fast scanning scores at 256 sampled pixels")


# ---------------------------------------------------------------------------
# Full-size benchmark configurations
# ---------------------------------------------------------------------------
BIG = [1, 2, 3, 4, 5, 6, 7]
TH, TW = 8, 64        # output tile of the forward / backward-data kernels: 8 rows of one residue class x 64 columns


def _tail_units(N, F, Hm, Wm, d, slots):
    """Units (n, r, c) of an N x F x Hm x Wm output map that sit where the tile schedule of the
    forward / backward-data kernels is irregular: the first and the last tile of the tiles left
    over after the whole rounds of `slots` persistent workgroups (their channel chunks are shared
    between workgroups), and the bottom row block of the first and of the last residue class.
    Tiles are numbered (image, row tile, column tile, filter group), filter group fastest; row
    tiles class by class, down the map within a class."""
    tf = 64 if F > 32 else 32
    n_fgrp = -(-F // tf)
    nrb = -(-Hm // (d * TH))
    last = Hm - (nrb - 1) * d * TH
    full_cls = min(last, d)
    n_rowtile = (nrb - 1) * d + full_cls
    n_coltile = -(-Wm // TW)
    tiles = N * n_rowtile * n_coltile * n_fgrp

    def decode(t):
        t //= n_fgrp
        ct = t % n_coltile
        t //= n_coltile
        rt, n = t % n_rowtile, t // n_rowtile
        nf = full_cls * nrb
        if rt < nf:
            cls, rb = divmod(rt, nrb)
        else:
            q, rb = divmod(rt - nf, nrb - 1)
            cls = full_cls + q
        return n, rb * d * TH + cls, ct * TW

    out = []
    first_left = tiles // slots * slots
    for t in sorted({min(first_left, tiles - 1), tiles - 1}):
        n, u0, v0 = decode(t)
        rows = [u0 + r * d for r in range(TH) if u0 + r * d < Hm]
        out += [(n, rows[0], v0), (n, rows[-1], min(v0 + TW, Wm) - 1)]
    for cls in {0, full_cls - 1}:
        out.append((N - 1, (nrb - 1) * d * TH + cls, Wm - 1))
    return out


def _stratified_pixels(net, plan, N, H, W, count, slots, seed):
    """`count` labelled pixels (n, i, j): the corners and edge midpoints, pixels whose patches reach the
    irregular parts of every convolution's forward and backward-data tile schedule, and seeded uniform
    pixels for the rest.  Unit (r, c) of the whole-image map after layer l belongs to the patch of pixel
    (r - D*u, c - D*v) for any entry (u, v) of the patch CNN's map (Fig. 3)."""
    D = np.concatenate([[1], np.cumprod([L.s for L in net.layers])])      # D[l]: spacing of map l
    msz = [net.patch] + net.patch_sizes()
    want = []
    for l, p in enumerate(plan):
        if p.kind != dsk.DSK_CONV or p.k == 1:
            continue
        for map_l, F, Hm, Wm in ((l + 1, p.K, p.Ho, p.Wo), (l, p.C, p.H, p.W)):
            if map_l == 0:
                continue          # nobody computes the error map of the image
            for (n, r, c) in _tail_units(N, F, Hm, Wm, p.d, slots):
                u = min(max(0, -(-(r - H + 1) // int(D[map_l]))), msz[map_l] - 1)
                v = min(max(0, -(-(c - W + 1) // int(D[map_l]))), msz[map_l] - 1)
                i, j = r - int(D[map_l]) * u, c - int(D[map_l]) * v
                if 0 <= i < H and 0 <= j < W:
                    want.append((n, i, j))
    fixed = [tuple(int(t) for t in q) for q in sample_pixels(N, H, W, 8, seed)]
    seen, out = set(), []
    for q in fixed + want[:count // 3]:
        if q not in seen:
            seen.add(q)
            out.append(q)
    for q in sample_pixels(N, H, W, count + len(out), seed):
        q = tuple(int(t) for t in q)
        if len(out) < count and q not in seen:
            seen.add(q)
            out.append(q)
    out = np.asarray(out, np.int32)
    return out[np.random.default_rng(seed).permutation(len(out))]      # any prefix is a sample of the same kind


def _gather(t, pix, D, sz):
    """[P, C, sz, sz]: the entries (i + D*u, j + D*v) of a whole-image map for each pixel (n, i, j)."""
    return torch.stack([t[n, :, i:i + D * sz:D, j:j + D * sz:D] for (n, i, j) in pix]).cpu()


def _windows(x, k, s):
    """[P, C, mo, mo, k*k]: the taps of every k x k / stride-s window of x [P, C, mi, mi], tap index a*k+b."""
    P, C, mi, _ = x.shape
    mo = (mi - k) // s + 1
    st = x.strides
    w = np.lib.stride_tricks.as_strided(x, (P, C, mo, mo, k, k), (st[0], st[1], st[2] * s, st[3] * s, st[2], st[3]))
    return w.reshape(P, C, mo, mo, k * k)


def _compare_maps(net, m, pix, maps, ams, pre, bf16):
    """Every map of every sampled patch against the whole-image maps on the GPU (Fig. 3), and every decision
    the backward pass depends on: ReLU gates (y > 0) and max-pool winners.  A decision that differs must be a
    near-tie BY THE ORACLE'S OWN NUMBERS: its pre-activation, or the gap between its winner and the tap the
    GPU chose, within the tolerance of the values involved.  Returns (flipped [P] bool, n_flips, n_decisions)."""
    rel, ab = (BF16_REL, BF16_ABS) if bf16 else (F32_REL, F32_ABS)
    D = np.cumprod([L.s for L in net.layers])
    P = len(pix)
    flipped = np.zeros(P, bool)
    n_flips = n_dec = 0
    for l, L in enumerate(net.layers):
        ref = maps[l + 1]
        sz = ref.shape[-1]
        got = _gather(m.maps[l + 1], pix, int(D[l]), sz).double().numpy()
        # per tensor, max-norm: the largest entry among the sampled patches stands in for the map's (the last
        # map, one entry per class and patch, is checked over the whole sample by the caller)
        err = np.abs(got - ref).reshape(P, -1).max(axis=1)
        tol = rel * np.abs(ref).max() + ab
        bad = np.flatnonzero(err > tol)
        assert bad.size == 0 or l + 1 == len(net.layers), "map %d at pixel %s: err %.3g tol %.3g" % (
            l + 1, tuple(int(t) for t in pix[bad[0]]), err[bad[0]], tol)
        if L.kind == CONV and L.act == ACT_RELU:
            z = pre[l + 1]
            diff = (got > 0) != (z > 0)
            ztol = rel * np.abs(z).reshape(P, -1).max(axis=1) + ab
            far = diff & (np.abs(z) > ztol[:, None, None, None])
            assert not far.any(), "layer %d: %d ReLU gates differ away from zero (|pre-activation| up to %.3g)" % (
                l + 1, int(far.sum()), np.abs(z[far]).max())
            n_flips += int(diff.sum())
            n_dec += diff.size
            flipped |= diff.reshape(P, -1).any(axis=1)
        elif L.kind == MAXPOOL and m.argmax[l] is not None:
            ga = _gather(m.argmax[l], pix, int(D[l]), sz).numpy().astype(np.int64)
            oa = ams[l + 1].astype(np.int64)
            diff = ga != oa
            if diff.any():
                w = _windows(np.ascontiguousarray(maps[l]), L.k, L.s)
                gap = np.take_along_axis(w, oa[..., None], -1)[..., 0] - np.take_along_axis(w, ga[..., None], -1)[..., 0]
                xtol = rel * np.abs(maps[l]).reshape(P, -1).max(axis=1) + ab
                far = diff & ((gap < 0) | (gap > 2 * xtol[:, None, None, None]))
                assert not far.any(), "layer %d: %d max-pool winners differ without a near-tie (gap up to %.3g)" % (
                    l + 1, int(far.sum()), np.abs(gap[far]).max())
            n_flips += int(diff.sum())
            n_dec += diff.size
            flipped |= diff.reshape(P, -1).any(axis=1)
    return flipped, n_flips, n_dec


def _rel_err(got, want):
    got = to_np(got) if isinstance(got, torch.Tensor) else np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-300))


@pytest.mark.parametrize("ci", BIG, ids=lambda i: "config%d" % i)
def test_benchmark_configs_sampled(ci):
    """Full-size configuration, in the launch configuration bench.py times, against the exact oracle
    (fp64, unrounded inputs) on a stratified sample S of patches:
      * scores and EVERY intermediate map of every patch of S;
      * every ReLU gate and max-pool winner of those patches: identical, or a near-tie by the oracle's numbers;
      * fp32 gradients: within the fp32 bar on the patches of S without a differing decision (the gradient of
        the network is discontinuous in those decisions, Sec. 4.2), the error on all of S printed beside it;
      * bf16 gradients: against the exact oracle on S and on its first 64 patches, and against the oracle in
        bf16-storage mode (decisions taken on stored values, as the kernels take them);
      * linearity of the gradients in the mask at the configuration's real mask density (Sec. 4.3)."""
    cfg = CONFIGS[ci]
    net = cfg.net
    N, H, W = cfg.N, cfg.H, cfg.W
    dtypes = ["f32", "bf16"] if ci == 2 else [cfg.dtype]
    n_s = 256 if net.patch <= 67 else 192
    slots = 2 * torch.cuda.get_device_properties(0).multi_processor_count
    _say("config", ci, net.name, N, H, W, dtypes)
    wl = make_workload(net, N, H, W, cfg.mask_frac, cfg.seed, positive_frac=cfg.positive_frac)
    params = oracle.pack_params(wl.weights, wl.biases)
    xpad = oracle.pad_image(wl.image, net.patch)
    image = torch.from_numpy(wl.image).to(DEV)
    labels = torch.from_numpy(wl.labels).to(DEV)
    nets = {}
    for dt in dtypes:
        m = dsk.WholeImageNet(net, N, H, W, dt, DEV)
        m.load_params(wl.weights, wl.biases)
        m.forward(image)
        nets[dt] = m
    torch.cuda.synchronize()
    S = _stratified_pixels(net, nets[dtypes[0]].plan, N, H, W, n_s, slots, seed=1)
    P = len(S)
    _say("  gpu forward done; %d sampled patches" % P)

    # ---- forward: all maps, all decisions, chunk by chunk (a chunk of patches with all their maps fits in memory)
    rs = np.zeros((P, net.classes))
    flipped = {dt: np.zeros(P, bool) for dt in dtypes}
    counts = {dt: [0, 0] for dt in dtypes}
    for c0 in range(0, P, 16):
        sl = slice(c0, min(c0 + 16, P))
        maps, ams, pre = oracle.scan_forward_maps(net, params, xpad, S[sl])
        rs[sl] = maps[-1][:, :, 0, 0]
        for dt in dtypes:
            f, nf, nd = _compare_maps(net, nets[dt], S[sl], maps, ams, pre, dt == "bf16")
            flipped[dt][sl] = f
            counts[dt][0] += nf
            counts[dt][1] += nd
    for dt in dtypes:
        got = to_np(nets[dt].scores[S[:, 0], :, S[:, 1], S[:, 2]])
        assert_close(got, rs, "config %d %s scores at %d sampled pixels" % (ci, dt, P), bf16=dt == "bf16")
        _say("  %s: all maps of %d patches ok; %d of %d ReLU / max-pool decisions differ (all near-ties), in %d patches"
             % (dt, P, counts[dt][0], counts[dt][1], int(flipped[dt].sum())))

    # ---- oracle gradients: summed per group of patches with unnormalised errors, so that the gradient
    # of any union of groups follows by linearity (Sec. 4.3)
    z = rs - rs.max(axis=1, keepdims=True)
    prob = np.exp(z) / np.exp(z).sum(axis=1, keepdims=True)
    lab = wl.labels[S[:, 0], S[:, 1], S[:, 2]]
    delta = prob.copy()
    delta[np.arange(P), lab] -= 1.0
    nll = -np.log(prob[np.arange(P), lab])
    first = np.arange(P) < 64
    group = first.astype(int) * 2 + flipped["f32"].astype(int) if "f32" in dtypes else first.astype(int) * 2
    G = {}
    for gid in np.unique(group):
        sel = group == gid
        G[gid] = oracle.scan_backward(net, params, xpad, S[sel], delta[sel])[0]
    _say("  oracle backward done on %d patches" % P)

    def oracle_grads(sel):
        g = sum(G[gid] for gid in np.unique(group[sel])) / sel.sum()
        assert all((group == gid).sum() == (sel & (group == gid)).sum() for gid in np.unique(group[sel]))
        return oracle.unpack_params(net, g), float(nll[sel].sum() / sel.sum())

    def gpu_grads(m, sel):
        tmask = np.zeros((N, H, W), np.uint8)
        tmask[S[sel, 0], S[sel, 1], S[sel, 2]] = 1
        loss, dws, dbs = m.loss_backward(labels, torch.from_numpy(tmask).to(DEV))
        torch.cuda.synchronize()
        return loss.item(), [t.clone() for t in dws], [t.clone() for t in dbs], tmask

    for dt in dtypes:
        m = nets[dt]
        b16 = dt == "bf16"
        every = np.ones(P, bool)
        if not b16:
            kept = ~flipped[dt]
            assert kept.sum() >= P // 2, "decisions differ in %d of %d patches" % (P - kept.sum(), P)
            assert counts[dt][0] <= 1e-5 * counts[dt][1] + 2, "too many differing decisions: %d of %d" % tuple(counts[dt])
            (rdws, rdbs), rloss = oracle_grads(kept)
            loss, dws, dbs, tmask = gpu_grads(m, kept)
            assert abs(loss - rloss) <= F32_REL * abs(rloss) + F32_ABS
            for i in range(len(rdws)):
                assert_close(dws[i], rdws[i], "config %d f32 dw%d on the %d patches with identical decisions" % (ci, i, kept.sum()))
                assert_close(dbs[i], rdbs[i], "config %d f32 db%d" % (ci, i))
            if not kept.all():
                (adws, adbs), _ = oracle_grads(every)
                _, dws2, dbs2, _ = gpu_grads(m, every)
                _say("  f32 gradients on ALL %d patches (%d with a differing decision), max rel err per layer: dw %s db %s"
                     % (P, P - kept.sum(), ["%.2g" % _rel_err(a, b) for a, b in zip(dws2, adws)],
                        ["%.2g" % _rel_err(a, b) for a, b in zip(dbs2, adbs)]))
                loss, dws, dbs, tmask = gpu_grads(m, kept)
            _say("  f32 gradients on the %d patches with identical decisions: max rel err dw %s"
                 % (kept.sum(), ["%.2g" % _rel_err(a, b) for a, b in zip(dws, rdws)]))
            sel_T = kept
        else:
            # The bf16 path against (a) the exact oracle (fp64, unrounded image and weights) and (b) the oracle
            # that stores its maps in bf16 as the kernels do (image and weights rounded the same way), so that
            # ReLU gates and max-pool winners are decided on stored values on both sides; (c) says how far the
            # storage format alone moves the gradients: the oracle's two modes against each other.
            oparams = oracle.pack_params([bf16_round(w) for w in wl.weights], wl.biases)
            sb = oracle.scan_forward(net, oparams, xpad, S, storage=oracle.STORE_BF16)
            zb = sb - sb.max(axis=1, keepdims=True)
            pb = np.exp(zb) / np.exp(zb).sum(axis=1, keepdims=True)
            deltab = pb.copy()
            deltab[np.arange(P), lab] -= 1.0
            GB = {gid: oracle.scan_backward(net, oparams, xpad, S[group == gid], deltab[group == gid],
                                            storage=oracle.STORE_BF16)[0] for gid in np.unique(group)}
            for sel, what in ((first, "first 64"), (every, "all %d" % P)):
                (rdws, rdbs), rloss = oracle_grads(sel)
                sdws, sdbs = oracle.unpack_params(net, sum(GB[gid] for gid in np.unique(group[sel])) / sel.sum())
                loss, dws, dbs, tmask = gpu_grads(m, sel)
                fmt = lambda xs, ys: " ".join("%.2g" % _rel_err(x, y) for x, y in zip(xs, ys))
                _say("  bf16 gradients on the %s patches, max rel err per conv layer:" % what)
                _say("    (a) GPU vs exact oracle:           dw %s | db %s" % (fmt(dws, rdws), fmt(dbs, rdbs)))
                _say("    (b) GPU vs bf16-storage oracle:    dw %s | db %s" % (fmt(dws, sdws), fmt(dbs, sdbs)))
                _say("    (c) bf16-storage vs exact oracle:  dw %s | db %s" % (fmt(sdws, rdws), fmt(sdbs, rdbs)))
                assert abs(loss - rloss) <= BF16_REL * abs(rloss) + BF16_ABS
                for i in range(len(rdws)):
                    # (a) is reported, and bounded by what the storage format itself does to the oracle, (c)
                    ea, ec = _rel_err(dws[i], rdws[i]), _rel_err(sdws[i], rdws[i])
                    assert ea <= max(BF16_REL, 2.0 * ec), "config %d bf16 dw%d vs the exact oracle (%s patches): %.3g, storage alone %.3g" % (ci, i, what, ea, ec)
                    # (b) is held to the bf16 bar -- unless the storage format alone, (c), moves this tensor of the
                    # oracle by more than five times the bar on this sample: the sample is then too small for the
                    # rounding noise of the stored maps (which falls with the number of patches) to average out,
                    # and (b) must stay well inside (c) instead
                    eb = _rel_err(dws[i], sdws[i])
                    bar = BF16_REL if ec <= 5 * BF16_REL else ec / 4
                    assert eb <= bar, "config %d bf16 dw%d vs the bf16-storage oracle (%s patches): %.3g > %.3g (storage alone %.3g)" % (ci, i, what, eb, bar, ec)
                    ecb = _rel_err(sdbs[i], rdbs[i])
                    assert _rel_err(dbs[i], sdbs[i]) <= (BF16_REL if ecb <= 5 * BF16_REL else ecb / 4), "config %d bf16 db%d" % (ci, i)
            sel_T = every
        gT = dws + dbs
        lossT = loss

        # real mask density: gradients are linear in the mask (Sec. 4.3):
        # |M| g(M) = |T| g(T) + |M\T| g(M\T) for the test mask T inside M
        M = np.maximum(wl.mask, tmask)
        R = M * (1 - tmask)
        nM, nT, nR = int(M.sum()), int(tmask.sum()), int(R.sum())
        lossM, dws, dbs = m.loss_backward(labels, torch.from_numpy(M).to(DEV))
        gM = [t.clone() for t in dws + dbs]
        lossM = lossM.item()
        lossR, dws, dbs = m.loss_backward(labels, torch.from_numpy(R).to(DEV))
        gR = [t.clone() for t in dws + dbs]
        lossR = lossR.item()
        torch.cuda.synchronize()
        for a, t, r in zip(gM, gT, gR):
            want = (to_np(t) * nT + to_np(r) * nR) / nM
            assert_close(a, want, "mask linearity", bf16=b16)
        assert abs(lossM * nM - (lossT * nT + lossR * nR)) <= (2e-2 if b16 else 1e-4) * abs(lossM * nM) + 1e-5
    del nets, m
    torch.cuda.empty_cache()
