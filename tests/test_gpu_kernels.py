"""Per-kernel parity of the HIP path (through the C-ABI) against the patch-scanning
oracle, element by element on the same seeded inputs.  Shapes span several tiles
of every kernel and have ragged tails; spacings d cover 1 and values that do not
divide the tile sizes."""
import numpy as np
import pytest
import torch

import oracle
import paper_1412_4526_amd as dsk
from gpu_common import (assert_close, to_np, bf16_round, oracle_conv_fwd, oracle_conv_bwd,
                        oracle_pool_fwd, oracle_pool_bwd)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _t(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(dtype).contiguous()


def _say(*a):
    print(*a, flush=True)


# (N, C, H, W, K, k, d, act)
CONV_CASES = [
    (1, 3, 23, 29, 8, 5, 1, 1),        # first layer: C = 3
    (2, 8, 40, 37, 16, 3, 2, 1),
    (1, 16, 30, 45, 10, 2, 4, 0),      # fc as a 2x2 conv, K not a multiple of anything
    (1, 5, 41, 33, 7, 1, 3, 2),        # 1x1, tanh
    (1, 32, 75, 141, 64, 5, 2, 1),     # several tiles + ragged tail in both directions
    (1, 40, 60, 92, 70, 4, 8, 1),      # C, K not multiples of 32; large spacing
    (2, 64, 37, 70, 33, 1, 8, 0),      # 1x1 with K = 33
    (1, 6, 64, 50, 48, 7, 1, 1),       # 7x7
    (1, 130, 20, 90, 2, 3, 3, 0),      # K = 2, C > 128
    (1, 10, 130, 150, 12, 7, 16, 0),   # 7x7 taps 16 apart: 96-column halo, weight gradient one tap column at a time
    (1, 8, 120, 140, 40, 7, 16, 1),    # the same with more than 32 filters
    (1, 4, 90, 100, 9, 6, 12, 2),      # 6x6 taps 12 apart, four input channels
    (1, 20, 50, 61, 150, 1, 1, 1),     # 1x1 with three filter groups; pixel count not a multiple of 128
    (3, 70, 9, 13, 3, 1, 2, 0),        # 1x1, planes smaller than one wave's 128 pixels
    (1, 300, 20, 33, 2, 1, 1, 0),      # 1x1, more than 256 channels, two filters
    (1, 40, 50, 70, 72, 3, 4, 1),      # 3x3 with three 32-filter blocks: two blocks per workgroup, one group half empty
    (1, 8, 40, 88, 40, 3, 2, 1),       # last rows and columns at most half a tile, forward and backward-data: half-size tiles
    (2, 6, 30, 80, 33, 3, 1, 2),       # the same with two images and two filter groups
    (1, 16, 20, 30, 16, 2, 4, 0),      # a map smaller than half a tile both ways: one rectangle of 4 x 32 tiles
    (1, 8, 36, 150, 16, 5, 2, 1),      # only the column strip is narrow forward, only the row strip low backward
    (1, 96, 40, 70, 80, 3, 2, 1),      # 80 filters forward, 96 backward: the last 16 / 32 run as a launch of 32-filter tiles
    (2, 65, 30, 64, 130, 4, 2, 0),     # ... a tail of 2 filters forward, of one backward
]


@pytest.mark.parametrize("algo", [0, 1], ids=["auto", "direct"])
@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "N%dC%dH%dW%dK%dk%dd%da%d" % c)
def test_conv_fwd(case, algo):
    N, C, H, W, K, k, d, act = case
    _say("conv_fwd", case, "algo", algo)
    rng = np.random.default_rng(hash(case) % 2**31)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, k, k)) * np.sqrt(2.0 / (C * k * k))).astype(np.float32)
    b = (rng.standard_normal(K) * 0.2).astype(np.float32)
    ref = oracle_conv_fwd(x, w, b, d, act)
    prev = dsk.dsk_set_conv_algo(algo)
    try:
        y = dsk.dsk_conv_fwd(_t(x), _t(w), _t(b), d, act)
        y_nobias = dsk.dsk_conv_fwd(_t(x), _t(w), None, d, dsk.DSK_ACT_NONE)
        torch.cuda.synchronize()
    finally:
        dsk.dsk_set_conv_algo(prev)
    assert_close(y, ref, "conv_fwd")
    if act == 0:
        assert_close(y_nobias, ref - b[None, :, None, None], "conv_fwd without bias")


@pytest.mark.parametrize("algo", [0, 1], ids=["auto", "direct"])
@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "N%dC%dH%dW%dK%dk%dd%da%d" % c)
def test_conv_bwd(case, algo):
    N, C, H, W, K, k, d, act = case
    _say("conv_bwd", case, "algo", algo)
    rng = np.random.default_rng(hash(case) % 2**31 + 1)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, k, k)) * np.sqrt(2.0 / (C * k * k))).astype(np.float32)
    b = (rng.standard_normal(K) * 0.2).astype(np.float32)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, K, Ho, Wo)).astype(np.float32)
    dy[rng.random(dy.shape) < 0.5] = 0.0          # error maps are sparse after a mask
    rdw, rdb, rdx = oracle_conv_bwd(x, w, b, d, act, dy)
    prev = dsk.dsk_set_conv_algo(algo)
    try:
        xt, wt = _t(x), _t(w)
        y = dsk.dsk_conv_fwd(xt, wt, _t(b), d, act)
        g = _t(dy)
        dsk.dsk_act_bwd(y, g, act)
        dw, db = dsk.dsk_conv_bwd_weight(xt, g, k, k, d)
        dw2, db2 = dsk.dsk_conv_bwd_weight(xt, g, k, k, d)
        dx = dsk.dsk_conv_bwd_data(g, wt, d, H, W)
        # the fused form: non-linearity backward and bias gradient in one pass
        g2 = _t(dy)
        db_fused = dsk.dsk_act_bwd_bias(y, g2, act)
        dw_nobias, none = dsk.dsk_conv_bwd_weight(xt, g2, k, k, d, want_db=False)
        torch.cuda.synchronize()
    finally:
        dsk.dsk_set_conv_algo(prev)
    assert_close(dw, rdw, "dw")
    assert_close(db, rdb, "db")
    assert_close(dx, rdx, "dx")
    assert none is None and torch.equal(g2, g) and torch.equal(dw_nobias, dw)
    assert_close(db_fused, rdb, "db (fused with the non-linearity backward)")
    assert torch.equal(dw, dw2) and torch.equal(db, db2), "bwd_weight is not run-to-run deterministic"


def _oracle_pair_bwd(x0, bA, actA, w, d, dy):
    """Two conv layers with no pool in between: A = 1x1 with identity weights, bias bA and non-linearity actA
    (so its stored output is actA(x0 + bA) and the error at its input equals the error behind its non-linearity),
    B = the layer under test (weights w, spacing d, no non-linearity).  Returns (error map behind A's
    non-linearity, A's bias gradient) for the error dy at B's output."""
    from workloads import Net, conv, maxpool
    N, C, H, W = x0.shape
    K, _, k, _ = w.shape
    layers = ((maxpool(1, d),) if d > 1 else ()) + (conv(C, 1, 1, actA), conv(K, k, 1, 0))
    net = Net("pair", C, 1 + (k - 1) * d, layers)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    n, i, j = np.meshgrid(np.arange(N), np.arange(Ho), np.arange(Wo), indexing="ij")
    pix = np.stack([n.ravel(), i.ravel(), j.ravel()], 1).astype(np.int32)
    eye = np.eye(C, dtype=np.float32).reshape(C, C, 1, 1)
    params = oracle.pack_params([eye, w], [bA, np.zeros(K, np.float32)])
    delta = np.asarray(dy, np.float64).transpose(0, 2, 3, 1).reshape(-1, K)
    g, dx = oracle.scan_backward(net, params, x0, pix, delta, want_dx=True)
    _, dbs = oracle.unpack_params(net, g)
    return dx, dbs[0]


# (N, C, H, W, K, k, d, act of the layer below)
PAIR_CASES = [
    (1, 64, 37, 70, 33, 1, 1, 1),      # one group of 64 channels
    (2, 150, 50, 61, 20, 1, 1, 1),     # three channel groups, the last one ragged; planes not a multiple of 128 pixels
    (3, 20, 9, 13, 70, 1, 2, 2),       # at most 32 channels (one 32-block), planes smaller than a wave's 128 pixels, tanh
    (1, 256, 40, 40, 33, 1, 1, 0),     # no non-linearity below: the bias gradient alone
    (1, 40, 130, 141, 33, 1, 1, 1),    # more than 128 waves: two groups of per-wave sums
    (2, 8, 40, 37, 16, 3, 2, 1),       # 3x3: the two passes one after the other
    (1, 16, 30, 45, 10, 2, 4, 2),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("algo", [0, 1], ids=["auto", "direct"])
@pytest.mark.parametrize("case", PAIR_CASES, ids=lambda c: "N%dC%dH%dW%dK%dk%dd%da%d" % c)
def test_conv_bwd_data_act_bias(case, algo, dtype):
    """Backward-data with the non-linearity backward and bias gradient of the conv layer below (Sec. 4.1)
    against the oracle's two-layer network, and bit for bit against the two separate calls."""
    N, C, H, W, K, k, d, act = case
    _say("conv_bwd_data_act_bias", case, "algo", algo, dtype)
    bf = dtype == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    rnd = (lambda a: bf16_round(a).astype(np.float32)) if bf else (lambda a: np.asarray(a, np.float32))
    rng = np.random.default_rng(hash(case) % 2**31 + 5)
    x0 = rnd(rng.uniform(-1, 1, (N, C, H, W)))
    bA = (rng.standard_normal(C) * 0.2).astype(np.float32)
    w = rnd(rng.standard_normal((K, C, k, k)) * np.sqrt(2.0 / (C * k * k)))
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, K, Ho, Wo)).astype(np.float32)
    dy[rng.random(dy.shape) < 0.5] = 0.0
    dy = rnd(dy)
    rdx, rdb = _oracle_pair_bwd(x0, bA, act, w, d, dy)
    prev = dsk.dsk_set_conv_algo(algo)
    try:
        eye = torch.eye(C, device=DEV).reshape(C, C, 1, 1).contiguous()
        x = dsk.dsk_conv_fwd(_t(x0, td), eye, _t(bA), 1, act)        # the stored output of the layer below
        g, wt = _t(dy, td), _t(w)
        dx, db = dsk.dsk_conv_bwd_data_act_bias(g, wt, x, d, act)
        dx2 = dsk.dsk_conv_bwd_data(g, wt, d, H, W)
        db2 = dsk.dsk_act_bwd_bias(x, dx2, act)
        dx3, db3 = dsk.dsk_conv_bwd_data_act_bias(g, wt, x, d, act)
        torch.cuda.synchronize()
    finally:
        dsk.dsk_set_conv_algo(prev)
    assert dx.dtype == td and db.dtype == torch.float32
    assert_close(dx, rdx, "dx behind the non-linearity", bf16=bf)
    assert_close(db, rdb, "db of the layer below", bf16=bf)
    assert torch.equal(dx, dx3) and torch.equal(db, db3), "not run-to-run deterministic"
    if k > 1 or algo == 1 or (not bf and act != 2):
        # the same kernels (fp32: the 1x1 kernel with and without the epilogue), so the same bits in dx
        assert torch.equal(dx, dx2), "differs from the two separate calls"
    else:
        assert_close(dx, to_np(dx2), "dx against the two separate calls", bf16=bf)
    assert_close(db, to_np(db2), "db against the two separate calls", bf16=bf)


@pytest.mark.parametrize("seed", range(16))
def test_conv_bwd_data_act_bias_random_1x1(seed):
    """The one-pass form on seeded random 1x1 layers: channel counts around the 32-channel groups, planes that end
    inside a wave's 128 pixels, one to three images, every non-linearity, both storage types."""
    r = np.random.default_rng(4000 + seed)
    C = int(r.choice([1, 7, 31, 32, 33, 64, 65, 100, 129, 200]))
    K = int(r.choice([1, 2, 5, 21, 33, 40, 64]))
    N, H, W = int(r.integers(1, 4)), int(r.integers(1, 40)), int(r.integers(1, 90))
    act, bf = int(r.integers(0, 3)), bool(seed % 2)
    _say("conv_bwd_data_act_bias random", seed, (N, C, H, W, K, act), "bf16" if bf else "f32")
    td = torch.bfloat16 if bf else torch.float32
    rnd = (lambda a: bf16_round(a).astype(np.float32)) if bf else (lambda a: np.asarray(a, np.float32))
    x0 = rnd(r.uniform(-1, 1, (N, C, H, W)))
    bA = (r.standard_normal(C) * 0.2).astype(np.float32)
    w = rnd(r.standard_normal((K, C, 1, 1)) * np.sqrt(2.0 / C))
    dy = rnd(r.standard_normal((N, K, H, W)))
    rdx, rdb = _oracle_pair_bwd(x0, bA, act, w, 1, dy)
    eye = torch.eye(C, device=DEV).reshape(C, C, 1, 1).contiguous()
    x = dsk.dsk_conv_fwd(_t(x0, td), eye, _t(bA), 1, act)
    dx, db = dsk.dsk_conv_bwd_data_act_bias(_t(dy, td), _t(w), x, 1, act)
    torch.cuda.synchronize()
    assert_close(dx, rdx, "dx behind the non-linearity", bf16=bf)
    assert_close(db, rdb, "db of the layer below", bf16=bf)


# More output tiles than the 512 workgroups the chip holds at once, and not a multiple of it:
# persistent workgroups take whole tiles first and share the channel chunks of the rest.
SPLIT_CASES = [
    (1, 24, 826, 322, 32, 3, 1, 1),    # fwd: 515 tiles, 3 left over, fewer chunks than workgroups
    (2, 16, 300, 400, 40, 3, 2, 1),    # fwd: 532 tiles of 2 chunks
    (1, 24, 500, 700, 16, 3, 1, 0),    # fwd: 693 tiles of 3 chunks, 181 left over
    (1, 48, 200, 200, 40, 3, 2, 1),    # fewer tiles than workgroups (104 of 6 chunks): every tile is shared
    (2, 20, 90, 150, 70, 4, 4, 1),     # the same with two filter groups and a ragged last chunk
    (1, 32, 120, 260, 33, 2, 1, 0),    # 4 chunks per tile
    (1, 20, 300, 300, 32, 7, 16, 0),   # large-halo kernels (two channels per chunk), 32-filter tiles
    (1, 16, 280, 280, 48, 7, 16, 1),   # ... and 64-filter tiles
]


@pytest.mark.parametrize("case", SPLIT_CASES, ids=lambda c: "N%dC%dH%dW%dK%dk%dd%da%d" % c)
def test_conv_split_tiles(case):
    N, C, H, W, K, k, d, act = case
    _say("conv split tiles", case)
    rng = np.random.default_rng(hash(case) % 2**31 + 2)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, k, k)) * np.sqrt(2.0 / (C * k * k))).astype(np.float32)
    b = (rng.standard_normal(K) * 0.2).astype(np.float32)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, K, Ho, Wo)).astype(np.float32)
    dy[rng.random(dy.shape) < 0.5] = 0.0
    ref = oracle_conv_fwd(x, w, b, d, dsk.DSK_ACT_NONE)
    rdw, rdb, rdx = oracle_conv_bwd(x, w, b, d, dsk.DSK_ACT_NONE, dy)
    xt, wt, g = _t(x), _t(w), _t(dy)
    y = dsk.dsk_conv_fwd(xt, wt, _t(b), d, dsk.DSK_ACT_NONE)
    dx = dsk.dsk_conv_bwd_data(g, wt, d, H, W)
    dx2 = dsk.dsk_conv_bwd_data(g, wt, d, H, W)
    torch.cuda.synchronize()
    assert_close(y, ref, "conv_fwd")
    assert_close(dx, rdx, "dx")
    assert torch.equal(dx, dx2), "bwd_data is not run-to-run deterministic"


@pytest.mark.parametrize("case", CONV_CASES + [(1, 32, 200, 300, 64, 5, 2, 1), (1, 64, 150, 600, 128, 4, 8, 1)],
                         ids=lambda c: "N%dC%dH%dW%dK%dk%dd%da%d" % c)
def test_conv_workspace_is_enough_and_respected(case):
    """The three conv calls stay inside the workspace size the library asks for: a guard band
    behind it keeps its pattern (no oracle here: results are covered by the parity tests)."""
    N, C, H, W, K, k, d, act = case
    _say("conv workspace", case)
    x = torch.rand((N, C, H, W), device=DEV) - 0.5
    w = torch.randn((K, C, k, k), device=DEV) * 0.1
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = torch.randn((N, K, Ho, Wo), device=DEV)
    guard = 1 << 16
    for which in (dsk.DSK_WS_CONV_FWD, dsk.DSK_WS_CONV_BWD_DATA, dsk.DSK_WS_CONV_BWD_WEIGHT):
        need = dsk.dsk_conv_workspace_bytes(which, N, C, H, W, K, k, k, d, dsk.DSK_F32)
        need16 = (need + 15) // 16 * 16
        buf = torch.full((need16 + guard,), 0xA5, dtype=torch.uint8, device=DEV)
        ws = buf[:max(need16, 16)]
        if which == dsk.DSK_WS_CONV_FWD:
            dsk.dsk_conv_fwd(x, w, None, d, act, ws=ws)
        elif which == dsk.DSK_WS_CONV_BWD_DATA:
            dsk.dsk_conv_bwd_data(dy, w, d, H, W, ws=ws)
        else:
            dsk.dsk_conv_bwd_weight(x, dy, k, k, d, ws=ws)
        torch.cuda.synchronize()
        assert bool((buf[need16:] == 0xA5).all()), "write beyond the workspace (call %d)" % which
    # backward-data with the backward of a conv layer below (per-wave bias sums behind the weights for 1x1 kernels)
    need = dsk.dsk_conv_bwd_data_act_bias_workspace_bytes(N, C, H, W, K, k, k, d, dsk.DSK_F32, dsk.DSK_F32)
    need16 = (need + 15) // 16 * 16
    buf = torch.full((need16 + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    dsk.dsk_conv_bwd_data_act_bias(dy, w, x, d, dsk.DSK_ACT_RELU, ws=buf[:max(need16, 16)])
    torch.cuda.synchronize()
    assert bool((buf[need16:] == 0xA5).all()), "write beyond the workspace (backward-data with the layer below)"


BF16_CASES = [
    (1, 32, 50, 77, 48, 3, 2, 1),      # whole 16-channel chunks both ways
    (1, 40, 60, 92, 70, 4, 8, 1),      # ragged last chunk both ways, 64-filter tiles
    (2, 24, 40, 100, 64, 5, 2, 0),     # 25 taps
    (1, 16, 30, 45, 10, 2, 4, 2),      # backward-data has 10 < 16 channels: fp32 matrix path
    (1, 48, 70, 110, 40, 3, 16, 0),    # 3x3 taps 16 apart: weight gradient on the bf16 matrix cores too
    (2, 32, 40, 64, 33, 3, 8, 1),
    (1, 32, 60, 90, 40, 5, 4, 1),      # 25 taps 4 apart: a lane's 8 pixels come as two 8-byte LDS reads
    (1, 20, 40, 70, 36, 3, 4, 2),
    (1, 32, 44, 60, 72, 3, 2, 1),      # three filter blocks, two per workgroup; 4-byte LDS reads
    (1, 16, 60, 110, 40, 3, 18, 0),    # tile too large for four-pixel items: pixel pairs
    (1, 16, 30, 66, 33, 3, 1, 1),      # 66-column tiles: the last group of four is half outside
    (1, 32, 40, 96, 100, 3, 8, 0),     # weight gradient: four filter blocks per workgroup, 16-byte operand reads
    (1, 32, 44, 60, 130, 3, 4, 1),     # ... 8-byte operand reads, a last group of two blocks
    (1, 32, 50, 80, 24, 4, 4, 0),      # 4x4 with one filter block: a tap column per wave
    (1, 32, 40, 64, 20, 3, 2, 0),      # 3x3 with one filter block: tap columns divided between waves
    (2, 48, 70, 72, 64, 1, 8, 1),      # 1x1 layer on the bf16 matrix cores (tiles of neighbouring rows)
]


def _random_f32_case(seed):
    """A small layer drawn from the shapes the fp32 matrix-core kernels branch on: 1-7 taps a side, any tap spacing,
    channel counts below and around the chunk sizes, filter counts around the 32 / 64 blocks (a last group of at
    most 32 filters runs as a second launch), maps that end inside a tile or inside half a tile."""
    r = np.random.default_rng(2000 + seed)
    k = int(r.choice([1, 2, 3, 3, 4, 5, 5, 6, 7]))
    d = int(r.choice([1, 1, 2, 3, 4, 5, 8, 16]))
    if (k - 1) * d > 96: d = 96 // (k - 1)
    C = int(r.choice([1, 3, 4, 8, 20, 32, 33, 64, 96, 130]))
    K = int(r.choice([1, 2, 21, 32, 33, 64, 65, 80, 96, 128, 160]))
    H = (k - 1) * d + int(r.integers(1, 50))
    W = (k - 1) * d + int(r.integers(1, 140))
    return (int(r.integers(1, 3)), C, H, W, K, k, d, int(r.integers(0, 3)))


@pytest.mark.parametrize("seed", range(24))
def test_conv_f32_random_shapes(seed):
    """Forward, backward-data and weight gradient on a seeded random small layer against the oracle."""
    case = _random_f32_case(seed)
    N, C, H, W, K, k, d, act = case
    _say("conv f32 random", seed, case)
    rng = np.random.default_rng(seed)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, k, k)) * np.sqrt(2.0 / (C * k * k))).astype(np.float32)
    b = (rng.standard_normal(K) * 0.2).astype(np.float32)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, K, Ho, Wo)).astype(np.float32)
    y = dsk.dsk_conv_fwd(_t(x), _t(w), _t(b), d, act)
    dw, db = dsk.dsk_conv_bwd_weight(_t(x), _t(dy), k, k, d)
    dx = dsk.dsk_conv_bwd_data(_t(dy), _t(w), d, H, W)
    torch.cuda.synchronize()
    assert_close(y, oracle_conv_fwd(x, w, b, d, act), "y")
    rdw, rdb, rdx = oracle_conv_bwd(x, w, b, d, 0, dy)
    assert_close(dw, rdw, "dw")
    assert_close(db, rdb, "db")
    assert_close(dx, rdx, "dx")


def _random_bf16_case(seed):
    """A small layer drawn from the shapes the bf16 matrix-core kernels branch on: kernel size, tap spacing (odd,
    2, 4, 8 and their multiples), even and odd widths, channel and filter counts around the 16 / 32 / 64 block sizes,
    maps that end inside a tile."""
    r = np.random.default_rng(1000 + seed)
    k = int(r.choice([1, 3, 3, 4, 4, 5, 5]))
    d = int(r.choice([1, 2, 2, 3, 4, 4, 6, 8, 8, 12, 16]))
    if (k - 1) * d > 48: d = 48 // (k - 1)
    C = int(r.choice([16, 17, 24, 32, 33, 48, 64, 70]))
    K = int(r.choice([1, 5, 16, 31, 32, 33, 64, 65, 96, 100, 130]))
    H = (k - 1) * d + int(r.integers(1, 40))
    W = (k - 1) * d + int(r.integers(1, 80))
    if seed % 3: W += W % 2      # two in three with even width (the four- and eight-pixel staging)
    return (int(r.integers(1, 3)), C, H, W, K, k, d, int(r.integers(0, 3)))


@pytest.mark.parametrize("seed", range(24))
def test_conv_bf16_random_shapes(seed):
    """The three bf16 calls on a seeded random small layer against the oracle on the rounded inputs."""
    case = _random_bf16_case(seed)
    N, C, H, W, K, k, d, act = case
    _say("conv bf16 random", seed, case)
    rng = np.random.default_rng(seed)
    x = bf16_round(rng.uniform(-1, 1, (N, C, H, W))).astype(np.float32)
    w = bf16_round(rng.standard_normal((K, C, k, k)) * np.sqrt(2.0 / (C * k * k))).astype(np.float32)
    b = (rng.standard_normal(K) * 0.2).astype(np.float32)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = bf16_round(rng.standard_normal((N, K, Ho, Wo))).astype(np.float32)
    xb, gb = _t(x, torch.bfloat16), _t(dy, torch.bfloat16)
    y = dsk.dsk_conv_fwd(xb, _t(w), _t(b), d, act, out_dtype=torch.float32)
    dw, db = dsk.dsk_conv_bwd_weight(xb, gb, k, k, d)
    dx = dsk.dsk_conv_bwd_data(gb, _t(w), d, H, W, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert_close(y, oracle_conv_fwd(x, w, b, d, act), "y")
    rdw, rdb, rdx = oracle_conv_bwd(x, w, b, d, 0, dy)
    assert_close(dw, rdw, "dw")
    assert_close(db, rdb, "db")
    assert_close(dx, rdx, "dx")


@pytest.mark.parametrize("case", BF16_CASES, ids=lambda c: "N%dC%dH%dW%dK%dk%dd%da%d" % c)
def test_conv_bf16_variant(case):
    """bf16 activations/weights, fp32 accumulate: within 2e-2 of the fp32 oracle on the
    unrounded inputs, and within fp32 tolerance of the oracle fed the rounded inputs.
    Algo 0: bf16 matrix cores where they apply; 1: plain kernels; 2: fp32 matrix path."""
    N, C, H, W, K, k, d, act = case
    rng = np.random.default_rng(7)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, k, k)) * np.sqrt(2.0 / (C * k * k))).astype(np.float32)
    b = (rng.standard_normal(K) * 0.2).astype(np.float32)
    for algo in (0, 1, 2):
        _say("conv bf16", case, "algo", algo)
        prev = dsk.dsk_set_conv_algo(algo)
        try:
            xb = _t(x, torch.bfloat16)
            y = dsk.dsk_conv_fwd(xb, _t(w), _t(b), d, act, out_dtype=torch.float32)
            yb = dsk.dsk_conv_fwd(xb, _t(w), _t(b), d, act)
            Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
            dy = rng.standard_normal((N, K, Ho, Wo)).astype(np.float32)
            gb = _t(dy, torch.bfloat16)
            dw, db = dsk.dsk_conv_bwd_weight(xb, gb, k, k, d)
            dx = dsk.dsk_conv_bwd_data(gb, _t(w), d, H, W, out_dtype=torch.float32)
            torch.cuda.synchronize()
        finally:
            dsk.dsk_set_conv_algo(prev)
        assert yb.dtype == torch.bfloat16
        assert_close(y, oracle_conv_fwd(x, w, b, d, act), "bf16 conv vs fp32 oracle", bf16=True)
        assert_close(yb, oracle_conv_fwd(x, w, b, d, act), "bf16-out conv vs fp32 oracle", bf16=True)
        xr, wr = bf16_round(x), bf16_round(w)
        assert_close(y, oracle_conv_fwd(xr, wr, b, d, act), "bf16 conv vs oracle on rounded inputs")
        rdw, rdb, rdx = oracle_conv_bwd(xr, wr, b, d, 0, bf16_round(dy))
        assert_close(dw, rdw, "bf16 dw vs oracle on rounded inputs")
        assert_close(db, rdb, "bf16 db vs oracle on rounded inputs")
        assert_close(dx, rdx, "bf16 dx vs oracle on rounded inputs")
        fdw, fdb, fdx = oracle_conv_bwd(x, w, b, d, 0, dy)
        assert_close(dw, fdw, "bf16 dw vs fp32 oracle", bf16=True)
        assert_close(dx, fdx, "bf16 dx vs fp32 oracle", bf16=True)


# (N, C, H, W, k, d)
POOL_CASES = [
    (1, 8, 51, 51, 2, 1), (2, 5, 46, 300, 2, 2), (1, 3, 70, 530, 2, 4), (1, 4, 90, 61, 2, 8),
    (1, 6, 64, 77, 3, 2), (2, 3, 40, 280, 3, 4), (1, 2, 60, 44, 4, 3), (1, 3, 33, 20, 8, 1),
    (1, 2, 9, 9, 2, 8),   # d larger than the output
    (1, 3, 100, 300, 8, 1), (1, 2, 90, 70, 8, 2), (2, 2, 50, 280, 4, 2),   # 8x8 and 4x4 windows over several tiles
    (1, 2, 40, 50, 5, 2), (1, 2, 30, 30, 6, 1),                            # window sizes without a tiled kernel
    (1, 2, 24, 770, 2, 2), (1, 1, 20, 1026, 2, 2), (1, 2, 40, 600, 3, 2),  # pixel pairs; 128, 256 and 64 threads along a row
    (1, 2, 30, 51, 8, 1), (2, 2, 33, 47, 8, 1), (1, 3, 21, 43, 4, 1), (1, 2, 26, 45, 4, 1), (1, 1, 70, 1063, 8, 1),  # d = 1: four pixels per thread
]


@pytest.mark.parametrize("case", POOL_CASES, ids=lambda c: "N%dC%dH%dW%dk%dd%d" % c)
@pytest.mark.parametrize("ties", [False, True], ids=["random", "ties"])
def test_maxpool_fwd_bwd(case, ties):
    N, C, H, W, k, d = case
    _say("maxpool", case, "ties", ties)
    rng = np.random.default_rng(hash(case) % 2**31)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    if ties:
        x = np.maximum(x, 0.0)                    # ReLU output: many exact zeros (some -0.0)
        x[rng.random(x.shape) < 0.05] = -0.0
    ry, ram = oracle_pool_fwd(x, k, d, True)
    y, am = dsk.dsk_maxpool_fwd(_t(x), k, d)
    y_only, none = dsk.dsk_maxpool_fwd(_t(x), k, d, want_argmax=False)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, C, Ho, Wo)).astype(np.float32)
    dx = dsk.dsk_maxpool_bwd(_t(dy), am, k, d, H, W)
    torch.cuda.synchronize()
    assert none is None
    assert np.array_equal(to_np(y), ry), "max-pool values must be exact"
    assert np.array_equal(to_np(y_only), ry)
    assert np.array_equal(am.cpu().numpy().astype(np.int32), ram), "argmax must be bit-exact"
    assert_close(dx, oracle_pool_bwd(x, k, d, True, dy), "maxpool dx")


@pytest.mark.parametrize("case", POOL_CASES, ids=lambda c: "N%dC%dH%dW%dk%dd%d" % c)
def test_avgpool_fwd_bwd(case):
    N, C, H, W, k, d = case
    _say("avgpool", case)
    rng = np.random.default_rng(hash(case) % 2**31 + 5)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    ry, _ = oracle_pool_fwd(x, k, d, False)
    y = dsk.dsk_avgpool_fwd(_t(x), k, d)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, C, Ho, Wo)).astype(np.float32)
    dx = dsk.dsk_avgpool_bwd(_t(dy), k, d, H, W)
    torch.cuda.synchronize()
    assert_close(y, ry, "avgpool y")
    assert_close(dx, oracle_pool_bwd(x, k, d, False, dy), "avgpool dx")


@pytest.mark.parametrize("case", [(1, 4, 40, 150, 2, 2), (1, 3, 30, 77, 2, 1), (1, 2, 40, 280, 3, 4), (1, 2, 50, 140, 8, 2),
                                  (2, 2, 36, 90, 4, 2)], ids=lambda c: "N%dC%dH%dW%dk%dd%d" % c)
def test_pool_bf16(case):
    N, C, H, W, k, d = case
    _say("pool bf16", case)
    rng = np.random.default_rng(3)
    x = bf16_round(rng.uniform(-1, 1, (N, C, H, W)))
    ry, ram = oracle_pool_fwd(x, k, d, True)
    y, am = dsk.dsk_maxpool_fwd(_t(x, torch.bfloat16), k, d)
    torch.cuda.synchronize()
    assert y.dtype == torch.bfloat16
    assert np.array_equal(to_np(y), ry) and np.array_equal(am.cpu().numpy().astype(np.int32), ram)
    ya = dsk.dsk_avgpool_fwd(_t(x, torch.bfloat16), k, d)
    assert_close(ya, oracle_pool_fwd(x, k, d, False)[0], "bf16 avgpool", bf16=True)
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = bf16_round(rng.standard_normal((N, C, Ho, Wo)))
    dx = dsk.dsk_maxpool_bwd(_t(dy, torch.bfloat16), am, k, d, H, W)
    assert dx.dtype == torch.bfloat16
    assert_close(dx, oracle_pool_bwd(x, k, d, True, dy), "bf16 maxpool dx", bf16=True)
    dxa = dsk.dsk_avgpool_bwd(_t(dy, torch.bfloat16), k, d, H, W)
    assert_close(dxa, oracle_pool_bwd(x, k, d, False, dy), "bf16 avgpool dx", bf16=True)


@pytest.mark.parametrize("shape", [(1, 10, 40, 40), (2, 33, 37, 61), (1, 2, 50, 9), (3, 1, 5, 7)],
                         ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("frac", [0.0, 0.1, 1.0])
def test_masked_softmax_xent(shape, frac):
    N, Cls, H, W = shape
    _say("softmax", shape, frac)
    rng = np.random.default_rng(N * 1000 + Cls)
    scores = (rng.standard_normal(shape) * 4).astype(np.float32)
    labels = rng.integers(0, Cls, (N, H, W)).astype(np.int32)
    mask = (rng.random((N, H, W)) < frac).astype(np.uint8) * rng.integers(1, 255, (N, H, W)).astype(np.uint8)
    rloss, rdelta, count = oracle.masked_softmax_xent(scores, labels, mask)
    loss, delta = dsk.dsk_masked_softmax_xent(_t(scores), _t(labels, torch.int32), _t(mask, torch.uint8))
    torch.cuda.synchronize()
    assert_close(loss, np.array([rloss]), "loss")
    assert_close(delta, rdelta, "dscores")
    # errors of unchosen pixels are exactly zero
    assert not to_np(delta)[np.broadcast_to((mask == 0)[:, None], shape)].any()
    lossb, deltab = dsk.dsk_masked_softmax_xent(_t(scores), _t(labels, torch.int32), _t(mask, torch.uint8),
                                                dscores_dtype=torch.bfloat16)
    assert_close(deltab, rdelta, "bf16 dscores", bf16=True)


def test_pad_image_and_act_bwd():
    rng = np.random.default_rng(0)
    img = rng.uniform(-1, 1, (2, 3, 17, 23)).astype(np.float32)
    for n in (1, 6, 15):
        lo = n // 2
        xp = dsk.dsk_pad_image(_t(img), lo, n - 1 - lo)
        assert np.array_equal(to_np(xp), oracle.pad_image(img, n))
    xpb = dsk.dsk_pad_image(_t(img), 3, 2, out_dtype=torch.bfloat16)
    assert np.array_equal(to_np(xpb)[:, :, 3:20, 3:26], bf16_round(img).astype(np.float64))
    y = rng.uniform(-1, 1, 1000).astype(np.float32)
    y[::7] = 0.0
    g = rng.standard_normal(1000).astype(np.float32)
    for act, ref in ((1, g * (y > 0)), (2, g * (1 - y.astype(np.float64) ** 2)), (0, g)):
        gt = _t(g.copy())
        dsk.dsk_act_bwd(_t(y), gt, act)
        assert_close(gt, ref, "act_bwd %d" % act)


def test_bf16_rounding_on_the_device():
    """The kernels round fp32 to bf16 with the hardware's conversion: nearest, ties to even, as torch does on the CPU
    -- exact ties both ways, values just off a tie, the largest finite values, signed zeros and infinities."""
    vals = []
    for base in (1.0, -1.0, 3.0e38, 1.5e-20, 0.3):
        u = np.float32(base).view(np.uint32)
        u0 = np.uint32(u & 0xffff0000)
        for low in (0x0000, 0x0001, 0x7fff, 0x8000, 0x8001, 0xffff):          # bit 16 clear: a tie goes down
            vals.append(np.uint32(u0 | low))
        for low in (0x7fff, 0x8000, 0x8001):                                  # bit 16 set: a tie goes up
            vals.append(np.uint32(u0 | 0x10000 | low))
    vals += [np.float32(v).view(np.uint32) for v in (0.0, -0.0, np.inf, -np.inf, 3.3895314e38)]
    img = np.array(vals, np.uint32).view(np.float32)
    img = np.resize(img, (1, 1, 8, 8)).astype(np.float32)
    got = to_np(dsk.dsk_pad_image(_t(img), 0, 0, out_dtype=torch.bfloat16)).astype(np.float32)
    want = bf16_round(img)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("shape", [(2, 5, 12, 20), (1, 3, 9, 7), (1, 40, 64, 96), (2, 4, 50, 66)],
                         ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_act_bwd_bias(shape, dt):
    """Non-linearity backward fused with the bias gradient; planes that are and are not multiples of 4."""
    _say("act_bwd_bias", shape, dt)
    rng = np.random.default_rng(11)
    y = rng.uniform(-1, 1, shape).astype(np.float32)
    y[rng.random(shape) < 0.3] = 0.0
    g = rng.standard_normal(shape).astype(np.float32)
    bf = dt == torch.bfloat16
    if bf:
        y, g = bf16_round(y), bf16_round(g)
    for act in (1, 2, 0):
        f = (y > 0) if act == 1 else (1 - y.astype(np.float64) ** 2) if act == 2 else 1.0
        ref = g * f
        if bf:
            ref = bf16_round(ref).astype(np.float64)      # the bias gradient sums what is stored
        gt = _t(g.copy(), dt)
        db = dsk.dsk_act_bwd_bias(_t(y, dt), gt, act)
        torch.cuda.synchronize()
        assert_close(gt, ref, "act_bwd_bias dy act %d" % act, bf16=bf)
        assert_close(db, to_np(gt).sum(axis=(0, 2, 3)), "act_bwd_bias db act %d" % act)
        gt2 = _t(g.copy(), dt)
        dsk.dsk_act_bwd(_t(y, dt), gt2, act)
        assert torch.equal(gt, gt2)


def test_launch_errors_are_reported_not_raised_as_faults():
    """Shapes the kernels cannot take are refused with a status before any launch."""
    x = torch.zeros((1, 2, 8, 8), device=DEV)
    w = torch.zeros((3, 2, 3, 3), device=DEV)
    with pytest.raises(dsk.DskError) as e:
        dsk.dsk_conv_fwd(x, w, None, 4)
    assert e.value.status == dsk.DSK_ESHAPE
    with pytest.raises(dsk.DskError) as e:
        dsk.dsk_maxpool_fwd(x, 2, 8)
    assert e.value.status == dsk.DSK_ESHAPE


# odd widths and spacings: 16-byte accesses at any alignment, partial groups at the row ends
WALK_CASES = [(1, 3, 37, 53, 2, 3), (2, 2, 41, 67, 3, 1), (1, 2, 150, 39, 2, 5), (1, 1, 300, 21, 3, 7), (1, 2, 19, 5, 2, 1),
              (1, 2, 200, 130, 2, 2), (1, 1, 33, 1030, 3, 6)]


@pytest.mark.parametrize("case", POOL_CASES[:7] + WALK_CASES, ids=lambda c: "N%dC%dH%dW%dk%dd%d" % c)
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("is_max", [True, False], ids=["max", "avg"])
def test_pool_bwd_act_bias(case, dt, is_max):
    """Pool gradient + non-linearity backward of the layer in front + its bias gradient in one call, against
    the oracle's pool gradient times act'(y) written out; also the pool kernels themselves on odd shapes."""
    N, C, H, W, k, d = case
    _say("pool_bwd_act_bias", case, dt, is_max)
    bf = dt == torch.bfloat16
    rng = np.random.default_rng(hash(case) % 2**31 + 9)
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    x[rng.random(x.shape) < 0.3] = 0.0          # closed gates of the ReLU in front of the pool
    Ho, Wo = H - (k - 1) * d, W - (k - 1) * d
    dy = rng.standard_normal((N, C, Ho, Wo)).astype(np.float32)
    if bf:
        x, dy = bf16_round(x), bf16_round(dy)
    ry, ram = oracle_pool_fwd(x, k, d, is_max)
    rdx = oracle_pool_bwd(x, k, d, is_max, dy)
    xt, gt = _t(x, dt), _t(dy, dt)
    if is_max:
        y, am = dsk.dsk_maxpool_fwd(xt, k, d)
        assert np.array_equal(to_np(y), ry) and np.array_equal(am.cpu().numpy().astype(np.int32), ram)
        plain = dsk.dsk_maxpool_bwd(gt, am, k, d, H, W)
    else:
        y, am = dsk.dsk_avgpool_fwd(xt, k, d), None
        assert_close(y, ry, "avgpool y", bf16=bf)
        plain = dsk.dsk_avgpool_bwd(gt, k, d, H, W)
    assert_close(plain, rdx, "pool dx", bf16=bf)
    kind = dsk.DSK_MAXPOOL if is_max else dsk.DSK_AVGPOOL
    for act in (1, 2, 0):
        f = (x > 0) if act == 1 else (1 - x.astype(np.float64) ** 2) if act == 2 else 1.0
        want = rdx * f
        dx, db = dsk.dsk_pool_bwd_act_bias(kind, gt, am, xt, k, d, H, W, act)
        torch.cuda.synchronize()
        assert_close(dx, want, "fused dx act %d" % act, bf16=bf)
        assert_close(db, to_np(dx).sum(axis=(0, 2, 3)), "fused db act %d (sum of the stored map)" % act)
        if not bf:
            assert_close(db, want.sum(axis=(0, 2, 3)), "fused db act %d" % act)
        # the same as the two separate calls, bit for bit
        sep = plain.clone()
        db2 = dsk.dsk_act_bwd_bias(xt, sep, act)
        assert torch.equal(dx, sep) or (bf and act == 2)      # bf16 tanh: the separate form rounds twice
        if not (bf and act == 2):
            assert_close(db, to_np(db2), "db of the two forms")
