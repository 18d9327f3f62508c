"""GPU parity: every entry point of libstanza against the CPU checker, element by element, on seeded
inputs at sizes the checker finishes in seconds and that span several tiles plus ragged tails."""
import copy

import numpy as np
import pytest
import torch

import workloads as wl_mod
from gpu_util import TOL_F32, dev, host, param_update_err, rel_err
from oracle import ConvGeom, PoolGeom
from oracle import network as onet

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    a.load()
    assert torch.cuda.is_available()
    return a


def rng(seed):
    return np.random.default_rng(seed)


# (N,H,W,C,K,R,S,stride,pad): vector and scalar loader paths, every tile shape, ragged M/N/K tails,
# strides 2 and 4, filters 1/3/5/7/11, enough pixels for several reduction slices in the filter gradient
CONV_CASES = [
    (2, 19, 17, 8, 24, 3, 3, 1, 1),
    (2, 16, 16, 3, 16, 3, 3, 1, 1),        # C = 3: scalar gather
    (3, 13, 13, 16, 72, 3, 3, 1, 1),       # K not a multiple of the tile
    (2, 14, 14, 64, 160, 3, 3, 1, 1),      # two 128-wide column tiles, ragged
    (1, 56, 56, 64, 64, 3, 3, 1, 1),       # 64-wide output, many row tiles
    (2, 28, 28, 20, 12, 1, 1, 1, 0),       # pointwise
    (2, 15, 15, 24, 40, 1, 1, 2, 0),       # strided pointwise (projection shortcut)
    (2, 29, 29, 16, 32, 3, 3, 2, 1),       # strided 3x3
    (2, 35, 33, 3, 16, 7, 7, 2, 3),        # stem
    (2, 27, 27, 12, 20, 5, 5, 1, 2),
    (1, 67, 67, 3, 24, 11, 11, 4, 2),
    (2, 20, 19, 8, 16, 5, 5, 3, 2),        # stride 3: nine stride classes of the data gradient, in three launches, odd class sizes
    (2, 9, 9, 6, 10, 3, 3, 1, 0),          # C, K not multiples of 4
    (4, 1, 1, 300, 70, 1, 1, 1, 0),        # an FC layer as a convolution
]


def _ids(c):
    return "n{}h{}w{}c{}k{}r{}s{}st{}p{}".format(*c)


@pytest.mark.parametrize("case", CONV_CASES, ids=_ids)
def test_conv_forward(api, o32, case):
    N, H, W, C, K, R, S, st, pad = case
    g = ConvGeom(N, H, W, C, K, R, S, st, pad)
    r = rng(1)
    x = r.standard_normal((N, H, W, C), dtype=np.float32)
    w = (r.standard_normal((K, R, S, C), dtype=np.float32) / np.sqrt(R * S * C)).astype(np.float32)
    b = r.standard_normal(K, dtype=np.float32)
    for relu in (False, True):
        ref = o32.conv_fwd(g, x, w, b, relu=relu)
        d = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS | (api.CONV_RELU if relu else 0))
        y = torch.full(ref.shape, float("nan"), device="cuda:0")
        api.stanza_conv_fwd(d, dev(x), dev(w), dev(b), y)
        e = rel_err(host(y), ref)
        assert e < TOL_F32, (case, relu, e)
    # no bias
    d = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, 0)
    y = torch.full(ref.shape, float("nan"), device="cuda:0")
    api.stanza_conv_fwd(d, dev(x), dev(w), None, y)
    assert rel_err(host(y), o32.conv_fwd(g, x, w, None)) < TOL_F32


@pytest.mark.parametrize("case", CONV_CASES, ids=_ids)
def test_conv_backward_data(api, o32, case):
    N, H, W, C, K, R, S, st, pad = case
    g = ConvGeom(N, H, W, C, K, R, S, st, pad)
    r = rng(2)
    w = (r.standard_normal((K, R, S, C), dtype=np.float32) / np.sqrt(R * S * K)).astype(np.float32)
    dy = r.standard_normal((N, g.Ho, g.Wo, K), dtype=np.float32)
    yfwd = r.standard_normal(dy.shape, dtype=np.float32)        # stands for the forward output (sign pattern)
    xin = r.standard_normal((N, H, W, C), dtype=np.float32)     # stands for the layer input (sign pattern)
    prev = r.standard_normal((N, H, W, C), dtype=np.float32)
    ref_plain = o32.conv_bwd_data(g, dy, w)
    d = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS)
    dx = torch.full(ref_plain.shape, float("nan"), device="cuda:0")
    api.stanza_conv_bwd_data(d, dev(dy), None, dev(w), None, dx)
    assert rel_err(host(dx), ref_plain) < TOL_F32
    # gated dy, accumulate onto prev, gate the result by the layer input's sign
    ref = o32.conv_bwd_data(g, o32.relu_bwd(dy, yfwd), w)
    ref = o32.relu_bwd((ref.astype(np.float64) + prev).astype(np.float32), xin)
    d2 = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_RELU | api.CONV_ACCUM)
    dx2 = dev(prev)
    api.stanza_conv_bwd_data(d2, dev(dy), dev(yfwd), dev(w), dev(xin), dx2)
    assert rel_err(host(dx2), ref) < TOL_F32
    np.testing.assert_array_equal(host(dx2) == 0, ref == 0)


@pytest.mark.parametrize("case", CONV_CASES, ids=_ids)
def test_conv_backward_weight(api, o32, case):
    N, H, W, C, K, R, S, st, pad = case
    g = ConvGeom(N, H, W, C, K, R, S, st, pad)
    r = rng(3)
    x = r.standard_normal((N, H, W, C), dtype=np.float32)
    dy = r.standard_normal((N, g.Ho, g.Wo, K), dtype=np.float32)
    yfwd = r.standard_normal(dy.shape, dtype=np.float32)
    for gate in (False, True):
        dye = o32.relu_bwd(dy, yfwd) if gate else dy
        ref_dw, ref_db = o32.conv_bwd_weight(g, x, dye)
        d = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS | (api.CONV_RELU if gate else 0))
        ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(d, 2)), dtype=torch.uint8, device="cuda:0")
        dw = torch.full(ref_dw.shape, float("nan"), device="cuda:0")
        db = torch.full(ref_db.shape, float("nan"), device="cuda:0")
        xd, dyd, yd = dev(x), dev(dy), dev(yfwd) if gate else None
        api.stanza_conv_bwd_weight(d, xd, dyd, yd, dw, db, ws)
        assert rel_err(host(dw), ref_dw) < TOL_F32, (case, gate)
        assert rel_err(host(db), ref_db) < TOL_F32, (case, gate)
        # run-to-run bit reproducibility (fixed-order reductions, no float atomics)
        dw2, db2 = torch.empty_like(dw), torch.empty_like(db)
        api.stanza_conv_bwd_weight(d, xd, dyd, yd, dw2, db2, ws)
        assert torch.equal(dw, dw2) and torch.equal(db, db2)


# 3x3 / stride 1 / pad 1 layers with at least 48 channels on both sides take the nine-tap filter-gradient kernel: strips of
# 28 pixels (56, 112), one strip per row (28, 17, 30), ragged strips (31 = 16 + 15, 33 = 17 + 16), several rows per stage
# (14: 2 rows, 7: 3 rows with a last block of 1, 5: 4 rows + 1, 3, 1), channel counts that do not fill the 64-wide tiles
# (52, 68, 100, 132), one image and many, slices that start in the middle of a column strip
NINE_TAP_CASES = [
    (2, 56, 56, 64, 64), (1, 28, 28, 128, 64), (3, 14, 14, 64, 128), (5, 7, 7, 64, 64), (2, 5, 5, 48, 52), (1, 3, 3, 64, 64),
    (4, 1, 1, 64, 64), (2, 31, 31, 52, 68), (1, 33, 17, 68, 52), (2, 17, 33, 100, 48), (1, 30, 30, 64, 132), (2, 9, 60, 48, 48),
    (7, 12, 10, 56, 60), (1, 112, 112, 64, 64), (16, 14, 14, 256, 192), (3, 8, 8, 512, 64),
    # image layers (4 input channels: an RGB image padded to 4) take the 36-column form of the kernel: strips of 56 pixels
    # (224 = 4 x 56), one short strip (32), ragged strips (61 = 31 + 30, 115 = 39 + 38 + 38), K that does not fill a tile
    (2, 32, 32, 4, 16), (1, 60, 61, 4, 64), (3, 9, 115, 4, 68), (2, 224, 224, 4, 64), (5, 3, 2, 4, 8), (1, 1, 1, 4, 132),
]


@pytest.mark.parametrize("case", NINE_TAP_CASES, ids=lambda c: "n{}h{}w{}c{}k{}".format(*c))
def test_conv_backward_weight_nine_tap_kernel(api, o32, case):
    N, H, W, C, K = case
    g = ConvGeom(N, H, W, C, K, 3, 3, 1, 1)
    r = rng(31)
    x = r.standard_normal((N, H, W, C), dtype=np.float32)
    dy = r.standard_normal((N, H, W, K), dtype=np.float32)
    yfwd = r.standard_normal(dy.shape, dtype=np.float32)
    # with CONV_NINE_TAP (on the small and odd-sized images of this list the library would otherwise take the implicit GEMM), and
    # once as the library chooses
    for gate, bias, force in ((False, True, True), (True, True, True), (False, False, True), (True, True, False)):
        dye = o32.relu_bwd(dy, yfwd) if gate else dy
        ref_dw, ref_db = o32.conv_bwd_weight(g, x, dye)
        d = api.conv_desc(N, H, W, C, K, 3, 3, 1, 1, api.F32,
                          (api.CONV_BIAS if bias else 0) | (api.CONV_RELU if gate else 0) | (api.CONV_NINE_TAP if force else 0))
        ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(d, 2)), dtype=torch.uint8, device="cuda:0")
        ws.fill_(0xFF)                                               # NaN bit patterns: every partial sum that is read was written
        dw = torch.full(ref_dw.shape, float("nan"), device="cuda:0")
        db = torch.full(ref_db.shape, float("nan"), device="cuda:0") if bias else None
        xd, dyd, yd = dev(x), dev(dy), dev(yfwd) if gate else None
        api.stanza_conv_bwd_weight(d, xd, dyd, yd, dw, db, ws)
        assert rel_err(host(dw), ref_dw) < TOL_F32, (case, gate, bias)
        if bias:
            assert rel_err(host(db), ref_db) < TOL_F32, (case, gate)
        dw2 = torch.empty_like(dw)                                   # fixed-order reductions: run-to-run identical
        api.stanza_conv_bwd_weight(d, xd, dyd, yd, dw2, torch.empty_like(db) if bias else None, ws)
        assert torch.equal(dw, dw2)


# forward pass of an image layer (4 input channels, 3x3 / stride 1 / pad 1): the kernel that keeps the filter in registers.
# Stages of 4 rows x 32 pixels: whole (224, 32), ragged in both directions (61 x 60, 9 x 115, 3 x 2, 1 x 1), K below, at and
# above one 64-channel tile and not a multiple of 16
@pytest.mark.parametrize("case", [(2, 32, 32, 16), (1, 60, 61, 64), (3, 9, 115, 68), (1, 224, 224, 64), (5, 3, 2, 8), (2, 1, 1, 132), (2, 17, 33, 20)],
                         ids=lambda c: "n{}h{}w{}k{}".format(*c))
def test_conv_forward_image_layer_kernel(api, o32, case):
    N, H, W, K = case
    g = ConvGeom(N, H, W, 4, K, 3, 3, 1, 1)
    r = rng(32)
    x = r.standard_normal((N, H, W, 4), dtype=np.float32)
    w = (r.standard_normal((K, 3, 3, 4), dtype=np.float32) / 6).astype(np.float32)
    b = r.standard_normal(K, dtype=np.float32)
    for bias, relu in ((True, True), (False, False), (True, False)):
        ref = o32.conv_fwd(g, x, w, b if bias else None, relu=relu)
        d = api.conv_desc(N, H, W, 4, K, 3, 3, 1, 1, api.F32, (api.CONV_BIAS if bias else 0) | (api.CONV_RELU if relu else 0))
        y = torch.full(ref.shape, float("nan"), device="cuda:0")
        api.stanza_conv_fwd(d, dev(x), dev(w), dev(b) if bias else None, y)
        assert rel_err(host(y), ref) < TOL_F32, (case, bias, relu)
        if relu:
            np.testing.assert_array_equal(host(y) == 0, ref == 0)


# shapes whose forward / backward-data launches are cut into reduction slices when a workspace is given: few tiles (all
# of them sliced), and several rounds of tiles with a partly filled last round (only the tail sliced)
SLICED_CASES = [
    (2, 14, 14, 64, 160, 3, 3, 1, 1),
    (4, 1, 1, 300, 70, 1, 1, 1, 0),
    (8, 1, 1, 2048, 256, 1, 1, 1, 0),
    (2, 27, 27, 12, 20, 5, 5, 1, 2),
    (16, 56, 56, 32, 128, 3, 3, 1, 1),       # 784 tiles of 64x128: three full rounds + a tail of 16
    (9, 56, 56, 256, 64, 3, 3, 1, 1),        # 64-wide tiles
    (2, 29, 29, 16, 32, 3, 3, 2, 1),         # strided: general gather path
]


@pytest.mark.parametrize("case", SLICED_CASES, ids=_ids)
def test_conv_sliced_launches(api, o32, case):
    N, H, W, C, K, R, S, st, pad = case
    g = ConvGeom(N, H, W, C, K, R, S, st, pad)
    r = rng(4)
    x = r.standard_normal((N, H, W, C), dtype=np.float32)
    w = (r.standard_normal((K, R, S, C), dtype=np.float32) / np.sqrt(R * S * C)).astype(np.float32)
    b = r.standard_normal(K, dtype=np.float32)
    dy = r.standard_normal((N, g.Ho, g.Wo, K), dtype=np.float32)
    yfwd = r.standard_normal(dy.shape, dtype=np.float32)
    prev = r.standard_normal((N, H, W, C), dtype=np.float32)
    d = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS | api.CONV_RELU)
    need = [api.stanza_conv_workspace_bytes(d, k) for k in (0, 1)]
    assert max(need) > 0, "this shape is expected to be sliced"
    ws = torch.empty(max(need + [16]), dtype=torch.uint8, device="cuda:0")
    xd, wd, bd, dyd = dev(x), dev(w), dev(b), dev(dy)
    if need[0]:
        ref = o32.conv_fwd(g, x, w, b, relu=True)
        y = torch.full(ref.shape, float("nan"), device="cuda:0")
        api.stanza_conv_fwd(d, xd, wd, bd, y, ws)
        assert rel_err(host(y), ref) < TOL_F32
        y2 = torch.full(ref.shape, float("nan"), device="cuda:0")
        api.stanza_conv_fwd(d, xd, wd, bd, y2, ws)
        assert torch.equal(y, y2)
        # a workspace that is too small is not an error: the launch is simply not cut
        y3 = torch.full(ref.shape, float("nan"), device="cuda:0")
        api.stanza_conv_fwd(d, xd, wd, bd, y3, ws[:256])
        assert rel_err(host(y3), ref) < TOL_F32
    if need[1]:
        ref = o32.conv_bwd_data(g, o32.relu_bwd(dy, yfwd), w)
        ref = o32.relu_bwd((ref.astype(np.float64) + prev).astype(np.float32), x)
        d2 = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_RELU | api.CONV_ACCUM)
        dx = dev(prev)
        api.stanza_conv_bwd_data(d2, dyd, dev(yfwd), wd, xd, dx, ws)
        assert rel_err(host(dx), ref) < TOL_F32
        np.testing.assert_array_equal(host(dx) == 0, ref == 0)
        d3 = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, 0)
        dx3 = torch.full(prev.shape, float("nan"), device="cuda:0")
        api.stanza_conv_bwd_data(d3, dyd, None, wd, None, dx3, ws)
        assert rel_err(host(dx3), o32.conv_bwd_data(g, dy, w)) < TOL_F32


POOL_CASES = [(2, 16, 16, 8, 2, 2, 0, True), (2, 15, 13, 12, 3, 2, 0, True), (2, 14, 15, 16, 3, 2, 1, True),
              (1, 9, 9, 3, 2, 2, 0, True), (1, 11, 11, 5, 3, 2, 1, False), (3, 8, 8, 4, 2, 2, 0, False),
              (1, 12, 12, 4, 3, 1, 1, True),
              # non-overlapping windows over whole images: the one-thread-per-output kernels
              (2, 12, 18, 24, 3, 3, 0, True), (5, 64, 64, 128, 2, 2, 0, True), (2, 20, 12, 36, 2, 2, 0, False)]


@pytest.mark.parametrize("case", POOL_CASES, ids=lambda c: "n{}h{}w{}c{}win{}s{}p{}r{}".format(*c))
def test_pool_relu(api, o32, case):
    N, H, W, C, win, st, pad, relu = case
    g = PoolGeom(N, H, W, C, win, st, pad, relu)
    r = rng(4)
    x = r.standard_normal((N, H, W, C), dtype=np.float32)
    x[0, :4, :4, :] = 0.25                     # ties
    x[0, 4:8, :, 0] = -np.abs(x[0, 4:8, :, 0]) - 1   # all-negative windows
    y_ref, am_ref = o32.pool_relu_fwd(g, x)
    d = api.pool_desc(N, H, W, C, win, st, pad, relu)
    y = torch.full(y_ref.shape, float("nan"), device="cuda:0")
    am = torch.full(y_ref.shape, 255, dtype=torch.uint8, device="cuda:0")
    api.stanza_pool_relu_fwd(d, dev(x), y, am)
    np.testing.assert_array_equal(host(y), y_ref)            # a max is exact
    np.testing.assert_array_equal(host(am), am_ref)          # index work is bit-exact
    dy = r.standard_normal(y_ref.shape, dtype=np.float32)
    dx_ref = o32.pool_relu_bwd(g, dy, y_ref, am_ref)
    dx = torch.full(x.shape, float("nan"), device="cuda:0")
    api.stanza_pool_relu_bwd(d, dev(dy), dev(y_ref), dev(am_ref), dx)
    assert rel_err(host(dx), dx_ref) < TOL_F32
    np.testing.assert_array_equal(host(dx) == 0, dx_ref == 0)


def test_add_relu_and_gap(api, o32):
    r = rng(5)
    for shape in ((2, 7, 7, 12), (1, 3, 3, 5), (3, 14, 14, 64)):
        a, b = r.standard_normal(shape, dtype=np.float32), r.standard_normal(shape, dtype=np.float32)
        o_ref = o32.add_relu_fwd(a, b)
        o = torch.full(shape, float("nan"), device="cuda:0")
        api.stanza_add_relu_fwd(dev(a), dev(b), o)
        assert rel_err(host(o), o_ref) < 1e-6
        dout = r.standard_normal(shape, dtype=np.float32)
        dz = torch.full(shape, float("nan"), device="cuda:0")
        api.stanza_add_relu_bwd(dev(dout), dev(o_ref), dz)
        np.testing.assert_array_equal(host(dz), o32.relu_bwd(dout, o_ref))
        f_ref = o32.gap_fwd(a)
        f = torch.full((shape[0], shape[3]), float("nan"), device="cuda:0")
        api.stanza_gap_fwd(dev(a), f)
        assert rel_err(host(f), f_ref.reshape(shape[0], shape[3])) < 1e-5
        df = r.standard_normal((shape[0], shape[3]), dtype=np.float32)
        dx = torch.full(shape, float("nan"), device="cuda:0")
        api.stanza_gap_bwd(dev(df), dx)
        assert rel_err(host(dx), o32.gap_bwd(df, shape)) < 1e-6


FC_CASES = [([2048, 256, 10], 8), ([520, 136, 50], 96), ([64, 1000], 130), ([300, 128, 64, 12], 33)]


@pytest.mark.parametrize("dims,n", FC_CASES, ids=lambda v: str(v).replace(" ", ""))
def test_fc_step(api, o32, dims, n):
    from paper_1812_10624_amd.netrun import FcWorker
    r = rng(6)
    feats = np.maximum(r.standard_normal((n, dims[0]), dtype=np.float32), 0)
    labels = r.integers(0, dims[-1], n).astype(np.int32)
    params = [((r.standard_normal((dims[i + 1], dims[i]), dtype=np.float32) * np.sqrt(2.0 / dims[i])).astype(np.float32),
               (r.standard_normal(dims[i + 1], dtype=np.float32) * 0.1).astype(np.float32)) for i in range(len(dims) - 1)]
    mom = [((r.standard_normal(w.shape, dtype=np.float32) * 1e-2).astype(np.float32),
            (r.standard_normal(b.shape, dtype=np.float32) * 1e-2).astype(np.float32)) for w, b in params]
    lr, m, wd = 0.05, 0.9, 1e-3
    p_ref, m_ref = copy.deepcopy(params), copy.deepcopy(mom)
    ref = onet.fc_step(o32, feats, labels, p_ref, m_ref, lr, m, wd)
    gp = [(dev(w), dev(b)) for w, b in params]
    gm = [(dev(w), dev(b)) for w, b in mom]
    fw = FcWorker(dims, n, gp, gm, lr, m, wd)
    fw.step(dev(feats), dev(labels))
    assert abs(float(host(fw.loss)[0]) - ref["loss"]) < 1e-5 * max(1.0, abs(ref["loss"]))
    np.testing.assert_array_equal(host(fw.pred), ref["pred"])
    assert rel_err(host(fw.dfeats), ref["dfeats"]) < TOL_F32
    for li in range(len(params)):
        for which in range(2):
            got, want, before = host(gp[li][which]), p_ref[li][which], params[li][which]
            # the update itself (new - old), which is what the step computes, after the one rounding of the stored parameter
            assert param_update_err(got, want, before) < TOL_F32, (li, which)
            assert rel_err(got, want) < 1e-5
            assert rel_err(host(gm[li][which]), m_ref[li][which]) < TOL_F32, (li, which)


@pytest.mark.parametrize("K", [1, 2, 3, 8, 16])
def test_ps_aggregate(api, o32, K):
    numels = [1000, 10, 4097, 2048 * 3 + 1, 2048, 64 * 3 * 3 * 64, 3]
    ws_, vs_, gs_ = wl_mod.gen_ps_case(numels, K, seed=11)
    w_ref, v_ref = copy.deepcopy(ws_), copy.deepcopy(vs_)
    for t in range(len(numels)):
        o32.ps_aggregate(w_ref[t], v_ref[t], gs_[t], 1.0, 0.01, 0.9, 5e-4)
    gw, gv = [dev(a) for a in ws_], [dev(a) for a in vs_]
    gg = [[dev(gs_[t][k]) for t in range(len(numels))] for k in range(K)]
    ws = torch.empty(api.stanza_ps_workspace_bytes(len(numels), K), dtype=torch.uint8, device="cuda:0")
    api.stanza_ps_aggregate(gw, gv, gg, 1.0, 0.01, 0.9, 5e-4, ws)
    for t in range(len(numels)):
        assert rel_err(host(gv[t]), v_ref[t]) < 1e-5, t
        assert rel_err(host(gw[t]), w_ref[t]) < 1e-6, t
    # second step through the planned entry point, other scale
    plan = api.stanza_ps_plan(gw, gv, gg, ws)
    api.stanza_ps_aggregate_planned(plan, 1.0 / K, 0.02, 0.5, 0.0, ws)
    for t in range(len(numels)):
        o32.ps_aggregate(w_ref[t], v_ref[t], gs_[t], 1.0 / K, 0.02, 0.5, 0.0)
        assert rel_err(host(gv[t]), v_ref[t]) < 1e-5, t
        assert rel_err(host(gw[t]), w_ref[t]) < 1e-6, t


@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 6, 8, 11, 16, 19])
def test_ps_aggregate_recursive_doubling(api, K):
    """Shards added in the order of the all-reduce of Sec. 4.1.2.  The sum itself is compared BIT-EXACT: with
    momentum 0, weight decay 0, scale 1 the velocity written is the sum (0*v + (1*s + 0*w) is exact), and both sides
    add float32 values in the same tree.  Then a full update at tolerance."""
    from oracle import allreduce as oar
    numels = [1000, 10, 4097, 4096 * 2 + 5, 4096, 3]
    ws_, vs_, gs_ = wl_mod.gen_ps_case(numels, K, seed=23)
    # make the order visible: large cancelling terms in some shards
    for t in range(len(numels)):
        for k in range(K):
            gs_[t][k][::7] *= np.float32(1e4 * (-1) ** k)
    gw, gv = [dev(a) for a in ws_], [dev(a) for a in vs_]
    gg = [[dev(gs_[t][k]) for t in range(len(numels))] for k in range(K)]
    ws = torch.empty(api.stanza_ps_workspace_bytes(len(numels), K), dtype=torch.uint8, device="cuda:0")
    api.stanza_ps_aggregate_ordered(api.SUM_RECURSIVE_DOUBLING, gw, gv, gg, 1.0, 1.0, 0.0, 0.0, ws)
    for t in range(len(numels)):
        want = oar.recursive_doubling_allreduce(gs_[t])[0][0]
        got = host(gv[t])
        np.testing.assert_array_equal(got, want, err_msg=f"tensor {t}")
        np.testing.assert_array_equal(host(gw[t]), ws_[t] - want)
    # full update through the planned entry point from fresh state
    gw, gv = [dev(a) for a in ws_], [dev(a) for a in vs_]
    plan = api.stanza_ps_plan(gw, gv, gg, ws)
    api.stanza_ps_aggregate_ordered_planned(api.SUM_RECURSIVE_DOUBLING, plan, 1.0 / K, 0.02, 0.9, 5e-4, ws)
    for t in range(len(numels)):
        w_ref, v_ref = ws_[t].copy(), vs_[t].copy()
        oar.ps_aggregate_rd(w_ref, v_ref, gs_[t], 1.0 / K, 0.02, 0.9, 5e-4)
        assert rel_err(host(gv[t]), v_ref) < 1e-5, t
        assert rel_err(host(gw[t]), w_ref) < 1e-6, t
    # index order through the same entry point equals stanza_ps_aggregate bit for bit
    a_w, a_v = [dev(a) for a in ws_], [dev(a) for a in vs_]
    b_w, b_v = [dev(a) for a in ws_], [dev(a) for a in vs_]
    api.stanza_ps_aggregate_ordered(api.SUM_INDEX_ORDER, a_w, a_v, gg, 1.0, 0.01, 0.9, 5e-4, ws)
    api.stanza_ps_aggregate(b_w, b_v, gg, 1.0, 0.01, 0.9, 5e-4, ws)
    for t in range(len(numels)):
        np.testing.assert_array_equal(host(a_w[t]), host(b_w[t]))
        np.testing.assert_array_equal(host(a_v[t]), host(b_v[t]))


def _gpu_params(params):
    return {n: (dev(w), dev(b)) for n, (w, b) in params.items()}


@pytest.mark.parametrize("name", ["tiny", "minires", "minimlp", "mlp"])
def test_layerwise_and_split_step(api, o32, name):
    """Gate 1: every op of the stack fed the checker's own inputs for that op, forward and backward.
    Gate 2: the whole layer-separated step (K workers -> FC worker -> workers -> aggregation) and its
    parameter updates."""
    from paper_1812_10624_amd.netrun import Aggregator, ConvWorker, FcWorker
    wl = wl_mod.get_workload(name)
    K, B, seed = wl.K, wl.B, 0
    imgs = [wl_mod.gen_images(wl, seed, k) for k in range(K)]
    labels = wl_mod.gen_labels(wl, seed)
    cp = wl_mod.gen_conv_params(wl, seed)
    fp = wl_mod.gen_fc_params(wl, seed)
    cm = {n: (np.zeros_like(w), np.zeros_like(b)) for n, (w, b) in cp.items()}
    fm = [(np.zeros_like(w), np.zeros_like(b)) for w, b in fp]
    cp_ref, cm_ref, fp_ref, fm_ref = (copy.deepcopy(a) for a in (cp, cm, fp, fm))
    ref = onet.split_step(o32, wl.ops, imgs, labels, cp_ref, cm_ref, fp_ref, fm_ref, wl.lr, wl.momentum, wl.weight_decay, keep=True)

    # ---- gate 1: layer-wise on worker 0, inputs taken from the checker
    bufs, bgr = ref["bufs"][0], ref["buf_grads"][0]
    gpar = _gpu_params(cp)
    for op in wl.ops:
        if op["op"] == "conv":
            x = bufs[op["src"]]
            n, h, w, c = x.shape
            d = api.conv_desc(n, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"], api.F32,
                              api.CONV_BIAS | (api.CONV_RELU if op["relu"] else 0))
            y = torch.empty(bufs[op["dst"]].shape, device="cuda:0")
            api.stanza_conv_fwd(d, dev(x), gpar[op["name"]][0], gpar[op["name"]][1], y)
            assert rel_err(host(y), bufs[op["dst"]]) < TOL_F32, op
        elif op["op"] == "pool":
            x = bufs[op["src"]]
            n, h, w, c = x.shape
            d = api.pool_desc(n, h, w, c, op["win"], op["stride"], op["pad"], op["relu"])
            y = torch.empty(bufs[op["dst"]].shape, device="cuda:0")
            am = torch.empty(bufs[op["dst"]].shape, dtype=torch.uint8, device="cuda:0")
            api.stanza_pool_relu_fwd(d, dev(x), y, am)
            np.testing.assert_array_equal(host(y), bufs[op["dst"]])
            np.testing.assert_array_equal(host(am), bufs[op["dst"] + "#argmax"])

    # ---- gate 2: the whole step on the GPU
    gfp = [(dev(w), dev(b)) for w, b in fp]
    gfm = [(dev(w), dev(b)) for w, b in fm]
    gcm = _gpu_params(cm)
    workers = [ConvWorker(wl.ops, wl.image, B, gpar) for _ in range(K)]
    fcw = FcWorker(wl.fc_dims, K * B, gfp, gfm, wl.lr, wl.momentum, wl.weight_decay)
    feats = torch.empty((K * B, wl.fc_dims[0]), device="cuda:0")
    for k, wk in enumerate(workers):
        feats[k * B:(k + 1) * B].copy_(wk.forward(dev(imgs[k])).view(B, -1))
    assert rel_err(host(feats), ref["feats"]) < TOL_F32
    dfeats = fcw.step(feats, dev(labels))
    assert abs(float(host(fcw.loss)[0]) - ref["loss"]) < 1e-5 * max(1.0, abs(ref["loss"]))
    np.testing.assert_array_equal(host(fcw.pred), ref["pred"])
    if name == "mlp":
        # 1024 x 4096 hidden pre-activations: a handful lie within rounding of zero, where the two sides may take the
        # ReLU gate differently and a whole row of the handed-back gradient moves by one term of its sum.  Rows whose
        # pre-activations all keep a margin from zero are unique and held to the tolerance; the others to direction.
        z1 = ref["feats"].astype(np.float64) @ fp[0][0].astype(np.float64).T + fp[0][1].astype(np.float64)
        clear = np.abs(z1).min(axis=1) > 1e-5
        assert clear.sum() > 0.9 * len(clear)
        got = host(dfeats)
        assert rel_err(got[clear], ref["dfeats"][clear]) < TOL_F32
        for i in np.nonzero(~clear)[0]:
            a, b = got[i].astype(np.float64), ref["dfeats"][i].astype(np.float64)
            assert a @ b / (np.linalg.norm(a) * np.linalg.norm(b)) > 0.99, i
        dfeats.copy_(dev(ref["dfeats"]))      # the workers continue from the checker's gradient
    else:
        assert rel_err(host(dfeats), ref["dfeats"]) < TOL_F32
    for k, wk in enumerate(workers):
        wk.backward(dfeats[k * B:(k + 1) * B])
        for nme in cp:
            assert rel_err(host(wk.grads[nme][0]), ref["worker_grads"][k][nme][0]) < TOL_F32, (k, nme)
            assert rel_err(host(wk.grads[nme][1]), ref["worker_grads"][k][nme][1]) < TOL_F32, (k, nme)
    names = list(cp)
    agg = Aggregator([gpar[n][i] for n in names for i in range(2)], [gcm[n][i] for n in names for i in range(2)],
                     [[wk.grads[n][i] for n in names for i in range(2)] for wk in workers])
    agg.step(1.0, wl.lr, wl.momentum, wl.weight_decay)
    # the momentum buffer is the update divided by lr: compare it at gradient accuracy, the parameter itself tightly
    for nme in names:
        for i in range(2):
            assert rel_err(host(gcm[nme][i]), cm_ref[nme][i]) < TOL_F32, (nme, i)
            assert rel_err(host(gpar[nme][i]), cp_ref[nme][i]) < 1e-5, (nme, i)
            assert not np.array_equal(host(gpar[nme][i]), cp[nme][i])
    for li in range(len(fp)):
        for i in range(2):
            got_m, got_p = host(gfm[li][i]), host(gfp[li][i])
            if name == "mlp" and li == 0:
                # same near-ties: a hidden unit whose pre-activation is within rounding of zero for some sample may get
                # that sample's term or not; the units that keep a margin for every sample are unique
                unit_clear = np.abs(z1).min(axis=0) > 1e-5
                assert unit_clear.sum() > 0.9 * len(unit_clear)
                assert rel_err(got_m[unit_clear], fm_ref[li][i][unit_clear]) < TOL_F32, (li, i)
                assert rel_err(got_p[unit_clear], fp_ref[li][i][unit_clear]) < 1e-5, (li, i)
                assert rel_err(got_p, fp_ref[li][i]) < 1e-2, (li, i)      # the others: off by at most one sample's term
                continue
            assert rel_err(got_m, fm_ref[li][i]) < TOL_F32, (li, i)
            # the parameter through the update it received (new - old), at gradient accuracy
            assert param_update_err(got_p, fp_ref[li][i], fp[li][i]) < TOL_F32, (li, i)
            assert rel_err(got_p, fp_ref[li][i]) < 1e-4, (li, i)
    # gate 1 for the backward ops: feed the checker's gradients of each buffer
    gpar0 = _gpu_params(cp)
    for op in wl.ops:
        dyv = np.ascontiguousarray(bgr[op["dst"]]) if op["op"] in ("pool", "conv") else None
        if op["op"] == "pool":
            n, h, w, c = bufs[op["src"]].shape
            d = api.pool_desc(n, h, w, c, op["win"], op["stride"], op["pad"], op["relu"])
            dx = torch.empty((n, h, w, c), device="cuda:0")
            api.stanza_pool_relu_bwd(d, dev(dyv), dev(bufs[op["dst"]]), dev(bufs[op["dst"] + "#argmax"]), dx)
            assert rel_err(host(dx), o32.pool_relu_bwd(PoolGeom(n, h, w, c, op["win"], op["stride"], op["pad"], op["relu"]),
                                                       dyv, bufs[op["dst"]], bufs[op["dst"] + "#argmax"])) < TOL_F32
        elif op["op"] == "conv":
            x = bufs[op["src"]]
            n, h, w, c = x.shape
            g = ConvGeom(n, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"])
            d = api.conv_desc(n, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"], api.F32,
                              api.CONV_BIAS | (api.CONV_RELU if op["relu"] else 0))
            yd = dev(bufs[op["dst"]]) if op["relu"] else None
            ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(d, 2)), dtype=torch.uint8, device="cuda:0")
            dw = torch.empty(cp[op["name"]][0].shape, device="cuda:0")
            db = torch.empty(op["K"], device="cuda:0")
            api.stanza_conv_bwd_weight(d, dev(x), dev(dyv), yd, dw, db, ws)
            assert rel_err(host(dw), ref["worker_grads"][0][op["name"]][0]) < TOL_F32, op
            assert rel_err(host(db), ref["worker_grads"][0][op["name"]][1]) < TOL_F32, op
            if op["src"] != "x0":
                dz = o32.relu_bwd(dyv, bufs[op["dst"]]) if op["relu"] else dyv
                dx = torch.empty(x.shape, device="cuda:0")
                api.stanza_conv_bwd_data(d, dev(dyv), yd, gpar0[op["name"]][0], None, dx)
                assert rel_err(host(dx), o32.conv_bwd_data(g, dz, cp[op["name"]][0])) < TOL_F32, op


def test_error_paths_on_device(api):
    d = api.conv_desc(1, 8, 8, 4, 4, 3, 3, 1, 1, api.F32, api.CONV_BIAS)
    x = torch.zeros(1, 8, 8, 4, device="cuda:0")
    w = torch.zeros(4, 3, 3, 4, device="cuda:0")
    y = torch.zeros(1, 8, 8, 4, device="cuda:0")
    with pytest.raises(api.StanzaError):
        api.stanza_conv_fwd(d, x, w, None, y)                       # bias flagged but missing
    dl = api.conv_desc(8, 32, 32, 4, 4, 3, 3, 1, 1, api.F32, api.CONV_BIAS)       # long reduction: needs a workspace
    xl = torch.zeros(8, 32, 32, 4, device="cuda:0")
    with pytest.raises(api.StanzaError):
        api.stanza_conv_bwd_weight(dl, xl, xl, None, w, torch.zeros(4, device="cuda:0"), torch.zeros(8, dtype=torch.uint8, device="cuda:0"))
    d16 = api.conv_desc(1, 8, 8, 4, 4, 3, 3, 1, 1, api.BF16, 0)
    with pytest.raises(api.StanzaError):
        api.stanza_conv_fwd(d16, x, w, None, y)


@pytest.mark.parametrize("name,K,n_f", [("tiny", 4, 2), ("minimlp", 6, 3)])
def test_several_fc_workers(api, o32, name, K, n_f):
    """Sec. 4.1.3 on the GPU: K CONV workers in n_f groups, one stanza_fc_grads per FC worker, recursive-doubling
    aggregation of the FC workers' gradient sets and of the CONV workers', against the checker's same iteration."""
    from paper_1812_10624_amd.netrun import Aggregator, ConvWorker, FcGradWorker
    wl = wl_mod.get_workload(name)
    B, seed = wl.B, 3
    n, per = K * B, K // n_f
    imgs = [wl_mod.gen_images(wl, seed, k) for k in range(K)]
    labels = wl_mod.gen_labels(wl, seed, n)
    cp, fp = wl_mod.gen_conv_params(wl, seed), wl_mod.gen_fc_params(wl, seed)
    r = rng(8)
    cm = {nm: (r.standard_normal(w.shape, dtype=np.float32) * np.float32(1e-2), r.standard_normal(b.shape, dtype=np.float32) * np.float32(1e-2))
          for nm, (w, b) in cp.items()}
    fm = [(r.standard_normal(w.shape, dtype=np.float32) * np.float32(1e-2), r.standard_normal(b.shape, dtype=np.float32) * np.float32(1e-2))
          for w, b in fp]
    cp_ref, cm_ref, fp_ref, fm_ref = (copy.deepcopy(a) for a in (cp, cm, fp, fm))
    ref = onet.multi_fc_split_step(o32, wl.ops, imgs, labels, cp_ref, cm_ref, fp_ref, fm_ref, wl.lr, 0.9, 1e-4, n_f)

    gpar, gcm = _gpu_params(cp), _gpu_params(cm)
    gfp = [(dev(w), dev(b)) for w, b in fp]
    gfm = [(dev(w), dev(b)) for w, b in fm]
    workers = [ConvWorker(wl.ops, wl.image, B, gpar) for _ in range(K)]
    fcs = [FcGradWorker(wl.fc_dims, per * B, n, gfp) for _ in range(n_f)]
    feats = torch.empty((n, wl.fc_dims[0]), device="cuda:0")
    for k, wk in enumerate(workers):
        feats[k * B:(k + 1) * B].copy_(wk.forward(dev(imgs[k])).view(B, -1))
    glab = dev(labels)
    loss = 0.0
    for f, fw in enumerate(fcs):
        rows = slice(f * per * B, (f + 1) * per * B)
        fw.step(feats[rows], glab[rows])
        loss += float(host(fw.loss)[0])
        np.testing.assert_array_equal(host(fw.pred), ref["pred"][rows])
        assert rel_err(host(fw.dfeats), ref["dfeats"][rows]) < TOL_F32
        for li in range(len(fp)):
            assert rel_err(host(fw.gW[li]), ref["fc_worker_grads"][f][li][0]) < TOL_F32, (f, li)
            assert rel_err(host(fw.gb[li]), ref["fc_worker_grads"][f][li][1]) < TOL_F32, (f, li)
    assert abs(loss - ref["loss"]) < 1e-5 * max(1.0, abs(ref["loss"]))
    for k, wk in enumerate(workers):
        f = k // per
        wk.backward(fcs[f].dfeats[(k - f * per) * B:(k - f * per + 1) * B])
    # all-reduce + update among the FC workers, then among the CONV workers, both in recursive-doubling order
    fc_agg = Aggregator([t for pair in gfp for t in pair], [t for pair in gfm for t in pair],
                        [[t for li in range(len(fp)) for t in (fw.gW[li], fw.gb[li])] for fw in fcs])
    fc_agg.step(1.0, wl.lr, 0.9, 1e-4, api.SUM_RECURSIVE_DOUBLING)
    names = list(cp)
    agg = Aggregator([gpar[nm][i] for nm in names for i in range(2)], [gcm[nm][i] for nm in names for i in range(2)],
                     [[wk.grads[nm][i] for nm in names for i in range(2)] for wk in workers])
    agg.step(1.0, wl.lr, 0.9, 1e-4, api.SUM_RECURSIVE_DOUBLING)
    for li in range(len(fp)):
        for i in range(2):
            assert rel_err(host(gfm[li][i]), fm_ref[li][i]) < TOL_F32, (li, i)
            assert param_update_err(host(gfp[li][i]), fp_ref[li][i], fp[li][i]) < TOL_F32, (li, i)
    for nm in names:
        for i in range(2):
            assert rel_err(host(gcm[nm][i]), cm_ref[nm][i]) < TOL_F32, (nm, i)
            assert rel_err(host(gpar[nm][i]), cp_ref[nm][i]) < 1e-5, (nm, i)


# residual join in the convolution's epilogue: vector and scalar output paths, sliced tiles (workspace), 64- and 128-wide tiles
@pytest.mark.parametrize("case", [(2, 14, 14, 64, 160, 1, 1, 1, 0), (3, 13, 13, 16, 72, 3, 3, 1, 1), (2, 9, 9, 6, 10, 3, 3, 1, 0),
                                  (2, 15, 15, 24, 40, 1, 1, 2, 0), (16, 56, 56, 32, 128, 1, 1, 1, 0), (8, 1, 1, 2048, 256, 1, 1, 1, 0)], ids=_ids)
@pytest.mark.parametrize("relu", [True, False])
def test_conv_forward_with_residual_join(api, o32, case, relu):
    N, H, W, C, K, R, S, st, pad = case
    g = ConvGeom(N, H, W, C, K, R, S, st, pad)
    r = rng(21)
    x = r.standard_normal((N, H, W, C), dtype=np.float32)
    w = (r.standard_normal((K, R, S, C), dtype=np.float32) / np.sqrt(R * S * C)).astype(np.float32)
    b = r.standard_normal(K, dtype=np.float32)
    res = r.standard_normal((N, g.Ho, g.Wo, K), dtype=np.float32)
    z = (o32.conv_fwd(g, x, w, b, relu=False).astype(np.float64) + res).astype(np.float32)
    ref = np.maximum(z, 0) if relu else z
    d = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS | (api.CONV_RELU if relu else 0))
    for with_ws in (False, True):
        ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(d, 0)), dtype=torch.uint8, device="cuda:0") if with_ws else None
        y = torch.full(ref.shape, float("nan"), device="cuda:0")
        api.stanza_conv_fwd_res(d, dev(x), dev(w), dev(b), dev(res), y, ws)
        assert rel_err(host(y), ref) < TOL_F32, (case, relu, with_ws)
    if relu:      # the same thing as the convolution followed by the join
        y1 = torch.empty(ref.shape, device="cuda:0")
        d0 = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS)
        api.stanza_conv_fwd(d0, dev(x), dev(w), dev(b), y1)
        o = torch.empty_like(y1)
        api.stanza_add_relu_fwd(y1, dev(res), o)
        y2 = torch.empty_like(y1)
        api.stanza_conv_fwd_res(d, dev(x), dev(w), dev(b), dev(res), y2)
        assert torch.equal(o, y2)
