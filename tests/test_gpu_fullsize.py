"""GPU parity at the full sizes of the benchmark's configurations, in the launch configuration the bench
times: each layer is run whole on the GPU and compared with the CPU checker on sampled outputs that the
checker computes one by one (plus corners and edges, where padding and ragged tiles live)."""
import numpy as np
import pytest
import torch

import workloads as wl_mod
from gpu_util import TOL_F32, dev, host
from oracle import ConvGeom

pytestmark = pytest.mark.gpu

NSAMP = 48


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    a.load()
    assert torch.cuda.is_available()
    return a


def _draw(shape, seed, scale=1.0):
    r = wl_mod.rng_for(seed, "full", *shape)
    a = r.standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return a


def _sample_idx(shape, seed, n=NSAMP):
    r = np.random.default_rng(seed)
    idx = [tuple(int(r.integers(0, d)) for d in shape) for _ in range(n)]
    # corners and last elements: padding taps, ragged tile edges
    idx += [tuple(0 for _ in shape), tuple(d - 1 for d in shape), tuple((d - 1) if i % 2 else 0 for i, d in enumerate(shape))]
    return idx


def _check(got, want, scale_ref, what):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    floor = 0.05 * scale_ref
    e = float((np.abs(got - want) / np.maximum(np.abs(want), floor)).max())
    assert e < TOL_F32, (what, e)


# name, (N,H,W,C,K,R,S,stride,pad): the distinct heavy shapes of configs 2-4 at their real batch sizes
FULL_CASES = [
    ("vgg_c1", (64, 224, 224, 3, 64, 3, 3, 1, 1)),
    ("vgg_c2", (64, 224, 224, 64, 64, 3, 3, 1, 1)),
    ("vgg_c5", (64, 56, 56, 128, 256, 3, 3, 1, 1)),
    ("vgg_c11", (64, 14, 14, 512, 512, 3, 3, 1, 1)),
    ("alex_c1", (128, 224, 224, 3, 96, 11, 11, 4, 2)),
    ("alex_c2", (128, 27, 27, 96, 256, 5, 5, 1, 2)),
    ("res_stem", (64, 224, 224, 3, 64, 7, 7, 2, 3)),
    ("res_s2_3x3", (64, 56, 56, 128, 128, 3, 3, 2, 1)),
    ("res_s2_proj", (64, 56, 56, 256, 512, 1, 1, 2, 0)),
    ("res_1x1", (64, 56, 56, 256, 64, 1, 1, 1, 0)),
]


@pytest.mark.parametrize("name,case", FULL_CASES, ids=[c[0] for c in FULL_CASES])
def test_conv_layer_full_size(api, o32, name, case):
    N, H, W, C, K, R, S, st, pad = case
    g = ConvGeom(N, H, W, C, K, R, S, st, pad)
    x = _draw((N, H, W, C), 1)
    w = _draw((K, R, S, C), 2, (2.0 / (R * S * C)) ** 0.5)
    b = _draw((K,), 3, 0.1)
    dy = _draw((N, g.Ho, g.Wo, K), 4)
    xd, wd, bd, dyd = dev(x), dev(w), dev(b), dev(dy)
    d = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS | api.CONV_RELU)
    # the workspace the bench's sequencer passes: with it the last round of tiles is cut into reduction slices
    ws01 = torch.empty(max(16, api.stanza_conv_workspace_bytes(d, 0), api.stanza_conv_workspace_bytes(d, 1)), dtype=torch.uint8, device="cuda:0")
    # forward (+bias, +ReLU)
    y = torch.empty((N, g.Ho, g.Wo, K), device="cuda:0")
    api.stanza_conv_fwd(d, xd, wd, bd, y, ws01)
    yh = host(y)
    idx = _sample_idx(yh.shape, 10)
    want = [o32.conv_fwd_at(g, x, w, b, True, *i) for i in idx]
    _check([yh[i] for i in idx], want, float(np.abs(yh).max()), name + " fwd")
    assert (yh >= 0).all()
    del y
    # backward-data (plain; the gating variants are covered at small sizes)
    if C > 3:
        d0 = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, 0)
        dx = torch.empty((N, H, W, C), device="cuda:0")
        api.stanza_conv_bwd_data(d0, dyd, None, wd, None, dx, ws01)
        dxh = host(dx)
        idx = _sample_idx(dxh.shape, 11)
        want = [o32.conv_bwd_data_at(g, dy, w, *i) for i in idx]
        _check([dxh[i] for i in idx], want, float(np.abs(dxh).max()), name + " bwd_data")
        del dx, dxh
    # backward-weight + bias gradient (ungated dy)
    db_desc = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS)
    ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(db_desc, 2)), dtype=torch.uint8, device="cuda:0")
    dw = torch.empty((K, R, S, C), device="cuda:0")
    db = torch.empty((K,), device="cuda:0")
    api.stanza_conv_bwd_weight(db_desc, xd, dyd, None, dw, db, ws)
    dwh, dbh = host(dw), host(db)
    idx = _sample_idx(dwh.shape, 12, 24)
    want = [o32.conv_bwd_weight_at(g, x, dy, *i) for i in idx]
    _check([dwh[i] for i in idx], want, float(np.abs(dwh).max()), name + " bwd_weight")
    cols = [0, K - 1, K // 2]
    _check([dbh[j] for j in cols], [o32.colsum_at(dy.reshape(-1, K), j) for j in cols], float(np.abs(dbh).max()), name + " dbias")


def test_fc_layers_full_size(api, o32):
    """The VGG-16-shaped FC worker's first layer (512 x 25088 -> 4096) through the engine the FC step uses,
    and a whole FC step at the ResNet-50-shaped size (1024 x 2048 -> 1000), sampled."""
    import copy
    from oracle import network as onet
    from paper_1812_10624_amd.netrun import FcWorker
    n, A, O = 512, 25088, 4096
    feats = np.maximum(_draw((n, A), 5), 0)
    w = _draw((O, A), 6, (2.0 / A) ** 0.5)
    b = _draw((O,), 7, 0.01)
    d = api.conv_desc(n, 1, 1, A, O, 1, 1, 1, 0, api.F32, api.CONV_BIAS | api.CONV_RELU)
    z = torch.empty((n, O), device="cuda:0")
    api.stanza_conv_fwd(d, dev(feats), dev(w), dev(b), z)
    zh = host(z)
    idx = _sample_idx(zh.shape, 13)
    _check([zh[i] for i in idx], [o32.fc_fwd_at(feats, w, b, i, o, relu=True) for i, o in idx], float(np.abs(zh).max()), "fc1 fwd")
    # whole step, ResNet-50-shaped FC worker
    dims, n2 = [2048, 1000], 1024
    f2 = np.maximum(_draw((n2, dims[0]), 8), 0)
    lab = wl_mod.rng_for(9, "lab").integers(0, dims[1], n2).astype(np.int32)
    p = [(_draw((dims[1], dims[0]), 9, (2.0 / dims[0]) ** 0.5), _draw((dims[1],), 10, 0.01))]
    m = [(np.zeros_like(p[0][0]), np.zeros_like(p[0][1]))]
    p_ref, m_ref = copy.deepcopy(p), copy.deepcopy(m)
    ref = onet.fc_step(o32, f2, lab, p_ref, m_ref, 0.01, 0.9, 0.0)
    gp, gm = [(dev(p[0][0]), dev(p[0][1]))], [(dev(m[0][0]), dev(m[0][1]))]
    fw = FcWorker(dims, n2, gp, gm, 0.01, 0.9, 0.0)
    fw.step(dev(f2), dev(lab))
    assert abs(float(host(fw.loss)[0]) - ref["loss"]) < 1e-5 * abs(ref["loss"])
    np.testing.assert_array_equal(host(fw.pred), ref["pred"])
    from gpu_util import rel_err
    assert rel_err(host(fw.dfeats), ref["dfeats"]) < TOL_F32
    assert rel_err(host(gm[0][0]), m_ref[0][0]) < TOL_F32
    assert rel_err(host(gm[0][1]), m_ref[0][1]) < TOL_F32
    assert rel_err(host(gp[0][0]), p_ref[0][0]) < 1e-5


@pytest.mark.parametrize("which", ["conv", "fc"])
def test_ps_aggregate_full_size(api, o32, which):
    """Config 5: K = 16 shards over the VGG-16-shaped conv set (26 tensors, 14.7 M parameters), whole-tensor
    comparison; for the 123.6 M-parameter FC set the two largest tensors are cut to their first 4 M elements
    on the checker side (the GPU still runs the full set)."""
    from gpu_util import rel_err
    wl = wl_mod.get_workload("vgg16")
    numels, fans = wl_mod.param_tensor_numels(wl, which)
    K = 16
    if which == "fc":
        K = 4      # host memory: 123.6 M x K shards
    ws_, vs_, gs_ = wl_mod.gen_ps_case(numels, K, seed=21, fan_ins=fans)
    gw, gv = [dev(a) for a in ws_], [dev(a) for a in vs_]
    gg = [[dev(gs_[t][k]) for t in range(len(numels))] for k in range(K)]
    ws = torch.empty(api.stanza_ps_workspace_bytes(len(numels), K), dtype=torch.uint8, device="cuda:0")
    api.stanza_ps_aggregate(gw, gv, gg, 1.0, 0.01, 0.9, 5e-4, ws)
    for t, ne in enumerate(numels):
        cut = min(ne, 4 << 20)
        w_ref, v_ref = ws_[t][:cut].copy(), vs_[t][:cut].copy()
        o32.ps_aggregate(w_ref, v_ref, [np.ascontiguousarray(gs_[t][k][:cut]) for k in range(K)], 1.0, 0.01, 0.9, 5e-4)
        assert rel_err(host(gv[t])[:cut], v_ref) < 1e-5, t
        assert rel_err(host(gw[t])[:cut], w_ref) < 1e-6, t
        tail_w = host(gw[t])[-8:]
        assert np.isfinite(tail_w).all() and not np.array_equal(tail_w, ws_[t][-8:])


def test_conv_input_of_two_gibibytes(api, o32):
    """Largest case: a 2 GiB float32 input (2^29 elements) is beyond the 32-bit byte offsets of the vector fetch path; the
    launch falls back to element-wise addressing and must still be right everywhere, the far end of the tensor included."""
    N, H, W, C, K, R, S, st, pad = 1, 2048, 2048, 128, 8, 3, 3, 1, 1
    g = ConvGeom(N, H, W, C, K, R, S, st, pad)
    r = wl_mod.rng_for(41, "huge")
    x = r.standard_normal((N, H, W, C), dtype=np.float32)
    w = r.standard_normal((K, R, S, C), dtype=np.float32) * np.float32((2.0 / (R * S * C)) ** 0.5)
    b = r.standard_normal(K, dtype=np.float32) * np.float32(0.1)
    assert x.nbytes == 1 << 31
    xd, wd, bd = dev(x), dev(w), dev(b)
    d = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS | api.CONV_RELU)
    y = torch.empty((N, H, W, K), device="cuda:0")
    api.stanza_conv_fwd(d, xd, wd, bd, y)
    yh = host(y)
    idx = _sample_idx(yh.shape, 14, 32) + [(0, 2047, 2047, 7), (0, 2047, 0, 0), (0, 1024, 2047, 3)]
    want = [o32.conv_fwd_at(g, x, w, b, True, *i) for i in idx]
    _check([yh[i] for i in idx], want, float(np.abs(yh).max()), "2 GiB input fwd")
    # filter gradient over the same input (dy small, x large)
    dy = r.standard_normal((N, H, W, K), dtype=np.float32)
    dd = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS)
    ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(dd, 2)), dtype=torch.uint8, device="cuda:0")
    dw = torch.empty((K, R, S, C), device="cuda:0")
    db = torch.empty((K,), device="cuda:0")
    api.stanza_conv_bwd_weight(dd, xd, dev(dy), None, dw, db, ws)
    dwh = host(dw)
    idx = _sample_idx(dwh.shape, 15, 12)
    want = [o32.conv_bwd_weight_at(g, x, dy, *i) for i in idx]
    _check([dwh[i] for i in idx], want, float(np.abs(dwh).max()), "2 GiB input bwd_weight")


def test_conv_tensor_beyond_2_gib(api, o32):
    """A layer whose input (and input gradient) is larger than 2 GiB: the vector fetch addresses tensors with 32-bit byte
    offsets, so the launch must fall back to element-indexed gathers; sampled against the checker in all three directions."""
    N, H, W, C, K = 86, 224, 224, 128, 8
    g = ConvGeom(N, H, W, C, K, 1, 1, 1, 0)
    r = np.random.default_rng(5)
    x = r.standard_normal((N, H, W, C), dtype=np.float32)
    assert x.nbytes > (1 << 31)
    w = (r.standard_normal((K, 1, 1, C), dtype=np.float32) / np.sqrt(C)).astype(np.float32)
    b = r.standard_normal(K, dtype=np.float32)
    dy = r.standard_normal((N, H, W, K), dtype=np.float32)
    xd, wd, dyd = dev(x), dev(w), dev(dy)
    d = api.conv_desc(N, H, W, C, K, 1, 1, 1, 0, api.F32, api.CONV_BIAS | api.CONV_RELU)
    y = torch.full((N, H, W, K), float("nan"), device="cuda:0")
    api.stanza_conv_fwd(d, xd, wd, dev(b), y)
    yh = host(y)
    assert np.isfinite(yh).all()
    idx = _sample_idx(yh.shape, 20)
    _check([yh[i] for i in idx], [o32.conv_fwd_at(g, x, w, b, True, *i) for i in idx], float(np.abs(yh).max()), "fwd > 2 GiB")
    del y, yh
    d0 = api.conv_desc(N, H, W, C, K, 1, 1, 1, 0, api.F32, 0)
    dx = torch.full((N, H, W, C), float("nan"), device="cuda:0")
    api.stanza_conv_bwd_data(d0, dyd, None, wd, None, dx)
    dxh = host(dx)
    assert np.isfinite(dxh).all()
    idx = _sample_idx(dxh.shape, 21)
    _check([dxh[i] for i in idx], [o32.conv_bwd_data_at(g, dy, w, *i) for i in idx], float(np.abs(dxh).max()), "bwd_data > 2 GiB")
    del dx, dxh
    ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(d0, 2)), dtype=torch.uint8, device="cuda:0")
    dw = torch.full((K, 1, 1, C), float("nan"), device="cuda:0")
    api.stanza_conv_bwd_weight(d0, xd, dyd, None, dw, None, ws)
    dwh = host(dw)
    idx = [(0, 0, 0, 0), (K - 1, 0, 0, C - 1), (3, 0, 0, 77), (5, 0, 0, 1)]
    _check([dwh[i] for i in idx], [o32.conv_bwd_weight_at(g, x, dy, *i) for i in idx], float(np.abs(dwh).max()), "bwd_weight > 2 GiB")
