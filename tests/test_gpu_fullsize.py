"""GPU parity at the full sizes of the benchmark's configurations, in the launch configuration the bench
times: each layer is run whole on the GPU and compared with the CPU checker on outputs that the checker
computes one by one: at least one in every 64 x 64 block of the output seen as the GEMM's matrix (every tile
shape of the kernels is a multiple of that, so every workgroup of the first round, of the last full round and of the
sliced tail is sampled), the corners, and the first and last image whole."""
import copy

import numpy as np
import pytest
import torch

import workloads as wl_mod
from gpu_util import TOL_F32, dev, host, note, param_update_err, rel_err
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


def _block_idx(shape, ncols, seed, block=64):
    """One index in every block x block tile of the tensor seen as a [numel / ncols, ncols] matrix (rows x columns of
    the GEMM that produces it), as tuples into `shape`."""
    numel = int(np.prod(shape))
    rows = numel // ncols
    r = np.random.default_rng(seed)
    rb, cb = (rows + block - 1) // block, (ncols + block - 1) // block
    r0 = (np.arange(rb) * block)[:, None] + np.zeros((1, cb), np.int64)
    c0 = np.zeros((rb, 1), np.int64) + (np.arange(cb) * block)[None, :]
    rr = r0 + r.integers(0, np.minimum(block, rows - r0))
    cc = c0 + r.integers(0, np.minimum(block, ncols - c0))
    flat = (rr * ncols + cc).ravel()
    return [tuple(int(v) for v in np.unravel_index(f, shape)) for f in flat]


def _check(got, want, scale_ref, what):
    e = note(got, want, scale_ref)
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
    ("res_s2_3x3_stride2", (64, 56, 56, 128, 128, 3, 3, 2, 1)),
    ("res_s2_proj", (64, 56, 56, 256, 512, 1, 1, 2, 0)),
    ("res_1x1", (64, 56, 56, 256, 64, 1, 1, 1, 0)),
    # shapes whose tile plan differs from the large layers': short reductions (64x64 and 64x128 tiles), fewer than two 128x128
    # tiles per CU with a medium reduction (smaller tiles, only the last round cut into slices), a 7x7 3x3 layer (its filter
    # gradient goes to the implicit GEMM, not the nine-tap kernel)
    ("res_s1_1x1_64", (64, 56, 56, 64, 64, 1, 1, 1, 0)),
    ("res_s1_1x1_256", (64, 56, 56, 64, 256, 1, 1, 1, 0)),
    ("res_s2_3x3", (64, 28, 28, 128, 128, 3, 3, 1, 1)),
    ("res_s4_1x1", (64, 7, 7, 512, 2048, 1, 1, 1, 0)),
    ("res_s4_3x3", (64, 7, 7, 512, 512, 3, 3, 1, 1)),
]


def _whole_image(N):
    return sorted({0, N - 1})


@pytest.mark.parametrize("name,case", FULL_CASES, ids=[c[0] for c in FULL_CASES])
def test_conv_layer_full_size(api, o32, name, case):
    N, H, W, C, K, R, S, st, pad = case
    g = ConvGeom(N, H, W, C, K, R, S, st, pad)
    g1 = ConvGeom(1, H, W, C, K, R, S, st, pad)
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
    idx = _sample_idx(yh.shape, 10) + _block_idx(yh.shape, K, 110)
    want = [o32.conv_fwd_at(g, x, w, b, True, *i) for i in idx]
    scale = float(np.abs(yh).max())
    _check([yh[i] for i in idx], want, scale, name + " fwd")
    for n in _whole_image(N):        # first and last image whole
        _check(yh[n], o32.conv_fwd(g1, np.ascontiguousarray(x[n:n + 1]), w, b, relu=True)[0], scale, name + " fwd image %d" % n)
    assert (yh >= 0).all()
    del y
    # backward-data (plain; the gating variants are covered at small sizes)
    if C > 3:
        d0 = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, 0)
        dx = torch.empty((N, H, W, C), device="cuda:0")
        api.stanza_conv_bwd_data(d0, dyd, None, wd, None, dx, ws01)
        dxh = host(dx)
        idx = _sample_idx(dxh.shape, 11) + _block_idx(dxh.shape, C, 111)
        want = [o32.conv_bwd_data_at(g, dy, w, *i) for i in idx]
        scale = float(np.abs(dxh).max())
        _check([dxh[i] for i in idx], want, scale, name + " bwd_data")
        for n in _whole_image(N):
            _check(dxh[n], o32.conv_bwd_data(g1, np.ascontiguousarray(dy[n:n + 1]), w)[0], scale, name + " bwd_data image %d" % n)
        del dx, dxh
    # backward-weight + bias gradient (ungated dy)
    db_desc = api.conv_desc(N, H, W, C, K, R, S, st, pad, api.F32, api.CONV_BIAS)
    ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(db_desc, 2)), dtype=torch.uint8, device="cuda:0")
    dw = torch.empty((K, R, S, C), device="cuda:0")
    db = torch.empty((K,), device="cuda:0")
    api.stanza_conv_bwd_weight(db_desc, xd, dyd, None, dw, db, ws)
    dwh, dbh = host(dw), host(db)
    idx = _sample_idx(dwh.shape, 12, 24) + _block_idx(dwh.shape, R * S * C, 112)
    want = [o32.conv_bwd_weight_at(g, x, dy, *i) for i in idx]
    _check([dwh[i] for i in idx], want, float(np.abs(dwh).max()), name + " bwd_weight")
    dy2 = dy.reshape(-1, K)
    _check(dbh, [o32.colsum_at(dy2, j) for j in range(K)], float(np.abs(dbh).max()), name + " dbias")


def _fc_step_against_checker(api, o32, dims, n, seed, lr=0.01, momentum=0.9, wd=5e-4):
    """One whole stanza_fc_step against the checker's fc_step, element by element: loss, predicted classes (bit-exact),
    the gradient handed back to the CONV workers, every momentum buffer and every parameter."""
    import fc_cases
    from oracle import network as onet
    from paper_1812_10624_amd.netrun import FcWorker
    feats, labels, params, mom, _ = fc_cases.fc_case(dims, n, seed)
    p_ref, m_ref = copy.deepcopy(params), copy.deepcopy(mom)
    ref = onet.fc_step(o32, feats, labels, p_ref, m_ref, lr, momentum, wd)
    for li, (dw, _) in enumerate(ref["grads"]):      # momentum buffers and gradients of like size: neither hides the other
        assert 0.1 < float(mom[li][0].std()) / float(dw.std()) < 10.0, li
    gp = [(dev(w), dev(b)) for w, b in params]
    gm = [(dev(w), dev(b)) for w, b in mom]
    fw = FcWorker(dims, n, gp, gm, lr, momentum, wd)
    fw.step(dev(feats), dev(labels))
    assert abs(float(host(fw.loss)[0]) - ref["loss"]) < 1e-5 * max(1.0, abs(ref["loss"]))
    np.testing.assert_array_equal(host(fw.pred), ref["pred"])
    assert rel_err(host(fw.dfeats), ref["dfeats"]) < TOL_F32
    for li in range(len(params)):
        for which in range(2):
            e_v = rel_err(host(gm[li][which]), m_ref[li][which])
            assert e_v < TOL_F32, ("momentum", li, which, e_v)
            e_p = param_update_err(host(gp[li][which]), p_ref[li][which], params[li][which])
            assert e_p < TOL_F32, ("parameter", li, which, e_p)
            assert not np.array_equal(p_ref[li][which], params[li][which])


def test_fc_step_vgg16_full_size(api, o32):
    """The FC worker of the VGG-16-shaped configuration at the size the bench times: 512 rows (8 CONV workers x 64),
    25088 -> 4096 -> 4096 -> 1000, non-zero momentum buffers and weight decay."""
    _fc_step_against_checker(api, o32, [25088, 4096, 4096, 1000], 512, seed=33)


def test_fc_step_alexnet_full_size(api, o32):
    """The FC worker of the AlexNet-shaped configuration: 512 rows (4 CONV workers x 128), 9216 -> 4096 -> 4096 -> 1000."""
    _fc_step_against_checker(api, o32, [9216, 4096, 4096, 1000], 512, seed=31)


def test_fc_step_resnet50_full_size(api, o32):
    """The FC worker of the ResNet-50-shaped configuration: 1024 rows (16 CONV workers x 64), 2048 -> 1000."""
    _fc_step_against_checker(api, o32, [2048, 1000], 1024, seed=35)


@pytest.mark.parametrize("which", ["conv", "fc"])
def test_ps_aggregate_full_size(api, o32, which):
    """Config 5: K = 16 shards over the VGG-16-shaped conv set (26 tensors, 14.7 M parameters) and over the FC set
    (6 tensors, 123.6 M parameters), one launch per set as the bench runs it, every tensor compared whole.  The host holds
    one tensor's shards at a time: they are drawn, uploaded and dropped, and drawn again for the checker."""
    wl = wl_mod.get_workload("vgg16")
    numels, fans = wl_mod.param_tensor_numels(wl, which)
    K, seed = 16, 21
    gw, gv, gg = [], [], [[] for _ in range(K)]
    for t, ne in enumerate(numels):
        w0, v0, shards = wl_mod.gen_ps_tensor(t, ne, K, seed, fans[t])
        gw.append(dev(w0))
        gv.append(dev(v0))
        for k in range(K):
            gg[k].append(dev(shards[k]))
        del w0, v0, shards
    ws = torch.empty(api.stanza_ps_workspace_bytes(len(numels), K), dtype=torch.uint8, device="cuda:0")
    api.stanza_ps_aggregate(gw, gv, gg, 1.0, 0.01, 0.9, 5e-4, ws)
    torch.cuda.synchronize()
    for t, ne in enumerate(numels):
        w_ref, v_ref, shards = wl_mod.gen_ps_tensor(t, ne, K, seed, fans[t])
        w0 = w_ref.copy()
        o32.ps_aggregate(w_ref, v_ref, shards, 1.0, 0.01, 0.9, 5e-4)
        del shards
        assert rel_err(host(gv[t]), v_ref) < 1e-5, t
        assert param_update_err(host(gw[t]), w_ref, w0) < TOL_F32, t
        assert rel_err(host(gw[t]), w_ref) < 1e-6, t


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
