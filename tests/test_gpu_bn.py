"""Batch normalisation on the GPU against the CPU checker: forward, statistics, running averages and backward
per call on shapes that span every thread mapping (scalar and 16-byte channel vectors, rows that fill a
fraction of / exactly / several workgroups' widths, one and many row slabs), then the whole layer-separated
step of the small normalised residual stack."""
import copy

import numpy as np
import pytest
import torch

import workloads as wl_mod
from gpu_util import TOL_BF16, TOL_F32, dev, host, rel_err
from oracle import network as onet

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    a.load()
    assert torch.cuda.is_available()
    return a


def _case(seed, rows, c):
    rng = wl_mod.rng_for(seed, "bn", rows, c)
    x = rng.standard_normal((rows, c), dtype=np.float32) * rng.uniform(0.5, 3.0, c).astype(np.float32) \
        + rng.uniform(-4, 4, c).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, c).astype(np.float32)
    beta = (rng.standard_normal(c) * 0.5).astype(np.float32)
    dy = rng.standard_normal((rows, c), dtype=np.float32)
    return x, gamma, beta, dy


def _gate32(x, gamma, beta, mean, istd):
    """Sign of the forward output as the library's contract states it: ((x - mean) * s) + beta with s = gamma * istd,
    every operation rounded to float32 (the decision is taken in the kernel's precision on both sides)."""
    f = np.float32
    s = (gamma.astype(f) * istd.astype(f)).astype(f)
    return (((x.astype(f) - mean.astype(f)).astype(f) * s).astype(f) + beta.astype(f)).astype(f) > 0


# rows, channels: scalar path (C % 4 != 0), a row narrower than / equal to / wider than 256 vectors, ragged slabs
SHAPES = [(1, 4), (33, 3), (61, 1030), (175, 4), (243, 7), (442, 48), (784, 512), (98, 2048), (300, 1028), (40000, 64), (12545, 256)]


@pytest.mark.parametrize("rows,c", SHAPES)
@pytest.mark.parametrize("relu", [False, True])
def test_bn_forward_backward(api, o32, rows, c, relu):
    x, gamma, beta, dy = _case(1, rows, c)
    eps = 1e-5
    rm0, rv0 = np.full(c, 0.25, np.float32), np.full(c, 1.5, np.float32)
    rm_ref, rv_ref = rm0.copy(), rv0.copy()
    y_ref, mean_ref, istd_ref = o32.bn_fwd(x, gamma, beta, eps, relu, rm_ref, rv_ref, 0.1)
    xd, gd, bd = dev(x), dev(gamma), dev(beta)
    y = torch.full((rows, c), float("nan"), device="cuda:0")
    mean, istd = torch.empty(c, device="cuda:0"), torch.empty(c, device="cuda:0")
    rm, rv = dev(rm0), dev(rv0)
    ws = torch.empty(max(16, api.stanza_bn_workspace_bytes(rows, c)), dtype=torch.uint8, device="cuda:0")
    api.stanza_bn_fwd(xd, gd, bd, y, mean, istd, ws, eps, relu, rm, rv, 0.1)
    assert rel_err(host(mean), mean_ref) < 1e-5
    if rows > 1:
        assert rel_err(host(istd), istd_ref) < TOL_F32
        assert rel_err(host(y), y_ref) < TOL_F32
        assert rel_err(host(rv), rv_ref) < TOL_F32
    else:
        assert np.allclose(host(istd), 1 / np.sqrt(eps), rtol=1e-5)       # one row: zero variance
    assert rel_err(host(rm), rm_ref) < 1e-5
    if rows == 1:
        return
    # backward on the checker's statistics
    gate = _gate32(x, gamma, beta, mean_ref, istd_ref) if relu else np.ones_like(x, bool)
    if relu:
        assert 0.05 < gate.mean() < 0.95
    g_in = np.where(gate, dy, np.float32(0))
    dx_ref, dg_ref, db_ref = o32.bn_bwd(x, np.ascontiguousarray(g_in), gamma, mean_ref, istd_ref)
    dx = torch.full((rows, c), float("nan"), device="cuda:0")
    dg, db = torch.empty(c, device="cuda:0"), torch.empty(c, device="cuda:0")
    api.stanza_bn_bwd(xd, dev(dy), gd, bd, dev(mean_ref), dev(istd_ref), dx, dg, db, ws, relu)
    assert rel_err(host(dg), dg_ref) < TOL_F32
    assert rel_err(host(db), db_ref) < TOL_F32
    assert rel_err(host(dx), dx_ref) < TOL_F32
    # the forward output's sign is what the backward pass recomputes
    if relu:
        np.testing.assert_array_equal(host(y) > 0, _gate32(x, gamma, beta, host(mean), host(istd)))


def test_bn_largest_layer_of_the_residual_network(api, o32):
    """The first normalisation layer of the ResNet-50-shaped stack at the paper's per-worker batch (64 x 112 x 112 pixels,
    64 channels: 1024 row slabs), every element against the checker."""
    rows, c = 64 * 112 * 112, 64
    x, gamma, beta, dy = _case(7, rows, c)
    y_ref, mean_ref, istd_ref = o32.bn_fwd(x, gamma, beta, 1e-5, True)
    xd = dev(x)
    y = torch.empty((rows, c), device="cuda:0")
    mean, istd = torch.empty(c, device="cuda:0"), torch.empty(c, device="cuda:0")
    ws = torch.empty(api.stanza_bn_workspace_bytes(rows, c), dtype=torch.uint8, device="cuda:0")
    api.stanza_bn_fwd(xd, dev(gamma), dev(beta), y, mean, istd, ws, 1e-5, True)
    assert rel_err(host(mean), mean_ref) < 1e-5 and rel_err(host(istd), istd_ref) < TOL_F32
    assert rel_err(host(y), y_ref) < TOL_F32
    gate = _gate32(x, gamma, beta, mean_ref, istd_ref)
    dx_ref, dg_ref, db_ref = o32.bn_bwd(x, np.ascontiguousarray(np.where(gate, dy, np.float32(0))), gamma, mean_ref, istd_ref)
    dx = torch.empty((rows, c), device="cuda:0")
    dg, db = torch.empty(c, device="cuda:0"), torch.empty(c, device="cuda:0")
    api.stanza_bn_bwd(xd, dev(dy), dev(gamma), dev(beta), dev(mean_ref), dev(istd_ref), dx, dg, db, ws, True)
    assert rel_err(host(dg), dg_ref) < TOL_F32 and rel_err(host(db), db_ref) < TOL_F32
    assert rel_err(host(dx), dx_ref) < TOL_F32


def test_bn_constant_and_offset_columns(api, o32):
    """A constant channel has zero variance (istd = 1/sqrt(eps), output beta); a channel with a large offset keeps its
    variance (the sums are taken about a value inside the data's range)."""
    rows, c = 4096, 8
    rng = wl_mod.rng_for(2, "bnconst")
    x = rng.standard_normal((rows, c), dtype=np.float32)
    x[:, 1] = 3.5
    x[:, 2] += 1000.0
    x[:, 3] = x[:, 3] * 1e-3 - 50.0
    gamma, beta = np.ones(c, np.float32), np.linspace(-1, 1, c).astype(np.float32)
    y_ref, mean_ref, istd_ref = o32.bn_fwd(x, gamma, beta, 1e-5, False)
    y = torch.empty((rows, c), device="cuda:0")
    mean, istd = torch.empty(c, device="cuda:0"), torch.empty(c, device="cuda:0")
    ws = torch.empty(api.stanza_bn_workspace_bytes(rows, c), dtype=torch.uint8, device="cuda:0")
    api.stanza_bn_fwd(dev(x), dev(gamma), dev(beta), y, mean, istd, ws, 1e-5, False)
    assert rel_err(host(istd), istd_ref) < TOL_F32
    assert np.all(host(y)[:, 1] == beta[1])
    # an offset of 1000 (50000) sigma costs the input itself ten (sixteen) bits: those channels are compared at that accuracy
    assert np.abs(host(y)[:, 2] - y_ref[:, 2]).max() < 2e-3 and np.abs(host(y)[:, 3] - y_ref[:, 3]).max() < 2e-2
    assert rel_err(host(y)[:, [0, 4, 5, 6, 7]], y_ref[:, [0, 4, 5, 6, 7]]) < TOL_F32


@pytest.mark.parametrize("rows,c", [(175, 8), (784, 512), (98, 2048), (40000, 64)])
def test_bn_bf16(api, o32, rows, c):
    x, gamma, beta, dy = _case(3, rows, c)
    x, dy = wl_mod.round_bf16(x), wl_mod.round_bf16(dy)
    y_ref, mean_ref, istd_ref = o32.bn_fwd(x, gamma, beta, 1e-5, True)
    xd = dev(x, torch.bfloat16)
    y = torch.empty((rows, c), device="cuda:0", dtype=torch.bfloat16)
    mean, istd = torch.empty(c, device="cuda:0"), torch.empty(c, device="cuda:0")
    ws = torch.empty(api.stanza_bn_workspace_bytes(rows, c, api.BF16), dtype=torch.uint8, device="cuda:0")
    api.stanza_bn_fwd(xd, dev(gamma), dev(beta), y, mean, istd, ws, 1e-5, True, dtype=api.BF16)
    assert rel_err(host(mean), mean_ref) < 1e-5 and rel_err(host(istd), istd_ref) < TOL_F32
    assert rel_err(host(y.float()), y_ref) < TOL_BF16
    gate = _gate32(x, gamma, beta, mean_ref, istd_ref)
    dx_ref, dg_ref, db_ref = o32.bn_bwd(x, np.ascontiguousarray(np.where(gate, dy, np.float32(0))), gamma, mean_ref, istd_ref)
    dx = torch.empty((rows, c), device="cuda:0", dtype=torch.bfloat16)
    dg, db = torch.empty(c, device="cuda:0"), torch.empty(c, device="cuda:0")
    api.stanza_bn_bwd(xd, dev(dy, torch.bfloat16), dev(gamma), dev(beta), dev(mean_ref), dev(istd_ref), dx, dg, db, ws, True, dtype=api.BF16)
    assert rel_err(host(dg), dg_ref) < TOL_F32 and rel_err(host(db), db_ref) < TOL_F32
    assert rel_err(host(dx.float()), dx_ref) < TOL_BF16


def _none_or(fn, t):
    return None if t is None else fn(t)


@pytest.mark.parametrize("K,B", [(2, 3), (3, 4)])
def test_normalised_residual_step(api, o32, K, B):
    """The layer-separated step of the small normalised residual stack: features, loss, handed-back gradient, every
    worker's filter / scale / shift gradients, the aggregated update."""
    from paper_1812_10624_amd.netrun import Aggregator, ConvWorker, FcWorker
    from gpu_util import param_update_err
    wl = wl_mod.get_workload("miniresbn")
    seed = 4
    # Whole-chain bound.  Every normalisation layer (gated at 1e-4 on its own in test_bn_forward_backward) divides by a standard
    # deviation taken over as few as B*4 values per channel in the last stage, and its backward pass subtracts two means:
    # the rounding of everything upstream is amplified by gamma*istd at each of the 13 layers.  Measured whole-chain
    # E(tau = 0.05) = 4.1e-4 (K=2, B=3) and 4.5e-4 (K=3, B=4); the same chain without normalisation (minires) stays at 1.3e-5.
    chain = 6e-4
    imgs = [wl_mod.gen_images(wl, seed, k, B) for k in range(K)]
    labels = wl_mod.gen_labels(wl, seed, K * B)
    cp = wl_mod.gen_conv_params(wl, seed)
    fp = wl_mod.gen_fc_params(wl, seed)
    cm = {n: (np.zeros_like(w), _none_or(np.zeros_like, b)) for n, (w, b) in cp.items()}
    fm = [(np.zeros_like(w), np.zeros_like(b)) for w, b in fp]
    cp_ref, cm_ref, fp_ref, fm_ref = (copy.deepcopy(a) for a in (cp, cm, fp, fm))
    lr, mom, wd = 0.05, 0.9, 1e-4
    ref = onet.split_step(o32, wl.ops, imgs, labels, cp_ref, cm_ref, fp_ref, fm_ref, lr, mom, wd, keep=True)

    gpar = {n: (dev(w), _none_or(dev, b)) for n, (w, b) in cp.items()}
    gcm = {n: (dev(w), _none_or(dev, b)) for n, (w, b) in cm.items()}
    gfp = [(dev(w), dev(b)) for w, b in fp]
    gfm = [(dev(w), dev(b)) for w, b in fm]
    feats = torch.full((K * B, wl.fc_dims[0]), float("nan"), device="cuda:0")
    workers = [ConvWorker(wl.ops, wl.image, B, gpar, feat_out=feats[k * B:(k + 1) * B]) for k in range(K)]   # hand-off without a copy
    fcw = FcWorker(wl.fc_dims, K * B, gfp, gfm, lr, mom, wd)
    for k, wk in enumerate(workers):
        wk.forward(dev(imgs[k]))
    assert rel_err(host(feats), ref["feats"]) < TOL_F32
    # every normalisation layer's saved statistics on worker 0
    for op in wl.ops:
        if op["op"] == "bn":
            mean_ref, istd_ref = ref["bufs"][0][op["dst"] + "#stats"][0]
            mean, istd = workers[0].bn_stats[op["name"]]
            assert np.abs(host(mean) - mean_ref).max() < 1e-5 * max(1.0, np.abs(mean_ref).max()), op["name"]
            assert rel_err(host(istd), istd_ref) < TOL_F32, op["name"]
    dfeats = fcw.step(feats, dev(labels))
    assert abs(float(host(fcw.loss)[0]) - ref["loss"]) < 1e-5 * max(1.0, abs(ref["loss"]))
    assert rel_err(host(dfeats), ref["dfeats"]) < TOL_F32
    for k, wk in enumerate(workers):
        wk.backward(dfeats[k * B:(k + 1) * B])
        for nme in cp:
            for i in range(2):
                if cp[nme][i] is None:
                    assert wk.grads[nme][i] is None
                    continue
                assert rel_err(host(wk.grads[nme][i]), ref["worker_grads"][k][nme][i]) < chain, (k, nme, i)
    flat = lambda d: [t for pair in d.values() for t in pair if t is not None]
    agg = Aggregator(flat(gpar), flat(gcm), [flat(wk.grads) for wk in workers])
    agg.step(1.0, lr, mom, wd)
    for nme in cp:
        for i in range(2):
            if cp[nme][i] is None:
                continue
            assert rel_err(host(gcm[nme][i]), cm_ref[nme][i]) < chain, (nme, i)
            assert param_update_err(host(gpar[nme][i]), cp_ref[nme][i], cp[nme][i]) < chain, (nme, i)
            assert not np.array_equal(host(gpar[nme][i]), cp[nme][i])


@pytest.mark.parametrize("rows,c,half", [(257, 12, False), (4096, 64, False), (33, 3, False), (3 * 14 * 14, 256, True), (4097, 24, True)])
def test_bn_forward_with_residual_join(api, o32, rows, c, half):
    """y = max(bn(x) + res, 0) in one call: against the checker's normalisation followed by its residual join, and (float32)
    bit for bit against the two library calls it replaces."""
    import workloads as wl_mod
    x, gamma, beta, _ = _case(11, rows, c)
    res = np.random.default_rng(12).standard_normal((rows, c), dtype=np.float32)
    if half:
        x, res = wl_mod.round_bf16(x), wl_mod.round_bf16(res)
    y_ref, mean_ref, istd_ref = o32.bn_fwd(x, gamma, beta, 1e-5, False)
    ref = o32.add_relu_fwd(y_ref.reshape(1, 1, rows, c), res.reshape(1, 1, rows, c)).reshape(rows, c)
    DT = api.BF16 if half else api.F32

    def up(a):
        if not half:
            return dev(a)
        return torch.from_numpy(wl_mod.bf16_bits(a).view(np.int16)).to("cuda:0").view(torch.bfloat16).reshape(a.shape)

    def down(t):
        if not half:
            return host(t)
        torch.cuda.synchronize()
        return wl_mod.bf16_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16)).reshape(tuple(t.shape))

    xd, rd, gd, bd = up(x), up(res), dev(gamma), dev(beta)
    y = torch.full((rows, c), float("nan"), device="cuda:0").to(torch.bfloat16 if half else torch.float32)
    mean, istd = torch.empty(c, device="cuda:0"), torch.empty(c, device="cuda:0")
    ws = torch.empty(max(16, api.stanza_bn_workspace_bytes(rows, c, DT)), dtype=torch.uint8, device="cuda:0")
    api.stanza_bn_fwd_res(xd, gd, bd, rd, y, mean, istd, ws, 1e-5, True, dtype=DT)
    assert rel_err(host(mean), mean_ref) < 1e-5 and rel_err(host(istd), istd_ref) < TOL_F32
    assert rel_err(down(y), ref) < (2e-2 if half else TOL_F32)
    assert (down(y) >= 0).all()
    if not half:
        y1, o = torch.empty_like(y), torch.empty_like(y)
        api.stanza_bn_fwd(xd, gd, bd, y1, mean, istd, ws, 1e-5, False)
        api.stanza_add_relu_fwd(y1, rd, o)
        assert torch.equal(o, y)


# N, H, W, C, K, R, stride, pad, bias, offset: tiles of 64 / 128 / 256 rows and 64 / 128 columns, ragged last tiles in both
# directions, launches whose tiles are all whole / all cut into reduction slices / both, a column mean far from zero
FUSED_CASES = [
    (2, 19, 17, 16, 64, 3, 1, 1, False, 0.0),       # 646 rows: a few 64-row tiles, ragged
    (4, 28, 28, 64, 256, 1, 1, 0, False, 0.0),      # short reduction: whole tiles only
    (8, 14, 14, 64, 128, 3, 1, 1, True, 0.0),       # under two rounds of tiles: every tile sliced (with a workspace)
    (3, 14, 14, 32, 192, 3, 1, 1, False, 0.0),      # three 64-wide column tiles
    (2, 15, 15, 48, 160, 3, 2, 1, True, 30.0),      # ragged column tile, stride 2, channel means 30 standard deviations out
    (16, 56, 56, 64, 64, 1, 1, 0, False, 0.0),      # 256-row tiles
    (25, 56, 56, 32, 128, 3, 1, 1, False, 0.0),     # 613 tiles: two whole rounds and a sliced tail
    (1, 7, 7, 512, 2048, 1, 1, 0, False, 0.0),      # 49 rows
]


@pytest.mark.parametrize("case", FUSED_CASES, ids=lambda c: "n%dh%dw%dc%dk%dr%ds%d" % c[:7])
@pytest.mark.parametrize("with_ws", [False, True])
def test_conv_statistics_feed_the_normalisation_layer(api, o32, case, with_ws):
    """stanza_conv_fwd_stats + stanza_bn_fwd_stats against stanza_conv_fwd + the checker's normalisation of that output: the
    convolution's output is bit for bit the plain call's, and the statistics taken from the epilogue's column sums agree with
    the checker's pass over the tensor."""
    from oracle import ConvGeom
    N, H, W, C, K, R, stride, pad, bias, offset = case
    rng = wl_mod.rng_for(21, "convbn", *case[:7])
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = (rng.standard_normal((K, R, R, C), dtype=np.float32) * np.sqrt(2.0 / (R * R * C))).astype(np.float32)
    b = (rng.standard_normal(K) * 0.5 + offset).astype(np.float32) if bias else None
    gamma = rng.uniform(0.5, 1.5, K).astype(np.float32)
    beta = (rng.standard_normal(K) * 0.5).astype(np.float32)
    d = api.conv_desc(N, H, W, C, K, R, R, stride, pad, flags=api.CONV_BIAS if bias else 0)
    ho, wo = api.conv_out_hw(d)
    rows = N * ho * wo
    need = api.stanza_conv_stats_bytes(d)
    assert need > 0
    ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(d, 0)), dtype=torch.uint8, device="cuda:0") if with_ws else None
    xd, wd, bd = dev(x), dev(w), None if b is None else dev(b)
    y_plain = torch.empty((N, ho, wo, K), device="cuda:0")
    api.stanza_conv_fwd(d, xd, wd, bd, y_plain, ws)
    y = torch.full((N, ho, wo, K), float("nan"), device="cuda:0")
    stats = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda:0")
    api.stanza_conv_fwd_stats(d, xd, wd, bd, y, stats, ws)
    assert torch.equal(y, y_plain)
    y_conv = host(y)
    if rows <= 4000:
        assert rel_err(y_conv, o32.conv_fwd(ConvGeom(N, H, W, C, K, R, R, stride, pad), x, w, b)) < TOL_F32
    for relu in (False, True):
        rm0, rv0 = np.full(K, 0.25, np.float32), np.full(K, 1.5, np.float32)
        rm_ref, rv_ref = rm0.copy(), rv0.copy()
        z_ref, mean_ref, istd_ref = o32.bn_fwd(y_conv.reshape(rows, K), gamma, beta, 1e-5, relu, rm_ref, rv_ref, 0.1)
        z = torch.full((rows, K), float("nan"), device="cuda:0")
        mean, istd = torch.empty(K, device="cuda:0"), torch.empty(K, device="cuda:0")
        rm, rv = dev(rm0), dev(rv0)
        api.stanza_bn_fwd_stats(y.view(rows, K), stats, dev(gamma), dev(beta), z, mean, istd, 1e-5, relu, running_mean=rm, running_var=rv)
        # the mean to a hundred-thousandth of the column's spread (these columns are centred near zero: an error relative to the
        # largest mean would measure nothing)
        assert (np.abs(host(mean) - mean_ref) * istd_ref).max() < 1e-5
        assert rel_err(host(istd), istd_ref) < TOL_F32
        assert rel_err(host(z), z_ref) < TOL_F32
        assert rel_err(host(rm), rm_ref) < 1e-5 and rel_err(host(rv), rv_ref) < TOL_F32
    # with the residual join, and bit for bit against the unfused layer given the same statistics
    res = rng.standard_normal((rows, K), dtype=np.float32)
    z2 = torch.empty((rows, K), device="cuda:0")
    api.stanza_bn_fwd_stats(y.view(rows, K), stats, dev(gamma), dev(beta), z2, mean, istd, 1e-5, True, res=dev(res))
    ref2 = o32.add_relu_fwd(o32.bn_fwd(y_conv.reshape(rows, K), gamma, beta, 1e-5, False)[0].reshape(1, 1, rows, K), res.reshape(1, 1, rows, K))
    assert rel_err(host(z2), ref2.reshape(rows, K)) < TOL_F32


def test_statistics_buffer_of_another_matrix_gives_nan(api):
    """The normalisation call checks the header that the convolution left: a buffer that was never written, or that describes
    another matrix, yields NaN statistics instead of reads outside it."""
    rows, c = 300, 64
    x = torch.randn((rows, c), device="cuda:0")
    y = torch.empty_like(x)
    mean, istd = torch.zeros(c, device="cuda:0"), torch.zeros(c, device="cuda:0")
    g, b = torch.ones(c, device="cuda:0"), torch.zeros(c, device="cuda:0")
    api.stanza_bn_fwd_stats(x, torch.zeros(4096, dtype=torch.uint8, device="cuda:0"), g, b, y, mean, istd)
    assert bool(torch.isnan(mean).all()) and bool(torch.isnan(istd).all())
    d = api.conv_desc(1, 10, 10, 16, 64, 1, 1, 1, 0)                     # a 100 x 64 matrix
    stats = torch.zeros(api.stanza_conv_stats_bytes(d), dtype=torch.uint8, device="cuda:0")
    api.stanza_conv_fwd_stats(d, torch.randn((1, 10, 10, 16), device="cuda:0"), torch.randn((64, 1, 1, 16), device="cuda:0"), None,
                              torch.empty((1, 10, 10, 64), device="cuda:0"), stats)
    api.stanza_bn_fwd_stats(x, stats, g, b, y, mean, istd)               # x has 300 rows
    assert bool(torch.isnan(mean).all())
