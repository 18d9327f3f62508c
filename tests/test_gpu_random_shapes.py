"""GPU parity on seeded random convolution geometries (both dtypes): every option of the three conv entry points drawn at
random per case -- bias, ReLU epilogue, gate of dy, accumulation, input-sign mask, per-axis padding, with and without the
optional slice workspace -- against the CPU checker, element by element.  The fixed cases of the other files are chosen
to hit known paths; these are chosen by a generator, to hit the ones nobody thought of."""
import numpy as np
import pytest
import torch

import workloads as wl_mod
from gpu_util import TOL_BF16, TOL_F32, dev, host, rel_err
from oracle import ConvGeom

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    a.load()
    assert torch.cuda.is_available()
    return a


def _geometry(seed, half, big=False):
    r = np.random.default_rng(1000 + seed)
    if big:
        # enough rows and columns for 128x128 tiles, several rounds of them, sliced tails and filter-gradient slices
        R = S = int(r.choice([1, 3, 3]))
        st = int(r.choice([1, 1, 2]))
        ph = pw = int(r.integers(0, R))
        H, W = int(r.integers(20, 41)), int(r.integers(20, 41))
        C, K = (8 if half else 4) * int(r.integers(10, 40)), (8 if half else 4) * int(r.integers(10, 40))
        N = int(r.integers(4, 17))
        while N > 1 and N * H * W * C * K * R * S // (st * st) > 2.0e9:        # keep the checker to seconds
            N -= 1
        opts = {k: bool(r.random() < 0.5) for k in ("bias", "relu", "gate", "accum", "xmask")}
        opts["ws"] = True
        return (N, H, W, C, K, R, S, st, ph, pw), opts
    R = int(r.choice([1, 1, 2, 3, 3, 5, 7]))
    S = R if r.random() < 0.7 else int(r.choice([1, 3, 5, 7]))
    st = int(r.choice([1, 1, 1, 2, 2, 3]))
    ph, pw = int(r.integers(0, R)), int(r.integers(0, S))                 # pad < window
    H = int(r.integers(max(R - 2 * ph, 1), 34))
    W = int(r.integers(max(S - 2 * pw, 1), 34))
    N = int(r.integers(1, 5))
    if half:
        C, K = 8 * int(r.integers(1, 12)), 8 * int(r.integers(1, 12))
    else:
        C, K = int(r.integers(1, 80)), int(r.integers(1, 80))
        if r.random() < 0.4:
            C = 4 * ((C + 3) // 4)
        if r.random() < 0.4:
            K = 4 * ((K + 3) // 4)
    opts = {k: bool(r.random() < 0.5) for k in ("bias", "relu", "gate", "accum", "xmask", "ws")}
    return (N, H, W, C, K, R, S, st, ph, pw), opts


def _run(api, o32, seed, half, big=False):
    (N, H, W, C, K, R, S, st, ph, pw), o = _geometry(seed, half, big)
    g = ConvGeom(N, H, W, C, K, R, S, st, ph, pw)
    r = np.random.default_rng(2000 + seed)
    q = wl_mod.round_bf16 if half else (lambda a: a)
    x = q(r.standard_normal((N, H, W, C), dtype=np.float32))
    w = q((r.standard_normal((K, R, S, C), dtype=np.float32) / np.sqrt(R * S * C)).astype(np.float32))
    b = r.standard_normal(K, dtype=np.float32)
    dy = q(r.standard_normal((N, g.Ho, g.Wo, K), dtype=np.float32))
    yf = q(r.standard_normal((N, g.Ho, g.Wo, K), dtype=np.float32))        # stands for the layer's output (its sign gates dy)
    xin = q(r.standard_normal((N, H, W, C), dtype=np.float32))             # stands for the layer's input (its sign masks dx)
    prev = q(r.standard_normal((N, H, W, C), dtype=np.float32))
    DT, tdt, tol = (api.BF16, torch.bfloat16, TOL_BF16) if half else (api.F32, torch.float32, TOL_F32)
    what = dict(seed=seed, geom=(N, H, W, C, K, R, S, st, ph, pw), **o)

    def up(a):
        if not half:
            return dev(a)
        bits = wl_mod.bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).to("cuda:0").view(torch.bfloat16).reshape(a.shape)

    def down(t):
        if not half:
            return host(t)
        torch.cuda.synchronize()
        return wl_mod.bf16_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16)).reshape(tuple(t.shape))

    def desc(flags):
        return api.conv_desc(N, H, W, C, K, R, S, st, ph, DT, flags, pad_w=pw)

    def workspace(d, which):
        if not o["ws"] and which != 2:
            return None
        return torch.empty(max(16, api.stanza_conv_workspace_bytes(d, which)), dtype=torch.uint8, device="cuda:0")

    # forward
    d = desc((api.CONV_BIAS if o["bias"] else 0) | (api.CONV_RELU if o["relu"] else 0))
    y = torch.full((N, g.Ho, g.Wo, K), float("nan"), device="cuda:0").to(tdt)
    api.stanza_conv_fwd(d, up(x), up(w), dev(b) if o["bias"] else None, y, workspace(d, 0))
    assert rel_err(down(y), o32.conv_fwd(g, x, w, b if o["bias"] else None, relu=o["relu"])) < tol, ("fwd", what)
    # backward-data
    d = desc((api.CONV_RELU if o["gate"] else 0) | (api.CONV_ACCUM if o["accum"] else 0))
    ref = o32.conv_bwd_data(g, o32.relu_bwd(dy, yf) if o["gate"] else dy, w)
    if o["accum"]:
        ref = (ref.astype(np.float64) + prev).astype(np.float32)
    if o["xmask"]:
        ref = o32.relu_bwd(ref, xin)
    dx = up(prev) if o["accum"] else torch.full((N, H, W, C), float("nan"), device="cuda:0").to(tdt)
    api.stanza_conv_bwd_data(d, up(dy), up(yf) if o["gate"] else None, up(w), up(xin) if o["xmask"] else None, dx, workspace(d, 1))
    assert rel_err(down(dx), ref) < tol, ("bwd_data", what)
    # backward-weight (float32 outputs in both dtypes)
    d = desc((api.CONV_BIAS if o["bias"] else 0) | (api.CONV_RELU if o["gate"] else 0))
    ref_dw, ref_db = o32.conv_bwd_weight(g, x, o32.relu_bwd(dy, yf) if o["gate"] else dy)
    dw = torch.full((K, R, S, C), float("nan"), device="cuda:0")
    db = torch.full((K,), float("nan"), device="cuda:0")
    api.stanza_conv_bwd_weight(d, up(x), up(dy), up(yf) if o["gate"] else None, dw, db if o["bias"] else None, workspace(d, 2))
    wtol = 1e-3 if half else tol          # bf16 products are exact in float32: only the summation order differs
    assert rel_err(host(dw), ref_dw) < wtol, ("bwd_weight", what)
    if o["bias"]:
        assert rel_err(host(db), ref_db) < wtol, ("dbias", what)


@pytest.mark.parametrize("seed", range(48))
def test_random_conv_f32(api, o32, seed):
    _run(api, o32, seed, False)


@pytest.mark.parametrize("seed", range(32))
def test_random_conv_bf16(api, o32, seed):
    _run(api, o32, 500 + seed, True)


@pytest.mark.parametrize("seed", range(8))
def test_random_large_conv_f32(api, o32, seed):
    _run(api, o32, 800 + seed, False, big=True)


@pytest.mark.parametrize("seed", range(6))
def test_random_large_conv_bf16(api, o32, seed):
    _run(api, o32, 900 + seed, True, big=True)


def _pool_case(seed):
    r = np.random.default_rng(3000 + seed)
    win = int(r.choice([2, 2, 3, 3, 4, 5]))
    st = int(r.integers(1, win + 1))
    pad = int(r.integers(0, (win + 1) // 2)) if r.random() < 0.5 else 0       # pad <= win / 2: every window reaches the image
    H, W = int(r.integers(win, 40)), int(r.integers(win, 40))
    N = int(r.integers(1, 5))
    C = int(r.integers(1, 70))
    return N, H, W, C, win, st, pad, bool(r.random() < 0.5)


@pytest.mark.parametrize("seed", range(40))
def test_random_pools(api, o32, seed):
    """Max pool (+ReLU) with its argmax byte and backward pass, and the average pool, float32 and (C % 8 == 0) bfloat16."""
    from oracle import PoolGeom
    N, H, W, C, win, st, pad, relu = _pool_case(seed)
    half = seed % 3 == 2
    if half:
        C = 8 * ((C + 7) // 8)
    g = PoolGeom(N, H, W, C, win, st, pad, relu)
    r = np.random.default_rng(4000 + seed)
    q = wl_mod.round_bf16 if half else (lambda a: a)
    x = q(r.standard_normal((N, H, W, C), dtype=np.float32))
    dy = q(r.standard_normal((N, g.Ho, g.Wo, C), dtype=np.float32))
    DT, tdt = (api.BF16, torch.bfloat16) if half else (api.F32, torch.float32)
    what = (seed, N, H, W, C, win, st, pad, relu, half)

    def up(a):
        if not half:
            return dev(a)
        return torch.from_numpy(wl_mod.bf16_bits(a).view(np.int16)).to("cuda:0").view(torch.bfloat16).reshape(a.shape)

    def down(t):
        if not half:
            return host(t)
        torch.cuda.synchronize()
        return wl_mod.bf16_to_f32(t.view(torch.int16).cpu().numpy().view(np.uint16)).reshape(tuple(t.shape))

    d = api.pool_desc(N, H, W, C, win, st, pad, relu)
    y_ref, am_ref = o32.pool_relu_fwd(g, x)
    y = torch.full(y_ref.shape, float("nan"), device="cuda:0").to(tdt)
    am = torch.full(y_ref.shape, 255, dtype=torch.uint8, device="cuda:0")
    api.stanza_pool_relu_fwd(d, up(x), y, am, DT)
    np.testing.assert_array_equal(down(y), y_ref, err_msg=str(what))            # a selection: bit-exact
    np.testing.assert_array_equal(host(am), am_ref, err_msg=str(what))
    dx = torch.full(x.shape, float("nan"), device="cuda:0").to(tdt)
    api.stanza_pool_relu_bwd(d, up(dy), y, am, dx, DT)
    # overlapping windows add their gradients: float32 sums in both dtypes, one rounding to bf16
    assert rel_err(down(dx), o32.pool_relu_bwd(g, dy, y_ref, am_ref)) < (2.0 ** -8 * 1.01 if half else 1e-5), what
    ya = torch.full(y_ref.shape, float("nan"), device="cuda:0").to(tdt)
    api.stanza_avgpool_fwd(d, up(x), ya, DT)
    assert rel_err(down(ya), o32.avgpool_fwd(g, x)) < (2.0 ** -8 * 1.01 if half else 1e-5), what
    dxa = torch.full(x.shape, float("nan"), device="cuda:0").to(tdt)
    api.stanza_avgpool_bwd(d, up(dy), dxa, DT)
    assert rel_err(down(dxa), o32.avgpool_bwd(g, dy)) < (2.0 ** -8 * 1.01 if half else 1e-5), what
