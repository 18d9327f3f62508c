"""Pins for the CPU checker: each operation is tied to something other than itself — an
explicitly built dense operator, a library routine on a special case, an adjoint identity,
a finite difference, a closed form, or the paper's split == monolithic invariant (Sec. 3.2)."""
import math

import numpy as np
import pytest
import scipy.signal
import scipy.special

from oracle import ConvGeom, PoolGeom

RNG = np.random.default_rng(1234)

GEOMS = [
    ConvGeom(2, 6, 7, 3, 4, 3, 3, 1, 1),
    ConvGeom(1, 9, 8, 2, 3, 3, 3, 2, 1),     # strided, padded
    ConvGeom(2, 11, 11, 2, 3, 5, 5, 2, 2),
    ConvGeom(1, 13, 12, 3, 2, 7, 7, 2, 3),   # stem-like
    ConvGeom(2, 5, 6, 4, 5, 1, 1, 1, 0),     # pointwise
    ConvGeom(1, 7, 7, 3, 4, 1, 1, 2, 0),     # strided pointwise (projection shortcut)
    ConvGeom(1, 23, 23, 1, 2, 11, 11, 4, 2),  # large filter, stride 4
    ConvGeom(2, 4, 4, 2, 3, 3, 3, 1, 0),     # no padding
    ConvGeom(2, 6, 9, 3, 4, 1, 7, 1, 0, 3),  # 1x7 filter, padded along the width only
    ConvGeom(1, 9, 6, 2, 3, 7, 1, 1, 3, 0),  # 7x1 filter, padded along the height only
    ConvGeom(2, 5, 4, 3, 2, 3, 1, 1, 1, 0),  # 3x1
]


def rnd(shape, dt=np.float64):
    return RNG.standard_normal(shape).astype(dt)


def toeplitz(g: ConvGeom, w):
    """Dense matrix T with vec(Y) = T vec(X), built one entry at a time."""
    T = np.zeros((g.N * g.Ho * g.Wo * g.K, g.N * g.H * g.W * g.C))
    for n in range(g.N):
        for p in range(g.Ho):
            for q in range(g.Wo):
                for k in range(g.K):
                    row = ((n * g.Ho + p) * g.Wo + q) * g.K + k
                    for r in range(g.R):
                        for s in range(g.S):
                            h, ww = p * g.stride - g.pad + r, q * g.stride - g.pw + s
                            if 0 <= h < g.H and 0 <= ww < g.W:
                                for c in range(g.C):
                                    T[row, ((n * g.H + h) * g.W + ww) * g.C + c] += w[k, r, s, c]
    return T


@pytest.mark.parametrize("g", GEOMS, ids=lambda g: f"{g.H}x{g.W}x{g.C}k{g.K}r{g.R}x{g.S}s{g.stride}p{g.pad}x{g.pw}")
def test_conv_against_dense_operator(o64, g):
    x, w, b = rnd((g.N, g.H, g.W, g.C)), rnd((g.K, g.R, g.S, g.C)), rnd((g.K,))
    dy = rnd((g.N, g.Ho, g.Wo, g.K))
    T = toeplitz(g, w)
    y = o64.conv_fwd(g, x, w, b)
    ref = (T @ x.reshape(-1)).reshape(y.shape) + b
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(o64.conv_fwd(g, x, w, b, relu=True), np.maximum(ref, 0), rtol=1e-12, atol=1e-12)
    dx = o64.conv_bwd_data(g, dy, w)
    np.testing.assert_allclose(dx.reshape(-1), T.T @ dy.reshape(-1), rtol=1e-12, atol=1e-12)
    # weight gradient: Y is linear in W, so dW = d<Y,dY>/dW; check through the dense operator of
    # unit filters (one-hot W gives one column of the Jacobian)
    dw, db = o64.conv_bwd_weight(g, x, dy)
    for _ in range(6):
        idx = tuple(RNG.integers(0, d) for d in w.shape)
        e = np.zeros_like(w)
        e[idx] = 1.0
        np.testing.assert_allclose(dw[idx], (toeplitz(g, e) @ x.reshape(-1)) @ dy.reshape(-1), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(db, dy.reshape(-1, g.K).sum(0), rtol=1e-12, atol=1e-12)


def test_conv_single_channel_is_library_correlation(o64):
    g = ConvGeom(1, 10, 9, 1, 1, 3, 3, 1, 1)
    x, w = rnd((1, 10, 9, 1)), rnd((1, 3, 3, 1))
    y = o64.conv_fwd(g, x, w)
    ref = scipy.signal.correlate2d(np.pad(x[0, :, :, 0], 1), w[0, :, :, 0], mode="valid")
    np.testing.assert_allclose(y[0, :, :, 0], ref, rtol=1e-12, atol=1e-12)
    # filter flip would give convolve2d instead: make sure the two differ on this input
    assert np.abs(ref - scipy.signal.convolve2d(np.pad(x[0, :, :, 0], 1), w[0, :, :, 0], mode="valid")).max() > 1e-3


def test_conv_special_cases(o64):
    # 1x1 stride-1 conv is a plain matrix product over pixels
    g = ConvGeom(2, 5, 6, 7, 4, 1, 1, 1, 0)
    x, w, b = rnd((2, 5, 6, 7)), rnd((4, 1, 1, 7)), rnd((4,))
    np.testing.assert_allclose(o64.conv_fwd(g, x, w, b).reshape(-1, 4), x.reshape(-1, 7) @ w.reshape(4, 7).T + b,
                               rtol=1e-12, atol=1e-12)
    # a filter as large as the image, no padding, is an FC layer over the NHWC flattening
    g = ConvGeom(3, 4, 5, 2, 6, 4, 5, 1, 0)
    x, w = rnd((3, 4, 5, 2)), rnd((6, 4, 5, 2))
    np.testing.assert_allclose(o64.conv_fwd(g, x, w).reshape(3, 6), x.reshape(3, -1) @ w.reshape(6, -1).T,
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(o64.fc_fwd(x.reshape(3, -1).copy(), w.reshape(6, -1).copy()),
                               o64.conv_fwd(g, x, w).reshape(3, 6), rtol=1e-12, atol=1e-12)
    # centre-tap delta filter per channel is the identity
    g = ConvGeom(1, 6, 6, 3, 3, 3, 3, 1, 1)
    w = np.zeros((3, 3, 3, 3))
    for c in range(3):
        w[c, 1, 1, c] = 1.0
    x = rnd((1, 6, 6, 3))
    np.testing.assert_array_equal(o64.conv_fwd(g, x, w), x)
    # a one-pixel-shift filter moves the image the way cross-correlation does: Y[p,q] = X[p+1,q]
    w = np.zeros((1, 3, 3, 1))
    w[0, 2, 1, 0] = 1.0
    g = ConvGeom(1, 5, 5, 1, 1, 3, 3, 1, 1)
    x = rnd((1, 5, 5, 1))
    y = o64.conv_fwd(g, x, w)
    np.testing.assert_array_equal(y[0, :-1, :, 0], x[0, 1:, :, 0])
    np.testing.assert_array_equal(y[0, -1, :, 0], 0)


@pytest.mark.parametrize("g", GEOMS[:6] + GEOMS[8:], ids=lambda g: f"r{g.R}x{g.S}s{g.stride}p{g.pad}x{g.pw}")
def test_conv_adjoint_identities(o64, g):
    x, w = rnd((g.N, g.H, g.W, g.C)), rnd((g.K, g.R, g.S, g.C))
    w2 = rnd(w.shape)
    dy = rnd((g.N, g.Ho, g.Wo, g.K))
    lhs = np.vdot(o64.conv_fwd(g, x, w), dy)
    assert abs(lhs - np.vdot(x, o64.conv_bwd_data(g, dy, w))) <= 1e-11 * abs(lhs) + 1e-11
    lhs2 = np.vdot(o64.conv_fwd(g, x, w2), dy)
    dw, _ = o64.conv_bwd_weight(g, x, dy)
    assert abs(lhs2 - np.vdot(w2, dw)) <= 1e-11 * abs(lhs2) + 1e-11


def test_f32_checker_matches_f64_checker(o32, o64):
    g = GEOMS[1]
    x, w, b = rnd((g.N, g.H, g.W, g.C), np.float32), rnd((g.K, g.R, g.S, g.C), np.float32), rnd((g.K,), np.float32)
    dy = rnd((g.N, g.Ho, g.Wo, g.K), np.float32)
    xd, wd_, bd, dyd = (a.astype(np.float64) for a in (x, w, b, dy))
    np.testing.assert_allclose(o32.conv_fwd(g, x, w, b), o64.conv_fwd(g, xd, wd_, bd), rtol=0, atol=2e-6)
    np.testing.assert_allclose(o32.conv_bwd_data(g, dy, w), o64.conv_bwd_data(g, dyd, wd_), rtol=0, atol=2e-6)
    np.testing.assert_allclose(o32.conv_bwd_weight(g, x, dy)[0], o64.conv_bwd_weight(g, xd, dyd)[0], rtol=0, atol=4e-6)


def test_sampled_entry_points_equal_full_tensors(o32):
    g = GEOMS[2]
    x, w, b = rnd((g.N, g.H, g.W, g.C), np.float32), rnd((g.K, g.R, g.S, g.C), np.float32), rnd((g.K,), np.float32)
    dy = rnd((g.N, g.Ho, g.Wo, g.K), np.float32)
    y = o32.conv_fwd(g, x, w, b, relu=True)
    dx = o32.conv_bwd_data(g, dy, w)
    dw, db = o32.conv_bwd_weight(g, x, dy)
    for _ in range(20):
        n, p, q, k = (RNG.integers(0, d) for d in y.shape)
        assert np.float32(o32.conv_fwd_at(g, x, w, b, True, n, p, q, k)) == y[n, p, q, k]
        n, h, ww, c = (RNG.integers(0, d) for d in dx.shape)
        assert np.float32(o32.conv_bwd_data_at(g, dy, w, n, h, ww, c)) == dx[n, h, ww, c]
        k, r, s, c = (RNG.integers(0, d) for d in dw.shape)
        assert np.float32(o32.conv_bwd_weight_at(g, x, dy, k, r, s, c)) == dw[k, r, s, c]
    assert np.float32(o32.colsum_at(dy.reshape(-1, g.K), 1)) == db[1]


# ------------------------------------------------------------------ pooling
POOLS = [PoolGeom(2, 8, 8, 3, 2, 2, 0, True), PoolGeom(1, 13, 11, 2, 3, 2, 0, True),
         PoolGeom(2, 9, 10, 2, 3, 2, 1, True), PoolGeom(1, 7, 7, 2, 3, 2, 1, False), PoolGeom(1, 6, 6, 2, 2, 2, 0, False)]


def np_pool(g: PoolGeom, x):
    """Window max through -inf padding and strided window views."""
    xp = np.pad(x, ((0, 0), (g.pad, g.pad), (g.pad, g.pad), (0, 0)), constant_values=-np.inf)
    win = np.lib.stride_tricks.sliding_window_view(xp, (g.win, g.win), axis=(1, 2))[:, ::g.stride, ::g.stride]
    win = win[:, :g.Ho, :g.Wo]                      # [N,Ho,Wo,C,win,win]
    flat = win.reshape(win.shape[:4] + (-1,))
    return flat.max(-1), flat.argmax(-1)            # argmax: first maximum, row-major in the window


@pytest.mark.parametrize("g", POOLS, ids=lambda g: f"w{g.win}s{g.stride}p{g.pad}r{int(g.relu)}")
def test_pool_forward_and_backward(o64, g):
    x = rnd((g.N, g.H, g.W, g.C))
    x[0, :4, :4, 0] = 0.5          # ties: first maximum in the window must win
    x[0, 4:, :, 1] = -1.0 - np.abs(x[0, 4:, :, 1])   # all-negative region: ReLU gates it
    y, am = o64.pool_relu_fwd(g, x)
    ref, ref_am = np_pool(g, x)
    np.testing.assert_array_equal(y, np.maximum(ref, 0) if g.relu else ref)
    np.testing.assert_array_equal(am, ref_am.astype(np.uint8))
    assert am.max() < g.win * g.win
    # fused == pool(relu(x)) as well
    if g.relu:
        y2, _ = o64.pool_relu_fwd(PoolGeom(g.N, g.H, g.W, g.C, g.win, g.stride, g.pad, False), np.maximum(x, 0))
        np.testing.assert_array_equal(y, y2)
    dy = rnd(y.shape)
    dx = o64.pool_relu_bwd(g, dy, y, am)
    gate = (y > 0) if g.relu else np.ones_like(y, bool)
    assert abs(dx.sum() - (dy * gate).sum()) < 1e-10           # mass conservation
    # scatter form written independently: route each output's gradient to its argmax pixel
    ref_dx = np.zeros_like(x)
    for n in range(g.N):
        for p in range(g.Ho):
            for q in range(g.Wo):
                for c in range(g.C):
                    if gate[n, p, q, c]:
                        i, j = divmod(int(ref_am[n, p, q, c]), g.win)
                        ref_dx[n, p * g.stride - g.pad + i, q * g.stride - g.pad + j, c] += dy[n, p, q, c]
    np.testing.assert_allclose(dx, ref_dx, rtol=1e-12, atol=1e-12)


def test_pool_finite_difference(o64):
    g = PoolGeom(1, 7, 7, 2, 3, 2, 0, True)
    x = rnd((1, 7, 7, 2))
    y, am = o64.pool_relu_fwd(g, x)
    dy = rnd(y.shape)
    dx = o64.pool_relu_bwd(g, dy, y, am)
    h = 1e-6
    for _ in range(30):
        idx = tuple(RNG.integers(0, d) for d in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (np.vdot(o64.pool_relu_fwd(g, xp)[0], dy) - np.vdot(o64.pool_relu_fwd(g, xm)[0], dy)) / (2 * h)
        assert abs(fd - dx[idx]) < 1e-6, (idx, fd, dx[idx])


# ------------------------------------------------------------------ FC and loss
def test_fc_against_matmul(o64):
    a, w, b = rnd((5, 13)), rnd((7, 13)), rnd((7,))
    dz = rnd((5, 7))
    np.testing.assert_allclose(o64.fc_fwd(a, w, b), a @ w.T + b, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(o64.fc_fwd(a, w, b, relu=True), np.maximum(a @ w.T + b, 0), rtol=1e-12, atol=1e-12)
    dw, db, da = o64.fc_bwd(a, w, dz)
    np.testing.assert_allclose(dw, dz.T @ a, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, dz.sum(0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(da, dz @ w, rtol=1e-12, atol=1e-12)
    assert abs(o64.fc_fwd_at(a, w, b, 2, 3) - (a[2] @ w[3] + b[3])) < 1e-12


def test_softmax_ce_invariants(o64):
    n, cls = 6, 10
    z = rnd((n, cls)) * 3
    lab = RNG.integers(0, cls, n).astype(np.int32)
    loss, dz, pred = o64.softmax_ce(z, lab)
    sm = dz * n
    sm[np.arange(n), lab] += 1
    np.testing.assert_allclose(sm.sum(1), 1.0, rtol=1e-12)
    np.testing.assert_allclose(dz.sum(1), 0.0, atol=1e-15)
    np.testing.assert_allclose(sm, scipy.special.softmax(z, axis=1), rtol=1e-11, atol=1e-15)
    ref = np.mean(scipy.special.logsumexp(z, axis=1) - z[np.arange(n), lab])
    assert abs(loss - ref) < 1e-12
    np.testing.assert_array_equal(pred, z.argmax(1))
    # shift invariance
    loss2, dz2, _ = o64.softmax_ce(z + 100.0, lab)
    assert abs(loss2 - loss) < 1e-10
    np.testing.assert_allclose(dz2, dz, atol=1e-13)
    # all-zero logits: loss = ln(classes), gradient (1/classes - onehot)/n, ties -> class 0
    for cls2 in (10, 1000):
        z0 = np.zeros((4, cls2))
        lab0 = np.array([0, 1, cls2 - 1, 5], np.int32)
        loss0, dz0, pred0 = o64.softmax_ce(z0, lab0)
        assert abs(loss0 - math.log(cls2)) < 1e-12
        e = np.zeros_like(z0)
        e[np.arange(4), lab0] = 1
        np.testing.assert_allclose(dz0, (1.0 / cls2 - e) / 4, rtol=1e-12, atol=1e-18)
        assert (pred0 == 0).all()
    # finite difference of the mean loss
    h = 1e-6
    for _ in range(10):
        i, j = RNG.integers(0, n), RNG.integers(0, cls)
        zp, zm = z.copy(), z.copy()
        zp[i, j] += h
        zm[i, j] -= h
        fd = (o64.softmax_ce(zp, lab)[0] - o64.softmax_ce(zm, lab)[0]) / (2 * h)
        assert abs(fd - dz[i, j]) < 1e-8


# ------------------------------------------------------------------ optimiser
def test_sgd_momentum_closed_form(o64):
    g = rnd((50,))
    w0 = rnd((50,))
    w, v = w0.copy(), np.zeros(50)
    lr, m = 0.01, 0.9
    acc = np.zeros(50)
    for t in range(1, 8):
        o64.sgd_momentum(w, v, g, lr, m, 0.0)
        vt = g * (1 - m ** t) / (1 - m)
        acc += vt
        np.testing.assert_allclose(v, vt, rtol=1e-12)
        np.testing.assert_allclose(w, w0 - lr * acc, rtol=1e-12, atol=1e-14)
    # no momentum, no decay: plain Eq.(1) step
    w, v = w0.copy(), np.zeros(50)
    o64.sgd_momentum(w, v, g, 0.1, 0.0, 0.0)
    np.testing.assert_allclose(w, w0 - 0.1 * g, rtol=1e-14)
    # weight decay enters the gradient before the momentum buffer
    w, v = w0.copy(), rnd((50,))
    v0 = v.copy()
    o64.sgd_momentum(w, v, g, 0.1, 0.5, 0.01)
    np.testing.assert_allclose(v, 0.5 * v0 + g + 0.01 * w0, rtol=1e-13)
    np.testing.assert_allclose(w, w0 - 0.1 * v, rtol=1e-13)


def test_ps_aggregate_properties(o64):
    K, ne = 5, 40
    gs = [rnd((ne,)) for _ in range(K)]
    w0, v0 = rnd((ne,)), rnd((ne,))
    w, v = w0.copy(), v0.copy()
    o64.ps_aggregate(w, v, gs, 1.0, 0.01, 0.9, 5e-4)
    w2, v2 = w0.copy(), v0.copy()
    o64.sgd_momentum(w2, v2, np.sum(gs, axis=0), 0.01, 0.9, 5e-4)
    np.testing.assert_allclose(w, w2, rtol=1e-13)
    np.testing.assert_allclose(v, v2, rtol=1e-13)
    # K copies of one gradient with scale 1/K is a single-shard step
    w, v = w0.copy(), v0.copy()
    o64.ps_aggregate(w, v, [gs[0]] * K, 1.0 / K, 0.01, 0.9, 0.0)
    w2, v2 = w0.copy(), v0.copy()
    o64.sgd_momentum(w2, v2, gs[0], 0.01, 0.9, 0.0)
    np.testing.assert_allclose(w, w2, rtol=1e-13)


def test_residual_and_gap(o64):
    a, b = rnd((2, 3, 4, 5)), rnd((2, 3, 4, 5))
    np.testing.assert_allclose(o64.add_relu_fwd(a, b), np.maximum(a + b, 0), rtol=1e-15)
    x = rnd((2, 3, 4, 5))
    np.testing.assert_allclose(o64.gap_fwd(x).reshape(2, 5), x.mean((1, 2)), rtol=1e-13)
    df = rnd((2, 5))
    dx = o64.gap_bwd(df, x.shape)
    np.testing.assert_allclose(dx, np.broadcast_to(df[:, None, None, :] / 12.0, x.shape), rtol=1e-15)
