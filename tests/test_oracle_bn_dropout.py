"""Pins for the CPU checker's batch normalisation and seeded dropout: library moments, closed forms, finite
differences of a scalar loss, orthogonality identities of the backward pass, the generator's published
known-answer vectors, mask statistics, and the whole normalised residual step (split == monolithic with
per-worker statistics, chained gradients == finite differences)."""
import copy
import os

import numpy as np
import pytest

import workloads as wl_mod
from oracle import dropout as dr
from oracle import network as onet

HERE = os.path.dirname(os.path.abspath(__file__))


def _case(seed, shape=(3, 4, 5, 6)):
    rng = np.random.default_rng(seed)
    c = shape[-1]
    x = rng.standard_normal(shape) * rng.uniform(0.5, 3.0, c) + rng.uniform(-4, 4, c)     # per-channel scale and offset
    return x, rng.uniform(0.5, 1.5, c), rng.standard_normal(c), rng.standard_normal(shape)


# ------------------------------------------------------------------ batch normalisation
@pytest.mark.parametrize("relu", [False, True])
def test_bn_forward_matches_library_moments(o64, relu):
    x, gamma, beta, _ = _case(0)
    eps = 1e-3
    y, mean, istd = o64.bn_fwd(x, gamma, beta, eps, relu)
    x2 = x.reshape(-1, x.shape[-1])
    mu, var = np.mean(x2, axis=0), np.var(x2, axis=0)                    # numpy's own moments (biased variance)
    np.testing.assert_allclose(mean, mu, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(istd, 1 / np.sqrt(var + eps), rtol=1e-13)
    ref = gamma * (x2 - mu) / np.sqrt(var + eps) + beta
    if relu:
        ref = np.maximum(ref, 0)
    np.testing.assert_allclose(y.reshape(ref.shape), ref, rtol=1e-12, atol=1e-12)


def test_bn_output_moments_closed_form(o64):
    """Per channel the output has mean beta and variance gamma^2 var/(var + eps), whatever the input's scale and offset;
    the output does not change when the input is shifted, nor (up to eps) when it is scaled."""
    x, gamma, beta, _ = _case(1)
    eps = 1e-2
    y, _, _ = o64.bn_fwd(x, gamma, beta, eps)
    y2, x2 = y.reshape(-1, y.shape[-1]), x.reshape(-1, x.shape[-1])
    np.testing.assert_allclose(y2.mean(0), beta, atol=1e-13)
    v = x2.var(0)
    np.testing.assert_allclose(y2.var(0), gamma ** 2 * v / (v + eps), rtol=1e-12)
    y_shift, _, _ = o64.bn_fwd(x + 7.25, gamma, beta, eps)
    np.testing.assert_allclose(y_shift, y, atol=1e-12)
    y_scaled, _, _ = o64.bn_fwd(np.ascontiguousarray(x * 3.0), gamma, beta, 9.0 * eps)
    np.testing.assert_allclose(y_scaled, y, atol=1e-12)


def test_bn_running_statistics(o64):
    x, gamma, beta, _ = _case(2)
    c = x.shape[-1]
    rm, rv = np.full(c, 0.5), np.full(c, 2.0)
    o64.bn_fwd(x, gamma, beta, 1e-5, False, rm, rv, 0.1)
    x2 = x.reshape(-1, c)
    np.testing.assert_allclose(rm, 0.9 * 0.5 + 0.1 * x2.mean(0), rtol=1e-13)
    np.testing.assert_allclose(rv, 0.9 * 2.0 + 0.1 * x2.var(0, ddof=1), rtol=1e-13)


def test_bn_backward_finite_differences(o64):
    """L = sum(r * bn(x)); the checker's dx, dgamma, dbeta against central differences of the checker's forward."""
    x, gamma, beta, r = _case(3, (2, 3, 3, 4))
    eps = 1e-3
    _, mean, istd = o64.bn_fwd(x, gamma, beta, eps)
    dx, dg, db = o64.bn_bwd(x, r, gamma, mean, istd)
    loss = lambda xx, gg, bb: float((o64.bn_fwd(np.ascontiguousarray(xx), gg, bb, eps)[0] * r).sum())
    h = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(25):
        idx = tuple(rng.integers(0, s) for s in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        fd = (loss(xp, gamma, beta) - loss(xm, gamma, beta)) / (2 * h)
        assert abs(fd - dx[idx]) < 1e-7 * max(1.0, abs(fd)), (idx, fd, dx[idx])
    for c in range(x.shape[-1]):
        e = np.zeros_like(gamma)
        e[c] = h
        fd_g = (loss(x, gamma + e, beta) - loss(x, gamma - e, beta)) / (2 * h)
        fd_b = (loss(x, gamma, beta + e) - loss(x, gamma, beta - e)) / (2 * h)
        assert abs(fd_g - dg[c]) < 1e-7 * max(1.0, abs(fd_g))
        assert abs(fd_b - db[c]) < 1e-7 * max(1.0, abs(fd_b))


def test_bn_backward_identities(o64):
    """Per channel dx is orthogonal to the constant vector (the output ignores a shift of the input) and, up to the
    closed-form remainder gamma istd^3 eps dgamma that eps leaves, to xhat (it ignores a scaling); dbeta and dgamma are
    plain column sums."""
    x, gamma, beta, dy = _case(4)
    eps = 1e-5
    _, mean, istd = o64.bn_fwd(x, gamma, beta, eps)
    dx, dg, db = o64.bn_bwd(x, dy, gamma, mean, istd)
    c = x.shape[-1]
    x2, dx2, dy2 = x.reshape(-1, c), dx.reshape(-1, c), dy.reshape(-1, c)
    xhat = (x2 - mean) * istd
    scale = np.abs(dx2).sum(0)
    assert np.all(np.abs(dx2.sum(0)) < 1e-12 * scale)
    assert np.all(np.abs((dx2 * xhat).sum(0) - gamma * istd ** 3 * eps * dg) < 1e-12 * scale)
    np.testing.assert_allclose(db, dy2.sum(0), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dg, (dy2 * xhat).sum(0), rtol=1e-12, atol=1e-12)


def test_bn_float_storage_agrees_with_double(o32, o64):
    x, gamma, beta, dy = _case(5, (4, 7, 7, 8))
    y64, m64, i64 = o64.bn_fwd(x, gamma, beta, 1e-5, True)
    f = lambda a: np.ascontiguousarray(a, np.float32)
    y32, m32, i32 = o32.bn_fwd(f(x), f(gamma), f(beta), 1e-5, True)
    np.testing.assert_allclose(y32, y64, rtol=2e-5, atol=2e-5)
    dx64 = o64.bn_bwd(x, dy, gamma, m64, i64)[0]
    dx32 = o32.bn_bwd(f(x), f(dy), f(gamma), m32, i32)[0]
    np.testing.assert_allclose(dx32, dx64, rtol=1e-4, atol=1e-5)


# ------------------------------------------------------------------ average pool, concatenation
@pytest.mark.parametrize("geom", [(2, 7, 6, 3, 3, 1, 1), (1, 8, 8, 2, 3, 2, 0), (2, 5, 5, 4, 2, 2, 1), (1, 6, 7, 2, 5, 3, 2)])
def test_avgpool_against_masked_library_sums(o64, geom):
    """Window sums of x and of the image's indicator through scipy's correlation: the mean over the valid part of
    each window is their ratio; the backward pass is the transpose (adjoint identity) and sums to sum(dy)."""
    import scipy.signal
    from oracle import PoolGeom
    n, h, w, c, win, stride, pad = geom
    g = PoolGeom(n, h, w, c, win, stride, pad, False)
    rng = np.random.default_rng(7)
    x = rng.standard_normal((n, h, w, c))
    y = o64.avgpool_fwd(g, x)
    ones = np.ones((win, win))
    cnt = scipy.signal.correlate2d(np.pad(np.ones((h, w)), pad), ones, mode="valid")[::stride, ::stride]
    assert cnt.shape == (g.Ho, g.Wo) and cnt.min() >= 1
    for i in range(n):
        for ch in range(c):
            tot = scipy.signal.correlate2d(np.pad(x[i, :, :, ch], pad), ones, mode="valid")[::stride, ::stride]
            np.testing.assert_allclose(y[i, :, :, ch], tot / cnt, rtol=1e-12, atol=1e-13)
    dy = rng.standard_normal(y.shape)
    dx = o64.avgpool_bwd(g, dy)
    assert abs(np.vdot(y, dy) - np.vdot(x, dx)) < 1e-11
    np.testing.assert_allclose(dx.sum(axis=(1, 2)), dy.sum(axis=(1, 2)), rtol=1e-11, atol=1e-12)
    # a constant image stays constant, padding or not
    np.testing.assert_allclose(o64.avgpool_fwd(g, np.full_like(x, 2.5)), 2.5, rtol=1e-13)


def test_inception_table_matches_published_network():
    """Main tower of the published network: 23.8M parameters (the 27M the paper prints, Sec. 2.3 table of models,
    include its auxiliary classifier, which is not built), 5.7 G multiply-adds per 299x299 image, 35/17/8 grids of
    288/768/2048 channels."""
    wl = wl_mod.get_workload("inception3")
    conv, fc = wl_mod.count_params(wl)
    assert conv + fc == 23_834_568
    assert 0.85 < (conv + fc) / 27e6 < 0.9
    sh = wl_mod.shape_pass(wl, 1)
    assert sh["a2"] == (1, 35, 35, 288) and sh["c3x"] == (1, 17, 17, 768) and sh["e1"] == (1, 8, 8, 2048)
    assert abs(wl_mod.conv_flops(wl, 1)[0] / 2 / 5.71e9 - 1) < 0.01


def test_mini_inception_gradients_match_finite_differences(o64):
    """Every kind of block (branches, concatenation, average and max pooling branches, 1xn / nx1 filters, grid
    reductions) through the chained gradients of the whole small stack."""
    wl = wl_mod.get_workload("miniinception")
    B = 2
    imgs, labels, cp, cm, fp, fm = _setup(o64, wl, 6, 1, B)

    def loss_of(params):
        buf = onet.conv_stack_forward(o64, wl.ops, imgs[0], params)
        return onet.fc_step(o64, buf["feat"].reshape(B, -1), labels, fp, fm, 0, 0, 0, update=False)["loss"]

    buf = onet.conv_stack_forward(o64, wl.ops, imgs[0], cp)
    fc = onet.fc_step(o64, buf["feat"].reshape(B, -1), labels, fp, fm, 0, 0, 0, update=False)
    pg, _ = onet.conv_stack_backward(o64, wl.ops, buf, cp, fc["dfeats"])
    rng = np.random.default_rng(3)
    names = [n for n in cp if not n.endswith("_bn")]
    for name in [names[i] for i in rng.choice(len(names), 16, replace=False)] + ["c1a", "a0_pool", "b_dblc", "c0x_d3", "d_7d", "e0_d3b"]:
        t = cp[name][0]
        idx = tuple(rng.integers(0, s) for s in t.shape)
        old = t[idx]
        got = pg[name][0][idx]
        errs = []
        for h in (1e-6, 1e-7):       # an early filter reaches so many units that the wider step may cross a ReLU kink
            t[idx] = old + h
            lp = loss_of(cp)
            t[idx] = old - h
            lm = loss_of(cp)
            t[idx] = old
            fd = (lp - lm) / (2 * h)
            errs.append(abs(fd - got) / max(abs(fd), 1e-2))
        assert min(errs) < 5e-6, (name, errs, got)


# ------------------------------------------------------------------ whole normalised residual step
def _arr(o, t):
    return None if t is None else o.arr(t)


def _setup(o, wl, seed, K, B):
    imgs = [o.arr(wl_mod.gen_images(wl, seed, k, B)) for k in range(K)]
    labels = wl_mod.gen_labels(wl, seed, K * B)
    cp = {n: (o.arr(w), _arr(o, b)) for n, (w, b) in wl_mod.gen_conv_params(wl, seed).items()}
    fp = [(o.arr(w), o.arr(b)) for w, b in wl_mod.gen_fc_params(wl, seed)]
    cm = {n: (np.zeros_like(w), None if b is None else np.zeros_like(b)) for n, (w, b) in cp.items()}
    fm = [(np.zeros_like(w), np.zeros_like(b)) for w, b in fp]
    return imgs, labels, cp, cm, fp, fm


def test_normalised_table_matches_published_parameter_counts():
    """Bias-free convolutions plus a scale and a shift per channel give the published totals of the residual networks."""
    c50 = wl_mod.count_params(wl_mod.get_workload("resnet50bn"))
    c152 = wl_mod.count_params(wl_mod.get_workload("resnet152bn"))
    assert abs(sum(c152) / 6.02e7 - 1) < 1e-3                   # Sec. 2.3, table of models: 60.2M
    assert sum(c50) < sum(c152) and c50[1] == c152[1] == 2048 * 1000 + 1000
    wl = wl_mod.get_workload("miniresbn")
    kinds = [op["op"] for op in wl.ops]
    assert kinds.count("bn") == kinds.count("conv") and all(not op["bias"] for op in wl.ops if op["op"] == "conv")


@pytest.mark.parametrize("K,B", [(2, 3), (3, 2)])
def test_normalised_split_equals_monolithic_with_per_worker_statistics(o64, K, B):
    """K workers that each normalise over their own batch train the model whose normalisation layers take their
    statistics per group of B samples; with whole-batch statistics the step differs."""
    wl = wl_mod.get_workload("miniresbn")
    imgs, labels, cp, cm, fp, fm = _setup(o64, wl, 5, K, B)
    cp2, cm2, fp2, fm2 = (copy.deepcopy(a) for a in (cp, cm, fp, fm))
    cp3, cm3, fp3, fm3 = (copy.deepcopy(a) for a in (cp, cm, fp, fm))
    r1 = onet.split_step(o64, wl.ops, imgs, labels, cp, cm, fp, fm, 0.05, 0.9, 1e-4)
    allimg = np.concatenate(imgs, 0)
    r2 = onet.monolithic_step(o64, wl.ops, allimg, labels, cp2, cm2, fp2, fm2, 0.05, 0.9, 1e-4, bn_groups=K)
    r3 = onet.monolithic_step(o64, wl.ops, allimg, labels, cp3, cm3, fp3, fm3, 0.05, 0.9, 1e-4, bn_groups=1)
    assert abs(r1["loss"] - r2["loss"]) < 1e-12
    assert abs(r1["loss"] - r3["loss"]) > 1e-6
    for n in cp:
        for a, b in zip(cp[n], cp2[n]):
            if a is not None:
                np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
    for (w, b), (w2, b2) in zip(fp, fp2):
        np.testing.assert_allclose(w, w2, rtol=0, atol=1e-13)


def test_normalised_stack_gradients_match_finite_differences(o64):
    """Loss of the whole network (normalised residual stack, FC layer, softmax cross-entropy) against its chained
    gradients: one entry of a filter, of a normalisation scale and of a shift per layer."""
    wl = wl_mod.get_workload("miniresbn")
    K, B = 1, 4
    imgs, labels, cp, cm, fp, fm = _setup(o64, wl, 8, K, B)

    def loss_of(params):
        buf = onet.conv_stack_forward(o64, wl.ops, imgs[0], params)
        return onet.fc_step(o64, buf["feat"].reshape(B, -1), labels, fp, fm, 0, 0, 0, update=False)["loss"]

    buf = onet.conv_stack_forward(o64, wl.ops, imgs[0], cp)
    fc = onet.fc_step(o64, buf["feat"].reshape(B, -1), labels, fp, fm, 0, 0, 0, update=False)
    pg, _ = onet.conv_stack_backward(o64, wl.ops, buf, cp, fc["dfeats"])
    rng = np.random.default_rng(1)
    h = 1e-6
    checked = 0
    for name, pair in cp.items():
        for which, t in enumerate(pair):
            if t is None:
                assert pg[name][which] is None
                continue
            idx = tuple(rng.integers(0, s) for s in t.shape)
            old = t[idx]
            t[idx] = old + h
            lp = loss_of(cp)
            t[idx] = old - h
            lm = loss_of(cp)
            t[idx] = old
            fd = (lp - lm) / (2 * h)
            got = pg[name][which][idx]
            assert abs(fd - got) < 2e-6 * max(abs(fd), 1e-2), (name, which, fd, got)
            checked += 1
    assert checked == 3 * sum(1 for op in wl.ops if op["op"] == "conv")


# ------------------------------------------------------------------ counter-based generator and dropout
def test_generator_known_answers():
    rows = [ln.split() for ln in open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        assert dr.philox4x32_10(v[0:4], v[4:6]) == tuple(v[6:10])


def test_vectorised_words_equal_block_function():
    seed, stream = 0x1234567890ABCDEF, (5 << 8) | 2
    words = dr.random_words(1003, seed, stream)
    for i in (0, 1, 2, 3, 4, 517, 1000, 1002):
        blk = dr.philox4x32_10((i // 4, 0, stream & 0xFFFFFFFF, stream >> 32), (seed & 0xFFFFFFFF, seed >> 32))
        assert int(words[i]) == blk[i % 4]
    assert dr.random_words(0, 1, 1).size == 0


@pytest.mark.parametrize("p", [0.0, 0.1, 0.5, 0.9])
def test_mask_statistics(p):
    n = 200_000
    keep = dr.keep_mask(n, p, 42, dr.fc_stream(3, 1))
    sigma = np.sqrt(max(p * (1 - p), 1e-12) / n)
    assert abs(keep.mean() - (1 - p)) <= 4 * sigma
    if p == 0.0:
        assert keep.all()
    else:
        other = dr.keep_mask(n, p, 42, dr.fc_stream(4, 1))                 # next iteration: an independent mask
        both = (keep & other).mean()
        assert abs(both - (1 - p) ** 2) <= 5 * np.sqrt((1 - p) ** 2 * (1 - (1 - p) ** 2) / n)
        assert not np.array_equal(keep, dr.keep_mask(n, p, 43, dr.fc_stream(3, 1)))
        # neighbouring elements are uncorrelated
        assert abs(np.corrcoef(keep[:-1], keep[1:])[0, 1]) < 5 / np.sqrt(n)


def test_threshold_is_taken_at_float32_precision():
    assert dr.keep_threshold(0.5) == 1 << 31
    assert dr.keep_threshold(0.0) == 0
    assert dr.keep_threshold(0.1) == int(np.floor(float(np.float32(0.1)) * 2.0 ** 32))


def test_dropout_is_scaled_selection_and_self_adjoint():
    rng = np.random.default_rng(0)
    x, y = rng.standard_normal((37, 29)), rng.standard_normal((37, 29))
    p, seed, stream = 0.3, 9, 77
    d = dr.dropout_fwd(x, p, seed, stream)
    keep = dr.keep_mask(x.size, p, seed, stream).reshape(x.shape)
    assert np.all(d[~keep] == 0)
    np.testing.assert_allclose(d[keep], x[keep] / (1 - float(np.float32(p))), rtol=1e-15)
    assert abs((d * y).sum() - (x * dr.dropout_bwd(y, p, seed, stream)).sum()) < 1e-10
    # unbiased: the mean over many masks returns x
    acc = sum(dr.dropout_fwd(x, p, seed, s) for s in range(400)) / 400
    assert np.abs(acc - x).max() < 0.5


def test_fc_step_with_dropout_matches_finite_differences(o64):
    wl = wl_mod.get_workload("minimlp")
    n = 6
    rng = np.random.default_rng(2)
    feats = np.abs(rng.standard_normal((n, wl.fc_dims[0])))
    labels = wl_mod.gen_labels(wl, 2, n)
    fp = [(o64.arr(w), o64.arr(b)) for w, b in wl_mod.gen_fc_params(wl, 2)]
    fm = [(np.zeros_like(w), np.zeros_like(b)) for w, b in fp]
    drop = (0.4, 17, 5)
    r = onet.fc_step(o64, feats, labels, fp, fm, 0, 0, 0, update=False, dropout=drop)
    r0 = onet.fc_step(o64, feats, labels, fp, fm, 0, 0, 0, update=False)
    assert abs(r["loss"] - r0["loss"]) > 1e-6
    rp0 = onet.fc_step(o64, feats, labels, fp, fm, 0, 0, 0, update=False, dropout=(0.0, 17, 5))
    assert rp0["loss"] == r0["loss"] and np.array_equal(rp0["dfeats"], r0["dfeats"])
    loss = lambda: onet.fc_step(o64, feats, labels, fp, fm, 0, 0, 0, update=False, dropout=drop)["loss"]
    h = 1e-6
    for li, (w, b) in enumerate(fp):
        for t, g in ((w, r["grads"][li][0]), (b, r["grads"][li][1])):
            for _ in range(4):
                idx = tuple(rng.integers(0, s) for s in t.shape)
                old = t[idx]
                t[idx] = old + h
                lp = loss()
                t[idx] = old - h
                lm = loss()
                t[idx] = old
                fd = (lp - lm) / (2 * h)
                assert abs(fd - g[idx]) < 1e-6 * max(abs(fd), 1e-3), (li, idx, fd, g[idx])
    for _ in range(6):
        idx = tuple(rng.integers(0, s) for s in feats.shape)
        old = feats[idx]
        feats[idx] = old + h
        lp = loss()
        feats[idx] = old - h
        lm = loss()
        feats[idx] = old
        fd = (lp - lm) / (2 * h)
        assert abs(fd - r["dfeats"][idx]) < 1e-6 * max(abs(fd), 1e-3)
