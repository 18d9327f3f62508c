"""Whole-step pins for the CPU checker: the split step equals the monolithic step (the paper's
equivalence claim, Sec. 3.2), the chained gradients match finite differences of the loss, and
the workload tables reproduce the parameter counts the paper prints."""
import copy
import os

import numpy as np
import pytest

import workloads as wl_mod
from oracle import network as onet

HERE = os.path.dirname(os.path.abspath(__file__))


def _setup(o, wl, seed, K, B, small_fc=None):
    imgs = [o.arr(wl_mod.gen_images(wl, seed, k, B)) for k in range(K)]
    labels = wl_mod.gen_labels(wl, seed, K * B)
    cp = {n: (o.arr(w), o.arr(b)) for n, (w, b) in wl_mod.gen_conv_params(wl, seed).items()}
    fp = [(o.arr(w), o.arr(b)) for w, b in wl_mod.gen_fc_params(wl, seed)]
    rng = np.random.default_rng(seed + 99)
    cm = {n: (o.arr(rng.standard_normal(w.shape) * 1e-2), o.arr(rng.standard_normal(b.shape) * 1e-2)) for n, (w, b) in cp.items()}
    fm = [(o.arr(rng.standard_normal(w.shape) * 1e-2), o.arr(rng.standard_normal(b.shape) * 1e-2)) for w, b in fp]
    return imgs, labels, cp, cm, fp, fm


@pytest.mark.parametrize("name,K,B", [("tiny", 1, 2), ("tiny", 2, 2), ("tiny", 3, 1), ("tiny", 4, 1), ("minires", 2, 2), ("minires", 3, 1),
                                        ("minimlp", 3, 2), ("minimlp", 2, 5)])
def test_split_equals_monolithic(o64, name, K, B):
    wl = wl_mod.get_workload(name)
    imgs, labels, cp, cm, fp, fm = _setup(o64, wl, 3, K, B)
    cp2, cm2, fp2, fm2 = (copy.deepcopy(a) for a in (cp, cm, fp, fm))
    cp0 = copy.deepcopy(cp)
    r1 = onet.split_step(o64, wl.ops, imgs, labels, cp, cm, fp, fm, 0.01, 0.9, 1e-4)
    r2 = onet.monolithic_step(o64, wl.ops, np.concatenate(imgs, 0), labels, cp2, cm2, fp2, fm2, 0.01, 0.9, 1e-4)
    assert abs(r1["loss"] - r2["loss"]) < 1e-12
    np.testing.assert_array_equal(r1["pred"], r2["pred"])
    for n in cp:
        for a, b, a0 in zip(cp[n], cp2[n], cp0[n]):
            step = np.abs(a - a0).max()
            assert step > 0                               # the parameters did move
            np.testing.assert_allclose(a, b, rtol=0, atol=1e-12 * max(1.0, step))
        for a, b in zip(cm[n], cm2[n]):
            np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-14)
    for (w, b), (w2, b2) in zip(fp, fp2):
        np.testing.assert_allclose(w, w2, rtol=0, atol=1e-13)
        np.testing.assert_allclose(b, b2, rtol=0, atol=1e-13)
    # the sum over workers of the per-worker gradients is the whole-batch gradient
    for n in cp:
        tot = sum(g[n][0] for g in r1["worker_grads"])
        np.testing.assert_allclose(tot, r2["worker_grads"][0][n][0], rtol=1e-9, atol=1e-13)


@pytest.mark.parametrize("name,K,B,n_f", [("tiny", 4, 1, 2), ("tiny", 4, 1, 4), ("minimlp", 6, 2, 3), ("minires", 2, 2, 2)])
def test_several_fc_workers_equal_one(o64, name, K, B, n_f):
    """Sec. 4.1.3: with the CONV workers split among n_f FC workers whose gradients are all-reduced, the iteration is
    still the monolithic step on the whole batch (loss parts add up to the global mean, every parameter moves alike)."""
    wl = wl_mod.get_workload(name)
    imgs, labels, cp, cm, fp, fm = _setup(o64, wl, 11, K, B)
    cp2, cm2, fp2, fm2 = (copy.deepcopy(a) for a in (cp, cm, fp, fm))
    r1 = onet.multi_fc_split_step(o64, wl.ops, imgs, labels, cp, cm, fp, fm, 0.01, 0.9, 1e-4, n_f)
    r2 = onet.monolithic_step(o64, wl.ops, np.concatenate(imgs, 0), labels, cp2, cm2, fp2, fm2, 0.01, 0.9, 1e-4)
    assert abs(r1["loss"] - r2["loss"]) < 1e-12
    np.testing.assert_array_equal(r1["pred"], r2["pred"])
    for n in cp:
        for a, b in zip(cp[n], cp2[n]):
            np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
        for a, b in zip(cm[n], cm2[n]):
            np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-13)
    for (w, b), (w2, b2) in zip(fp, fp2):
        np.testing.assert_allclose(w, w2, rtol=0, atol=1e-13)
        np.testing.assert_allclose(b, b2, rtol=0, atol=1e-13)
    for (w, b), (w2, b2) in zip(fm, fm2):
        np.testing.assert_allclose(w, w2, rtol=1e-9, atol=1e-13)
        np.testing.assert_allclose(b, b2, rtol=1e-9, atol=1e-13)


def test_partial_softmax_ce_parts_add_up(o64):
    r = np.random.default_rng(3)
    z = r.standard_normal((12, 7))
    y = r.integers(0, 7, 12).astype(np.int32)
    loss, dz, pred = o64.softmax_ce(z, y)
    parts = [o64.softmax_ce_part(z[a:b], y[a:b], 12) for a, b in ((0, 4), (4, 8), (8, 12))]
    assert abs(sum(p[0] for p in parts) - loss) < 1e-14
    np.testing.assert_allclose(np.concatenate([p[1] for p in parts]), dz, rtol=1e-14, atol=0)
    np.testing.assert_array_equal(np.concatenate([p[2] for p in parts]), pred)
    # a worker holding every row is the single-worker function
    l2, dz2, _ = o64.softmax_ce_part(z, y, 12)
    assert l2 == loss
    np.testing.assert_array_equal(dz2, dz)


def _loss_only(o, wl, imgs, labels, cp, fp):
    feats = np.concatenate([onet.conv_stack_forward(o, wl.ops, im, cp)["feat"].reshape(im.shape[0], -1) for im in imgs], 0)
    a = feats
    for li, (w, b) in enumerate(fp):
        a = o.fc_fwd(a, w, b, relu=li < len(fp) - 1)
    return o.softmax_ce(a, labels)[0]


@pytest.mark.parametrize("name", ["tiny", "minires", "minimlp"])
def test_chain_gradients_match_finite_differences(o64, name):
    """Central differences of the mean loss over the global batch with respect to single conv and FC
    parameters, against the gradients the split step sums over workers."""
    wl = wl_mod.get_workload(name)
    K, B = 2, 1
    imgs, labels, cp, cm, fp, fm = _setup(o64, wl, 5, K, B)
    cp_w, fp_w = copy.deepcopy(cp), copy.deepcopy(fp)
    res = onet.split_step(o64, wl.ops, imgs, labels, cp_w, copy.deepcopy(cm), fp_w, copy.deepcopy(fm), 0.0, 0.0, 0.0)
    rng = np.random.default_rng(0)
    h = 1e-5
    names = list(cp)
    checked = 0
    for trial in range(24):
        n = names[trial % len(names)]
        which = trial % 2
        t = cp[n][which]
        idx = tuple(rng.integers(0, d) for d in t.shape)
        g = sum(wg[n][which][idx] for wg in res["worker_grads"])
        old = t[idx]
        t[idx] = old + h
        lp = _loss_only(o64, wl, imgs, labels, cp, fp)
        t[idx] = old - h
        lm = _loss_only(o64, wl, imgs, labels, cp, fp)
        t[idx] = old
        fd = (lp - lm) / (2 * h)
        assert abs(fd - g) <= 2e-6 * max(1.0, abs(g)) + 1e-8, (n, which, idx, fd, g)
        checked += abs(g) > 1e-9
    assert checked >= 8
    for li in range(len(fp)):
        for which in range(2):
            t = fp[li][which]
            idx = tuple(rng.integers(0, d) for d in t.shape)
            g = res["fc_grads"][li][which][idx]
            old = t[idx]
            t[idx] = old + h
            lp = _loss_only(o64, wl, imgs, labels, cp, fp)
            t[idx] = old - h
            lm = _loss_only(o64, wl, imgs, labels, cp, fp)
            t[idx] = old
            assert abs((lp - lm) / (2 * h) - g) <= 2e-6 * max(1.0, abs(g)) + 1e-8
    # gradient handed back to the workers: perturb one feature through the FC stack alone
    feats = res["feats"].copy()
    for _ in range(4):
        i, j = rng.integers(0, feats.shape[0]), rng.integers(0, feats.shape[1])

        def fc_loss(f):
            a = f
            for li, (w, b) in enumerate(fp):
                a = o64.fc_fwd(a, w, b, relu=li < len(fp) - 1)
            return o64.softmax_ce(a, labels)[0]
        fpl, fml = feats.copy(), feats.copy()
        fpl[i, j] += h
        fml[i, j] -= h
        assert abs((fc_loss(fpl) - fc_loss(fml)) / (2 * h) - res["dfeats"][i, j]) < 1e-7


def test_update_uses_preupdate_weights_and_global_mean(o64):
    """With lr > 0 the gradient handed back must be computed from the weights before the update, and
    the loss gradient must carry 1/n for the global n = K*B (Eq. 1), not the per-worker batch."""
    wl = wl_mod.get_workload("tiny")
    imgs, labels, cp, cm, fp, fm = _setup(o64, wl, 7, 2, 1)
    a = onet.split_step(o64, wl.ops, imgs, labels, copy.deepcopy(cp), copy.deepcopy(cm), copy.deepcopy(fp), copy.deepcopy(fm), 0.5, 0.9, 0.0)
    b = onet.split_step(o64, wl.ops, imgs, labels, copy.deepcopy(cp), copy.deepcopy(cm), copy.deepcopy(fp), copy.deepcopy(fm), 0.0, 0.9, 0.0)
    np.testing.assert_array_equal(a["dfeats"], b["dfeats"])
    # one worker alone on its own sample sees a gradient twice as large for that sample (n halves)
    solo = onet.split_step(o64, wl.ops, imgs[:1], labels[:1], copy.deepcopy(cp), copy.deepcopy(cm), copy.deepcopy(fp), copy.deepcopy(fm), 0.0, 0.9, 0.0)
    np.testing.assert_allclose(solo["dfeats"][0], 2 * b["dfeats"][0], rtol=1e-12, atol=1e-16)


def test_workload_tables_match_printed_counts():
    want = {}
    for line in open(os.path.join(HERE, "golden", "param_counts.txt")):
        if line.strip() and not line.startswith("#"):
            name, part, val, tol = line.split()
            want[(name, part)] = (float(val), float(tol))
    for (name, part), (val, tol) in want.items():
        wl = wl_mod.get_workload(name)
        conv, fc = wl_mod.count_params(wl)
        got = {"conv": conv, "fc": fc, "total": conv + fc, "features": wl.fc_dims[0]}[part]
        assert abs(got - val) <= tol * val + (0 if tol else 0), (name, part, got, val)
    # exact counts of the five configurations, derived from their layer lists
    exact = {"tiny": (5088, 527114), "alexnet": (3747200, 58631144), "vgg16": (14714688, 123642856),
             "resnet50": (23481472, 2049000),
             # MLP of the paper's last table, 3072 inputs: front 3072-1024-1024, back 1024-4096-10
             "mlp": (3072 * 1024 + 1024 + 1024 * 1024 + 1024, 1024 * 4096 + 4096 + 4096 * 10 + 10)}
    for name, pair in exact.items():
        assert wl_mod.count_params(wl_mod.get_workload(name)) == pair
    for name in wl_mod.WORKLOAD_NAMES:
        wl = wl_mod.get_workload(name)
        n, h, w, c = wl_mod.shape_pass(wl)["feat"]
        assert h * w * c == wl.fc_dims[0]
