"""Seeded dropout on the GPU against the CPU checker: the generator's words bit for bit (through the kept / dropped
pattern at several thresholds), the scaled selection, and the FC worker's step with dropout after its hidden layers."""
import copy

import numpy as np
import pytest
import torch

import workloads as wl_mod
from gpu_util import TOL_F32, dev, host, rel_err
from oracle import dropout as odr
from oracle import network as onet

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    a.load()
    assert torch.cuda.is_available()
    return a


@pytest.mark.parametrize("numel", [1, 3, 4, 5, 1023, 4096, 100003, 512 * 4096])      # the last: a VGG-16 hidden layer at n = 512
@pytest.mark.parametrize("p,seed,stream", [(0.5, 0, 0), (0.1, 0x1234567890ABCDEF, (7 << 8) | 1), (0.9, 2 ** 64 - 1, 2 ** 56 + 5), (0.0, 5, 5)])
def test_dropout_mask_and_scale(api, numel, p, seed, stream):
    x = wl_mod.rng_for(1, "drop", numel).standard_normal(numel, dtype=np.float32)
    x[x == 0] = 1.0
    y = torch.full((numel,), float("nan"), device="cuda:0")
    api.stanza_dropout(dev(x), y, p, seed, stream)
    got = host(y)
    keep = odr.keep_mask(numel, p, seed, stream)
    np.testing.assert_array_equal(got != 0, keep)                    # integer work: bit-exact
    ref = odr.dropout_fwd(x, p, seed, stream)
    assert np.abs(got - ref).max() <= 2e-7 * np.abs(ref).max()
    if p == 0.0:
        np.testing.assert_array_equal(got, x)
    # in place
    xd = dev(x)
    api.stanza_dropout(xd, xd, p, seed, stream)
    np.testing.assert_array_equal(host(xd), got)


def test_words_bit_exact_through_thresholds(api):
    """Thirty-two thresholds p = j/32 recover the top five bits of every word: the GPU's pattern equals the checker's."""
    numel, seed, stream = 8192, 99, 12345
    words = odr.random_words(numel, seed, stream)
    x = dev(np.ones(numel, np.float32))
    y = torch.empty(numel, device="cuda:0")
    top = np.zeros(numel, np.int64)
    for j in range(1, 32):
        api.stanza_dropout(x, y, j / 32.0, seed, stream)
        top += host(y) != 0
    np.testing.assert_array_equal(top, words >> 27)


@pytest.mark.parametrize("name,n", [("minimlp", 15), ("tiny", 8)])
def test_fc_step_with_dropout(api, o32, name, n):
    from paper_1812_10624_amd.netrun import FcWorker
    wl = wl_mod.get_workload(name)
    dims = wl.fc_dims if name != "minimlp" else [24, 56, 40, 10]      # two hidden layers: two different streams
    rng = wl_mod.rng_for(3, "dropfc", name)
    feats = np.abs(rng.standard_normal((n, dims[0]), dtype=np.float32))
    labels = rng.integers(0, dims[-1], size=n, dtype=np.int32)
    fp = [((rng.standard_normal((o, i), dtype=np.float32) * np.float32((2.0 / i) ** 0.5)), (rng.standard_normal(o) * 0.1).astype(np.float32))
          for i, o in zip(dims[:-1], dims[1:])]
    fm = [(np.zeros_like(w), np.zeros_like(b)) for w, b in fp]
    p, seed = 0.4, 2024
    gfp = [(dev(w), dev(b)) for w, b in fp]
    gfm = [(dev(w), dev(b)) for w, b in fm]
    fcw = FcWorker(dims, n, gfp, gfm, 0.05, 0.9, 1e-4, dropout=(p, seed))
    fp_ref, fm_ref = copy.deepcopy(fp), copy.deepcopy(fm)
    losses = []
    for step in range(3):                                             # three iterations: three different masks
        ref = onet.fc_step(o32, feats, labels, fp_ref, fm_ref, 0.05, 0.9, 1e-4, dropout=(p, seed, step))
        dfeats = fcw.step(dev(feats), dev(labels))
        assert abs(float(host(fcw.loss)[0]) - ref["loss"]) < 1e-5 * max(1.0, abs(ref["loss"])), step
        assert rel_err(host(dfeats), ref["dfeats"]) < TOL_F32, step
        losses.append(ref["loss"])
        for li in range(len(fp)):
            for i in range(2):
                assert rel_err(host(gfm[li][i]), fm_ref[li][i]) < TOL_F32, (step, li, i)
                assert rel_err(host(gfp[li][i]), fp_ref[li][i]) < 1e-4, (step, li, i)
    assert len(set(losses)) == 3
    # the same worker without dropout takes a different step
    fcw0 = FcWorker(dims, n, [(dev(w), dev(b)) for w, b in fp], [(dev(w), dev(b)) for w, b in fm], 0.05, 0.9, 1e-4)
    fcw0.step(dev(feats), dev(labels))
    ref0 = onet.fc_step(o32, feats, labels, copy.deepcopy(fp), copy.deepcopy(fm), 0.05, 0.9, 1e-4)
    assert abs(float(host(fcw0.loss)[0]) - ref0["loss"]) < 1e-5 * max(1.0, abs(ref0["loss"]))
