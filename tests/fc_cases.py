"""Seeded inputs for whole-step tests of the FC worker at the sizes of the benchmark's configurations.

The FC worker's hidden layers end in ReLU, and the backward pass gates on the sign of each hidden unit: a float32
comparison that decides a 0/1 factor.  Among 512 x 4096 pre-activations per layer a handful fall within rounding of
zero, where a float64-accumulating sum and a float32 one may land on different sides; the gradients of that sample then
differ by a whole term, and both answers are right.  So that the step has ONE right answer, a sample whose hidden
pre-activations (or whose two largest logits) come closer than `margin` is drawn again from its own stream until none
does.  This conditions each row on an event of probability about one half and leaves the distributions (features
max(0, N(0,1)), normal weights of variance 2/fan_in, uniform labels) what the bench's are.
The margins are evaluated with numpy float64 matrix products: selection of inputs, not part of the comparison."""
import numpy as np

import workloads as wl_mod


def _forward64(feats, params64):
    """Hidden pre-activations and logits of the given rows, float64."""
    zs, a = [], feats.astype(np.float64)
    for li, (w, b) in enumerate(params64):
        z = a @ w.T + b
        zs.append(z)
        a = np.maximum(z, 0)
    return zs


def row_margin(zs):
    """Per row: the smallest |hidden pre-activation| and the gap between the two largest logits."""
    m = np.full(zs[0].shape[0], np.inf)
    for z in zs[:-1]:
        m = np.minimum(m, np.abs(z).min(axis=1))
    top = np.partition(zs[-1], -2, axis=1)
    return np.minimum(m, top[:, -1] - top[:, -2])


def fc_case(dims, n, seed, margin=1e-4, mom_scale=None):
    """feats [n, dims[0]] = max(0, N(0,1)), labels, params [(W, b)] (normal variance 2/fan_in; biases uniform within
    1/sqrt(fan_in)), momentum buffers ~ N(0, mom_scale[l]^2) (default 5e-4: about the size of the gradients, so that
    neither term of v = m v + g hides the other).  Returns (feats, labels, params, mom, redraws)."""
    L = len(dims) - 1
    params = []
    for li in range(L):
        i, o = dims[li], dims[li + 1]
        w = wl_mod.rng_for(seed, "fcw", li).standard_normal((o, i), dtype=np.float32)
        w *= np.float32((2.0 / i) ** 0.5)
        b = ((wl_mod.rng_for(seed, "fcb", li).random(o, dtype=np.float32) * 2 - 1) * np.float32(i ** -0.5)).astype(np.float32)
        params.append((w, b))
    params64 = [(w.astype(np.float64), b.astype(np.float64)) for w, b in params]
    feats = np.empty((n, dims[0]), np.float32)
    todo = np.arange(n)
    redraws = 0
    for attempt in range(64):
        for i in todo:
            feats[i] = np.maximum(wl_mod.rng_for(seed, "fcx", int(i), attempt).standard_normal(dims[0], dtype=np.float32), 0)
        bad = row_margin(_forward64(feats[todo], params64)) <= margin
        todo = todo[bad]
        if todo.size == 0:
            break
        redraws += int(todo.size)
    assert todo.size == 0, "rows still within the margin after 64 draws"
    labels = wl_mod.rng_for(seed, "fcy").integers(0, dims[-1], size=n, dtype=np.int32)
    ms = mom_scale if mom_scale is not None else [5e-4] * L
    mom = []
    for li, (w, b) in enumerate(params):
        vw = wl_mod.rng_for(seed, "fcvw", li).standard_normal(w.shape, dtype=np.float32)
        vw *= np.float32(ms[li])
        vb = (wl_mod.rng_for(seed, "fcvb", li).standard_normal(b.shape, dtype=np.float32) * np.float32(ms[li])).astype(np.float32)
        mom.append((vw, vb))
    return feats, labels, params, mom, redraws
