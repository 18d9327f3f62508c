"""Helpers for the GPU parity tests: the tolerance metric, its report, and host<->device plumbing."""
import json
import os

import numpy as np
import torch

TAU = 0.05
TOL_F32 = 1e-4     # max relative error of the fp32 path (spec tolerance)
TOL_BF16 = 2e-2
# End of a chain of bf16 operations (an FC worker's gradients, a stack's features).  Each operand of a late product carries L
# earlier roundings of relative rms 2^-9 * sqrt(2/3) each (L = 4..6: activations forward, gradients backward, filter copies), so a
# Kd-term sum of size max|ref| ~ 4 sigma has an error of rms ~ sqrt(L) * 2^-9 * 0.82 * sigma; against the floor tau * max|ref| =
# 0.2 sigma that is E ~ 0.016 * sqrt(L) per element and 4.5 times that at the largest of ~1e6 elements: 0.07 * sqrt(L / 4) + the
# final rounding.  Measured on this suite: 0.054 - 0.075.  One bound for all such ends:
TOL_BF16_CHAIN = 0.1
REPORT_TAUS = (1e-3, 1e-2, 0.05)

# every comparison of a run: test id -> [count, E(tau) for tau in REPORT_TAUS, plain inf-norm ratio] (maxima over the test's calls)
REPORT = {}


def _errors(got, ref):
    """(E at each of REPORT_TAUS, |got-ref|_inf / |ref|_inf) for two float64 arrays of one shape."""
    diff = np.abs(got - ref)
    aref = np.abs(ref)
    scale = float(aref.max()) if aref.size else 0.0
    if scale == 0.0:
        m = float(diff.max()) if diff.size else 0.0
        return [m] * len(REPORT_TAUS), m
    return [float((diff / np.maximum(aref, t * scale)).max()) for t in REPORT_TAUS], float(diff.max()) / scale


def note(got, ref, scale_ref=None, tag=""):
    """Record one comparison under the running test's name; returns E at TAU.  scale_ref: max|ref| of the whole tensor
    when got / ref are samples of it; tag: suffix of the report line (e.g. "#chain" for a diagnostic that is not gated)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if scale_ref is None:
        es, linf = _errors(got, ref)
    else:
        diff = np.abs(got - ref)
        s = float(scale_ref) if scale_ref else 1.0
        es = [float((diff / np.maximum(np.abs(ref), t * s)).max()) for t in REPORT_TAUS]
        linf = float(diff.max()) / s
    _record(tag, es, linf)
    return es[REPORT_TAUS.index(TAU)]


def _record(suffix, es, linf):
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0] + suffix
    rec = REPORT.setdefault(test, [0, [0.0] * len(REPORT_TAUS), 0.0])
    rec[0] += 1
    rec[1] = [max(a, b) for a, b in zip(rec[1], es)]
    rec[2] = max(rec[2], linf)


def rel_err(got, ref):
    """E = max_i |got_i - ref_i| / max(|ref_i|, TAU * max|ref|): element-wise relative error with a floor
    for entries that are (near) zero by cancellation.  Every call is also recorded at the other floors (see note)."""
    return note(got, ref)


def param_update_err(got, want, before):
    """A parameter after the step, through the update it received.  The step computes delta = -lr * v and stores
    before + delta rounded to float32 once; that rounding (half a unit in the last place of the PARAMETER, which is
    far larger than the update's own accuracy when |delta| << |w|) lands both sides on the same float or on
    neighbours.  So: E of (got - before) against (want - before) after allowing one unit in the last place of want."""
    got, want, before = (np.asarray(a, np.float64) for a in (got, want, before))
    delta = want - before
    slack = np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)
    excess = np.maximum(np.abs(got - want) - slack, 0.0)
    dmax = float(np.abs(delta).max())
    es = [float((excess / np.maximum(np.abs(delta), t * dmax)).max()) if dmax > 0 else float(excess.max()) for t in REPORT_TAUS]
    _record("#param-update", es, float(excess.max()) / dmax if dmax > 0 else float(excess.max()))
    return es[REPORT_TAUS.index(TAU)]


def families():
    """The report folded to test functions (parametrisations merged): name -> (comparisons, E per tau, inf-norm ratio)."""
    fam = {}
    for test, (cnt, es, linf) in REPORT.items():
        key = test.split("[")[0] + (test[test.index("#"):] if "#" in test and "[" in test else "")
        f = fam.setdefault(key, [0, [0.0] * len(REPORT_TAUS), 0.0])
        f[0] += cnt
        f[1] = [max(a, b) for a, b in zip(f[1], es)]
        f[2] = max(f[2], linf)
    return fam


def write_report(path):
    with open(path, "w") as fh:
        json.dump({"taus": REPORT_TAUS, "tests": REPORT, "families": families()}, fh, indent=1)


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to("cuda:0")


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()
