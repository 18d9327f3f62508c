"""Performance model and node assignment (Sec. 4.2, Sec. 7.1): the checker's closed forms are pinned to the values the
paper prints, and the library's host functions are compared with the checker."""
import math
import os
import random

import pytest

from oracle import perf_model as pm

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    rows = []
    for line in open(os.path.join(HERE, "golden", "perf_model.txt")):
        if line.strip() and not line.startswith("#"):
            rows.append(line.split())
    return rows


def test_checker_matches_printed_values():
    for row in _golden():
        if row[0] == "ps_comm":
            comm = pm.ps_time(float(row[2]) * 1e6, 0.0, 4, 1, 10e9)
            assert abs(comm - float(row[3])) < 0.0051, row          # printed to two decimals
        elif row[0] == "ps_total":
            P, nw, gb, iters, epochs, hours = float(row[2]) * 1e6, int(row[3]), float(row[4]), int(row[5]), int(row[6]), float(row[7])
            total_h = pm.ps_time(P, 0.0, nw, 1, gb * 2 ** 30) * iters * epochs / 3600
            assert 0 <= total_h - hours < 0.01, (row, total_h)        # 3.257 h, printed truncated as 3.25
        elif row[0] == "rounds":
            assert pm.allreduce_rounds(int(row[1])) == int(row[2]), row


def test_checker_structure():
    args = dict(T_c=0.3, T_f=0.01, A=9216, K=128, P_c=3.7e6, bw=10e9)
    # one conv worker, one FC worker: no all-reduce term
    t = pm.stanza_time(n_c=1, n_f=1, **args)
    assert abs(t - (0.3 + 0.01 + 2 * 9216 * 128 * 32 / 10e9)) < 1e-12
    # infinite bandwidth leaves Eq. (2)
    big = dict(args, bw=1e30)
    assert abs(pm.stanza_time(n_c=6, n_f=2, **big) - (0.3 + 3 * 0.01)) < 1e-9
    # assignment really is the arg max over all splits, and its throughput is n_c K / t_s
    for N in (2, 3, 8, 17, 80):
        nc, nf, th = pm.assign(N=N, **args)
        assert nc + nf == N and nc >= 1 and nf >= 1
        assert all(th >= pm.stanza_throughput(n_c=c, n_f=N - c, **args) - 1e-9 for c in range(1, N))
        assert abs(th - nc * 128 / pm.stanza_time(n_c=nc, n_f=nf, **args)) < 1e-9
    # an FC-heavy model pulls workers to the FC side
    heavy = dict(args, T_f=0.5)
    assert pm.assign(N=16, **heavy)[1] > pm.assign(N=16, **args)[1]


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    if not os.path.exists(a.LIB_PATH):
        from paper_1812_10624_amd.build import build_library
        build_library()
    a.load()
    return a


def test_library_matches_checker(api):
    rnd = random.Random(7)
    for n in range(1, 200):
        assert api.stanza_model_allreduce_rounds(n) == pm.allreduce_rounds(n)
    for _ in range(300):
        T_c, T_f = rnd.uniform(1e-3, 2), rnd.uniform(1e-4, 0.5)
        A, K, P_c = rnd.choice([2048, 9216, 25088]), rnd.choice([32, 64, 128]), rnd.uniform(1e6, 3e7)
        bw = rnd.choice([2.6 * 2 ** 30, 10e9, 25e9, 100e9, 153e9 * 8])
        m = api.ModelParams(T_c, T_f, A, K, P_c, bw)
        n_c, n_f = rnd.randint(1, 64), rnd.randint(1, 8)
        ref = pm.stanza_time(T_c, T_f, A, K, P_c, bw, n_c, n_f)
        assert math.isclose(api.stanza_model_stanza_time(m, n_c, n_f), ref, rel_tol=1e-12)
        assert math.isclose(api.stanza_model_stanza_throughput(m, n_c, n_f), n_c * K / ref, rel_tol=1e-12)
        N = rnd.randint(2, 100)
        got = api.stanza_model_assign(m, N)
        want = pm.assign(T_c, T_f, A, K, P_c, bw, N)
        assert got[:2] == want[:2] and math.isclose(got[2], want[2], rel_tol=1e-12)
        P, T_ps, nw, ns = rnd.uniform(1e6, 2e8), rnd.uniform(0.01, 2), rnd.randint(1, 64), rnd.randint(1, 8)
        assert math.isclose(api.stanza_model_ps_time(P, T_ps, nw, ns, bw), pm.ps_time(P, T_ps, nw, ns, bw), rel_tol=1e-12)
        assert math.isclose(api.stanza_model_ps_throughput(P, T_ps, K, nw, ns, bw), pm.ps_throughput(P, T_ps, K, nw, ns, bw), rel_tol=1e-12)


def test_library_rejects_bad_arguments(api):
    m = api.ModelParams(0.1, 0.01, 100, 32, 1e6, 1e9)
    assert api.stanza_model_stanza_time(m, 0, 1) < 0
    assert api.stanza_model_stanza_time(m, 1, 0) < 0
    assert api.stanza_model_stanza_time(api.ModelParams(0.1, 0.01, 100, 32, 1e6, 0.0), 1, 1) < 0
    assert api.stanza_model_ps_time(1e6, 0.1, 0, 1, 1e9) < 0
    with pytest.raises(api.StanzaError):
        api.stanza_model_assign(m, 1)
