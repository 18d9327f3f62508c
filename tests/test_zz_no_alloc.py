"""The aggregation entry point that allocates nothing (stanza_ps_aggregate_static: its pointer table lives in a fixed array of
the library's device image) against the workspace form it is a variant of, through the C ABI: two calls in a row, the second
with a smaller input, so that what the first call left in the array lies behind the second call's table."""
import numpy as np
import pytest
import torch

import workloads as wl_mod
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    a.load()
    assert torch.cuda.is_available()
    return a


def _run_both(api, numels, K, seed, order, hyper):
    ws_, vs_, gs_ = wl_mod.gen_ps_case(numels, K, seed=seed)
    out = []
    for static in (False, True):
        gw, gv = [dev(a) for a in ws_], [dev(a) for a in vs_]
        gg = [[dev(gs_[t][k]) for t in range(len(numels))] for k in range(K)]
        if static:
            api.stanza_ps_aggregate_static(order, gw, gv, gg, *hyper)
        else:
            ws = torch.empty(api.stanza_ps_workspace_bytes(len(numels), K), dtype=torch.uint8, device="cuda:0")
            api.stanza_ps_aggregate_ordered(order, gw, gv, gg, *hyper, ws)
        out.append(([host(t) for t in gw], [host(t) for t in gv]))
    (w_ws, v_ws), (w_st, v_st) = out
    for t in range(len(numels)):
        # same kernel, same table contents, fixed summation order: the two forms agree bit for bit
        np.testing.assert_array_equal(w_st[t], w_ws[t])
        np.testing.assert_array_equal(v_st[t], v_ws[t])
        assert not np.array_equal(w_st[t], ws_[t])
    return w_st, v_st, (ws_, vs_, gs_)


def test_static_aggregation_equals_workspace_form_on_two_calls(api, o32):
    from gpu_util import rel_err
    hyper = (1.0, 0.01, 0.9, 5e-4)
    # first call: 40 tensors, K = 16 (801 table words: two fill launches), ragged and whole chunks
    big = [4096 * 3 + 5, 1000, 64 * 27, 64, 4097, 8, 4096, 12345] * 5
    _run_both(api, big, 16, 51, api.SUM_INDEX_ORDER, hyper)
    # second call, smaller in every way (3 tensors, K = 3: 22 words), other summation order
    small = [5000, 17, 4096]
    w_st, v_st, (ws_, vs_, gs_) = _run_both(api, small, 3, 52, api.SUM_RECURSIVE_DOUBLING, hyper)
    # and the small call against the checker
    from oracle import allreduce as oar
    for t in range(len(small)):
        w_ref, v_ref = ws_[t].copy(), vs_[t].copy()
        oar.ps_aggregate_rd(w_ref, v_ref, gs_[t], *hyper)
        assert rel_err(v_st[t], v_ref) < 1e-5 and rel_err(w_st[t], w_ref) < 1e-6


def test_static_aggregation_refuses_what_does_not_fit(api):
    n = 2000                       # 2000 * (16 + 4) + 1 words > 32768
    w = [torch.zeros(8, device="cuda:0") for _ in range(n)]
    with pytest.raises(api.StanzaError, match="capacity"):
        api.stanza_ps_aggregate_static(api.SUM_INDEX_ORDER, w, w, [w] * 16, 1.0, 0.01, 0.9, 0.0)
