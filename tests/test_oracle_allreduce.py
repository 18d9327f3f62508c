"""Pins for the checker's recursive-doubling all-reduce (Sec. 4.1.2): properties the paper states, a tree typed out
by hand, exact integer sums, a brute-force simulation of the message exchange written independently, and a case in
which the order of the additions is visible in the result."""
import math

import numpy as np
import pytest

from oracle import allreduce as ar
from oracle import perf_model as pm


def _grads(K, n, seed, dtype=np.float32):
    r = np.random.default_rng(seed)
    return [r.standard_normal(n).astype(dtype) for _ in range(K)]


@pytest.mark.parametrize("K", list(range(1, 18)) + [31, 32, 33])
def test_every_worker_holds_the_same_bits_and_the_round_count(K):
    held, rounds = ar.recursive_doubling_allreduce(_grads(K, 257, K))
    assert len(held) == K
    for h in held[1:]:
        assert np.array_equal(h.view(np.uint32), held[0].view(np.uint32))
    # Sec. 4.1.2: log2 K rounds for a power of two, floor(log2 K) + 2 otherwise
    if K == 1:
        assert rounds == 0
    elif K & (K - 1) == 0:
        assert rounds == int(math.log2(K))
    else:
        assert rounds == int(math.floor(math.log2(K))) + 2
    assert rounds == pm.allreduce_rounds(K)


def test_eight_workers_take_three_rounds():
    # the paper's worked count: "log2 8, i.e. 3 rounds ... with 8 CONV workers"
    assert ar.recursive_doubling_allreduce(_grads(8, 5, 0))[1] == 3


def test_power_of_two_is_the_balanced_tree_typed_out():
    g = _grads(8, 1000, 3)
    f = np.float32
    want = ((g[0] + g[1]) + (g[2] + g[3])) + ((g[4] + g[5]) + (g[6] + g[7]))
    assert want.dtype == f
    got = ar.recursive_doubling_allreduce(g)[0][0]
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    g = _grads(4, 1000, 4)
    want = (g[0] + g[1]) + (g[2] + g[3])
    assert np.array_equal(ar.recursive_doubling_allreduce(g)[0][3].view(np.uint32), want.view(np.uint32))


def test_surplus_workers_are_folded_in_before_the_tree():
    # K = 6: P = 4, surplus workers 4 and 5 send to workers 0 and 1
    g = _grads(6, 1000, 5)
    want = (((g[0] + g[4]) + (g[1] + g[5])) + (g[2] + g[3]))
    held = ar.recursive_doubling_allreduce(g)[0]
    for h in held:
        assert np.array_equal(h.view(np.uint32), want.view(np.uint32))
    # K = 3: P = 2, worker 2 sends to worker 0
    g = _grads(3, 1000, 6)
    want = (g[0] + g[2]) + g[1]
    assert np.array_equal(ar.recursive_doubling_allreduce(g)[0][1].view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("K", [2, 3, 5, 8, 11, 16])
def test_integer_gradients_sum_exactly(K):
    r = np.random.default_rng(K)
    g = [r.integers(-1000, 1000, 300).astype(np.float32) for _ in range(K)]
    got = ar.recursive_doubling_allreduce(g)[0][0]
    assert np.array_equal(got, np.sum(np.stack(g).astype(np.int64), axis=0).astype(np.float32))


@pytest.mark.parametrize("K", [2, 3, 7, 8, 13, 16])
def test_close_to_the_exact_sum(K):
    g = _grads(K, 4000, 100 + K)
    got = ar.recursive_doubling_allreduce(g)[0][0].astype(np.float64)
    exact = np.sum(np.stack(g).astype(np.float64), axis=0)
    bound = (math.ceil(math.log2(K)) + 1) * 2.0 ** -24 * np.sum(np.abs(np.stack(g).astype(np.float64)), axis=0)
    assert np.all(np.abs(got - exact) <= bound + 1e-30)


def test_the_order_of_additions_is_the_trees_not_the_index_order():
    # 1e8 + 1 rounds to 1e8 in float32, so the grouping decides the result
    f = np.float32
    g = [np.array([v], f) for v in (1e8, 1.0, -1e8, 1.0)]
    tree = ar.recursive_doubling_allreduce(g)[0][0][0]
    assert tree == f(f(f(1e8) + f(1.0)) + f(f(-1e8) + f(1.0)))
    index = f(f(f(f(1e8) + f(1.0)) + f(-1e8)) + f(1.0))
    assert tree == 0.0 and index == 1.0


def test_against_a_message_passing_simulation():
    """Every worker as its own object that only sees the messages it receives."""
    class Worker:
        def __init__(self, rank, g):
            self.rank, self.buf, self.inbox = rank, g.copy(), None

    for K in (2, 5, 8, 12):
        g = _grads(K, 64, 200 + K)
        ws = [Worker(j, g[j]) for j in range(K)]
        P = 1 << (K.bit_length() - 1)
        for i in range(K - P):
            ws[i].buf = ws[i].buf + ws[P + i].buf
        rnd = 1
        while (1 << (rnd - 1)) < P:
            d = 1 << (rnd - 1)          # the partner is 2^(i-1) places away in round i
            for j in range(P):
                ws[j ^ d].inbox = ws[j].buf.copy()
            for j in range(P):
                ws[j].buf = ws[j].buf + ws[j].inbox
            rnd += 1
        for i in range(K - P):
            ws[P + i].buf = ws[i].buf.copy()
        held = ar.recursive_doubling_allreduce(g)[0]
        for j in range(K):
            assert np.array_equal(held[j].view(np.uint32), ws[j].buf.view(np.uint32))


def test_update_after_the_allreduce(o64):
    K, n = 6, 50
    g = _grads(K, n, 9, np.float64)
    r = np.random.default_rng(1)
    w0, v0 = r.standard_normal(n), r.standard_normal(n)
    w, v = w0.copy(), v0.copy()
    ar.ps_aggregate_rd(w, v, g, 0.5, 0.01, 0.9, 5e-4)
    w2, v2 = w0.copy(), v0.copy()
    o64.sgd_momentum(w2, v2, 0.5 * ar.recursive_doubling_allreduce(g)[0][0], 0.01, 0.9, 5e-4)
    np.testing.assert_allclose(w, w2, rtol=1e-13)
    np.testing.assert_allclose(v, v2, rtol=1e-13)
