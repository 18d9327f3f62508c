"""CPU checker (test infrastructure only) for the all-reduce among CONV workers, Sec. 4.1.2 of the paper.

The schedule is recursive doubling.  Every worker keeps a buffer; in round i = 1, 2, ... worker j sends its buffer
to the worker 2^(i-1) places away (j xor 2^(i-1)), receives that worker's buffer and adds it to its own.  After
log2 K rounds every worker holds the sum of all K gradients.  (The paper prints the distance as "2i-1"; the
algorithm it cites, and its own count of log2 8 = 3 rounds for 8 workers, fix it as 2^(i-1).)

When K is not a power of two, K - P "surplus" workers (P = 2^floor(log2 K)) first send their gradients to K - P of
the others, recursive doubling runs on the P workers, and a last round returns the result to the surplus workers:
floor(log2 K) + 2 rounds.  The paper picks the surplus workers and their partners at random; the reading taken here
and by the library under test is: the surplus workers are the last K - P, and surplus worker P + i is paired with
worker i.

The tensors are float32 in the software the paper ran, and the point of the schedule (footnote of Sec. 4.1.2) is
that every worker ends with the same bits, so this file adds in the precision of its inputs, one rounding per
addition, and simulates every worker rather than computing one tree.

This file shares nothing with the GPU library and is never imported by it.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np


def recursive_doubling_allreduce(grads: List[np.ndarray]) -> Tuple[List[np.ndarray], int]:
    """Simulate the all-reduce over K = len(grads) workers.  Returns (what every worker holds at the end, number of
    communication rounds).  Additions are done in the dtype of the inputs."""
    K = len(grads)
    assert K >= 1
    dtype = grads[0].dtype
    buf = [np.array(g, dtype=dtype, copy=True) for g in grads]
    if K == 1:
        return buf, 0
    P = 1
    while P * 2 <= K:
        P *= 2
    surplus = K - P
    rounds = 0
    if surplus:
        # extra round before: surplus worker P + i -> worker i
        for i in range(surplus):
            received = buf[P + i]
            buf[i] = (buf[i] + received).astype(dtype)
        rounds += 1
    dist = 1
    while dist < P:
        # all P workers exchange at once: build the new buffers from the old ones
        old = buf[:P]
        new = []
        for j in range(P):
            received = old[j ^ dist]
            new.append((old[j] + received).astype(dtype))
        buf[:P] = new
        dist *= 2
        rounds += 1
    if surplus:
        # extra round after: worker i returns the result to surplus worker P + i
        for i in range(surplus):
            buf[P + i] = buf[i].copy()
        rounds += 1
    return buf, rounds


def ps_aggregate_rd(w: np.ndarray, v: np.ndarray, grads: List[np.ndarray], scale: float, lr: float, momentum: float,
                    wd: float) -> None:
    """All-reduce as above, then the momentum-SGD update of Sec. 6.1 on the result (worker 0's copy; all copies are
    identical), in place on w and v.  The update itself is evaluated in float64 and stored in the dtype of w."""
    held, _ = recursive_doubling_allreduce(grads)
    s = held[0].astype(np.float64)
    g = scale * s + wd * w.astype(np.float64)
    vel = momentum * v.astype(np.float64) + g
    v[...] = vel.astype(v.dtype)
    w[...] = (w.astype(np.float64) - lr * vel).astype(w.dtype)
