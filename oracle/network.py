"""CPU checker (test infrastructure only): one training iteration with the CONV and FC
layers on separate workers, and its monolithic twin.

The sequence follows the paper's training process with layer separation (Sec. 3.2):
every CONV worker runs its conv stack forward on its own batch and hands the
activations after the last pooling layer to the FC worker; the FC worker
concatenates them, finishes the forward pass, computes the loss over the global
batch, backpropagates through the FC layers down to the gradient of the received
activations, hands each worker its slice back and updates the FC parameters; the
CONV workers finish backpropagation, their gradients are summed over workers and
the conv parameters are updated.  Only sequencing, slicing and concatenation happen
here; every number is produced by the loops in stanza_oracle.c.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import ConvGeom, Oracle, PoolGeom


def conv_stack_forward(o: Oracle, ops: List[dict], x0, params) -> Dict[str, np.ndarray]:
    """Run the op list; returns every named buffer plus '<dst>#argmax' for pools."""
    buf = {"x0": x0}
    for op in ops:
        kind = op["op"]
        if kind == "conv":
            x = buf[op["src"]]
            n, h, w, c = x.shape
            g = ConvGeom(n, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"])
            wt, b = params[op["name"]]
            buf[op["dst"]] = o.conv_fwd(g, x, wt, b, relu=op["relu"])
        elif kind == "pool":
            x = buf[op["src"]]
            n, h, w, c = x.shape
            g = PoolGeom(n, h, w, c, op["win"], op["stride"], op["pad"], op["relu"])
            buf[op["dst"]], buf[op["dst"] + "#argmax"] = o.pool_relu_fwd(g, x)
        elif kind == "add_relu":
            buf[op["dst"]] = o.add_relu_fwd(buf[op["a"]], buf[op["b"]])
        elif kind == "gap":
            buf[op["dst"]] = o.gap_fwd(buf[op["src"]])
        else:
            raise ValueError(kind)
    return buf


def conv_stack_backward(o: Oracle, ops: List[dict], buf, params, dfeat):
    """Backpropagate dfeat (gradient of the stack's output) through the op list.
    Returns ({conv name: (dW, db)}, {buffer name: gradient}) ."""
    grad: Dict[str, np.ndarray] = {"feat": dfeat.reshape(buf["feat"].shape)}
    pgrads = {}

    def give(name, g):
        grad[name] = g if name not in grad else o.arr(grad[name].astype(np.float64) + g.astype(np.float64))

    for op in reversed(ops):
        kind = op["op"]
        if kind == "conv":
            x = buf[op["src"]]
            n, h, w, c = x.shape
            g = ConvGeom(n, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"])
            dy = grad[op["dst"]]
            if op["relu"]:
                dy = o.relu_bwd(dy, buf[op["dst"]])
            wt, _ = params[op["name"]]
            pgrads[op["name"]] = o.conv_bwd_weight(g, x, dy)
            if op["src"] != "x0":
                give(op["src"], o.conv_bwd_data(g, dy, wt))
        elif kind == "pool":
            x = buf[op["src"]]
            n, h, w, c = x.shape
            g = PoolGeom(n, h, w, c, op["win"], op["stride"], op["pad"], op["relu"])
            give(op["src"], o.pool_relu_bwd(g, grad[op["dst"]], buf[op["dst"]], buf[op["dst"] + "#argmax"]))
        elif kind == "add_relu":
            dz = o.relu_bwd(grad[op["dst"]], buf[op["dst"]])
            give(op["a"], dz)
            give(op["b"], dz)
        elif kind == "gap":
            give(op["src"], o.gap_bwd(grad[op["dst"]], buf[op["src"]].shape))
        else:
            raise ValueError(kind)
    return pgrads, grad


def fc_step(o: Oracle, feats, labels, fc_params, fc_mom, lr, momentum, wd, update=True):
    """FC worker: forward, mean softmax cross-entropy over all rows of feats, backward with the
    pre-update weights, then the momentum-SGD update in place.  Returns a dict with loss, pred,
    dfeats, the activations and the raw gradients."""
    acts = [feats]
    L = len(fc_params)
    for li, (w, b) in enumerate(fc_params):
        acts.append(o.fc_fwd(acts[-1], w, b, relu=(li < L - 1)))
    loss, dz, pred = o.softmax_ce(acts[-1], labels)
    grads = [None] * L
    for li in range(L - 1, -1, -1):
        w, _ = fc_params[li]
        dw, db, da = o.fc_bwd(acts[li], w, dz, need_da=True)
        grads[li] = (dw, db)
        if li > 0:
            dz = o.relu_bwd(da, acts[li])
        else:
            dfeats = da
    if update:
        for (w, b), (vw, vb), (dw, db) in zip(fc_params, fc_mom, grads):
            o.sgd_momentum(w, vw, dw, lr, momentum, wd)
            o.sgd_momentum(b, vb, db, lr, momentum, wd)
    return dict(loss=loss, pred=pred, dfeats=dfeats, acts=acts, grads=grads, dlogits=None)


def fc_grads(o: Oracle, feats, labels, fc_params, n_global):
    """One of several FC workers (Sec. 4.1.3): forward over its own rows, its share of the loss of the global batch,
    backward.  No update: the FC workers first all-reduce their gradients.  Returns loss part, pred, dfeats, grads."""
    acts = [feats]
    L = len(fc_params)
    for li, (w, b) in enumerate(fc_params):
        acts.append(o.fc_fwd(acts[-1], w, b, relu=(li < L - 1)))
    loss, dz, pred = o.softmax_ce_part(acts[-1], labels, n_global)
    grads = [None] * L
    for li in range(L - 1, -1, -1):
        w, _ = fc_params[li]
        dw, db, da = o.fc_bwd(acts[li], w, dz, need_da=True)
        grads[li] = (dw, db)
        if li > 0:
            dz = o.relu_bwd(da, acts[li])
        else:
            dfeats = da
    return dict(loss=loss, pred=pred, dfeats=dfeats, grads=grads)


def multi_fc_split_step(o: Oracle, ops, images: List[np.ndarray], labels, conv_params, conv_mom, fc_params, fc_mom,
                        lr, momentum, wd, n_f: int):
    """The layer-separated iteration with n_f FC workers (Sec. 4.1.3): the K CONV workers are split into n_f equal
    groups, FC worker f serves group f with its own complete copy of the FC layers, the FC workers all-reduce their
    gradients by recursive doubling and every copy applies the same update; the CONV workers all-reduce theirs the
    same way (Sec. 4.1.2).  One copy of the FC parameters is kept here because all copies stay identical."""
    from . import allreduce as ar
    K = len(images)
    assert K % n_f == 0
    per = K // n_f
    B = images[0].shape[0]
    n = K * B
    bufs = [conv_stack_forward(o, ops, o.arr(im), conv_params) for im in images]
    loss, preds, dfeats, fc_worker_grads = 0.0, [], [], []
    for f in range(n_f):
        rows = slice(f * per * B, (f + 1) * per * B)
        feats = np.concatenate([bufs[k]["feat"].reshape(B, -1) for k in range(f * per, (f + 1) * per)], axis=0)
        r = fc_grads(o, feats, labels[rows], fc_params, n)
        loss += r["loss"]
        preds.append(r["pred"])
        dfeats.append(r["dfeats"])
        fc_worker_grads.append(r["grads"])
    dfeats = np.concatenate(dfeats, axis=0)
    worker_grads = []
    for k in range(K):
        pg, _ = conv_stack_backward(o, ops, bufs[k], conv_params, dfeats[k * B:(k + 1) * B])
        worker_grads.append(pg)
    for li, ((w, b), (vw, vb)) in enumerate(zip(fc_params, fc_mom)):
        ar.ps_aggregate_rd(w.reshape(-1), vw.reshape(-1), [np.ascontiguousarray(g[li][0]).reshape(-1) for g in fc_worker_grads],
                           1.0, lr, momentum, wd)
        ar.ps_aggregate_rd(b, vb, [g[li][1] for g in fc_worker_grads], 1.0, lr, momentum, wd)
    for name, (w, b) in conv_params.items():
        vw, vb = conv_mom[name]
        ar.ps_aggregate_rd(w.reshape(-1), vw.reshape(-1), [np.ascontiguousarray(g[name][0]).reshape(-1) for g in worker_grads],
                           1.0, lr, momentum, wd)
        ar.ps_aggregate_rd(b, vb, [g[name][1] for g in worker_grads], 1.0, lr, momentum, wd)
    return dict(loss=loss, pred=np.concatenate(preds), dfeats=dfeats, worker_grads=worker_grads, fc_worker_grads=fc_worker_grads)


def split_step(o: Oracle, ops, images: List[np.ndarray], labels, conv_params, conv_mom, fc_params, fc_mom,
               lr, momentum, wd, keep=False):
    """One layer-separated iteration over K = len(images) CONV workers.  Parameters and momentum
    buffers are updated in place.  Returns loss, pred, per-worker conv gradients and (keep=True)
    all intermediates."""
    K = len(images)
    bufs = [conv_stack_forward(o, ops, o.arr(im), conv_params) for im in images]
    B = images[0].shape[0]
    feats = np.concatenate([b["feat"].reshape(B, -1) for b in bufs], axis=0)
    fc = fc_step(o, feats, labels, fc_params, fc_mom, lr, momentum, wd)
    worker_grads, worker_bgrads = [], []
    for k in range(K):
        pg, bg = conv_stack_backward(o, ops, bufs[k], conv_params, fc["dfeats"][k * B:(k + 1) * B])
        worker_grads.append(pg)
        worker_bgrads.append(bg)
    for name, (w, b) in conv_params.items():
        vw, vb = conv_mom[name]
        o.ps_aggregate(w.reshape(-1), vw.reshape(-1), [np.ascontiguousarray(g[name][0]).reshape(-1) for g in worker_grads],
                       1.0, lr, momentum, wd)
        o.ps_aggregate(b, vb, [g[name][1] for g in worker_grads], 1.0, lr, momentum, wd)
    out = dict(loss=fc["loss"], pred=fc["pred"], worker_grads=worker_grads, feats=feats, dfeats=fc["dfeats"],
               fc_grads=fc["grads"], fc_acts=fc["acts"])
    if keep:
        out["bufs"] = bufs
        out["buf_grads"] = worker_bgrads
    return out


def monolithic_step(o: Oracle, ops, images_all, labels, conv_params, conv_mom, fc_params, fc_mom, lr, momentum, wd):
    """The same iteration as one model on the whole batch (one worker, no hand-offs)."""
    return split_step(o, ops, [images_all], labels, conv_params, conv_mom, fc_params, fc_mom, lr, momentum, wd)
