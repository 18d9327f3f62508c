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


def conv_stack_forward(o: Oracle, ops: List[dict], x0, params, bn_groups: int = 1) -> Dict[str, np.ndarray]:
    """Run the op list; returns every named buffer plus '<dst>#argmax' for pools and '<dst>#stats' for normalisation
    layers.  bn_groups > 1: x0 stacks the batches of that many workers, and every normalisation layer takes its
    statistics over each worker's rows separately (what the workers do when each runs the stack on its own batch)."""
    buf = {"x0": x0}
    for op in ops:
        kind = op["op"]
        if kind == "conv":
            x = buf[op["src"]]
            n, h, w, c = x.shape
            g = ConvGeom(n, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"], op.get("pad_w", -1))
            wt, b = params[op["name"]]
            buf[op["dst"]] = o.conv_fwd(g, x, wt, b, relu=op["relu"])
        elif kind == "pool":
            x = buf[op["src"]]
            n, h, w, c = x.shape
            g = PoolGeom(n, h, w, c, op["win"], op["stride"], op["pad"], op["relu"])
            buf[op["dst"]], buf[op["dst"] + "#argmax"] = o.pool_relu_fwd(g, x)
        elif kind == "avgpool":
            x = buf[op["src"]]
            n, h, w, c = x.shape
            buf[op["dst"]] = o.avgpool_fwd(PoolGeom(n, h, w, c, op["win"], op["stride"], op["pad"], False), x)
        elif kind == "concat":
            buf[op["dst"]] = np.concatenate([buf[sname] for sname in op["srcs"]], axis=3)
        elif kind == "bn":
            x = buf[op["src"]]
            gamma, beta = params[op["name"]]
            per = x.shape[0] // bn_groups
            assert per * bn_groups == x.shape[0]
            parts = [o.bn_fwd(np.ascontiguousarray(x[i * per:(i + 1) * per]), gamma, beta, op["eps"], op["relu"])
                     for i in range(bn_groups)]
            buf[op["dst"]] = np.concatenate([p[0] for p in parts], axis=0)
            buf[op["dst"] + "#stats"] = [(p[1], p[2]) for p in parts]
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
            g = ConvGeom(n, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"], op.get("pad_w", -1))
            dy = grad[op["dst"]]
            if op["relu"]:
                dy = o.relu_bwd(dy, buf[op["dst"]])
            wt, bias = params[op["name"]]
            dw, db = o.conv_bwd_weight(g, x, dy)
            pgrads[op["name"]] = (dw, db if bias is not None else None)
            if op["src"] != "x0":
                give(op["src"], o.conv_bwd_data(g, dy, wt))
        elif kind == "pool":
            x = buf[op["src"]]
            n, h, w, c = x.shape
            g = PoolGeom(n, h, w, c, op["win"], op["stride"], op["pad"], op["relu"])
            give(op["src"], o.pool_relu_bwd(g, grad[op["dst"]], buf[op["dst"]], buf[op["dst"] + "#argmax"]))
        elif kind == "avgpool":
            n, h, w, c = buf[op["src"]].shape
            give(op["src"], o.avgpool_bwd(PoolGeom(n, h, w, c, op["win"], op["stride"], op["pad"], False), np.ascontiguousarray(grad[op["dst"]])))
        elif kind == "concat":
            at = 0
            for sname in op["srcs"]:
                cs = buf[sname].shape[3]
                give(sname, np.ascontiguousarray(grad[op["dst"]][..., at:at + cs]))
                at += cs
        elif kind == "bn":
            x, dy = buf[op["src"]], grad[op["dst"]]
            if op["relu"]:
                dy = o.relu_bwd(dy, buf[op["dst"]])
            gamma, _ = params[op["name"]]
            stats = buf[op["dst"] + "#stats"]
            per = x.shape[0] // len(stats)
            dxs, dg, db = [], 0.0, 0.0
            for i, (mean, istd) in enumerate(stats):
                rows = slice(i * per, (i + 1) * per)
                dxi, dgi, dbi = o.bn_bwd(np.ascontiguousarray(x[rows]), np.ascontiguousarray(dy[rows]), gamma, mean, istd)
                dxs.append(dxi)
                dg, db = dg + dgi.astype(np.float64), db + dbi.astype(np.float64)
            pgrads[op["name"]] = (o.arr(dg), o.arr(db))
            give(op["src"], np.concatenate(dxs, axis=0))
        elif kind == "add_relu":
            dz = o.relu_bwd(grad[op["dst"]], buf[op["dst"]])
            give(op["a"], dz)
            give(op["b"], dz)
        elif kind == "gap":
            give(op["src"], o.gap_bwd(grad[op["dst"]], buf[op["src"]].shape))
        else:
            raise ValueError(kind)
    return pgrads, grad


def fc_step(o: Oracle, feats, labels, fc_params, fc_mom, lr, momentum, wd, update=True, dropout=None):
    """FC worker: forward, mean softmax cross-entropy over all rows of feats, backward with the
    pre-update weights, then the momentum-SGD update in place.  Returns a dict with loss, pred,
    dfeats, the activations and the raw gradients.
    dropout = (p, seed, step): every hidden layer's ReLU output passes through seeded dropout (oracle/dropout.py);
    the next layer reads the dropped activations, and the gradient returns through the mask and then the ReLU."""
    from . import dropout as dr
    acts = [feats]            # what each layer reads
    hidden = [None]           # the ReLU outputs before dropout
    L = len(fc_params)
    for li, (w, b) in enumerate(fc_params):
        h = o.fc_fwd(acts[-1], w, b, relu=(li < L - 1))
        hidden.append(h)
        if dropout is not None and li < L - 1:
            h = dr.dropout_fwd(h, dropout[0], dropout[1], dr.fc_stream(dropout[2], li))
        acts.append(h)
    loss, dz, pred = o.softmax_ce(acts[-1], labels)
    grads = [None] * L
    for li in range(L - 1, -1, -1):
        w, _ = fc_params[li]
        dw, db, da = o.fc_bwd(acts[li], w, dz, need_da=True)
        grads[li] = (dw, db)
        if li > 0:
            if dropout is not None:
                da = dr.dropout_bwd(da, dropout[0], dropout[1], dr.fc_stream(dropout[2], li - 1))
            dz = o.relu_bwd(da, hidden[li])
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
        if b is not None:
            ar.ps_aggregate_rd(b, vb, [g[name][1] for g in worker_grads], 1.0, lr, momentum, wd)
    return dict(loss=loss, pred=np.concatenate(preds), dfeats=dfeats, worker_grads=worker_grads, fc_worker_grads=fc_worker_grads)


def split_step(o: Oracle, ops, images: List[np.ndarray], labels, conv_params, conv_mom, fc_params, fc_mom,
               lr, momentum, wd, keep=False, bn_groups: int = 1, dropout=None):
    """One layer-separated iteration over K = len(images) CONV workers.  Parameters and momentum
    buffers are updated in place.  Returns loss, pred, per-worker conv gradients and (keep=True)
    all intermediates."""
    K = len(images)
    bufs = [conv_stack_forward(o, ops, o.arr(im), conv_params, bn_groups) for im in images]
    B = images[0].shape[0]
    feats = np.concatenate([b["feat"].reshape(B, -1) for b in bufs], axis=0)
    fc = fc_step(o, feats, labels, fc_params, fc_mom, lr, momentum, wd, dropout=dropout)
    worker_grads, worker_bgrads = [], []
    for k in range(K):
        pg, bg = conv_stack_backward(o, ops, bufs[k], conv_params, fc["dfeats"][k * B:(k + 1) * B])
        worker_grads.append(pg)
        worker_bgrads.append(bg)
    for name, (w, b) in conv_params.items():
        vw, vb = conv_mom[name]
        o.ps_aggregate(w.reshape(-1), vw.reshape(-1), [np.ascontiguousarray(g[name][0]).reshape(-1) for g in worker_grads],
                       1.0, lr, momentum, wd)
        if b is not None:
            o.ps_aggregate(b, vb, [g[name][1] for g in worker_grads], 1.0, lr, momentum, wd)
    out = dict(loss=fc["loss"], pred=fc["pred"], worker_grads=worker_grads, feats=feats, dfeats=fc["dfeats"],
               fc_grads=fc["grads"], fc_acts=fc["acts"])
    if keep:
        out["bufs"] = bufs
        out["buf_grads"] = worker_bgrads
    return out


def monolithic_step(o: Oracle, ops, images_all, labels, conv_params, conv_mom, fc_params, fc_mom, lr, momentum, wd,
                    bn_groups: int = 1, dropout=None):
    """The same iteration as one model on the whole batch (one worker, no hand-offs).  For stacks with normalisation
    layers, bn_groups = K keeps the statistics per worker batch, which is the model the K workers train together."""
    return split_step(o, ops, [images_all], labels, conv_params, conv_mom, fc_params, fc_mom, lr, momentum, wd,
                      bn_groups=bn_groups, dropout=dropout)
