"""Workload tables and seeded synthetic inputs shared by the tests, the bench and the checker.

This module holds shapes and random draws only: no convolution, GEMM, loss or
optimiser arithmetic lives here.  Both the HIP path's Python binding and the CPU
checker are driven from the same tables and the same seeded tensors, so that the
two are compared on identical inputs while sharing no code of the method itself.

Layouts (all C-contiguous numpy arrays):
  activations  NHWC float32                 [N][H][W][C]
  conv weights [Kout][R][S][Cin] float32
  FC weights   [out][in] float32
  features     [n][A], A is the NHWC flattening (h*W + w)*C + c of the last map
  labels       int32

The networks are the CNN shapes the paper trains (Evaluation, Setup: table of
models and per-worker batch sizes) at ImageNet / CIFAR input shapes; the images
are N(0,1) noise standing in for those datasets.

A conv stack is an op list over named buffers; every op is a dict:
  {"op": "conv", "name", "src", "dst", "K","R","S","stride","pad","relu","bias"}   bias False: no bias term
  {"op": "bn", "name", "src", "dst", "relu", "eps"}   batch normalisation over the worker's own batch (+ReLU)
  {"op": "pool", "src", "dst", "win","stride","pad","relu"}
  {"op": "avgpool", "src", "dst", "win","stride","pad"}   mean over the part of the window inside the image
  {"op": "concat", "srcs": [...], "dst"}       channel concatenation, in the order listed
  {"op": "add_relu", "a", "b", "dst"}          dst = max(0, a + b)
A conv may carry "pad_w" (and S != R) for the 1xn / nx1 filters of the Inception blocks: "pad" is then the vertical padding.
  {"op": "gap", "src", "dst"}                  global average pool
The first buffer is "x0" (the images) and the last op writes "feat".
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

__all__ = [
    "Workload", "get_workload", "WORKLOAD_NAMES", "shape_pass", "conv_param_shapes",
    "fc_param_shapes", "gen_images", "gen_labels", "gen_conv_params", "gen_fc_params",
    "gen_ps_case", "gen_ps_tensor", "rng_for", "conv_flops", "fc_flops", "count_params", "bn_param_shapes", "flat_tensors",
]


@dataclass
class Workload:
    name: str
    K: int                      # number of conv workers feeding the FC worker
    B: int                      # per-worker batch
    image: Tuple[int, int, int]  # H, W, C
    ops: List[dict]
    fc_dims: List[int]          # A, hidden..., classes
    lr: float = 0.01
    momentum: float = 0.9
    weight_decay: float = 0.0
    notes: str = ""

    @property
    def n(self) -> int:
        return self.K * self.B

    @property
    def classes(self) -> int:
        return self.fc_dims[-1]


def _conv(name, src, dst, K, R, stride=1, pad=0, relu=True, S=None, bias=True, pad_w=None):
    d = dict(op="conv", name=name, src=src, dst=dst, K=K, R=R, S=R if S is None else S,
             stride=stride, pad=pad, relu=relu, bias=bias)
    if pad_w is not None and pad_w != pad:
        d["pad_w"] = pad_w
    return d


def _bn(name, src, dst, relu, eps=1e-5):
    return dict(op="bn", name=name, src=src, dst=dst, relu=relu, eps=eps)


def _pool(src, dst, win, stride, pad=0, relu=True):
    return dict(op="pool", src=src, dst=dst, win=win, stride=stride, pad=pad, relu=relu)


def _chain(spec):
    """spec: list of ("c", K, R, stride, pad) / ("p", win, stride, pad) -> linear op list."""
    ops, cur, ci, pi = [], "x0", 0, 0
    for s in spec:
        if s[0] == "c":
            ci += 1
            dst = f"c{ci}"
            ops.append(_conv(f"conv{ci}", cur, dst, s[1], s[2], s[3], s[4], relu=True))
        else:
            pi += 1
            dst = f"p{pi}"
            ops.append(_pool(cur, dst, s[1], s[2], s[3], relu=True))
        cur = dst
    ops[-1]["dst"] = "feat"
    return ops


def _tiny_ops():
    return _chain([("c", 16, 3, 1, 1), ("p", 2, 2, 0), ("c", 32, 3, 1, 1), ("p", 2, 2, 0)])


def _alexnet_ops():
    return _chain([("c", 96, 11, 4, 2), ("p", 3, 2, 0), ("c", 256, 5, 1, 2), ("p", 3, 2, 0),
                   ("c", 384, 3, 1, 1), ("c", 384, 3, 1, 1), ("c", 256, 3, 1, 1), ("p", 3, 2, 0)])


def _vgg16_ops(reps_per_stage=(2, 2, 3, 3, 3)):
    spec = []
    for width, reps in zip((64, 128, 256, 512, 512), reps_per_stage):
        spec += [("c", width, 3, 1, 1)] * reps + [("p", 2, 2, 0)]
    return _chain(spec)


def _res_unit(ops, name, src, K, R, stride, pad, relu, bn):
    """conv (+ReLU), or with bn: bias-free conv -> batch normalisation (+ReLU).  Returns the output buffer's name."""
    if not bn:
        ops.append(_conv(name, src, name, K, R, stride, pad, relu=relu))
        return name
    ops.append(_conv(name, src, name + "_z", K, R, stride, pad, relu=False, bias=False))
    ops.append(_bn(name + "_bn", name + "_z", name, relu=relu))
    return name


def _bottleneck_stack(stem_width, stages, bn):
    """stages: [(width, blocks, stride of the first block)].  Stem 7x7/2, 3x3/2 max-pool (pad 1), bottleneck blocks
    1x1 -> 3x3 (carries the stride) -> 1x1 with a projection shortcut in the first block of each stage, global
    average pool.  bn: every convolution is bias-free and followed by batch normalisation (the published network);
    otherwise the convolutions carry biases and nothing is normalised."""
    ops = []
    cur = _res_unit(ops, "stem", "x0", stem_width, 7, 2, 3, True, bn)
    ops.append(_pool(cur, "s0", 3, 2, 1, relu=True))
    cur = "s0"
    for si, (width, blocks, first_stride) in enumerate(stages, start=1):
        for bi in range(blocks):
            stride = first_stride if bi == 0 else 1
            tag = f"s{si}b{bi}"
            a = _res_unit(ops, tag + "a", cur, width, 1, 1, 0, True, bn)
            b = _res_unit(ops, tag + "b", a, width, 3, stride, 1, True, bn)
            c = _res_unit(ops, tag + "c", b, 4 * width, 1, 1, 0, False, bn)
            short = _res_unit(ops, tag + "sc", cur, 4 * width, 1, stride, 0, False, bn) if bi == 0 else cur
            ops.append(dict(op="add_relu", a=c, b=short, dst=tag + "o"))
            cur = tag + "o"
    ops.append(dict(op="gap", src=cur, dst="feat"))
    return ops


def _resnet50_ops(depths=(3, 4, 6, 3), bn=False):
    """Stages [3,4,6,3] ([3,8,36,3] for the 152-layer network) of widths 64..512, stride 2 from the second stage on."""
    return _bottleneck_stack(64, [(w, d, 1 if i == 0 else 2) for i, (w, d) in enumerate(zip((64, 128, 256, 512), depths))], bn)


def _mini_res_ops(bn=False, mult=1):
    """A three-block residual stack small enough for exhaustive checks: exercises 7x7/2,
    padded 3x3/2 pooling, 1x1, strided 3x3, projection and identity shortcuts, GAP.  mult scales every width
    (2: all channel counts are multiples of 8, as a bf16 stack needs)."""
    ops = []
    cur = _res_unit(ops, "stem", "x0", 8 * mult, 7, 2, 3, True, bn)
    ops.append(_pool(cur, "s0", 3, 2, 1, relu=True))
    cur = "s0"
    for bi, (width, stride, proj) in enumerate(((4 * mult, 1, True), (4 * mult, 1, False), (8 * mult, 2, True))):
        tag = f"b{bi}"
        a = _res_unit(ops, tag + "a", cur, width, 1, 1, 0, True, bn)
        b = _res_unit(ops, tag + "b", a, width, 3, stride, 1, True, bn)
        c = _res_unit(ops, tag + "c", b, 4 * width, 1, 1, 0, False, bn)
        short = _res_unit(ops, tag + "sc", cur, 4 * width, 1, stride, 0, False, bn) if proj else cur
        ops.append(dict(op="add_relu", a=c, b=short, dst=tag + "o"))
        cur = tag + "o"
    ops.append(dict(op="gap", src=cur, dst="feat"))
    return ops


def _inception_v3_ops(width_div=1, blocks=(3, 4, 2)):
    """The Inception-V3 conv stack as published (Szegedy et al., "Rethinking the Inception architecture"; the variant
    with factorised 7x7 filters and the expanded 8x8 blocks), main tower only: every convolution is bias-free and
    followed by batch normalisation (eps 1e-3) and ReLU.  Stem 3x3/2, 3x3, 3x3 (padded), 3x3/2 max-pool, 1x1, 3x3,
    3x3/2 max-pool; three 35x35 blocks; a grid reduction; four 17x17 blocks with 1x7 / 7x1 filters; a grid reduction;
    two 8x8 blocks with split 1x3 / 3x1 filters; global average pool.  In every block the pooling branch comes last.
    width_div divides every channel count and `blocks` sets how many blocks of each kind: small stacks for exhaustive
    checks."""
    ops = []
    wd = lambda c: max(c // width_div, 2)

    def unit(name, src, K, R, S=None, stride=1, pad=0, pad_w=None):
        ops.append(_conv(name, src, name + "_z", wd(K), R, stride, pad, relu=False, S=S, bias=False, pad_w=pad_w))
        ops.append(_bn(name + "_bn", name + "_z", name, relu=True, eps=1e-3))
        return name

    cur = unit("c1a", "x0", 32, 3, stride=2)
    cur = unit("c2a", cur, 32, 3)
    cur = unit("c2b", cur, 64, 3, pad=1)
    ops.append(_pool(cur, "p1", 3, 2, 0, relu=False)); cur = "p1"
    cur = unit("c3b", cur, 80, 1)
    cur = unit("c4a", cur, 192, 3)
    ops.append(_pool(cur, "p2", 3, 2, 0, relu=False)); cur = "p2"

    def avg(src, dst):
        ops.append(dict(op="avgpool", src=src, dst=dst, win=3, stride=1, pad=1))
        return dst

    def cat(tag, srcs):
        ops.append(dict(op="concat", srcs=srcs, dst=tag))
        return tag

    for i, pf in enumerate((32, 64, 64)[:blocks[0]]):          # 35x35 blocks
        t = f"a{i}"
        b1 = unit(t + "_1x1", cur, 64, 1)
        b5 = unit(t + "_5x5b", unit(t + "_5x5a", cur, 48, 1), 64, 5, pad=2)
        b3 = unit(t + "_3x3c", unit(t + "_3x3b", unit(t + "_3x3a", cur, 64, 1), 96, 3, pad=1), 96, 3, pad=1)
        bp = unit(t + "_pool", avg(cur, t + "_avg"), pf, 1)
        cur = cat(t, [b1, b5, b3, bp])
    # grid reduction 35 -> 17
    b3 = unit("b_3x3", cur, 384, 3, stride=2)
    bd = unit("b_dblc", unit("b_dblb", unit("b_dbla", cur, 64, 1), 96, 3, pad=1), 96, 3, stride=2)
    ops.append(_pool(cur, "b_max", 3, 2, 0, relu=False))
    cur = cat("b", [b3, bd, "b_max"])
    for i, c7 in enumerate((128, 160, 160, 192)[:blocks[1]]):  # 17x17 blocks
        t = f"c{i}x"
        b1 = unit(t + "_1x1", cur, 192, 1)
        b7 = unit(t + "_7c", unit(t + "_7b", unit(t + "_7a", cur, c7, 1), c7, 1, S=7, pad=0, pad_w=3), 192, 7, S=1, pad=3, pad_w=0)
        d = unit(t + "_d1", cur, c7, 1)
        d = unit(t + "_d2", d, c7, 7, S=1, pad=3, pad_w=0)
        d = unit(t + "_d3", d, c7, 1, S=7, pad=0, pad_w=3)
        d = unit(t + "_d4", d, c7, 7, S=1, pad=3, pad_w=0)
        d = unit(t + "_d5", d, 192, 1, S=7, pad=0, pad_w=3)
        bp = unit(t + "_pool", avg(cur, t + "_avg"), 192, 1)
        cur = cat(t, [b1, b7, d, bp])
    # grid reduction 17 -> 8
    b3 = unit("d_3b", unit("d_3a", cur, 192, 1), 320, 3, stride=2)
    b7 = unit("d_7a", cur, 192, 1)
    b7 = unit("d_7b", b7, 192, 1, S=7, pad=0, pad_w=3)
    b7 = unit("d_7c", b7, 192, 7, S=1, pad=3, pad_w=0)
    b7 = unit("d_7d", b7, 192, 3, stride=2)
    ops.append(_pool(cur, "d_max", 3, 2, 0, relu=False))
    cur = cat("d", [b3, b7, "d_max"])
    for i in range(blocks[2]):                                  # 8x8 blocks
        t = f"e{i}"
        b1 = unit(t + "_1x1", cur, 320, 1)
        m = unit(t + "_3a", cur, 384, 1)
        m1 = unit(t + "_3b1", m, 384, 1, S=3, pad=0, pad_w=1)
        m2 = unit(t + "_3b2", m, 384, 3, S=1, pad=1, pad_w=0)
        d = unit(t + "_d2", unit(t + "_d1", cur, 448, 1), 384, 3, pad=1)
        d1 = unit(t + "_d3a", d, 384, 1, S=3, pad=0, pad_w=1)
        d2 = unit(t + "_d3b", d, 384, 3, S=1, pad=1, pad_w=0)
        bp = unit(t + "_pool", avg(cur, t + "_avg"), 192, 1)
        cur = cat(t, [b1, m1, m2, d1, d2, bp])
    ops.append(dict(op="gap", src=cur, dst="feat"))
    return ops


def _mlp_front_ops(widths):
    """The front part of a layer-separated multilayer perceptron (Discussion, "Beyond CNNs"): fully connected
    layers with ReLU, written as 1x1 convolutions over a 1x1 "image" whose channels are the input vector, so that
    the front workers run through the same entry points as CONV workers."""
    ops, cur = [], "x0"
    for i, wdt in enumerate(widths, start=1):
        ops.append(_conv(f"fc_front{i}", cur, f"h{i}", wdt, 1, 1, 0, relu=True))
        cur = f"h{i}"
    ops[-1]["dst"] = "feat"
    return ops


def get_workload(name: str) -> Workload:
    if name == "tiny":
        return Workload("tiny", K=2, B=4, image=(32, 32, 3), ops=_tiny_ops(), fc_dims=[2048, 256, 10])
    if name == "alexnet":
        return Workload("alexnet", K=4, B=128, image=(224, 224, 3), ops=_alexnet_ops(),
                        fc_dims=[9216, 4096, 4096, 1000])
    if name == "vgg16":
        return Workload("vgg16", K=8, B=64, image=(224, 224, 3), ops=_vgg16_ops(),
                        fc_dims=[25088, 4096, 4096, 1000])
    if name == "resnet50":
        return Workload("resnet50", K=16, B=64, image=(224, 224, 3), ops=_resnet50_ops(),
                        fc_dims=[2048, 1000])
    if name == "minires":
        return Workload("minires", K=2, B=3, image=(33, 35, 3), ops=_mini_res_ops(),
                        fc_dims=[32, 7], notes="small residual stack for exhaustive parity")
    # two more networks of the paper's table of models, at its per-worker batch sizes
    if name == "vgg19":
        return Workload("vgg19", K=8, B=64, image=(224, 224, 3), ops=_vgg16_ops((2, 2, 4, 4, 4)),
                        fc_dims=[25088, 4096, 4096, 1000])
    if name == "resnet152":
        return Workload("resnet152", K=8, B=32, image=(224, 224, 3), ops=_resnet50_ops((3, 8, 36, 3)),
                        fc_dims=[2048, 1000], notes="without normalisation layers, like resnet50 here")
    # the residual networks as published: bias-free convolutions, each followed by batch normalisation
    if name == "resnet50bn":
        return Workload("resnet50bn", K=16, B=64, image=(224, 224, 3), ops=_resnet50_ops(bn=True), fc_dims=[2048, 1000])
    if name == "resnet152bn":
        return Workload("resnet152bn", K=8, B=32, image=(224, 224, 3), ops=_resnet50_ops((3, 8, 36, 3), bn=True),
                        fc_dims=[2048, 1000])
    if name == "inception3":
        return Workload("inception3", K=8, B=32, image=(299, 299, 3), ops=_inception_v3_ops(), fc_dims=[2048, 1000],
                        notes="main tower; the auxiliary classifier of the published network is not built")
    if name == "miniinception":
        ops = _inception_v3_ops(width_div=16, blocks=(1, 1, 1))
        return Workload("miniinception", K=2, B=2, image=(139, 139, 3), ops=ops, fc_dims=[2048 // 16, 10],
                        notes="one block of each kind at a sixteenth of the widths, for exhaustive parity")
    if name == "miniinception8":
        ops = _inception_v3_ops(width_div=2, blocks=(1, 1, 1))
        return Workload("miniinception8", K=2, B=2, image=(139, 139, 3), ops=ops, fc_dims=[2048 // 2, 10],
                        notes="one block of each kind at half the widths (every width a multiple of 8), for the bf16 stack")
    if name == "miniresbn":
        return Workload("miniresbn", K=2, B=3, image=(33, 35, 3), ops=_mini_res_ops(bn=True),
                        fc_dims=[32, 7], notes="small normalised residual stack for exhaustive parity")
    if name == "miniresbn16":
        return Workload("miniresbn16", K=2, B=3, image=(33, 35, 3), ops=_mini_res_ops(bn=True, mult=2),
                        fc_dims=[64, 7], notes="the small normalised residual stack with every width doubled (multiples of 8)")
    if name == "mlp":
        # 3 hidden layers of 1024, 1024, 4096 units on 3x32x32 inputs, separated after the second hidden layer;
        # the largest row of the paper's table: total batch 1024, base learning rate 0.08, vanilla SGD
        return Workload("mlp", K=8, B=128, image=(1, 1, 3072), ops=_mlp_front_ops([1024, 1024]),
                        fc_dims=[1024, 4096, 10], lr=0.08, momentum=0.0,
                        notes="layer-separated MLP: front workers 3072-1024-1024, back worker 1024-4096-10")
    if name == "minimlp":
        return Workload("minimlp", K=3, B=5, image=(1, 1, 52), ops=_mlp_front_ops([40, 24]),
                        fc_dims=[24, 56, 10], lr=0.08, momentum=0.0, notes="small MLP for exhaustive parity")
    raise KeyError(name)


WORKLOAD_NAMES = ("tiny", "alexnet", "vgg16", "resnet50", "minires", "mlp", "minimlp", "vgg19", "resnet152",
                  "resnet50bn", "resnet152bn", "miniresbn", "miniresbn16", "inception3", "miniinception", "miniinception8")


def _out_dim(h, win, stride, pad):
    return (h + 2 * pad - win) // stride + 1


def shape_pass(wl: Workload, batch: int | None = None) -> Dict[str, Tuple[int, int, int, int]]:
    """NHWC shape of every named buffer for a batch of `batch` images (default wl.B)."""
    n = wl.B if batch is None else batch
    shapes = {"x0": (n,) + tuple(wl.image)}
    for op in wl.ops:
        if op["op"] == "conv":
            _, h, w, _ = shapes[op["src"]]
            shapes[op["dst"]] = (n, _out_dim(h, op["R"], op["stride"], op["pad"]),
                                 _out_dim(w, op["S"], op["stride"], op.get("pad_w", op["pad"])), op["K"])
        elif op["op"] == "concat":
            parts = [shapes[sname] for sname in op["srcs"]]
            assert all(p[:3] == parts[0][:3] for p in parts), (op, parts)
            shapes[op["dst"]] = parts[0][:3] + (sum(p[3] for p in parts),)
        elif op["op"] in ("pool", "avgpool"):
            _, h, w, c = shapes[op["src"]]
            shapes[op["dst"]] = (n, _out_dim(h, op["win"], op["stride"], op["pad"]),
                                 _out_dim(w, op["win"], op["stride"], op["pad"]), c)
        elif op["op"] == "bn":
            shapes[op["dst"]] = shapes[op["src"]]
        elif op["op"] == "add_relu":
            assert shapes[op["a"]] == shapes[op["b"]], (op, shapes[op["a"]], shapes[op["b"]])
            shapes[op["dst"]] = shapes[op["a"]]
        elif op["op"] == "gap":
            _, h, w, c = shapes[op["src"]]
            shapes[op["dst"]] = (n, 1, 1, c)
        else:
            raise ValueError(op)
    return shapes


def conv_param_shapes(wl: Workload) -> List[Tuple[str, Tuple[int, int, int, int]]]:
    """[(conv name, (Kout, R, S, Cin))] in op order."""
    shapes = shape_pass(wl, 1)
    return [(op["name"], (op["K"], op["R"], op["S"], shapes[op["src"]][3]))
            for op in wl.ops if op["op"] == "conv"]


def fc_param_shapes(wl: Workload) -> List[Tuple[int, int]]:
    """[(out, in)] per FC layer."""
    d = wl.fc_dims
    return [(d[i + 1], d[i]) for i in range(len(d) - 1)]


def bn_param_shapes(wl: Workload) -> List[Tuple[str, int]]:
    """[(normalisation layer name, channels)] in op order."""
    shapes = shape_pass(wl, 1)
    return [(op["name"], shapes[op["src"]][3]) for op in wl.ops if op["op"] == "bn"]


def count_params(wl: Workload) -> Tuple[int, int]:
    """(parameters on the CONV workers: filters, biases, normalisation scales and shifts; parameters on the FC worker)."""
    has_bias = {op["name"]: op.get("bias", True) for op in wl.ops if op["op"] == "conv"}
    conv = sum(k * r * s * c + (k if has_bias[name] else 0) for name, (k, r, s, c) in conv_param_shapes(wl))
    conv += sum(2 * c for _, c in bn_param_shapes(wl))
    fc = sum(o * i + o for o, i in fc_param_shapes(wl))
    return conv, fc


def conv_flops(wl: Workload, batch: int | None = None) -> Tuple[float, float]:
    """(forward, backward) multiply-add flops of the conv stack, 2*M*N*Kd per GEMM pass;
    the first conv has no backward-data pass."""
    shapes = shape_pass(wl, batch)
    fwd = bwd = 0.0
    for op in wl.ops:
        if op["op"] != "conv":
            continue
        n, ho, wo, k = shapes[op["dst"]]
        c = shapes[op["src"]][3]
        f = 2.0 * n * ho * wo * k * c * op["R"] * op["S"]
        fwd += f
        bwd += f if op["src"] == "x0" else 2 * f
    return fwd, bwd


def fc_flops(wl: Workload) -> float:
    """Forward + both backward GEMMs of the FC stack (dA of the first layer included)."""
    return sum(3 * 2.0 * wl.n * o * i for o, i in fc_param_shapes(wl))


# ----------------------------------------------------------------------------
# seeded draws
# ----------------------------------------------------------------------------

def rng_for(seed: int, *stream) -> np.random.Generator:
    """Independent generator per (seed, stream key); the key is hashed position by position
    so that tensors can be drawn in any order and at any subset."""
    key = [int(seed)]
    for s in stream:
        if isinstance(s, str):
            key += [len(s)] + [ord(ch) for ch in s]
        else:
            key.append(int(s))
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(key)))


def gen_images(wl: Workload, seed: int, worker: int, batch: int | None = None) -> np.ndarray:
    n = wl.B if batch is None else batch
    h, w, c = wl.image
    return rng_for(seed, "img", worker).standard_normal((n, h, w, c), dtype=np.float32)


def gen_labels(wl: Workload, seed: int, n: int | None = None) -> np.ndarray:
    n = wl.n if n is None else n
    return rng_for(seed, "lab").integers(0, wl.classes, size=n, dtype=np.int32)


def _kaiming(rng, shape, fan_in):
    w = rng.standard_normal(shape, dtype=np.float32)
    w *= np.float32(math.sqrt(2.0 / fan_in))
    return w


def _bias(rng, n, fan_in):
    b = rng.random(n, dtype=np.float32)
    bound = np.float32(1.0 / math.sqrt(fan_in))
    return (b * 2 - 1) * bound


def gen_conv_params(wl: Workload, seed: int):
    """Parameters held by a CONV worker, in op order.  Convolutions: {name: (W [K,R,S,C], b [K] or None)}, normal
    weights with variance 2/fan_in (scaled down at the joins of a residual stack without normalisation, see below), uniform biases.  Normalisation layers: {name: (gamma [C], beta [C])} drawn around
    1 and 0 (a trained state rather than the initial one, so that neither drops out of the arithmetic)."""
    has_bias = {op["name"]: op.get("bias", True) for op in wl.ops if op["op"] == "conv"}
    conv_shapes = dict(conv_param_shapes(wl))
    bn_shapes = dict(bn_param_shapes(wl))
    # Residual stacks WITHOUT normalisation: with variance-2/fan_in filters everywhere the activations' energy triples at
    # every join (16 joins: features of a few thousand, a loss of hundreds, and momentum SGD at lr 0.01 overflows within
    # two steps).  As in the usual normalisation-free initialisations, the last convolution of a residual branch is
    # scaled by (2 J)^-1/2 (J joins in the stack: the energy then grows by about e over the whole stack) and a projection
    # shortcut by 2^-1/2 (it has no ReLU behind it to halve its output).
    joins = [op for op in wl.ops if op["op"] == "add_relu"]
    scale = {}
    if joins and not bn_shapes:
        produced_by = {op["dst"]: op for op in wl.ops if op["op"] == "conv"}
        for j in joins:
            if j["a"] in produced_by:
                scale[produced_by[j["a"]]["name"]] = (2.0 * len(joins)) ** -0.5
            if j["b"] in produced_by:
                scale[produced_by[j["b"]]["name"]] = 2.0 ** -0.5
    out = {}
    for op in wl.ops:
        name = op.get("name")
        if op["op"] == "conv":
            k, r, s, c = conv_shapes[name]
            fan = r * s * c
            w = _kaiming(rng_for(seed, "cw", name), (k, r, s, c), fan)
            if name in scale:
                w *= np.float32(scale[name])
            out[name] = (w, _bias(rng_for(seed, "cb", name), k, fan) if has_bias[name] else None)
        elif op["op"] == "bn":
            c = bn_shapes[name]
            g = rng_for(seed, "bng", name).standard_normal(c, dtype=np.float32) * np.float32(0.2) + np.float32(1.0)
            b = rng_for(seed, "bnb", name).standard_normal(c, dtype=np.float32) * np.float32(0.2)
            out[name] = (g, b)
    return out


def flat_tensors(d):
    """The tensors of a {name: (a, b)} dict in order, skipping absent biases (None)."""
    return [t for pair in d.values() for t in pair if t is not None]


def gen_fc_params(wl: Workload, seed: int):
    """[(W [out,in], b [out])] per FC layer."""
    out = []
    for li, (o, i) in enumerate(fc_param_shapes(wl)):
        out.append((_kaiming(rng_for(seed, "fw", li), (o, i), i),
                    _bias(rng_for(seed, "fb", li), o, i)))
    return out


def gen_ps_tensor(ti: int, ne: int, K: int, seed: int, fan_in: int = 64, shards: bool = True):
    """Aggregation inputs of ONE tensor (index ti of its set): w (normal, variance 2/fan_in), momentum v ~ N(0, 1e-3^2)
    and (shards=True) the K gradient shards ~ N(0, 1e-3^2).  Every array has its own stream, so a set can be drawn
    tensor by tensor, in any order, and a tensor's shards drawn again later without holding the whole set."""
    w = _kaiming(rng_for(seed, "psw", ti), (ne,), fan_in)
    v = rng_for(seed, "psv", ti).standard_normal(ne, dtype=np.float32)
    v *= np.float32(1e-3)
    shard = []
    for k in range(K if shards else 0):
        g = rng_for(seed, "psg", ti, k).standard_normal(ne, dtype=np.float32)
        g *= np.float32(1e-3)
        shard.append(g)
    return w, v, shard


def gen_ps_case(numels: List[int], K: int, seed: int, fan_ins: List[int] | None = None):
    """Parameter-server aggregation inputs of a whole set: lists over tensors of w, v and the K shards (gen_ps_tensor)."""
    ws, vs, gs = [], [], []
    for ti, ne in enumerate(numels):
        w, v, shard = gen_ps_tensor(ti, ne, K, seed, fan_ins[ti] if fan_ins is not None else 64)
        ws.append(w)
        vs.append(v)
        gs.append(shard)
    return ws, vs, gs


def param_tensor_numels(wl: Workload, which: str) -> Tuple[List[int], List[int]]:
    """(numels, fan_ins) of the per-layer parameter tensors (W then b per layer)."""
    numels, fans = [], []
    if which == "conv":
        has_bias = {op["name"]: op.get("bias", True) for op in wl.ops if op["op"] == "conv"}
        for name, (k, r, s, c) in conv_param_shapes(wl):
            numels += [k * r * s * c] + ([k] if has_bias[name] else [])
            fans += [r * s * c] * (2 if has_bias[name] else 1)
        for _, c in bn_param_shapes(wl):
            numels += [c, c]
            fans += [1, 1]
    else:
        for o, i in fc_param_shapes(wl):
            numels += [o * i, o]
            fans += [i, i]
    return numels, fans


# ----------------------------------------------------------------------------
# bfloat16 storage of seeded tensors (input preparation only: round to nearest even)
# ----------------------------------------------------------------------------

def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly representable in bfloat16."""
    return bf16_to_f32(bf16_bits(a)).reshape(np.shape(a))
