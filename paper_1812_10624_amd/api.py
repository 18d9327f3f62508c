"""ctypes binding of libstanza.so: the same names as include/stanza.h, argument marshalling only.

Tensors are torch CUDA(ROCm) tensors used purely as device buffers; every function passes
`tensor.data_ptr()` and the current stream's handle through the C ABI.  There is no fallback: if
the library is missing or a call returns an error, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("STANZA_LIB", os.path.join(_HERE, "libstanza.so"))   # override: an alternative build of the same library

F32, BF16 = 0, 1
CONV_BIAS, CONV_RELU, CONV_ACCUM, CONV_NINE_TAP = 1, 2, 4, 8
POOL_RELU = 1

EXPORTS = (
    "stanza_strerror", "stanza_version", "stanza_conv_workspace_bytes", "stanza_conv_fwd", "stanza_conv_fwd_res", "stanza_conv_bwd_data",
    "stanza_conv_bwd_weight", "stanza_pool_relu_fwd", "stanza_pool_relu_bwd", "stanza_add_relu_fwd",
    "stanza_add_relu_bwd", "stanza_gap_fwd", "stanza_gap_bwd", "stanza_cast_f32_to_bf16", "stanza_cast_bf16_to_f32",
    "stanza_cast_workspace_bytes", "stanza_cast_plan", "stanza_cast_f32_to_bf16_planned",
    "stanza_bn_workspace_bytes", "stanza_bn_fwd", "stanza_bn_fwd_res", "stanza_bn_bwd", "stanza_conv_stats_bytes", "stanza_conv_fwd_stats",
    "stanza_bn_fwd_stats", "stanza_avgpool_fwd", "stanza_avgpool_bwd", "stanza_copy2d",
    "stanza_fc_workspace_bytes", "stanza_fc_step", "stanza_fc_grads", "stanza_dropout", "stanza_ps_workspace_bytes", "stanza_ps_plan",
    "stanza_ps_aggregate_planned", "stanza_ps_aggregate", "stanza_ps_aggregate_ordered_planned", "stanza_ps_aggregate_ordered", "stanza_ps_aggregate_static",
    "stanza_model_allreduce_rounds", "stanza_model_stanza_time", "stanza_model_stanza_throughput", "stanza_model_assign",
    "stanza_model_ps_time", "stanza_model_ps_throughput",
)


class StanzaError(RuntimeError):
    pass


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "W", "C", "K", "R", "S", "stride_h", "stride_w", "pad_h", "pad_w", "dtype")] + \
               [("flags", C.c_uint32)]


class PoolDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("N", "H", "W", "C", "win_h", "win_w", "stride_h", "stride_w", "pad_h", "pad_w")] + \
               [("flags", C.c_uint32)]


class ModelParams(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("T_c", "T_f", "A", "K", "P_c", "bandwidth_bits")]


class FcDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("host_dims", C.POINTER(C.c_int32)), ("n_samples", C.c_int32),
                ("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float),
                ("dropout_p", C.c_float), ("dropout_seed", C.c_uint64), ("dropout_step", C.c_uint64), ("compute_dtype", C.c_int32)]


_lib = None
_tape = None             # while a list: every library call made through this module is also appended to it as (function, arguments)


class _Taping:
    """Stands in for the library while calls are being taped: passes each call on and notes it."""

    def __getattr__(self, name):
        fn = getattr(_lib, name)

        if fn.restype is not C.c_int or name in ("stanza_version",):      # a query, not a launch: nothing to issue again
            return fn

        def call(*args):
            _tape.append((fn, args, name))
            return fn(*args)
        return call


_taping = _Taping()


def tape_calls(tape):
    """tape: a list, or None to stop.  A sequencer whose calls never change (same buffers, same descriptors, same stream) can
    tape one pass and afterwards issue the taped library calls directly, without marshalling their arguments again.  The
    argument objects on the tape keep descriptors alive; the tensors behind the raw pointers are the caller's to keep."""
    global _tape
    load()
    _tape = tape


def replay_call(entry):
    """Issue one taped call again, with the error check of the call that taped it."""
    fn, args, name = entry
    rc = fn(*args)
    if rc:
        _check(rc, name)


def load() -> C.CDLL:
    """Load libstanza.so (built beforehand by `__graft_entry__.build()` / `python -m paper_1812_10624_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib if _tape is None else _taping
    if not os.path.exists(LIB_PATH):
        raise StanzaError(f"{LIB_PATH} is missing: build it with `python -m paper_1812_10624_amd.build` (no CPU fallback exists)")
    lib = C.CDLL(LIB_PATH)
    vp, sz, i32, i64, f32 = C.c_void_p, C.c_size_t, C.c_int32, C.c_int64, C.c_float
    lib.stanza_strerror.restype = C.c_char_p
    lib.stanza_strerror.argtypes = [C.c_int]
    lib.stanza_version.restype = C.c_int
    lib.stanza_conv_workspace_bytes.restype = sz
    lib.stanza_conv_workspace_bytes.argtypes = [C.POINTER(ConvDesc), C.c_int]
    lib.stanza_conv_fwd.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp, vp, sz, vp]
    lib.stanza_conv_fwd_res.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stanza_conv_bwd_data.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stanza_conv_bwd_weight.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stanza_pool_relu_fwd.argtypes = [C.POINTER(PoolDesc), i32, vp, vp, vp, vp]
    lib.stanza_pool_relu_bwd.argtypes = [C.POINTER(PoolDesc), i32, vp, vp, vp, vp, vp]
    lib.stanza_add_relu_fwd.argtypes = [i64, i32, vp, vp, vp, vp]
    lib.stanza_add_relu_bwd.argtypes = [i64, i32, vp, vp, vp, vp]
    lib.stanza_gap_fwd.argtypes = [i32, i32, i32, i32, vp, vp, vp]
    lib.stanza_gap_bwd.argtypes = [i32, i32, i32, i32, vp, vp, vp]
    lib.stanza_cast_f32_to_bf16.argtypes = [i64, vp, vp, vp]
    lib.stanza_cast_workspace_bytes.restype = sz
    lib.stanza_cast_workspace_bytes.argtypes = [i32]
    lib.stanza_cast_plan.argtypes = [i32, vp, vp, vp, vp, sz, vp]
    lib.stanza_cast_f32_to_bf16_planned.argtypes = [i32, vp, vp, sz, vp]
    lib.stanza_cast_bf16_to_f32.argtypes = [i64, vp, vp, vp]
    lib.stanza_avgpool_fwd.argtypes = [C.POINTER(PoolDesc), i32, vp, vp, vp]
    lib.stanza_avgpool_bwd.argtypes = [C.POINTER(PoolDesc), i32, vp, vp, vp]
    lib.stanza_copy2d.argtypes = [i64, i32, vp, i64, vp, i64, vp]
    lib.stanza_bn_workspace_bytes.restype = sz
    lib.stanza_bn_workspace_bytes.argtypes = [i64, i32, i32]
    lib.stanza_bn_fwd.argtypes = [i64, i32, i32, f32, i32, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, sz, vp]
    lib.stanza_bn_fwd_res.argtypes = [i64, i32, i32, f32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, sz, vp]
    lib.stanza_conv_stats_bytes.argtypes = [C.POINTER(ConvDesc)]
    lib.stanza_conv_stats_bytes.restype = sz
    lib.stanza_conv_fwd_stats.argtypes = [C.POINTER(ConvDesc), vp, vp, vp, vp, vp, sz, vp, sz, vp]
    lib.stanza_bn_fwd_stats.argtypes = [i64, i32, f32, i32, vp, vp, sz, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp]
    lib.stanza_bn_bwd.argtypes = [i64, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stanza_fc_workspace_bytes.restype = sz
    lib.stanza_fc_workspace_bytes.argtypes = [C.POINTER(FcDesc)]
    lib.stanza_fc_step.argtypes = [C.POINTER(FcDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stanza_fc_grads.argtypes = [C.POINTER(FcDesc), i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.stanza_dropout.argtypes = [i64, f32, C.c_uint64, C.c_uint64, vp, vp, vp]
    lib.stanza_ps_workspace_bytes.restype = sz
    lib.stanza_ps_workspace_bytes.argtypes = [i32, i32]
    lib.stanza_ps_plan.argtypes = [i32, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.stanza_ps_aggregate_planned.argtypes = [i32, vp, i32, f32, f32, f32, f32, vp, sz, vp]
    lib.stanza_ps_aggregate.argtypes = [i32, vp, vp, vp, vp, i32, f32, f32, f32, f32, vp, sz, vp]
    lib.stanza_ps_aggregate_ordered_planned.argtypes = [i32, i32, vp, i32, f32, f32, f32, f32, vp, sz, vp]
    lib.stanza_ps_aggregate_ordered.argtypes = [i32, i32, vp, vp, vp, vp, i32, f32, f32, f32, f32, vp, sz, vp]
    lib.stanza_ps_aggregate_static.argtypes = [i32, i32, vp, vp, vp, vp, i32, f32, f32, f32, f32, vp]
    f64 = C.c_double
    lib.stanza_model_allreduce_rounds.restype = i32
    lib.stanza_model_allreduce_rounds.argtypes = [i32]
    lib.stanza_model_stanza_time.restype = f64
    lib.stanza_model_stanza_time.argtypes = [C.POINTER(ModelParams), i32, i32]
    lib.stanza_model_stanza_throughput.restype = f64
    lib.stanza_model_stanza_throughput.argtypes = [C.POINTER(ModelParams), i32, i32]
    lib.stanza_model_assign.argtypes = [C.POINTER(ModelParams), i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(f64)]
    lib.stanza_model_ps_time.restype = f64
    lib.stanza_model_ps_time.argtypes = [f64, f64, i32, i32, f64]
    lib.stanza_model_ps_throughput.restype = f64
    lib.stanza_model_ps_throughput.argtypes = [f64, f64, f64, i32, i32, f64]
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        raise StanzaError(f"{what}: {load().stanza_strerror(rc).decode()} ({rc})")


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor expected"
    return C.c_void_p(t.data_ptr())


_issue_stream = None     # torch.cuda.Stream that the next calls are enqueued on instead of torch's current stream


def set_stream(stream):
    """Every following call goes to `stream` (None: back to torch's current stream).  For a sequencer that spreads independent
    calls over several streams and orders them with events; cheaper than switching torch's current stream around each call."""
    global _issue_stream
    _issue_stream = stream


def _stream():
    return C.c_void_p((torch.cuda.current_stream() if _issue_stream is None else _issue_stream).cuda_stream)


def _ws(t: Optional[torch.Tensor]):
    return (None, 0) if t is None else (_ptr(t), t.numel() * t.element_size())


def conv_desc(N, H, W, Cin, K, R, S, stride, pad, dtype=F32, flags=0, pad_w=None) -> ConvDesc:
    return ConvDesc(N, H, W, Cin, K, R, S, stride, stride, pad, pad if pad_w is None else pad_w, dtype, flags)


def pool_desc(N, H, W, Cc, win, stride, pad, relu=True) -> PoolDesc:
    return PoolDesc(N, H, W, Cc, win, win, stride, stride, pad, pad, POOL_RELU if relu else 0)


def conv_out_hw(d: ConvDesc):
    return ((d.H + 2 * d.pad_h - d.R) // d.stride_h + 1, (d.W + 2 * d.pad_w - d.S) // d.stride_w + 1)


def stanza_conv_workspace_bytes(d: ConvDesc, which: int) -> int:
    return int(load().stanza_conv_workspace_bytes(C.byref(d), which))


def stanza_conv_fwd(d: ConvDesc, x, w, bias, y, ws=None):
    p, n = _ws(ws)
    _check(load().stanza_conv_fwd(C.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), p, n, _stream()), "stanza_conv_fwd")


def stanza_conv_fwd_res(d: ConvDesc, x, w, bias, res, y, ws=None):
    p, n = _ws(ws)
    _check(load().stanza_conv_fwd_res(C.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(res), _ptr(y), p, n, _stream()), "stanza_conv_fwd_res")


def stanza_conv_bwd_data(d: ConvDesc, dy, y, w, x_mask, dx, ws=None):
    p, n = _ws(ws)
    _check(load().stanza_conv_bwd_data(C.byref(d), _ptr(dy), _ptr(y), _ptr(w), _ptr(x_mask), _ptr(dx), p, n, _stream()),
           "stanza_conv_bwd_data")


def stanza_conv_bwd_weight(d: ConvDesc, x, dy, y, dw, dbias, ws):
    p, n = _ws(ws)
    _check(load().stanza_conv_bwd_weight(C.byref(d), _ptr(x), _ptr(dy), _ptr(y), _ptr(dw), _ptr(dbias), p, n, _stream()),
           "stanza_conv_bwd_weight")


def stanza_pool_relu_fwd(d: PoolDesc, x, y, argmax, dtype=F32):
    _check(load().stanza_pool_relu_fwd(C.byref(d), dtype, _ptr(x), _ptr(y), _ptr(argmax), _stream()), "stanza_pool_relu_fwd")


def stanza_pool_relu_bwd(d: PoolDesc, dy, y, argmax, dx, dtype=F32):
    _check(load().stanza_pool_relu_bwd(C.byref(d), dtype, _ptr(dy), _ptr(y), _ptr(argmax), _ptr(dx), _stream()), "stanza_pool_relu_bwd")


def stanza_add_relu_fwd(a, b, o, dtype=F32):
    _check(load().stanza_add_relu_fwd(a.numel(), dtype, _ptr(a), _ptr(b), _ptr(o), _stream()), "stanza_add_relu_fwd")


def stanza_add_relu_bwd(dout, o, dz, dtype=F32):
    _check(load().stanza_add_relu_bwd(dout.numel(), dtype, _ptr(dout), _ptr(o), _ptr(dz), _stream()), "stanza_add_relu_bwd")


def stanza_gap_fwd(x, f, dtype=F32):
    n, h, w, c = x.shape
    _check(load().stanza_gap_fwd(n, h * w, c, dtype, _ptr(x), _ptr(f), _stream()), "stanza_gap_fwd")


def stanza_gap_bwd(df, dx, dtype=F32):
    n, h, w, c = dx.shape
    _check(load().stanza_gap_bwd(n, h * w, c, dtype, _ptr(df), _ptr(dx), _stream()), "stanza_gap_bwd")


def stanza_cast_f32_to_bf16(src, dst):
    _check(load().stanza_cast_f32_to_bf16(src.numel(), _ptr(src), _ptr(dst), _stream()), "stanza_cast_f32_to_bf16")


class CastPlan:
    """float32 -> bfloat16 copies of a list of tensors in one launch (stanza_cast_plan + stanza_cast_f32_to_bf16_planned)."""

    def __init__(self, srcs, dsts):
        import torch
        assert len(srcs) == len(dsts) and len(srcs) > 0
        for a, b in zip(srcs, dsts):
            assert a.is_cuda and b.is_cuda and a.is_contiguous() and b.is_contiguous() and a.numel() == b.numel()
            assert a.dtype == torch.float32 and b.dtype == torch.bfloat16
        self.n = len(srcs)
        self.numel = (C.c_int64 * self.n)(*[t.numel() for t in srcs])
        self.keep = (list(srcs), list(dsts))                 # the table holds their addresses
        self.ws = torch.empty(int(load().stanza_cast_workspace_bytes(self.n)), dtype=torch.uint8, device=srcs[0].device)
        _check(load().stanza_cast_plan(self.n, self.numel, _ptr_array(srcs), _ptr_array(dsts), _ptr(self.ws), self.ws.numel(), _stream()),
               "stanza_cast_plan")

    def run(self):
        _check(load().stanza_cast_f32_to_bf16_planned(self.n, self.numel, _ptr(self.ws), self.ws.numel(), _stream()),
               "stanza_cast_f32_to_bf16_planned")


def stanza_cast_bf16_to_f32(src, dst):
    _check(load().stanza_cast_bf16_to_f32(src.numel(), _ptr(src), _ptr(dst), _stream()), "stanza_cast_bf16_to_f32")


def stanza_avgpool_fwd(d: PoolDesc, x, y, dtype=F32):
    _check(load().stanza_avgpool_fwd(C.byref(d), dtype, _ptr(x), _ptr(y), _stream()), "stanza_avgpool_fwd")


def stanza_avgpool_bwd(d: PoolDesc, dy, dx, dtype=F32):
    _check(load().stanza_avgpool_bwd(C.byref(d), dtype, _ptr(dy), _ptr(dx), _stream()), "stanza_avgpool_bwd")


def stanza_copy2d(rows: int, cols: int, src, src_off: int, src_ld: int, dst, dst_off: int, dst_ld: int):
    """dst[dst_off + r*dst_ld + j] = src[src_off + r*src_ld + j] for r < rows, j < cols, in elements of the tensors' type.
    The library copies 4-byte elements: bfloat16 tensors go as pairs, so every length and offset must be even."""
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous() and src.dtype == dst.dtype
    assert src.dtype in (torch.float32, torch.bfloat16)
    assert src_off + (rows - 1) * src_ld + cols <= src.numel() and dst_off + (rows - 1) * dst_ld + cols <= dst.numel()
    if src.dtype == torch.bfloat16:
        assert cols % 2 == 0 and src_off % 2 == 0 and src_ld % 2 == 0 and dst_off % 2 == 0 and dst_ld % 2 == 0
        cols, src_off, src_ld, dst_off, dst_ld = cols // 2, src_off // 2, src_ld // 2, dst_off // 2, dst_ld // 2
    _check(load().stanza_copy2d(rows, cols, C.c_void_p(src.data_ptr() + 4 * src_off), src_ld, C.c_void_p(dst.data_ptr() + 4 * dst_off), dst_ld,
                                _stream()), "stanza_copy2d")


def stanza_copy_channels(src, src_off: int, dst, dst_off: int, cols: int):
    """stanza_copy2d over NHWC tensors: src[..., src_off:src_off+cols] -> dst[..., dst_off:dst_off+cols] (C fastest)."""
    cs, cd = src.shape[-1], dst.shape[-1]
    rows = src.numel() // cs
    assert rows == dst.numel() // cd and src_off + cols <= cs and dst_off + cols <= cd
    stanza_copy2d(rows, cols, src, src_off, cs, dst, dst_off, cd)


def stanza_bn_workspace_bytes(rows: int, channels: int, dtype=F32) -> int:
    return int(load().stanza_bn_workspace_bytes(rows, channels, dtype))


def stanza_bn_fwd(x, gamma, beta, y, save_mean, save_istd, ws, eps=1e-5, relu=False, running_mean=None, running_var=None,
                  momentum=0.1, dtype=F32):
    c = x.shape[-1]
    p, n = _ws(ws)
    _check(load().stanza_bn_fwd(x.numel() // c, c, dtype, eps, int(relu), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(save_mean),
                                _ptr(save_istd), _ptr(running_mean), _ptr(running_var), momentum, p, n, _stream()), "stanza_bn_fwd")


def stanza_bn_fwd_res(x, gamma, beta, res, y, save_mean, save_istd, ws, eps=1e-5, relu=True, running_mean=None, running_var=None,
                      momentum=0.1, dtype=F32):
    c = x.shape[-1]
    p, n = _ws(ws)
    _check(load().stanza_bn_fwd_res(x.numel() // c, c, dtype, eps, int(relu), _ptr(x), _ptr(gamma), _ptr(beta), _ptr(res), _ptr(y),
                                    _ptr(save_mean), _ptr(save_istd), _ptr(running_mean), _ptr(running_var), momentum, p, n, _stream()),
           "stanza_bn_fwd_res")


def stanza_conv_stats_bytes(d: ConvDesc) -> int:
    return int(load().stanza_conv_stats_bytes(C.byref(d)))


def stanza_conv_fwd_stats(d: ConvDesc, x, w, bias, y, stats, ws=None):
    p, n = _ws(ws)
    _check(load().stanza_conv_fwd_stats(C.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), _ptr(stats), stats.numel() * stats.element_size(),
                                        p, n, _stream()), "stanza_conv_fwd_stats")


def stanza_bn_fwd_stats(x, stats, gamma, beta, y, save_mean, save_istd, eps=1e-5, relu=False, res=None, running_mean=None, running_var=None,
                        momentum=0.1):
    c = x.shape[-1]
    _check(load().stanza_bn_fwd_stats(x.numel() // c, c, eps, int(relu), _ptr(x), _ptr(stats), stats.numel() * stats.element_size(),
                                      _ptr(gamma), _ptr(beta), _ptr(res), _ptr(y), _ptr(save_mean), _ptr(save_istd), _ptr(running_mean),
                                      _ptr(running_var), momentum, _stream()), "stanza_bn_fwd_stats")


def stanza_bn_bwd(x, dy, gamma, beta, save_mean, save_istd, dx, dgamma, dbeta, ws, relu=False, dtype=F32):
    c = x.shape[-1]
    p, n = _ws(ws)
    _check(load().stanza_bn_bwd(x.numel() // c, c, dtype, int(relu), _ptr(x), _ptr(dy), _ptr(gamma), _ptr(beta), _ptr(save_mean),
                                _ptr(save_istd), _ptr(dx), _ptr(dgamma), _ptr(dbeta), p, n, _stream()), "stanza_bn_bwd")


class FcPlan:
    """Host-side descriptor of an FC stack plus its keep-alive arrays."""

    def __init__(self, dims: Sequence[int], n_samples: int, lr: float, momentum: float, weight_decay: float,
                 dropout_p: float = 0.0, dropout_seed: int = 0, dropout_step: int = 0, compute_dtype: int = F32):
        self.dims = (C.c_int32 * len(dims))(*dims)
        self.desc = FcDesc(len(dims) - 1, self.dims, n_samples, lr, momentum, weight_decay, dropout_p, dropout_seed, dropout_step,
                           compute_dtype)

    def workspace_bytes(self) -> int:
        return int(load().stanza_fc_workspace_bytes(C.byref(self.desc)))


def _ptr_array(ts: Sequence[torch.Tensor]):
    for t in ts:
        assert t.is_cuda and t.is_contiguous()
    return (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])


def stanza_fc_step(plan: FcPlan, feats, labels, W: List[torch.Tensor], b, vW, vb, dfeats, loss, pred, ws):
    p, n = _ws(ws)
    _check(load().stanza_fc_step(C.byref(plan.desc), _ptr(feats), _ptr(labels), _ptr_array(W), _ptr_array(b), _ptr_array(vW),
                                 _ptr_array(vb), _ptr(dfeats), _ptr(loss), _ptr(pred), p, n, _stream()), "stanza_fc_step")


def stanza_fc_grads(plan: FcPlan, n_global: int, feats, labels, W: List[torch.Tensor], b, gW, gb, dfeats, loss_part, pred, ws):
    p, n = _ws(ws)
    _check(load().stanza_fc_grads(C.byref(plan.desc), n_global, _ptr(feats), _ptr(labels), _ptr_array(W), _ptr_array(b),
                                  _ptr_array(gW), _ptr_array(gb), _ptr(dfeats), _ptr(loss_part), _ptr(pred), p, n, _stream()),
           "stanza_fc_grads")


def stanza_dropout(x, y, p: float, seed: int, stream_id: int):
    _check(load().stanza_dropout(x.numel(), p, seed, stream_id, _ptr(x), _ptr(y), _stream()), "stanza_dropout")


def stanza_ps_workspace_bytes(n_tensors: int, K: int) -> int:
    return int(load().stanza_ps_workspace_bytes(n_tensors, K))


def _ps_args(w, v, grads):
    """w, v: lists of tensors; grads: list over shards of lists over tensors."""
    nt, K = len(w), len(grads)
    numel = (C.c_int64 * nt)(*[t.numel() for t in w])
    flat = [g for shard in grads for g in shard]
    assert len(flat) == nt * K
    return nt, K, numel, _ptr_array(w), _ptr_array(v), _ptr_array(flat)


def stanza_ps_plan(w, v, grads, ws):
    nt, K, numel, pw, pv, pg = _ps_args(w, v, grads)
    p, n = _ws(ws)
    _check(load().stanza_ps_plan(nt, numel, pw, pv, pg, K, p, n, _stream()), "stanza_ps_plan")
    return nt, K, numel


def stanza_ps_aggregate_planned(plan, scale, lr, momentum, weight_decay, ws):
    nt, K, numel = plan
    p, n = _ws(ws)
    _check(load().stanza_ps_aggregate_planned(nt, numel, K, scale, lr, momentum, weight_decay, p, n, _stream()),
           "stanza_ps_aggregate_planned")


def stanza_ps_aggregate(w, v, grads, scale, lr, momentum, weight_decay, ws):
    nt, K, numel, pw, pv, pg = _ps_args(w, v, grads)
    p, n = _ws(ws)
    _check(load().stanza_ps_aggregate(nt, numel, pw, pv, pg, K, scale, lr, momentum, weight_decay, p, n, _stream()),
           "stanza_ps_aggregate")


SUM_INDEX_ORDER, SUM_RECURSIVE_DOUBLING = 0, 1


def stanza_ps_aggregate_ordered_planned(order, plan, scale, lr, momentum, weight_decay, ws):
    nt, K, numel = plan
    p, n = _ws(ws)
    _check(load().stanza_ps_aggregate_ordered_planned(order, nt, numel, K, scale, lr, momentum, weight_decay, p, n, _stream()),
           "stanza_ps_aggregate_ordered_planned")


def stanza_ps_aggregate_ordered(order, w, v, grads, scale, lr, momentum, weight_decay, ws):
    nt, K, numel, pw, pv, pg = _ps_args(w, v, grads)
    p, n = _ws(ws)
    _check(load().stanza_ps_aggregate_ordered(order, nt, numel, pw, pv, pg, K, scale, lr, momentum, weight_decay, p, n, _stream()),
           "stanza_ps_aggregate_ordered")


def stanza_ps_aggregate_static(order, w, v, grads, scale, lr, momentum, weight_decay):
    """The aggregation without a workspace: the pointer table lives in a fixed array of the library's device image."""
    nt, K, numel, pw, pv, pg = _ps_args(w, v, grads)
    _check(load().stanza_ps_aggregate_static(order, nt, numel, pw, pv, pg, K, scale, lr, momentum, weight_decay, _stream()),
           "stanza_ps_aggregate_static")


# ---- performance model (host arithmetic)
def stanza_model_allreduce_rounds(n_c: int) -> int:
    return int(load().stanza_model_allreduce_rounds(n_c))


def stanza_model_stanza_time(m: ModelParams, n_c: int, n_f: int) -> float:
    return float(load().stanza_model_stanza_time(C.byref(m), n_c, n_f))


def stanza_model_stanza_throughput(m: ModelParams, n_c: int, n_f: int) -> float:
    return float(load().stanza_model_stanza_throughput(C.byref(m), n_c, n_f))


def stanza_model_assign(m: ModelParams, N: int):
    nc, nf, th = C.c_int32(), C.c_int32(), C.c_double()
    _check(load().stanza_model_assign(C.byref(m), N, C.byref(nc), C.byref(nf), C.byref(th)), "stanza_model_assign")
    return nc.value, nf.value, th.value


def stanza_model_ps_time(P, T_ps, n_w, n_s, bandwidth_bits) -> float:
    return float(load().stanza_model_ps_time(P, T_ps, n_w, n_s, bandwidth_bits))


def stanza_model_ps_throughput(P, T_ps, K, n_w, n_s, bandwidth_bits) -> float:
    return float(load().stanza_model_ps_throughput(P, T_ps, K, n_w, n_s, bandwidth_bits))
