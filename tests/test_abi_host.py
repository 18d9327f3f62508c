"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol that
include/stanza.h declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    if not os.path.exists(a.LIB_PATH):
        from paper_1812_10624_amd.build import build_library
        build_library()
    a.load()
    return a


def test_every_declared_symbol_is_exported(api):
    header = open(os.path.join(ROOT, "include", "stanza.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(stanza_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = api.load()
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in stanza.h but not exported"
    assert declared == set(api.EXPORTS)


def test_status_strings_and_version(api):
    lib = api.load()
    assert lib.stanza_version() >= 100
    assert lib.stanza_strerror(0) == b"ok"
    for code in range(-7, 0):
        assert lib.stanza_strerror(code) not in (b"ok", b"unknown status")
    assert lib.stanza_strerror(-99) == b"unknown status"


def test_conv_errors_before_launch(api):
    lib = api.load()
    good = api.conv_desc(2, 8, 8, 4, 8, 3, 3, 1, 1, api.F32, api.CONV_BIAS)
    p16, p4 = C.c_void_p(0x1000), C.c_void_p(0x1004)
    assert lib.stanza_conv_fwd(None, p16, p16, p16, p16, None, 0, None) == -2
    assert lib.stanza_conv_fwd(C.byref(good), None, p16, p16, p16, None, 0, None) == -2
    assert lib.stanza_conv_fwd(C.byref(good), p16, p16, None, p16, None, 0, None) == -2       # bias flagged, missing
    assert lib.stanza_conv_fwd(C.byref(good), p4, p16, p16, p16, None, 0, None) == -3
    for field, val in (("N", 0), ("C", -1), ("stride_h", 0), ("pad_h", 3), ("pad_w", -1), ("R", 11)):
        d = api.conv_desc(2, 8, 8, 4, 8, 3, 3, 1, 1, api.F32, 0)
        setattr(d, field, val)
        assert lib.stanza_conv_fwd(C.byref(d), p16, p16, None, p16, None, 0, None) == -1, field
    big = api.conv_desc(4096, 1024, 1024, 64, 8, 3, 3, 1, 1, api.F32, 0)                       # >= 2^31 elements
    assert lib.stanza_conv_fwd(C.byref(big), p16, p16, None, p16, None, 0, None) == -1
    # bfloat16 tensors are addressed with 32-bit byte offsets: 2 GiB and more is refused before any launch
    big16 = api.conv_desc(2048, 256, 256, 8, 8, 1, 1, 1, 0, api.BF16, 0)                       # 2^30 elements = 2 GiB
    assert lib.stanza_conv_fwd(C.byref(big16), p16, p16, None, p16, None, 0, None) == -4
    bad_dtype = api.conv_desc(2, 8, 8, 4, 8, 3, 3, 1, 1, 7, 0)
    assert lib.stanza_conv_fwd(C.byref(bad_dtype), p16, p16, None, p16, None, 0, None) == -4
    # residual join in the epilogue: the residual is required and aligned like every tensor
    assert lib.stanza_conv_fwd_res(C.byref(good), p16, p16, p16, None, p16, None, 0, None) == -2
    assert lib.stanza_conv_fwd_res(C.byref(good), p16, p16, p16, p4, p16, None, 0, None) == -3
    assert lib.stanza_conv_fwd_res(None, p16, p16, p16, p16, p16, None, 0, None) == -2
    assert lib.stanza_conv_bwd_data(C.byref(good), p16, None, p16, None, None, None, 0, None) == -2
    assert lib.stanza_conv_bwd_data(C.byref(good), p16, None, p16, p4, p16, None, 0, None) == -3
    # filter gradient: workspace is mandatory and sized by the query
    long_red = api.conv_desc(8, 32, 32, 4, 8, 3, 3, 1, 1, api.F32, api.CONV_BIAS)       # 8192 pixels: the reduction is split
    need = lib.stanza_conv_workspace_bytes(C.byref(long_red), 2)
    assert need > 0 and lib.stanza_conv_workspace_bytes(C.byref(long_red), 0) == 0
    assert lib.stanza_conv_bwd_weight(C.byref(long_red), p16, p16, None, p16, p16, p16, need - 1, None) == -5
    assert lib.stanza_conv_bwd_weight(C.byref(long_red), p16, p16, None, p16, p16, None, need, None) == -2
    assert lib.stanza_conv_bwd_weight(C.byref(long_red), p16, p16, None, p16, None, p16, need, None) == -2   # dbias missing


def test_pool_and_elementwise_errors(api):
    lib = api.load()
    p16 = C.c_void_p(0x1000)
    d = api.pool_desc(1, 8, 8, 4, 2, 2, 0)
    assert lib.stanza_pool_relu_fwd(C.byref(d), api.F32, None, p16, p16, None) == -2
    assert lib.stanza_pool_relu_fwd(C.byref(d), 5, p16, p16, p16, None) == -4
    d.pad_h = 2
    assert lib.stanza_pool_relu_fwd(C.byref(d), api.F32, p16, p16, p16, None) == -1          # pad >= window
    d = api.pool_desc(1, 8, 8, 4, 16, 16, 0)
    assert lib.stanza_pool_relu_fwd(C.byref(d), api.F32, p16, p16, p16, None) == -1          # window code > 255 / larger than image
    assert lib.stanza_add_relu_fwd(0, api.F32, p16, p16, p16, None) == -1
    assert lib.stanza_add_relu_fwd(16, api.F32, p16, None, p16, None) == -2
    assert lib.stanza_gap_fwd(1, 0, 4, api.F32, p16, p16, None) == -1


def test_fc_and_ps_errors(api):
    lib = api.load()
    p16 = C.c_void_p(0x1000)
    plan = api.FcPlan([64, 32, 10], 8, 0.01, 0.9, 0.0)
    need = plan.workspace_bytes()
    assert need > 0
    arr = (C.c_void_p * 2)(0x1000, 0x2000)
    assert lib.stanza_fc_step(C.byref(plan.desc), p16, p16, arr, arr, arr, arr, p16, p16, None, p16, need - 1, None) == -5
    assert lib.stanza_fc_step(C.byref(plan.desc), None, p16, arr, arr, arr, arr, p16, p16, None, p16, need, None) == -2
    nullarr = (C.c_void_p * 2)(0x1000, None)
    assert lib.stanza_fc_step(C.byref(plan.desc), p16, p16, nullarr, arr, arr, arr, p16, p16, None, p16, need, None) == -2
    assert lib.stanza_fc_grads(C.byref(plan.desc), 7, p16, p16, arr, arr, arr, arr, p16, p16, None, p16, need, None) == -1   # n_global < rows
    assert lib.stanza_fc_grads(C.byref(plan.desc), 16, p16, p16, arr, arr, None, arr, p16, p16, None, p16, need, None) == -2
    assert lib.stanza_fc_grads(C.byref(plan.desc), 16, p16, p16, arr, arr, arr, arr, p16, p16, None, p16, need - 1, None) == -5
    # every parameter and momentum pointer is checked for 16-byte alignment before any launch, the bias momentum included
    odd = (C.c_void_p * 2)(0x1000, 0x2004)
    for pos in range(4):
        args = [arr, arr, arr, arr]
        args[pos] = odd
        assert lib.stanza_fc_step(C.byref(plan.desc), p16, p16, *args, p16, p16, None, p16, need, None) == -3, pos
        assert lib.stanza_fc_grads(C.byref(plan.desc), 16, p16, p16, *args, p16, p16, None, p16, need, None) == -3, pos
    bad = api.FcPlan([64, 0, 10], 8, 0.01, 0.9, 0.0)
    assert bad.workspace_bytes() == 0
    assert lib.stanza_ps_workspace_bytes(0, 4) == 0
    need = lib.stanza_ps_workspace_bytes(2, 3)
    numel = (C.c_int64 * 2)(100, 0)
    w = (C.c_void_p * 2)(0x1000, 0x2000)
    g = (C.c_void_p * 6)(*([0x3000] * 6))
    assert lib.stanza_ps_plan(2, numel, w, w, g, 3, p16, need, None) == -1                     # empty tensor
    numel = (C.c_int64 * 2)(100, 50)
    assert lib.stanza_ps_plan(2, numel, w, w, g, 3, p16, need - 1, None) == -5
    g_bad = (C.c_void_p * 6)(0x3000, 0x3000, 0x3004, 0x3000, 0x3000, 0x3000)
    assert lib.stanza_ps_plan(2, numel, w, w, g_bad, 3, p16, need, None) == -3
    assert lib.stanza_ps_aggregate_planned(2, numel, 3, 1.0, 0.1, 0.9, 0.0, None, need, None) == -2
    assert lib.stanza_ps_aggregate_ordered_planned(7, 2, numel, 3, 1.0, 0.1, 0.9, 0.0, p16, need, None) == -1   # unknown order
    assert lib.stanza_ps_aggregate_ordered_planned(1, 2, numel, 3, 1.0, 0.1, 0.9, 0.0, None, need, None) == -2
    assert lib.stanza_ps_aggregate_ordered(9, 2, numel, w, w, g, 3, 1.0, 0.1, 0.9, 0.0, p16, need, None) == -1
    # the form without a workspace: its fixed table holds 32768 words; beyond that it refuses before touching the device
    assert lib.stanza_ps_aggregate_static(9, 2, numel, w, w, g, 3, 1.0, 0.1, 0.9, 0.0, None) == -1
    assert lib.stanza_ps_aggregate_static(0, 0, numel, w, w, g, 3, 1.0, 0.1, 0.9, 0.0, None) == -1
    assert lib.stanza_ps_aggregate_static(0, 1639, numel, w, w, g, 16, 1.0, 0.1, 0.9, 0.0, None) == -7
    assert lib.stanza_ps_aggregate_static(0, 8, numel, w, w, g, 4093, 1.0, 0.1, 0.9, 0.0, None) == -7


def test_cast_plan_errors(api):
    lib = api.load()
    p16, p4 = C.c_void_p(0x1000), C.c_void_p(0x1004)
    assert lib.stanza_cast_workspace_bytes(0) == 0 and lib.stanza_cast_workspace_bytes(-3) == 0
    need = lib.stanza_cast_workspace_bytes(2)
    assert need >= 8 * (2 * 2 + 1) + 8 * 2 * 2 and need % 256 == 0
    numel = (C.c_int64 * 2)(100, 50)
    ok = (C.c_void_p * 2)(0x1000, 0x2000)
    assert lib.stanza_cast_plan(0, numel, ok, ok, p16, need, None) == -1
    assert lib.stanza_cast_plan(2, (C.c_int64 * 2)(100, 0), ok, ok, p16, need, None) == -1        # empty tensor
    assert lib.stanza_cast_plan(2, None, ok, ok, p16, need, None) == -2
    assert lib.stanza_cast_plan(2, numel, ok, ok, None, need, None) == -2
    assert lib.stanza_cast_plan(2, numel, (C.c_void_p * 2)(0x1000, 0), ok, p16, need, None) == -2
    assert lib.stanza_cast_plan(2, numel, ok, (C.c_void_p * 2)(0x1000, 0x2004), p16, need, None) == -3
    assert lib.stanza_cast_plan(2, numel, ok, ok, p4, need, None) == -3
    assert lib.stanza_cast_plan(2, numel, ok, ok, p16, need - 1, None) == -5
    assert lib.stanza_cast_plan(2, (C.c_int64 * 2)(1 << 42, 1 << 42), ok, ok, p16, need, None) == -1   # more blocks than a grid holds
    assert lib.stanza_cast_f32_to_bf16(0, p16, p16, None) == -1 and lib.stanza_cast_bf16_to_f32(-5, p16, p16, None) == -1
    assert lib.stanza_cast_f32_to_bf16(1 << 44, p16, p16, None) == -1 and lib.stanza_cast_bf16_to_f32(1 << 44, p16, p16, None) == -1
    assert lib.stanza_cast_f32_to_bf16(16, None, p16, None) == -2 and lib.stanza_cast_bf16_to_f32(16, p16, None, None) == -2
    assert lib.stanza_cast_f32_to_bf16_planned(0, numel, p16, need, None) == -1
    assert lib.stanza_cast_f32_to_bf16_planned(2, None, p16, need, None) == -2
    assert lib.stanza_cast_f32_to_bf16_planned(2, numel, None, need, None) == -2
    assert lib.stanza_cast_f32_to_bf16_planned(2, numel, p16, need - 1, None) == -5
    assert lib.stanza_cast_f32_to_bf16_planned(2, (C.c_int64 * 2)(100, -1), p16, need, None) == -1


def test_bn_errors(api):
    import ctypes as C
    lib = api.load()
    p16, p4 = C.c_void_p(0x1000), C.c_void_p(0x1004)
    need = lib.stanza_bn_workspace_bytes(100, 8, api.F32)
    assert need > 0
    call = lambda rows=100, c=8, dt=api.F32, eps=1e-5, x=p16, ws=p16, nbytes=need, mom=0.1: lib.stanza_bn_fwd(
        rows, c, dt, eps, 0, x, p16, p16, p16, p16, p16, None, None, mom, ws, nbytes, None)
    assert call(rows=0) == -1 and call(c=0) == -1 and call(eps=0.0) == -1 and call(mom=1.5) == -1
    assert call(rows=1 << 29, c=8) == -1
    assert call(dt=api.BF16, c=12) == -4 and call(dt=9) == -4
    assert call(x=None) == -2 and call(x=p4) == -3 and call(nbytes=8) == -5
    assert lib.stanza_bn_workspace_bytes(0, 8, api.F32) == 0
    assert lib.stanza_bn_bwd(100, 8, api.F32, 0, p16, None, p16, p16, p16, p16, p16, p16, p16, p16, need, None) == -2
    # the residual-join forward: the residual is required and aligned like x
    assert lib.stanza_bn_fwd_res(100, 8, api.F32, 1e-5, 1, p16, p16, p16, None, p16, p16, p16, None, None, 0.1, p16, need, None) == -2
    assert lib.stanza_bn_fwd_res(100, 8, api.F32, 1e-5, 1, p16, p16, p16, p4, p16, p16, p16, None, None, 0.1, p16, need, None) == -3


def test_conv_statistics_errors(api):
    lib = api.load()
    p16, p4 = C.c_void_p(0x1000), C.c_void_p(0x1004)
    good = api.conv_desc(2, 8, 8, 4, 8, 3, 3, 1, 1, api.F32, 0)
    need = lib.stanza_conv_stats_bytes(C.byref(good))
    assert need >= 32 and need % 256 == 0
    # float32, output channels a multiple of 4, no fused ReLU: everything else has no statistics form
    for d in (api.conv_desc(2, 8, 8, 8, 8, 3, 3, 1, 1, api.BF16, 0), api.conv_desc(2, 8, 8, 4, 6, 3, 3, 1, 1, api.F32, 0),
              api.conv_desc(2, 8, 8, 4, 8, 3, 3, 1, 1, api.F32, api.CONV_RELU)):
        assert lib.stanza_conv_stats_bytes(C.byref(d)) == 0
        assert lib.stanza_conv_fwd_stats(C.byref(d), p16, p16, None, p16, p16, 1 << 20, None, 0, None) == -4
    bad = api.conv_desc(0, 8, 8, 4, 8, 3, 3, 1, 1, api.F32, 0)
    assert lib.stanza_conv_stats_bytes(C.byref(bad)) == 0 and lib.stanza_conv_stats_bytes(None) == 0
    assert lib.stanza_conv_fwd_stats(C.byref(bad), p16, p16, None, p16, p16, 1 << 20, None, 0, None) == -1
    assert lib.stanza_conv_fwd_stats(None, p16, p16, None, p16, p16, need, None, 0, None) == -2
    assert lib.stanza_conv_fwd_stats(C.byref(good), p16, p16, None, p16, None, need, None, 0, None) == -2
    assert lib.stanza_conv_fwd_stats(C.byref(good), p16, p16, None, p16, p4, need, None, 0, None) == -3
    assert lib.stanza_conv_fwd_stats(C.byref(good), p16, p16, None, p16, p16, need - 1, None, 0, None) == -5
    assert lib.stanza_conv_fwd_stats(C.byref(good), None, p16, None, p16, p16, need, None, 0, None) == -2
    call = lambda rows=128, c=8, eps=1e-5, x=p16, st=p16, nbytes=need, res=None, mom=0.1: lib.stanza_bn_fwd_stats(
        rows, c, eps, 0, x, st, nbytes, p16, p16, res, p16, p16, p16, None, None, mom, None)
    assert call(rows=0) == -1 and call(eps=0.0) == -1 and call(mom=-0.1) == -1
    assert call(c=6) == -4
    assert call(x=None) == -2 and call(st=None) == -2
    assert call(x=p4) == -3 and call(st=p4) == -3 and call(res=p4) == -3
    assert call(nbytes=16) == -5


def test_dropout_errors(api):
    lib = api.load()
    p16, p4 = C.c_void_p(0x1000), C.c_void_p(0x1004)
    assert lib.stanza_dropout(0, 0.5, 1, 1, p16, p16, None) == -1
    assert lib.stanza_dropout(16, 1.0, 1, 1, p16, p16, None) == -1
    assert lib.stanza_dropout(16, -0.1, 1, 1, p16, p16, None) == -1
    assert lib.stanza_dropout(16, 0.5, 1, 1, None, p16, None) == -2
    assert lib.stanza_dropout(16, 0.5, 1, 1, p16, p4, None) == -3
    plan = api.FcPlan([64, 32, 10], 8, 0.01, 0.9, 0.0, dropout_p=1.0)
    arr = (C.c_void_p * 2)(0x1000, 0x2000)
    need = plan.workspace_bytes()
    assert lib.stanza_fc_step(C.byref(plan.desc), p16, p16, arr, arr, arr, arr, p16, p16, None, p16, need, None) == -1


def test_avgpool_and_copy_errors(api):
    lib = api.load()
    p16, p4, p2 = C.c_void_p(0x1000), C.c_void_p(0x1004), C.c_void_p(0x1002)
    d = api.pool_desc(1, 8, 8, 4, 3, 1, 1, False)
    assert lib.stanza_avgpool_fwd(C.byref(d), api.F32, None, p16, None) == -2
    assert lib.stanza_avgpool_fwd(C.byref(d), api.BF16, p16, p16, None) == -4
    assert lib.stanza_avgpool_bwd(C.byref(d), api.F32, p16, p4, None) == -3
    d.pad_h = 3
    assert lib.stanza_avgpool_fwd(C.byref(d), api.F32, p16, p16, None) == -1
    assert lib.stanza_copy2d(0, 4, p16, 4, p16, 4, None) == -1
    assert lib.stanza_copy2d(4, 8, p16, 4, p16, 8, None) == -1          # leading dimension shorter than a row
    assert lib.stanza_copy2d(1 << 30, 4, p16, 4, p16, 4, None) == -1
    assert lib.stanza_copy2d(4, 4, None, 4, p16, 4, None) == -2
    assert lib.stanza_copy2d(4, 4, p2, 4, p16, 4, None) == -3


def test_fc_compute_dtype_errors(api):
    assert api.FcPlan([64, 32, 10], 8, 0.01, 0.9, 0.0, compute_dtype=7).workspace_bytes() == 0
    assert api.FcPlan([64, 36, 10], 8, 0.01, 0.9, 0.0, compute_dtype=api.BF16).workspace_bytes() == 0     # width not a multiple of 8
    # bfloat16 hidden layers: an operand of 2 GiB and more is refused by the layout query, before anything runs
    assert api.FcPlan([1 << 20, 1024, 10], 1024, 0.01, 0.9, 0.0, compute_dtype=api.BF16).workspace_bytes() == 0
    assert api.FcPlan([1 << 20, 1024, 10], 512, 0.01, 0.9, 0.0, compute_dtype=api.BF16).workspace_bytes() == 0   # the weights
    f32 = api.FcPlan([64, 32, 10], 8, 0.01, 0.9, 0.0).workspace_bytes()
    assert api.FcPlan([64, 32, 10], 8, 0.01, 0.9, 0.0, compute_dtype=api.BF16).workspace_bytes() > f32


def test_bench_refuses_more_than_one_gpu():
    """One GPU's share is what this build measures: the bench script says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""

