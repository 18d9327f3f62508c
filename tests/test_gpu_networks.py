"""Whole conv stacks of the benchmark's configs 2-4 at their real layer shapes (224 x 224 images, every layer,
the residual DAG) and a reduced per-worker batch, GPU sequencer against the CPU checker: features handed to the FC
worker, per-layer filter and bias gradients, then the FC step on those features."""
import numpy as np
import pytest
import torch

import workloads as wl_mod
from gpu_util import dev, host, note, rel_err
from oracle import network as onet

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def api():
    from paper_1812_10624_amd import api as a
    a.load()
    assert torch.cuda.is_available()
    return a


@pytest.mark.parametrize("name,B", [("alexnet", 2), ("vgg16", 1), ("resnet50", 2)])
def test_conv_stack_real_shapes(api, o32, name, B):
    from paper_1812_10624_amd.netrun import ConvWorker
    wl = wl_mod.get_workload(name)
    img = wl_mod.gen_images(wl, 0, 0, B)
    cp = wl_mod.gen_conv_params(wl, 0)
    bufs = onet.conv_stack_forward(o32, wl.ops, img, cp)
    feat_ref = bufs["feat"].reshape(B, -1)
    dfeat = (wl_mod.rng_for(5, "dfeat", name).standard_normal(feat_ref.shape, dtype=np.float32) / np.float32(feat_ref.shape[0]))
    pg, bgr = onet.conv_stack_backward(o32, wl.ops, bufs, cp, dfeat)
    gcp = {n: (dev(w), dev(b)) for n, (w, b) in cp.items()}
    wk = ConvWorker(wl.ops, wl.image, B, gcp)
    feat = wk.forward(dev(img)).view(B, -1)
    e_feat = rel_err(host(feat), feat_ref)
    assert e_feat < 1e-4, (name, e_feat)
    wk.backward(dev(dfeat))
    # Whole chain: far down a deep stack a last-bit difference flips a few ReLU masks / pool argmaxes and moves single
    # entries, so the end-to-end gradients are held to direction and size ...
    for n in cp:
        for which in range(2):
            a, b = host(wk.grads[n][which]).ravel().astype(np.float64), pg[n][which].ravel().astype(np.float64)
            cos = float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b) + 1e-300))
            assert cos > 0.9999, (name, n, which, cos)
            assert abs(np.linalg.norm(a) / np.linalg.norm(b) - 1) < 1e-2, (name, n, which)
            note(a, b, tag="#chain")         # element-wise E of the whole chain: reported, not gated (see above)
    # ... and every conv layer's backward is held to the 1e-4 bound on the checker's own inputs for that layer.
    from oracle import ConvGeom
    worst = 0.0
    for op in wl.ops:
        if op["op"] != "conv":
            continue
        x = bufs[op["src"]]
        n_, h, w, c = x.shape
        g = ConvGeom(n_, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"])
        dy = np.ascontiguousarray(bgr[op["dst"]])
        dz = o32.relu_bwd(dy, bufs[op["dst"]]) if op["relu"] else dy
        d = api.conv_desc(n_, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"], api.F32,
                          api.CONV_BIAS | (api.CONV_RELU if op["relu"] else 0))
        yd = dev(bufs[op["dst"]]) if op["relu"] else None
        ws = torch.empty(max(16, api.stanza_conv_workspace_bytes(d, 2)), dtype=torch.uint8, device="cuda:0")
        dw, db = torch.empty(cp[op["name"]][0].shape, device="cuda:0"), torch.empty(op["K"], device="cuda:0")
        xd, dyd = dev(x), dev(dy)
        api.stanza_conv_bwd_weight(d, xd, dyd, yd, dw, db, ws)
        ref_dw, ref_db = o32.conv_bwd_weight(g, x, dz)
        e1, e2 = rel_err(host(dw), ref_dw), rel_err(host(db), ref_db)
        assert e1 < 1e-4 and e2 < 1e-4, (name, op["name"], e1, e2)
        worst = max(worst, e1, e2)
        if op["src"] != "x0":
            dx = torch.empty(x.shape, device="cuda:0")
            api.stanza_conv_bwd_data(d, dyd, yd, gcp[op["name"]][0], None, dx)
            e3 = rel_err(host(dx), o32.conv_bwd_data(g, dz, cp[op["name"]][0]))
            assert e3 < 1e-4, (name, op["name"], e3)
            worst = max(worst, e3)
    print(f"{name}: features E={e_feat:.2e}, worst layer-wise backward E={worst:.2e}")


@pytest.mark.parametrize("name,half", [("tiny", False), ("minires", False), ("miniresbn16", True), ("miniinception8", True)])
def test_step_graph_replays_equal_eager_steps(api, name, half):
    """The whole layer-separated step captured as a HIP graph: three replays, with eager work and synchronisations between
    them, leave every parameter bit-identical to three eager steps from the same state (all reductions are fixed-order)."""
    import copy
    from paper_1812_10624_amd.netrun import Aggregator, ConvWorker, FcWorker, StepGraph
    wl = wl_mod.get_workload(name)
    K, B = wl.K, wl.B
    cp = {n: (dev(w), None if b is None else dev(b)) for n, (w, b) in wl_mod.gen_conv_params(wl, 0).items()}   # bias-free convolutions: None
    cm = {n: (torch.zeros_like(w), None if b is None else torch.zeros_like(b)) for n, (w, b) in cp.items()}
    fp = [(dev(w), dev(b)) for w, b in wl_mod.gen_fc_params(wl, 0)]
    fm = [(torch.zeros_like(w), torch.zeros_like(b)) for w, b in fp]
    imgs = [dev(wl_mod.gen_images(wl, 0, k)) for k in range(K)]
    labels = dev(wl_mod.gen_labels(wl, 0))
    feats = torch.empty((K * B, wl.fc_dims[0]), device="cuda:0")
    # every worker writes its hand-off straight into its rows of the FC worker's feature buffer
    # (half: the bf16 stacks, whose per-step filter copies are one planned multi-tensor cast inside the captured step)
    dt = api.BF16 if half else api.F32
    workers = [ConvWorker(wl.ops, wl.image, B, cp, dtype=dt, feat_out=feats[k * B:(k + 1) * B]) for k in range(K)]
    fc_dt = api.BF16 if half and all(d % 8 == 0 for d in wl.fc_dims[:-1]) else api.F32
    fcw = FcWorker(wl.fc_dims, K * B, fp, fm, wl.lr, 0.9, 1e-4, dtype=fc_dt)  # momentum on, so the velocity buffers are exercised
    agg = Aggregator(wl_mod.flat_tensors(cp), wl_mod.flat_tensors(cm), [wl_mod.flat_tensors(wk.grads) for wk in workers])

    def step():
        for k, wk in enumerate(workers):
            wk.forward(imgs[k])
        fcw.step(feats, labels)
        for k, wk in enumerate(workers):
            wk.backward(fcw.dfeats[k * B:(k + 1) * B])
        agg.step(1.0, wl.lr, 0.9, 1e-4)

    state = [t for pair in list(cp.values()) + list(cm.values()) + fp + fm for t in pair if t is not None]
    saved = [t.clone() for t in state]

    def restore():
        for t, s in zip(state, saved):
            t.copy_(s)

    for _ in range(3):
        step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in state]
    eager_loss = float(fcw.loss.cpu()[0])
    restore()
    g = StepGraph(step, warmup=1)
    restore()
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device="cuda:0")
    for _ in range(3):
        g.replay()
        scratch.add_(1.0)                       # the program's own eager work between replays
        torch.cuda.synchronize()
    for t, e in zip(state, eager):
        assert torch.equal(t, e)
    assert float(fcw.loss.cpu()[0]) == eager_loss
    assert not torch.equal(state[0], saved[0])


@pytest.mark.parametrize("K,numels", [(16, [4096 * 3, 1000, 64 * 27, 64, 4097, 8]), (3, [300] * 70)], ids=["k16", "k3_70tensors"])
def test_plain_aggregation_call_inside_a_graph_capture(api, o32, K, numels):
    """stanza_ps_aggregate itself (pointer table written by its own fill launches, then the aggregation launch) recorded in
    a stream capture: nothing in it allocates, copies through the runtime or waits.  Three replays with eager work and
    synchronisations between them; every replay is compared with the checker's step from the same state.  The second
    case's table (70 tensors: 491 words) needs two fill launches."""
    import copy
    from gpu_util import host, param_update_err, rel_err
    ws_, vs_, gs_ = wl_mod.gen_ps_case(numels, K, seed=77)
    gw, gv = [dev(a) for a in ws_], [dev(a) for a in vs_]
    gg = [[dev(gs_[t][k]) for t in range(len(numels))] for k in range(K)]
    ws = torch.empty(api.stanza_ps_workspace_bytes(len(numels), K), dtype=torch.uint8, device="cuda:0")
    ws.fill_(0xAB)                       # the capture must bring its own table
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.stanza_ps_aggregate(gw, gv, gg, 1.0, 0.01, 0.9, 5e-4, ws)
    torch.cuda.synchronize()
    # capture launches nothing: the state is still the initial one
    for t in range(len(numels)):
        np.testing.assert_array_equal(host(gw[t]), ws_[t])
    w_ref, v_ref = copy.deepcopy(ws_), copy.deepcopy(vs_)
    for rep in range(3):
        before = [w.copy() for w in w_ref]
        ws.fill_(0)                      # eager work between replays, on the table itself
        scratch = torch.randn(1 << 16, device="cuda:0").sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(scratch)
        for t in range(len(numels)):
            o32.ps_aggregate(w_ref[t], v_ref[t], gs_[t], 1.0, 0.01, 0.9, 5e-4)
            assert rel_err(host(gv[t]), v_ref[t]) < 1e-5, (rep, t)
            assert param_update_err(host(gw[t]), w_ref[t], before[t]) < 1e-4, (rep, t)
            assert rel_err(host(gw[t]), w_ref[t]) < 1e-6, (rep, t)


@pytest.mark.parametrize("name,B,dt", [("resnet50", 4, "f32"), ("inception3", 2, "f32"), ("vgg16", 2, "f32"), ("resnet50bn", 3, "f32"),
                                       ("resnet50", 3, "bf16"), ("inception3", 2, "bf16"),
                                       # at the batch sizes bench.py times, where the launches are as long and as many-tiled as there
                                       ("resnet50", 64, "f32"), ("inception3", 32, "f32"), ("vgg16", 64, "f32"), ("resnet50bn", 64, "bf16")])
def test_passes_on_several_streams_equal_one_stream(api, name, B, dt):
    """The CONV worker's passes (Sec. 3.2) spread calls that do not depend on each other over several streams: a layer's filter
    gradient beside its data gradient, the branches of an Inception module or a projection shortcut beside each other.  Same
    kernels, same operands, so the hand-off and every gradient must come out bit for bit as on one stream -- also where a residual
    join's gradient, which other calls read, is later accumulated into by the shortcut's side, where several branches accumulate
    into the gradient of their common input, and over repeated steps (the streams of one pass against the caller's stream before
    and after it)."""
    from paper_1812_10624_amd.netrun import ConvWorker
    wl = wl_mod.get_workload(name)
    img = dev(wl_mod.gen_images(wl, 3, 0, B))
    gcp = {n: tuple(None if t is None else dev(t) for t in ts) for n, ts in wl_mod.gen_conv_params(wl, 3).items()}
    wk = ConvWorker(wl.ops, wl.image, B, gcp, dtype=api.BF16 if dt == "bf16" else api.F32)
    assert wk.n_streams == (2 if name == "vgg16" else 4)
    wk.multi_stream = False
    feat_ref = wk.forward(img).clone()
    dfeat = torch.randn(feat_ref.shape, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(11)) / B
    wk.backward(dfeat)
    torch.cuda.synchronize()
    ref = {n: tuple(None if g is None else g.clone() for g in gs) for n, gs in wk.grads.items()}
    wk.multi_stream = True
    for rep in range(3):
        for t in list(wk.buf.values()) + [g for gs in wk.grads.values() for g in gs if g is not None]:
            if t is not wk.buf["x0"]:
                t.fill_(float("nan"))                # on the caller's stream: the passes must order their streams behind this
        feat = wk.forward().clone()                  # caller's stream, no synchronisation in between
        wk.backward(dfeat)
        got = {n: tuple(None if g is None else g.clone() for g in gs) for n, gs in wk.grads.items()}
        torch.cuda.synchronize()
        assert torch.equal(feat, feat_ref), (name, rep)
        for n in ref:
            for which in range(2):
                if ref[n][which] is not None:
                    assert torch.equal(got[n][which], ref[n][which]), (name, rep, n, which)
    # the second and third repetition were issued from the tape of the first (same buffers, same stream), across events
    assert len(wk.sched.plans) == 2 and sum(len(e[2]) for e in wk.sched.plans["backward"]) > 0
    assert all(len(e[4]) >= 1 for e in wk.sched.plans["forward"])
    # other tensors handed in: the pass is worked out and taped anew, same bits
    dfeat2 = dfeat.clone()
    wk.backward(dfeat2)
    torch.cuda.synchronize()
    assert wk.sched.keys["backward"][1] == dfeat2.data_ptr()
    for n in ref:
        for which in range(2):
            if ref[n][which] is not None:
                assert torch.equal(wk.grads[n][which], ref[n][which]), (name, "new dfeat", n, which)
