"""Sequencing of libstanza calls for one CONV worker, the FC worker and the gradient aggregation.

This is the role the training loop plays in the paper (Sec. 3.2, Fig. 5): it owns device buffers
(torch tensors) and issues the C-ABI calls in order.  It performs no arithmetic of its own.
"""
from __future__ import annotations

import inspect
from typing import Dict, List, Optional

import torch

from . import api


# Filter gradients run beside the data gradients (on another stream) for layers of at most this many 128 x 128 tiles of dy.  Measured
# at batch 64, images/s with the limit at 800 / 1,600 / 3,200 / 6,400 / 12,800 / none against one stream: VGG-16-shaped 1,333 / 1,332 /
# 1,341 / 1,344 / 1,343 / 1,319 against 1,328; ResNet-50-shaped 3,841 / 3,935 / 3,958 / 3,948 / 3,946 / 3,947 against 3,635;
# Inception-V3-shaped 1,634 / 1,637 / 1,645 / 1,646 / 1,645 / 1,643 against 1,539.  Only the two 224 x 224 x 64 layers of the VGG
# stacks (25,088 tiles) lose.
OVERLAP_MAX_TILES = 8192
# ... and of at least this many: a smaller launch is over before an event has passed from one stream to the other (the two 128-row
# layers of the MLP-shaped workload, 8 tiles: 0.58 against 0.56 ms per step in float32, 0.43 against 0.39 in bf16, with their filter
# gradients on a second stream).
OVERLAP_MIN_TILES = 16

# Arguments that a call WRITES (or updates in place); every other tensor argument is read.  The workspace counts as written.
_WRITES = {
    "stanza_conv_fwd": ("y", "ws"), "stanza_conv_fwd_res": ("y", "ws"), "stanza_conv_fwd_stats": ("y", "stats", "ws"),
    "stanza_conv_bwd_data": ("dx", "ws"), "stanza_conv_bwd_weight": ("dw", "dbias", "ws"),
    "stanza_pool_relu_fwd": ("y", "argmax"), "stanza_pool_relu_bwd": ("dx",),
    "stanza_avgpool_fwd": ("y",), "stanza_avgpool_bwd": ("dx",),
    "stanza_add_relu_fwd": ("o",), "stanza_add_relu_bwd": ("dz",),
    "stanza_gap_fwd": ("f",), "stanza_gap_bwd": ("dx",),
    "stanza_cast_f32_to_bf16": ("dst",), "stanza_cast_bf16_to_f32": ("dst",), "stanza_copy_channels": ("dst",),
    "stanza_bn_fwd": ("y", "save_mean", "save_istd", "ws", "running_mean", "running_var"),
    "stanza_bn_fwd_res": ("y", "save_mean", "save_istd", "ws", "running_mean", "running_var"),
    "stanza_bn_fwd_stats": ("y", "save_mean", "save_istd", "running_mean", "running_var"),
    "stanza_bn_bwd": ("dx", "dgamma", "dbeta", "ws"),
}
_PARAMS = {name: tuple(inspect.signature(getattr(api, name)).parameters) for name in _WRITES}


class StreamSchedule:
    """Spreads the calls of one pass (a CONV worker's forward or backward pass, Sec. 3.2) over a few streams of default priority
    and orders them with events, so that launches that do not depend on each other -- the branches of an Inception module, a
    projection shortcut beside its block, a layer's filter gradient beside its data gradient -- run side by side and fill each
    other's partly empty rounds of workgroups.

    begin / call / end issue a pass call by call and work it out on the way.  The caller names a stream for every call (a hint:
    any choice is correct); which call must wait for which is found from the calls themselves: a call waits for the last writer
    of every tensor it touches, and a writer also for every reader since (tensors are told apart by their storage, so views of
    one buffer count as that buffer).  Every library call made on the way is taped with its marshalled arguments.

    replay issues the pass again from that tape: the same library calls on the same streams between the same events, with no
    sequencing logic and no argument conversion (this is most of the host's time for a stack of short kernels).  The tape holds
    raw device addresses, so it stands only while the pass works on the same buffers from the same caller's stream: the
    sequencer's own buffers never move, and the addresses of what the caller hands in are the tape's key.

    A pass starts with every stream it uses waiting for the caller's stream and ends with the caller's stream waiting for them,
    so nothing outside the pass sees more than one stream.  Under graph capture, or switched off, calls go straight to the
    current stream."""

    def __init__(self, dev, n_streams: int):
        self.side = [torch.cuda.Stream(device=dev) for _ in range(n_streams - 1)]
        self.n = n_streams
        self.plans: Dict[str, list] = {}         # pass -> per call (stream index, entry point, events to wait for, event to record, tape)
        self.keys: Dict[str, tuple] = {}         # pass -> (caller's stream, addresses of the caller's tensors) its tape was made with
        self.used: Dict[str, list] = {}          # pass -> the side streams it uses
        self.ev_fork = torch.cuda.Event()
        self.ev_join = [torch.cuda.Event() for _ in self.side]
        self.on = False

    def _fork(self, main, active):
        if active:
            self.ev_fork.record(main)
        for st in active:
            st.wait_event(self.ev_fork)

    def _join(self, main, active):
        for st, ev in zip(active, self.ev_join):
            ev.record(st)
            main.wait_event(ev)

    def replay(self, tag: str, enabled: bool, key=()) -> bool:
        """Issue the pass `tag` from its tape.  False when there is no tape that fits (none yet, other tensors handed in, another
        caller's stream, graph capture, switched off): the pass then has to be issued call by call."""
        plan = self.plans.get(tag)
        if not enabled or plan is None or torch.cuda.is_current_stream_capturing():
            return False
        main = torch.cuda.current_stream()
        if self.keys[tag] != (main.cuda_stream,) + tuple(key):
            return False
        streams = [main] + self.side
        active = [self.side[i - 1] for i in self.used[tag]]      # a stream that the pass does not use is not made to join in
        self._fork(main, active)
        issue = api.replay_call
        for s, _, waits, ev, tape in plan:
            st = streams[s]
            for w in waits:
                st.wait_event(w)
            for entry in tape:
                issue(entry)
            if ev is not None:
                ev.record(st)
        self._join(main, active)
        return True

    def begin(self, tag: str, enabled: bool, key=()):
        self.on = enabled and not torch.cuda.is_current_stream_capturing()
        if not self.on:
            return
        self.tag, self.key = tag, key
        self.main = torch.cuda.current_stream()
        self.streams = [self.main] + self.side
        self.new, self.seq = [], 0
        self.last_writer: Dict[int, tuple] = {}      # storage -> (stream index, sequence number, event)
        self.readers: Dict[int, list] = {}           # storage -> the same, for every reader since the last writer
        self.seen = [dict() for _ in range(self.n)]  # per stream: other stream -> latest sequence number already waited for
        self._fork(self.main, self.side)

    def _work_out(self, s: int, name: str, args, kw):
        deps: Dict[int, tuple] = {}

        def need(dep):
            o, q, ev = dep
            if o != s and q > self.seen[s].get(o, -1) and (o not in deps or deps[o][0] < q):
                deps[o] = (q, ev)                        # a stream runs in order: its latest event stands for the earlier ones
        reads, writes = [], []
        for pname, val in list(zip(_PARAMS[name], args)) + list(kw.items()):
            if isinstance(val, torch.Tensor):
                (writes if pname in _WRITES[name] else reads).append(val.untyped_storage().data_ptr())
        for k in reads:
            if k in self.last_writer:
                need(self.last_writer[k])
        for k in writes:
            if k in self.last_writer:
                need(self.last_writer[k])
            for r in self.readers.get(k, ()):
                need(r)
        ev = torch.cuda.Event()
        me = (s, self.seq, ev)
        self.seq += 1
        for k in reads:
            self.readers.setdefault(k, []).append(me)
        for k in writes:
            self.last_writer[k] = me
            self.readers[k] = []
        for o, (q, _) in deps.items():
            self.seen[s][o] = q
        return [e for _, e in deps.values()], ev

    def call(self, s: int, name: str, *args, **kw):
        fn = getattr(api, name)
        if not self.on:
            return fn(*args, **kw)
        waits, ev = self._work_out(s, name, args, kw)
        st = self.streams[s]
        for w in waits:
            st.wait_event(w)
        tape = []
        api.set_stream(st)
        api.tape_calls(tape)
        try:
            fn(*args, **kw)
        finally:
            api.set_stream(None)
            api.tape_calls(None)
        ev.record(st)
        self.new.append((s, name, waits, ev, tape))

    def end(self):
        if not self.on:
            return
        waited = {id(e) for _, _, waits, _, _ in self.new for e in waits}       # replays record only the events somebody waits for
        self.plans[self.tag] = [(s, name, waits, ev if id(ev) in waited else None, tape) for s, name, waits, ev, tape in self.new]
        self.keys[self.tag] = (self.main.cuda_stream,) + tuple(self.key)
        self.used[self.tag] = sorted({e[0] for e in self.new} - {0})
        self._join(self.main, self.side)
        self.on = False


class ConvWorker:
    """One CONV worker: its conv stack forward up to the activations handed to the FC worker, and the
    backward pass from the gradient of those activations to per-layer filter/bias gradients.

    dtype=api.BF16 keeps activations, activation gradients and a per-step copy of the filters in bfloat16
    (master filters, filter/bias gradients, images, features and feature gradients stay float32); the image
    layer (C = 3) runs with its channels zero-padded to 8; any other conv whose channel counts are not multiples of 8 runs in
    float32 between casts.

    With multi_stream (the default on a GPU) the passes are issued from a tape after the first one (StreamSchedule): the tensors in
    `params` and `feat_out` must stay the same tensors for the life of the worker (they are updated in place by the aggregation and
    the FC worker); the gradient handed to backward may be another tensor at any time, the pass is then taped anew.  One thread
    issues the passes of all workers: the issue stream and the tape are state of the binding module."""

    def __init__(self, ops: List[dict], image_shape, batch: int, params: Dict[str, tuple], device="cuda:0", dtype=api.F32,
                 feat_out: Optional[torch.Tensor] = None):
        """feat_out: this worker's rows of the FC worker's [n, A] feature buffer (float32, contiguous).  The last op of the stack
        then writes the hand-off straight into it and no copy is made; without it the worker owns its feature buffer."""
        self.ops = ops
        self.dev = torch.device(device)
        self.dtype = dtype
        self.tdt = torch.bfloat16 if dtype == api.BF16 else torch.float32
        self.params = params                      # name -> (W [K,R,S,C], b [K]) float32 device tensors (shared between workers)
        self.shapes = {"x0": (batch,) + tuple(image_shape)}
        self.producer = {}
        self.descs = {}
        self.f32_layer = {}                       # op index -> True when a conv runs in float32 inside a bf16 stack
        self.padded = {}                          # op index -> true channel count of an image layer run with padded channels
        for i, op in enumerate(ops):
            kind = op["op"]
            if kind == "conv":
                n, h, w, c = self.shapes[op["src"]]
                flags = (api.CONV_BIAS if op.get("bias", True) else 0) | (api.CONV_RELU if op["relu"] else 0)
                # the image layer of a bf16 stack (3 channels): channels padded with zeros to a multiple of 8, so that it runs
                # through the bf16 kernels like every other layer instead of in float32 between casts of its output
                # (float32 stacks: to a multiple of 4, so that the image and the filter are fetched as 16-byte vectors)
                vec = 8 if dtype == api.BF16 else 4
                pad_c = op["src"] == "x0" and c % vec != 0 and (dtype != api.BF16 or op["K"] % 8 == 0)
                if pad_c:
                    self.padded[i] = c
                    c = (c + vec - 1) // vec * vec
                low = dtype == api.BF16 and c % 8 == 0 and op["K"] % 8 == 0
                self.f32_layer[i] = dtype == api.BF16 and not low
                d = api.conv_desc(n, h, w, c, op["K"], op["R"], op["S"], op["stride"], op["pad"], api.BF16 if low else api.F32, flags,
                                  pad_w=op.get("pad_w"))
                ho, wo = api.conv_out_hw(d)
                self.shapes[op["dst"]] = (n, ho, wo, op["K"])
                self.descs[i] = d
            elif kind in ("pool", "avgpool"):
                n, h, w, c = self.shapes[op["src"]]
                d = api.pool_desc(n, h, w, c, op["win"], op["stride"], op["pad"], op.get("relu", False))
                ho = (h + 2 * op["pad"] - op["win"]) // op["stride"] + 1
                wo = (w + 2 * op["pad"] - op["win"]) // op["stride"] + 1
                self.shapes[op["dst"]] = (n, ho, wo, c)
                self.descs[i] = d
            elif kind == "bn":
                self.shapes[op["dst"]] = self.shapes[op["src"]]
            elif kind == "concat":
                parts = [self.shapes[sname] for sname in op["srcs"]]
                self.shapes[op["dst"]] = parts[0][:3] + (sum(p[3] for p in parts),)
            elif kind == "add_relu":
                self.shapes[op["dst"]] = self.shapes[op["a"]]
            elif kind == "gap":
                n, h, w, c = self.shapes[op["src"]]
                self.shapes[op["dst"]] = (n, 1, 1, c)
            self.producer[op["dst"]] = op
        # A convolution (or normalisation layer) without ReLU whose only reader is the residual join that follows it in the op list
        # runs as stanza_conv_fwd_res (stanza_bn_fwd_res): the join's output is written by its epilogue and its own output never
        # exists.  (Backward is unchanged: the join's gate reads the join's output, the layer takes the gated gradient as it is.)
        self.joined = {}                          # op index -> (join op index, name of the other addend)
        self.join_desc = {}                       # conv op index -> its descriptor with the join's ReLU
        for i, op in enumerate(ops[:-1]):
            nxt = ops[i + 1]
            if op["op"] not in ("conv", "bn") or op["relu"] or nxt["op"] != "add_relu" or op["dst"] not in (nxt["a"], nxt["b"]) \
                    or nxt["a"] == nxt["b"]:
                continue
            readers = sum(1 for o in ops if op["dst"] in (o.get("src"), o.get("a"), o.get("b")) or op["dst"] in o.get("srcs", ()))
            if readers != 1 or (op["op"] == "conv" and (i in self.padded or self.f32_layer[i])):
                continue
            other = nxt["b"] if nxt["a"] == op["dst"] else nxt["a"]
            self.joined[i] = (i + 1, other)
            if op["op"] == "conv":
                self.join_desc[i] = api.ConvDesc.from_buffer_copy(self.descs[i])
                self.join_desc[i].flags |= api.CONV_RELU
        self.skip_fwd = {j for j, _ in self.joined.values()}
        # A float32 convolution whose output goes to a normalisation layer leaves the column statistics of its output behind
        # (stanza_conv_fwd_stats), and the layer reads them instead of making a pass of its own over the tensor.
        self.stats_conv = {}                      # conv op index -> index of the normalisation layer that takes its statistics
        stats_bytes = 0
        if dtype == api.F32:
            for i, op in enumerate(ops[:-1]):
                nxt = ops[i + 1]
                if op["op"] != "conv" or nxt["op"] != "bn" or nxt["src"] != op["dst"] or op["relu"] or i in self.joined or i in self.padded:
                    continue
                need = api.stanza_conv_stats_bytes(self.descs[i])
                if need:
                    self.stats_conv[i] = i + 1
                    stats_bytes = max(stats_bytes, need)
        self.stats_bn = set(self.stats_conv.values())
        self.stats_at: Dict[str, int] = {}        # conv output -> index of the statistics buffer its last forward pass wrote
        self.stats_buf = torch.empty(stats_bytes, device=self.dev, dtype=torch.uint8) if stats_bytes else None
        if dtype == api.BF16:
            assert all(op["op"] in ("conv", "pool", "avgpool", "concat", "bn", "add_relu", "gap") for op in ops)
        self.buf = {name: torch.empty(shape, device=self.dev, dtype=torch.float32 if name == "x0" else self.tdt)
                    for name, shape in self.shapes.items()}
        if feat_out is not None:
            assert feat_out.is_contiguous() and feat_out.dtype == torch.float32 and feat_out.numel() == self.buf["feat"].numel()
            if dtype == api.F32:
                self.buf["feat"] = feat_out.view(self.shapes["feat"])
        self.argmax = {op["dst"]: torch.empty(self.shapes[op["dst"]], device=self.dev, dtype=torch.uint8)
                       for op in ops if op["op"] == "pool"}
        self.gbuf: Dict[str, torch.Tensor] = {}
        self.grads = {name: (torch.empty_like(w), None if b is None else torch.empty_like(b)) for name, (w, b) in params.items()}
        # normalisation layers: saved statistics per layer, one workspace for all
        self.bn_stats = {}
        bn_ws = 16
        for op in ops:
            if op["op"] == "bn":
                shp = self.shapes[op["src"]]
                rows, c = shp[0] * shp[1] * shp[2], shp[3]
                self.bn_stats[op["name"]] = (torch.empty(c, device=self.dev), torch.empty(c, device=self.dev))
                bn_ws = max(bn_ws, api.stanza_bn_workspace_bytes(rows, c, dtype))
        self.bn_ws = torch.empty(bn_ws, device=self.dev, dtype=torch.uint8) if self.bn_stats else None
        # one workspace serves every conv call: the largest need over forward, backward-data and backward-weight
        ws_bytes = max([api.stanza_conv_workspace_bytes(d, which) for i, d in self.descs.items() if ops[i]["op"] == "conv"
                        for which in (0, 1, 2)] + [16])
        self.ws = torch.empty(ws_bytes, device=self.dev, dtype=torch.uint8)
        # Calls that do not depend on each other go to different streams (StreamSchedule): in the backward pass a layer's filter
        # gradient beside its data gradient (both start from dy, neither reads what the other writes, and nothing reads a filter
        # gradient before the aggregation), and where the op list forks (Inception modules, projection shortcuts) the branches
        # beside each other, forward and backward.  Every stream has its own workspaces.  multi_stream = False: every call on
        # the caller's stream (per-call timing; under graph capture a pass takes one stream by itself).
        uses: Dict[str, int] = {}
        for op in ops:
            for nm in ([op["src"]] if "src" in op else []) + list(op.get("srcs", ())) + [op[k] for k in ("a", "b") if k in op]:
                uses[nm] = uses.get(nm, 0) + 1
        self.n_streams = 4 if max(uses.values()) > 1 else 2
        self.multi_stream = self.dev.type == "cuda"
        self.sched = StreamSchedule(self.dev, self.n_streams) if self.dev.type == "cuda" else None
        self.wss = [self.ws] + [torch.empty(ws_bytes, device=self.dev, dtype=torch.uint8) for _ in range(self.n_streams - 1)]
        self.bn_wss = [self.bn_ws] + [None if self.bn_ws is None else torch.empty_like(self.bn_ws) for _ in range(self.n_streams - 1)]
        self.stats_bufs = [self.stats_buf] + [None if self.stats_buf is None else torch.empty_like(self.stats_buf)
                                              for _ in range(self.n_streams - 1)]
        for i in self.padded:
            cp = self.descs[i].C
            k, r, s_, _ = params[ops[i]["name"]][0].shape
            self.wpad32 = torch.zeros((k, r, s_, cp), device=self.dev)          # pad channels stay zero
            self.dwpad32 = torch.empty((k, r, s_, cp), device=self.dev)
            self.x0pad32 = torch.zeros(self.shapes["x0"][:3] + (cp,), device=self.dev)
        if dtype == api.BF16:
            self.w16 = {op["name"]: torch.empty_like(params[op["name"]][0], dtype=torch.bfloat16)
                        for i, op in enumerate(ops) if op["op"] == "conv" and not self.f32_layer[i] and i not in self.padded}
            plain = list(self.w16)                   # every bf16 filter copy of a step is written by one launch
            self.cast_plan = api.CastPlan([params[n][0] for n in plain], [self.w16[n] for n in plain]) if plain else None
            for i in self.padded:
                name = ops[i]["name"]
                self.w16[name] = torch.empty(self.wpad32.shape, device=self.dev, dtype=torch.bfloat16)
                self.x0pad16 = torch.empty(self.x0pad32.shape, device=self.dev, dtype=torch.bfloat16)
            big = max(int(torch.tensor(self.shapes[op["dst"]]).prod()) for i, op in enumerate(ops) if op["op"] == "conv" and self.f32_layer[i]) \
                if any(self.f32_layer.values()) else 0
            self.tmp32 = torch.empty(max(big, 1), device=self.dev, dtype=torch.float32)   # float32 staging of a mixed layer's y / dy
            self.feat32 = feat_out.view(self.shapes["feat"]) if feat_out is not None else \
                torch.empty(self.shapes["feat"], device=self.dev, dtype=torch.float32)
            self.dfeat16 = torch.empty(self.shapes["feat"], device=self.dev, dtype=torch.bfloat16)

    # ------------------------------------------------------------------ forward
    def forward(self, images: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Returns the float32 activations handed to the FC worker."""
        if images is not None:
            self.buf["x0"].copy_(images)
        if self.dtype == api.BF16 and self.cast_plan is not None:
            self.cast_plan.run()                     # this step's bf16 copies of the master filters
        sched, ns = self.sched, self.n_streams
        if sched.replay("forward", self.multi_stream):
            return self.feat32 if self.dtype == api.BF16 else self.buf["feat"]
        sched.begin("forward", self.multi_stream)
        q = sched.call
        # Stream hints: the first reader of a buffer goes on where the buffer was written, the k-th reader k streams further.
        at_stream: Dict[str, int] = {}           # buffer -> stream of its writer
        taken: Dict[str, int] = {}               # buffer -> readers issued so far

        def stream_for(name):
            k = taken.get(name, 0)
            taken[name] = k + 1
            return (at_stream.get(name, 0) + k) % ns
        for i, op in enumerate(self.ops):
            kind = op["op"]
            if i in self.skip_fwd:                  # a residual join computed by the preceding convolution's epilogue
                continue
            s = stream_for(op["src"] if "src" in op else op["srcs"][-1] if "srcs" in op else op["a"])
            at_stream[op["dst"]] = s
            if i in self.joined:
                at_stream[self.ops[self.joined[i][0]]["dst"]] = s
            if kind == "conv" and i in self.joined:
                w, b = self.params[op["name"]]
                j, other = self.joined[i]
                if self.dtype == api.BF16:
                    w = self.w16[op["name"]]
                q(s, "stanza_conv_fwd_res", self.join_desc[i], self.buf[op["src"]], w, b, self.buf[other], self.buf[self.ops[j]["dst"]],
                  self.wss[s])
            elif kind == "conv":
                w, b = self.params[op["name"]]
                if i in self.padded:
                    c = self.padded[i]
                    q(s, "stanza_copy_channels", self.buf["x0"], 0, self.x0pad32, 0, c)
                    q(s, "stanza_copy_channels", w, 0, self.wpad32, 0, c)
                    if self.dtype == api.BF16:
                        q(s, "stanza_cast_f32_to_bf16", self.x0pad32, self.x0pad16)
                        q(s, "stanza_cast_f32_to_bf16", self.wpad32, self.w16[op["name"]])
                        q(s, "stanza_conv_fwd", self.descs[i], self.x0pad16, self.w16[op["name"]], b, self.buf[op["dst"]], self.wss[s])
                    else:
                        q(s, "stanza_conv_fwd", self.descs[i], self.x0pad32, self.wpad32, b, self.buf[op["dst"]], self.wss[s])
                elif self.dtype == api.BF16 and not self.f32_layer[i]:
                    q(s, "stanza_conv_fwd", self.descs[i], self.buf[op["src"]], self.w16[op["name"]], b, self.buf[op["dst"]], self.wss[s])
                elif self.f32_layer[i]:
                    y32 = self.tmp32[: self.buf[op["dst"]].numel()].view(self.shapes[op["dst"]])
                    q(s, "stanza_conv_fwd", self.descs[i], self.buf[op["src"]], w, b, y32, self.wss[s])
                    q(s, "stanza_cast_f32_to_bf16", y32, self.buf[op["dst"]])
                elif i in self.stats_conv:
                    q(s, "stanza_conv_fwd_stats", self.descs[i], self.buf[op["src"]], w, b, self.buf[op["dst"]], self.stats_bufs[s],
                      self.wss[s])
                    self.stats_at[op["dst"]] = s
                else:
                    q(s, "stanza_conv_fwd", self.descs[i], self.buf[op["src"]], w, b, self.buf[op["dst"]], self.wss[s])
            elif kind == "pool":
                q(s, "stanza_pool_relu_fwd", self.descs[i], self.buf[op["src"]], self.buf[op["dst"]], self.argmax[op["dst"]], self.dtype)
            elif kind == "avgpool":
                q(s, "stanza_avgpool_fwd", self.descs[i], self.buf[op["src"]], self.buf[op["dst"]], self.dtype)
            elif kind == "concat":
                at = 0
                for sname in op["srcs"]:
                    cs = self.shapes[sname][3]
                    q(s, "stanza_copy_channels", self.buf[sname], 0, self.buf[op["dst"]], at, cs)
                    at += cs
            elif kind == "bn" and i in self.stats_bn:
                gamma, beta = self.params[op["name"]]
                mean, istd = self.bn_stats[op["name"]]
                stats = self.stats_bufs[self.stats_at[op["src"]]]      # where the producing convolution left them
                if i in self.joined:
                    j, other = self.joined[i]
                    q(s, "stanza_bn_fwd_stats", self.buf[op["src"]], stats, gamma, beta, self.buf[self.ops[j]["dst"]], mean, istd,
                      op["eps"], True, res=self.buf[other])
                else:
                    q(s, "stanza_bn_fwd_stats", self.buf[op["src"]], stats, gamma, beta, self.buf[op["dst"]], mean, istd, op["eps"],
                      op["relu"])
            elif kind == "bn" and i in self.joined:
                gamma, beta = self.params[op["name"]]
                mean, istd = self.bn_stats[op["name"]]
                j, other = self.joined[i]
                q(s, "stanza_bn_fwd_res", self.buf[op["src"]], gamma, beta, self.buf[other], self.buf[self.ops[j]["dst"]], mean, istd,
                  self.bn_wss[s], op["eps"], True, dtype=self.dtype)
            elif kind == "bn":
                gamma, beta = self.params[op["name"]]
                mean, istd = self.bn_stats[op["name"]]
                q(s, "stanza_bn_fwd", self.buf[op["src"]], gamma, beta, self.buf[op["dst"]], mean, istd, self.bn_wss[s], op["eps"],
                  op["relu"], dtype=self.dtype)
            elif kind == "add_relu":
                q(s, "stanza_add_relu_fwd", self.buf[op["a"]], self.buf[op["b"]], self.buf[op["dst"]], self.dtype)
            elif kind == "gap":
                # the features are float32 in every stack: a bf16 stack's global average pool widens as it sums
                q(s, "stanza_gap_fwd", self.buf[op["src"]], self.feat32 if self.dtype == api.BF16 else self.buf[op["dst"]], self.dtype)
        out = self.buf["feat"]
        if self.dtype == api.BF16:
            if self.producer["feat"]["op"] != "gap":
                q(at_stream.get("feat", 0), "stanza_cast_bf16_to_f32", self.buf["feat"], self.feat32)
            out = self.feat32
        sched.end()
        return out

    # ------------------------------------------------------------------ backward
    def _grad_buffer(self, name, like=None):
        if name not in self.gbuf:
            self.gbuf[name] = torch.empty(self.shapes[like or name], device=self.dev, dtype=self.tdt)
        return self.gbuf[name]

    def backward(self, dfeat: torch.Tensor):
        """dfeat: float32 gradient of the activations handed to the FC worker, [B, A] or the buffer's own shape."""
        dfeat = dfeat.reshape(self.shapes["feat"])
        sched, ns = self.sched, self.n_streams
        key = (dfeat.data_ptr(),) if dfeat.is_contiguous() and dfeat.dtype == torch.float32 else (None, id(dfeat))
        if key[0] is not None and sched.replay("backward", self.multi_stream, key):
            return self.grads
        sched.begin("backward", self.multi_stream, key)
        q = sched.call
        if self.dtype == api.BF16 and self.producer["feat"]["op"] != "gap":
            q(0, "stanza_cast_f32_to_bf16", dfeat.contiguous(), self.dfeat16)
            dfeat = self.dfeat16
        have: Dict[str, torch.Tensor] = {"feat": dfeat}
        gated = {"feat": False}   # True when the stored gradient is already multiplied by [buffer > 0]
        at_stream: Dict[str, int] = {"feat": 0}      # buffer -> stream of the last writer of its gradient (a hint, like forward's)

        def wgrad(s, d, *a):
            """A filter-gradient call: two streams on from its layer's data gradient.  Layers with more than OVERLAP_MAX_TILES
            128 x 128 tiles of dy stay on that stream: their launches run many full rounds of workgroups, there is little of a
            last round to fill, and the two kernels then only take each other's cache and HBM bandwidth."""
            ho, wo = api.conv_out_hw(d)
            tiles = -(-d.N * ho * wo // 128) * -(-d.K // 128)
            if OVERLAP_MIN_TILES <= tiles <= OVERLAP_MAX_TILES:
                s = (s + ns // 2) % ns
            q(s, "stanza_conv_bwd_weight", d, *a, self.wss[s])
            return s
        for i in reversed(range(len(self.ops))):
            op = self.ops[i]
            kind = op["op"]
            s = at_stream.get(op["dst"], 0)
            if kind == "conv":
                d = self.descs[i]
                dy = have.pop(op["dst"])
                # ReLU backward: already applied by whoever produced dy, or gate while loading
                y = None if (gated.get(op["dst"], False) or not op["relu"]) else self.buf[op["dst"]]
                w, _ = self.params[op["name"]]
                dw, db = self.grads[op["name"]]
                if i in self.padded:
                    sw = wgrad(s, d, self.x0pad16 if self.dtype == api.BF16 else self.x0pad32, dy, y, self.dwpad32, db)
                    q(sw, "stanza_copy_channels", self.dwpad32, 0, dw, 0, self.padded[i])
                    continue
                if self.f32_layer.get(i, False):
                    # mixed layer (first conv of a bf16 stack): float32 filter gradient from a float32 copy of dy
                    assert op["src"] == "x0", "a float32 conv inside a bf16 stack must be the first layer"
                    if y is not None:
                        raise NotImplementedError("ungated gradient into a mixed-precision first layer")
                    dy32 = self.tmp32[: dy.numel()].view(dy.shape)
                    q(s, "stanza_cast_bf16_to_f32", dy, dy32)
                    q(s, "stanza_conv_bwd_weight", d, self.buf["x0"], dy32, None, dw, db, self.wss[s])
                    continue
                wk = self.w16[op["name"]] if self.dtype == api.BF16 else w
                wgrad(s, d, self.buf[op["src"]], dy, y, dw, db)
                src = op["src"]
                if src != "x0":
                    prod = self.producer[src]
                    x_mask = self.buf[src] if (prod["op"] == "conv" and prod["relu"]) else None
                    dd = api.ConvDesc.from_buffer_copy(d)
                    if src in have:
                        # (a join's gradient is shared by both addends: adding into it waits, like any writer, for the calls
                        # that read it on other streams)
                        dd.flags |= api.CONV_ACCUM
                        dx = have[src]
                    else:
                        dx = self._grad_buffer(src)
                        have[src] = dx
                    q(s, "stanza_conv_bwd_data", dd, dy, y, wk, x_mask, dx, self.wss[s])
                    gated[src] = x_mask is not None
                    at_stream[src] = s
            elif kind == "avgpool":
                dx = self._grad_buffer(op["src"])
                assert op["src"] not in have, "a pooling branch must be the last reader of its input in the op list"
                q(s, "stanza_avgpool_bwd", self.descs[i], have.pop(op["dst"]), dx, self.dtype)
                have[op["src"]] = dx
                gated[op["src"]] = False
                at_stream[op["src"]] = s
            elif kind == "concat":
                wide = have.pop(op["dst"])
                at = 0
                for k, sname in enumerate(op["srcs"]):
                    cs = self.shapes[sname][3]
                    part = self._grad_buffer(sname)
                    assert sname not in have
                    sk = (s + k) % ns                 # every branch of the module takes its part of the gradient to a stream of its own
                    q(sk, "stanza_copy_channels", wide, at, part, 0, cs)
                    have[sname] = part
                    gated[sname] = False
                    at_stream[sname] = sk
                    at += cs
            elif kind == "bn":
                # the layer undoes its own ReLU from x, whether or not the incoming gradient is gated already
                gamma, beta = self.params[op["name"]]
                mean, istd = self.bn_stats[op["name"]]
                dgamma, dbeta = self.grads[op["name"]]
                dx = self._grad_buffer(op["src"])
                assert op["src"] not in have
                q(s, "stanza_bn_bwd", self.buf[op["src"]], have.pop(op["dst"]), gamma, beta, mean, istd, dx, dgamma, dbeta, self.bn_wss[s],
                  op["relu"], dtype=self.dtype)
                have[op["src"]] = dx
                gated[op["src"]] = False
                at_stream[op["src"]] = s
            elif kind == "pool":
                dx = self._grad_buffer(op["src"])
                assert op["src"] not in have
                q(s, "stanza_pool_relu_bwd", self.descs[i], have.pop(op["dst"]), self.buf[op["dst"]], self.argmax[op["dst"]], dx, self.dtype)
                have[op["src"]] = dx
                gated[op["src"]] = bool(op["relu"])   # [P>0] at the argmax equals [Y>0] there
                at_stream[op["src"]] = s
            elif kind == "add_relu":
                dz = self._grad_buffer(op["dst"] + "#dz", like=op["dst"])
                q(s, "stanza_add_relu_bwd", have.pop(op["dst"]), self.buf[op["dst"]], dz, self.dtype)
                # Both addends receive dz.  They share one tensor: in the reversed op order every reader of
                # the main-branch gradient is issued before the first accumulation into the shortcut's gradient.
                for k, name in enumerate((op["a"], op["b"])):
                    assert name not in have
                    have[name] = dz
                    gated[name] = False
                    at_stream[name] = (s + k) % ns    # a projection shortcut's backward beside the block's
            elif kind == "gap":
                dx = self._grad_buffer(op["src"])
                q(s, "stanza_gap_bwd", have.pop(op["dst"]).view(self.shapes[op["dst"]][0], -1), dx, self.dtype)
                have[op["src"]] = dx
                gated[op["src"]] = False
                at_stream[op["src"]] = s
        sched.end()
        return self.grads


class FcWorker:
    """The FC worker: owns the FC parameters and momentum buffers and runs stanza_fc_step."""

    def __init__(self, dims, n_samples, fc_params, fc_mom, lr, momentum, weight_decay, device="cuda:0", dropout=None, dtype=api.F32):
        """dropout = (p, seed): seeded dropout after every hidden layer; the iteration counter that separates the
        masks of successive steps is kept here (a captured HIP graph replays the step it was captured with)."""
        self.dev = torch.device(device)
        p, seed = dropout if dropout is not None else (0.0, 0)
        self.plan = api.FcPlan(dims, n_samples, lr, momentum, weight_decay, p, seed, 0, dtype)
        self.W = [w for w, _ in fc_params]
        self.b = [b for _, b in fc_params]
        self.vW = [w for w, _ in fc_mom]
        self.vb = [b for _, b in fc_mom]
        self.ws = torch.empty(self.plan.workspace_bytes(), device=self.dev, dtype=torch.uint8)
        self.dfeats = torch.empty((n_samples, dims[0]), device=self.dev, dtype=torch.float32)
        self.loss = torch.zeros(1, device=self.dev, dtype=torch.float32)
        self.pred = torch.empty(n_samples, device=self.dev, dtype=torch.int32)

    def step(self, feats: torch.Tensor, labels: torch.Tensor):
        api.stanza_fc_step(self.plan, feats, labels, self.W, self.b, self.vW, self.vb, self.dfeats, self.loss, self.pred, self.ws)
        self.plan.desc.dropout_step += 1
        return self.dfeats


class FcGradWorker:
    """One of several FC workers: forward, its share of the global-mean loss, backward; gradients are written out
    (no update) for the all-reduce among the FC workers.  n_samples rows are its own, n_global the whole batch."""

    def __init__(self, dims: List[int], n_samples: int, n_global: int, fc_params, device="cuda:0", dtype=api.F32):
        self.dev = torch.device(device)
        self.plan = api.FcPlan(dims, n_samples, 0.0, 0.0, 0.0, compute_dtype=dtype)
        self.n_global = n_global
        self.W = [w for w, _ in fc_params]
        self.b = [b for _, b in fc_params]
        self.gW = [torch.empty_like(w) for w in self.W]
        self.gb = [torch.empty_like(b) for b in self.b]
        self.ws = torch.empty(self.plan.workspace_bytes(), device=self.dev, dtype=torch.uint8)
        self.dfeats = torch.empty((n_samples, dims[0]), device=self.dev, dtype=torch.float32)
        self.loss = torch.zeros(1, device=self.dev, dtype=torch.float32)
        self.pred = torch.empty(n_samples, device=self.dev, dtype=torch.int32)

    def step(self, feats: torch.Tensor, labels: torch.Tensor):
        api.stanza_fc_grads(self.plan, self.n_global, feats, labels, self.W, self.b, self.gW, self.gb, self.dfeats, self.loss,
                            self.pred, self.ws)
        return self.dfeats


class Aggregator:
    """Sum of K workers' gradient shards + momentum-SGD update over a list of parameter tensors."""

    def __init__(self, w: List[torch.Tensor], v: List[torch.Tensor], grads: List[List[torch.Tensor]], device="cuda:0"):
        self.w, self.v, self.grads = w, v, grads
        self.ws = torch.empty(api.stanza_ps_workspace_bytes(len(w), len(grads)), device=device, dtype=torch.uint8)
        self.plan = api.stanza_ps_plan(w, v, grads, self.ws)

    def step(self, scale, lr, momentum, weight_decay, order=api.SUM_INDEX_ORDER):
        api.stanza_ps_aggregate_ordered_planned(order, self.plan, scale, lr, momentum, weight_decay, self.ws)


class StepGraph:
    """A fixed sequence of libstanza launches (one training step, or any part of it) captured once as a HIP graph and
    replayed: for networks made of many short kernels (residual stacks at small batch, the MLP) the launches themselves
    take a noticeable share of the step.  `fn` must only enqueue work on the current stream over buffers that stay put;
    it is run `warmup` times first so that lazily created buffers exist before the capture.  The library records no memset
    nodes, every kernel overwrites or updates its outputs in place, so a replay does exactly what the eager calls do."""

    def __init__(self, fn, warmup: int = 1):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            fn()

    def replay(self):
        self.graph.replay()
