"""Single-GPU multiplexing run (paper section 5 "Multiplexing", the ablation of section 7.2): a foreground
VGG-16 training step at per-GPU batch 2 -- the small-batch shard that leaves the GPU underused -- beside a
background ResNet-50 training step at batch 64 that soaks up the idle capacity.

Host logic only: every launch is a call of the C ABI; this module orders the calls, paces them and times them.
The paper's runtime gives the foreground a high-priority stream; stream priorities are not usable on this
machine pool, so both jobs run on streams of the DEFAULT priority and the two mechanisms the paper adds on top of
priorities carry the run:
  * launch pacing: the background queue holds at most `pace` un-finished launches (an event per launch, the
    launcher waits for the event `pace` launches back), so a foreground kernel never waits behind a deep
    background queue;
  * graphs split into small pieces: the foreground step is captured as several small device graphs (a few
    layers each) instead of one whole-iteration graph, so foreground launches cost one call per piece while the
    background can still slip in between the pieces.
Ladder (one row each): foreground alone, background alone, both with neither mechanism, + pacing, + pacing and
foreground graphs.  Reported: foreground step latency and slowdown, background and combined TFLOP/s, and the
foreground's per-layer latency alone versus collocated.
"""
import threading
import time


def _median(v):
    v = sorted(v)
    return v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2])


class _Job:
    """Pre-marshalled calls of one training step (forward through the layers, then backward from the last) on one stream."""

    def __init__(self, torch, dp, Layer, specs, linears, n, gen, dev, stream):
        self.stream, self.n = stream, n
        self.layers = [Layer(torch, dp, l, n, gen, dev, True) for l in specs] + [Layer(torch, dp, l, n, gen, dev, False) for l in linears]
        self.mult = [l.spec.count if l.is_conv else 1 for l in self.layers]
        descs = [l.desc(dp, n) for l in self.layers]
        ws_bytes = max(l.ws_bytes(dp, n) for l in self.layers)
        self.ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=dev)
        self.calls = []   # (layer index, pass name, zero-argument launch, nominal flops)
        with torch.cuda.stream(stream):
            for l, d in zip(self.layers, descs):    # the measured kernel choice times its candidates here, job alone on the GPU
                for _, fn, _ in l.passes():
                    fn(dp, d, self.ws, stream)
                    torch.cuda.synchronize()
        for li, (l, d, m) in enumerate(zip(self.layers, descs, self.mult)):
            for _ in range(m):
                self.calls.append((li, "fwd", l.bound("fwd", dp, d, self.ws, stream), l.flops(n)))
        for li in reversed(range(len(self.layers))):
            l, d = self.layers[li], descs[li]
            for _ in range(self.mult[li]):
                self.calls.append((li, "wgrad", l.bound("wgrad", dp, d, self.ws, stream), l.flops(n)))
                if l.needs_dx:
                    self.calls.append((li, "dgrad", l.bound("dgrad", dp, d, self.ws, stream), l.flops(n)))
        self.step_flops = sum(c[3] for c in self.calls)

    def run_step(self):
        for _, _, call, _ in self.calls:
            call()


def run(args, dp, torch, dev, Layer):
    from . import workloads as W
    gen = torch.Generator(device=dev)
    gen.manual_seed(20211210)
    dp.dp_set_autotune(0 if args.no_autotune else 2 if args.autotune == "cold" else 1)
    fg_stream, bg_stream = torch.cuda.Stream(), torch.cuda.Stream()   # both at the default priority
    fg = _Job(torch, dp, Layer, W.vgg16_convs(), W.vgg16_linears(), args.fg_batch, gen, dev, fg_stream)
    bg = _Job(torch, dp, Layer, W.resnet50_convs(), [], args.bg_batch, gen, dev, bg_stream)
    steps = max(3, args.steps)

    # ---- foreground pieces: a few layers per device graph ----
    def capture_pieces(per_piece):
        pieces = []
        for i in range(0, len(fg.calls), per_piece):
            chunk = fg.calls[i:i + per_piece]
            g = torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=fg_stream):
                for _, _, call, _ in chunk:
                    call()
            pieces.append(g)
        torch.cuda.synchronize()
        return pieces

    def fg_eager_step(events=None):
        if events is None:
            fg.run_step()
            return
        for i, (_, _, call, _) in enumerate(fg.calls):
            events[i][0].record(fg_stream)
            call()
            events[i][1].record(fg_stream)

    def time_fg(step_fn, with_layers):
        """Median step latency (HIP events on the foreground stream around each step, nothing between the calls) and, in
        separate eager steps, the latency of each call between two events of its own, summed per layer."""
        lat, per_call = [], [[] for _ in fg.calls]
        for _ in range(steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(fg_stream)
            step_fn()
            e1.record(fg_stream)
            e1.synchronize()
            lat.append(e0.elapsed_time(e1) * 1e3)
        layer_us = {}
        if with_layers:
            for _ in range(steps):
                evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in fg.calls]
                fg_eager_step(evs)
                fg_stream.synchronize()
                for i, (a, b) in enumerate(evs):
                    per_call[i].append(a.elapsed_time(b) * 1e3)
            for i, (li, _, _, _) in enumerate(fg.calls):
                name = fg.layers[li].name
                layer_us[name] = layer_us.get(name, 0.0) + _median(per_call[i])
        return _median(lat), layer_us

    # ---- background launcher thread: loops over its step until told to stop ----
    class Background:
        def __init__(self, pace):
            self.pace, self.stop, self.done_calls, self.thread = pace, False, 0, None
            self.t0 = self.t1 = 0.0

        def loop(self):
            torch.cuda.set_device(dev)
            ring = [torch.cuda.Event() for _ in range(self.pace)] if self.pace > 0 else None
            i = 0
            self.t0 = time.perf_counter()
            while not self.stop:
                for _, _, call, _ in bg.calls:
                    if ring is not None:
                        if i >= self.pace:
                            ring[i % self.pace].synchronize()     # at most `pace` launches of this queue are unfinished
                        call()
                        ring[i % self.pace].record(bg_stream)
                    else:
                        call()
                        if i % 64 == 63:                          # unpaced: only keep the runtime's queue from growing without bound
                            bg_stream.synchronize()
                    i += 1
                    if self.stop:
                        break
            bg_stream.synchronize()
            self.t1 = time.perf_counter()
            self.done_calls = i

        def start(self):
            self.thread = threading.Thread(target=self.loop)
            self.thread.start()
            time.sleep(0.05)   # let the queue fill

        def finish(self):
            self.stop = True
            self.thread.join()
            full, rest = divmod(self.done_calls, len(bg.calls))
            flops = full * bg.step_flops + sum(c[3] for c in bg.calls[:rest])
            return flops / (self.t1 - self.t0) / 1e12

    for _ in range(2):
        fg.run_step()
        bg.run_step()
    torch.cuda.synchronize()
    pieces = capture_pieces(args.graph_piece)

    def fg_graph_step():
        with torch.cuda.stream(fg_stream):   # a replay goes to the current stream
            for g in pieces:
                g.replay()

    ladder = []
    fg_alone_us, layer_alone = time_fg(fg_eager_step, True)
    fg_alone_graph_us, _ = time_fg(fg_graph_step, False)
    b = Background(0)
    b.start()
    time.sleep(0.3)
    bg_alone = b.finish()
    fg_tflops = lambda us: fg.step_flops / us / 1e6
    ladder.append({"config": "foreground alone (eager)", "fg_step_us": fg_alone_us, "fg_slowdown": 1.0, "bg_tflops": 0.0, "combined_tflops": fg_tflops(fg_alone_us)})
    ladder.append({"config": "foreground alone (split graphs)", "fg_step_us": fg_alone_graph_us, "fg_slowdown": fg_alone_graph_us / fg_alone_us, "bg_tflops": 0.0,
                   "combined_tflops": fg_tflops(fg_alone_graph_us)})
    ladder.append({"config": "background alone", "fg_step_us": None, "fg_slowdown": None, "bg_tflops": bg_alone, "combined_tflops": bg_alone})
    layer_colloc = {}
    for label, pace, graphs in (("collocated, no pacing, eager foreground", 0, False),
                                (f"collocated, background paced to {args.pace} launches, eager foreground", args.pace, False),
                                (f"collocated, background paced to {args.pace} launches, foreground as split graphs", args.pace, True),
                                ("collocated, background paced to 1 launch, foreground as split graphs", 1, True)):
        b = Background(pace)
        b.start()
        if graphs:
            us, _ = time_fg(fg_graph_step, False)
        else:
            us, lay = time_fg(fg_eager_step, True)
            if pace > 0:
                layer_colloc = lay
        bg_tf = b.finish()
        wall_share = fg_tflops(us)
        ladder.append({"config": label, "fg_step_us": us, "fg_slowdown": us / fg_alone_us, "bg_tflops": bg_tf, "combined_tflops": bg_tf + wall_share})
    best = max((r for r in ladder if r["fg_step_us"] and r["bg_tflops"]), key=lambda r: r["combined_tflops"])
    return {
        "metric": "single-GPU multiplexing: foreground VGG-16 step latency (batch 2) beside a background ResNet-50 step (batch 64); combined TFLOP/s",
        "value": best["combined_tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "higher_is_better": True, "dtype": "bf16",
        "data": "synthetic (seeded N(0,1) activations/gradients, He-normal weights)",
        "config": {"workload": f"foreground: VGG-16 13 conv + 3 FC, fwd + dgrad + wgrad at per-GPU batch {args.fg_batch}, one stream; background: ResNet-50 "
                               f"53 convs (23 unique shapes with multiplicities), fwd + dgrad + wgrad at batch {args.bg_batch}, looping on a second stream; "
                               "both streams at the default priority (prioritised streams are not usable on this machine pool)",
                   "pace": args.pace, "graph_piece_calls": args.graph_piece, "fg_graph_pieces": len(pieces)},
        "best_config": best["config"], "ladder": ladder,
        "fg_layer_latency_us": {name: [layer_alone[name], layer_colloc.get(name)] for name in layer_alone},
        "fg_layer_latency_columns": ["alone", f"collocated (background paced to {args.pace}, eager foreground)"],
    }
