"""Benchmark of the binarized-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: the binarized layers of the Sketch-A-Net trunk at batch 256 (config 3 of
the benchmark spec: conv2..conv6 + fc7 on synthetic sketches).  One step is one pass of the whole
path over the batch: for every layer, alpha/beta estimation of its filters, weight bit
packing, activation bit packing and the binary convolution / fully-connected product.  The
fp32 inputs of all layers and the fp32 weights are resident in HBM before the timed region.

A step is launched as one captured HIP graph: the weight sides of all layers (they depend on
no activation) run on side streams while the main stream packs the activations of all layers;
the products follow on two streams (each on the one with less product time so far).  The timed
region is K graph launches.

Prints one JSON line: the metric (effective binary MACs/s), the roofline of the dominant
call (the binary product of the largest layer) from HIP-event timings of an eager pass over
the same kernels, and the CPU oracle timed on the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Rooflines of the binary product on MI355X.
#   MFMA, fp4 operands (the kernel that ships): published dense peak 10.1 PFLOP/s = 5.05e15 MAC/s.
#   Vector ALU popcount form, for comparison: 256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-ops/s and
#   one AND + one BCNT per 32 binary MACs of a lane, i.e. at most 6.29e14 binary MAC/s.
#   HBM: 8 TB/s; a layer writes 4 bytes per output and reads its packed/expanded operands.
MFMA_FP4_FLOPS = 10.1e15
MFMA_BF16_FLOPS = 2.5e15
VALU_PAIR_MACS = 256 * 64 * 2.4e9 * 16
HBM_BYTES_PER_S = 8.0e12
# HBM bytes of one conv2 call at batch 256 (prepare + main kernel), from the FETCH_SIZE and WRITE_SIZE
# counter runs summarised in profiles/bench_config3_hbm_counters.md
CONV2_CALL_HBM_BYTES = 157136400


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=256, help="images per step (the metric is quoted at 256)")
    ap.add_argument("--cpu-batch", type=int, default=256, help="images of the CPU-oracle sample (0 = skip)")
    ap.add_argument("--product-streams", type=int, default=2,
                    help="streams the binary products alternate over (1 = all on the main stream)")
    ap.add_argument("--side-streams", type=int, default=2,
                    help="HIP streams for the weight side (estimation + weight packing) of the layers; 0 = one stream")
    ap.add_argument("--no-graph", action="store_true",
                    help="time eager launches instead of one captured HIP graph per step")
    ap.add_argument("--wait-all", action="store_true",
                    help="let the first product wait for the weight sides of all layers (default: each product waits "
                         "only for its own layer's weights, so later layers' weight sides run beside earlier products)")
    ap.add_argument("--no-fused", action="store_true", help="skip the measurements beside the headline (fused chain, training side, weights-only layers)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 256 MiB device-to-device copies (a known-size kernel that scales the "
                         "HBM byte counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


class LayerState:
    """Device buffers of one binarized layer, allocated once."""

    def __init__(self, L, W, X, tau, dab, torch):
        self.L, self.W, self.X, self.tau = L, W, X, tau
        B = X.shape[0]
        dev = X.device
        self.B = B
        self.W2 = W.reshape(L.F, -1)
        if L.is_fc:
            self.desc = None
            self.Y = torch.empty((B, L.F), dtype=torch.float32, device=dev)
            self.A = torch.empty((B, 1, 1, dab.words_per_pixel(L.C)), dtype=torch.int32, device=dev)
        else:
            self.desc = dab.dab_conv_desc(B, L.C, L.H, L.W, L.F, L.kh, L.kw, L.pad, L.pad, L.stride, L.stride)
            self.Y = torch.empty((B, L.Ho, L.Wo, L.F), dtype=torch.float32, device=dev)
            self.A = torch.empty((B, L.H, L.W, dab.words_per_pixel(L.C)), dtype=torch.int32, device=dev)
        self.macs = L.macs(B)
        nbytes = (dab.lib().dab_binfc_workspace_bytes(B, L.C, L.F) if L.is_fc
                  else dab.lib().dab_binconv2d_workspace_bytes(ctypes.byref(self.desc)))
        self.ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=dev)
        self.est = dab.estimate_outputs(L.F, dev)
        self.EW = dab.pack_weights_outputs(L.F, W.shape[1], W.shape[2], W.shape[3], dev)
        self.est_ws = torch.empty(max(dab.lib().dab_estimate_workspace_bytes(L.F, self.W2.shape[1]), 1),
                                  dtype=torch.uint8, device=dev)


def weight_side(s, dab):
    """alpha/beta estimation and weight bit packing of one layer (independent of the activations)."""
    est = dab.dab_estimate_alpha_beta(s.W2, out=s.est, ws=s.est_ws)
    dab.dab_pack_weights(s.W, est["thr_val"], est["thr_idx"], est["alpha_is_upper"], out=s.EW)


def activation_side(s, dab):
    dab.dab_pack_activations(s.X, dab.DAB_LAYOUT_NHWC, s.tau, out=s.A)


def product(s, dab):
    if s.desc is None:
        dab.dab_binfc(s.A.view(s.B, -1), s.EW[0], s.est["alpha"], s.est["beta"], s.L.C, out=s.Y, ws=s.ws)
    else:
        dab.dab_binconv2d(s.desc, s.A, s.EW[0], s.est["alpha"], s.est["beta"], out=s.Y, ws=s.ws)


def run_layer(s, dab, events=None):
    """estimate -> pack weights -> pack activations -> binary product, all on the current stream."""
    weight_side(s, dab)
    activation_side(s, dab)
    if events is not None:
        events[0].record()
    product(s, dab)
    if events is not None:
        events[1].record()
    return s.Y


class Schedule:
    """One step of all layers over HIP streams of equal (default) priority.

    The weight side of a layer (estimation, weight packing) depends on no activation, so the
    weight sides run on side streams (the heaviest layer alone, the others dealt out in layer order) while the current
    stream packs the activations of all layers (every input is resident when the step starts;
    memory-bound work beside the LDS-bound estimation).  The binary products then go, in layer
    order, to the current stream and one more (to the one with less product time so far, or
    alternating when the durations are not given): a product waits for its own layer's weights only
    (an event per layer), so the weight sides of later layers run beside the products of earlier
    ones, and with two product streams the prepare kernel of the next layer runs beside the
    main kernel of this one, whose last workgroups hand their compute units straight to the next
    main kernel.  A step forks from and joins back into the current stream, so steps never
    overlap, and the whole step can be captured into one HIP graph.
    """

    def __init__(self, states, n_side, torch, per_layer=True, n_product=2, product_ms=None):
        self.torch = torch
        self.states = states
        self.side = [torch.cuda.Stream() for _ in range(n_side)]
        self.extra = [torch.cuda.Stream() for _ in range(max(n_product, 1) - 1)] if n_side > 0 else []
        # the layer with by far the most weights (conv6) has a side stream to itself; the others are
        # dealt out in layer order over the remaining side streams, so that their weights become
        # ready in the order the products need them
        self.assign = [[] for _ in range(max(n_side, 1))]
        heavy = max(range(len(states)), key=lambda i: states[i].W2.numel())
        if n_side >= 2:
            self.assign[0].append(heavy)
            rest = [i for i in range(len(states)) if i != heavy]
            for k, i in enumerate(rest):
                self.assign[1 + k % (n_side - 1)].append(i)
        else:
            self.assign[0] = list(range(len(states)))
        # products: in layer order, each on the product stream with the least work so far when the
        # durations of the products are known (the small late layers then run beside a large one
        # instead of alone at the end), else alternating
        n_q = 1 + len(self.extra)
        self.product_on = [i % n_q for i in range(len(states))]
        if product_ms is not None and n_q > 1:
            load = [0.0] * n_q
            for i, ms in enumerate(product_ms):
                q = min(range(n_q), key=lambda j: load[j])
                self.product_on[i] = q
                load[q] += ms
        self.fork = torch.cuda.Event()
        self.packed = torch.cuda.Event()
        self.ready = [torch.cuda.Event() for _ in self.side]
        self.joined = [torch.cuda.Event() for _ in self.extra]
        self.layer_ready = [torch.cuda.Event() for _ in states]
        self.per_layer = per_layer

    def step(self, dab):
        torch, states = self.torch, self.states
        if not self.side:
            for s in states:
                run_layer(s, dab)
            return
        main = torch.cuda.current_stream()
        self.fork.record(main)
        # the main stream's first kernel is enqueued (and captured) before the side work, so that a
        # graph launch starts the main chain at once instead of behind the longest weight side
        activation_side(states[0], dab)
        for q, idxs, done in zip(self.side, self.assign, self.ready):
            q.wait_event(self.fork)
            with torch.cuda.stream(q):
                for i in idxs:
                    weight_side(states[i], dab)
                    if self.per_layer:
                        self.layer_ready[i].record(q)
            done.record(q)
        for s in states[1:]:
            activation_side(s, dab)
        self.packed.record(main)
        streams = [main] + self.extra
        for q in self.extra:
            q.wait_event(self.packed)
        if not self.per_layer:
            for q in streams:
                for done in self.ready:
                    q.wait_event(done)
        for i, s in enumerate(states):
            q = streams[self.product_on[i]]
            if self.per_layer:
                q.wait_event(self.layer_ready[i])
            with torch.cuda.stream(q):
                product(s, dab)
        for q, done in zip(self.extra, self.joined):
            done.record(q)
            main.wait_event(done)
        for done in self.ready:
            main.wait_event(done)

    def capture(self, dab):
        """The step as one HIP graph (kernel launches and stream dependencies only)."""
        torch = self.torch
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            self.step(dab)
        return graph


class FusedChain:
    """The same six layers with the re-binarizing epilogue: bits are handed from layer to layer
    (3/2 max-pooling as an OR on the bits after conv2 and conv5), so between conv2 and fc7 no fp32
    activation is written or read.  conv2 packs its fp32 input as in the plain step and fc7 writes
    fp32.  Thresholds of the hand-over are the per-channel means the plain step uses.  The weight
    sides run on the side streams of the schedule it is given (bench.py: one, in layer order)."""

    def __init__(self, states, sched, dab, torch):
        self.states, self.sched, self.torch = states, sched, torch
        self.bits = []
        for s in states:
            L = s.L
            if L.is_fc:
                self.bits.append(None)
                continue
            out = torch.empty((s.B, L.Ho, L.Wo, dab.words_per_pixel(L.F)), dtype=torch.int32, device=s.X.device)
            pooled = None
            if L.pool_after:
                pooled = torch.empty((s.B, (L.Ho - 3) // 2 + 1, (L.Wo - 3) // 2 + 1, dab.words_per_pixel(L.F)),
                                     dtype=torch.int32, device=s.X.device)
            self.bits.append((out, pooled))

    def step(self, dab, events=None):
        torch, states, sched = self.torch, self.states, self.sched
        main = torch.cuda.current_stream()
        sched.fork.record(main)
        activation_side(states[0], dab)
        for q, idxs, done in zip(sched.side, sched.assign, sched.ready):
            q.wait_event(sched.fork)
            with torch.cuda.stream(q):
                for i in idxs:
                    weight_side(states[i], dab)
                    sched.layer_ready[i].record(q)
            done.record(q)
        A = states[0].A
        for i, s in enumerate(states):
            main.wait_event(sched.layer_ready[i])
            if events is not None:
                events[i][0].record()
            if s.desc is None:
                dab.dab_binfc(A.view(s.B, -1), s.EW[0], s.est["alpha"], s.est["beta"], s.L.C, out=s.Y, ws=s.ws)
            else:
                out, pooled = self.bits[i]
                dab.dab_binconv2d_bits(s.desc, A, s.EW[0], s.est["alpha"], s.est["beta"], states[i + 1].tau, out=out,
                                       ws=s.ws)
                A = out
                if pooled is not None:
                    dab.dab_pool_bits(out, s.L.F, 3, 3, 2, 2, out=pooled)
                    A = pooled
            if events is not None:
                events[i][1].record()
        for done in sched.ready:
            main.wait_event(done)

    def capture(self, dab):
        torch = self.torch
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            self.step(dab)
        return graph


def build_states(batch, dab, torch, wl):
    """Synthetic sketches -> fp32 conv1 features -> inputs of all six layers (chained through the GPU path)."""
    dev = torch.device("cuda:0")
    imgs = wl.sketch_images(batch)
    w1, ws = wl.config3_weights()
    x = wl.config3_conv1_features(imgs, w1, device=dev)            # [B, 64, 35, 35], untimed fp32 prologue
    x = x.permute(0, 2, 3, 1).contiguous()                        # NHWC
    states = []
    for L, W in zip(wl.CFG3_LAYERS, ws):
        if L.is_fc:
            x = x.reshape(batch, -1).contiguous()
            tau = x.mean(dim=0)
        else:
            tau = x.mean(dim=(0, 1, 2))
        s = LayerState(L, torch.from_numpy(W).to(dev), x, tau.contiguous(), dab, torch)
        states.append(s)
        y = run_layer(s, dab).clone()
        if L.pool_after:
            y = torch.nn.functional.max_pool2d(y.permute(0, 3, 1, 2), 3, 2).permute(0, 2, 3, 1).contiguous()
        x = y
    torch.cuda.synchronize()
    return states


def training_weight_side(states, dab, torch, args):
    """The weight side of one training iteration (Algorithm 2, Theorem 4) for the six layers, measured
    beside the headline: MeanCenter + Clamp, estimation inside a window around the previous split,
    weight packing, W~, and the gradient factor applied to an upstream gradient.  The layers are
    independent: the one with by far the most weights has a stream to itself, the others are dealt
    over two more; one HIP graph.  Algorithmic bytes: nine passes over arrays of the size of W (the raw weights read once,
    the centred weights read by four kernels, the upstream gradient read once; centred weights, W~ and
    the gradient written) plus the packed bits."""
    bufs = []
    for s in states:
        bufs.append({"Wc": torch.empty_like(s.W), "Wt": torch.empty_like(s.W2), "G": torch.empty_like(s.W2),
                     "up": torch.randn_like(s.W2), "prev": {k: v.clone() for k, v in s.est.items()}})

    def layer(s, b):
        dab.dab_mean_center_clamp(s.W, dab.DAB_CENTER_FILTER, -1.0, 1.0, out=b["Wc"])
        W2 = b["Wc"].view(s.L.F, -1)
        est = dab.dab_estimate_alpha_beta_bounded(W2, b["prev"]["K"], b["prev"]["alpha_is_upper"],
                                                  max(1, W2.shape[1] // 64), out=b["prev"], ws=s.est_ws)
        dab.dab_pack_weights(b["Wc"], est["thr_val"], est["thr_idx"], est["alpha_is_upper"], out=s.EW)
        dab.dab_binarized_weights(W2, est["alpha"], est["beta"], est["thr_val"], est["thr_idx"],
                                  est["alpha_is_upper"], out=b["Wt"])
        dab.dab_weight_gradient(W2, est["thr_val"], est["thr_idx"], est["alpha_is_upper"], upstream=b["up"],
                                out=b["G"])

    heavy = max(range(len(states)), key=lambda i: states[i].W2.numel())
    rest = [i for i in range(len(states)) if i != heavy]
    groups = [[heavy], rest[0::2], rest[1::2]]                   # the current stream takes the last group
    sides = [torch.cuda.Stream() for _ in groups[:-1]]
    fork = torch.cuda.Event()
    joined = [torch.cuda.Event() for _ in sides]

    def step():
        main = torch.cuda.current_stream()
        fork.record(main)
        for q, idxs, done in zip(sides, groups, joined):
            q.wait_event(fork)
            with torch.cuda.stream(q):
                for i in idxs:
                    layer(states[i], bufs[i])
                done.record(q)
        for i in groups[-1]:
            layer(states[i], bufs[i])
        for done in joined:
            main.wait_event(done)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
        step()
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        graph.replay()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    weights = sum(s.W.numel() for s in states)
    nbytes = weights * 4 * 9 + sum(s.EW[0].numel() * 4 for s in states)
    # leave the plain step's packed weights as they were
    for s in states:
        weight_side(s, dab)
    torch.cuda.synchronize()
    return {"what": "MeanCenter + Clamp, windowed estimate, pack weights, W~, Theorem 4 gradient for the six layers; "
                    "three streams (the largest layer alone), one HIP graph",
            "ms_per_step": round(1e3 * dt / args.steps, 4), "weights": weights, "algorithmic_bytes": nbytes,
            "gb_per_s": round(nbytes / (dt / args.steps) / 1e9, 1)}


def weights_only_products(states, dab, torch, args):
    """The six layers as weights-only binarized layers (WBin of Section 5.1) on their real-valued inputs,
    one call after the other on one stream: HIP events around each dab_wbin_conv2d / dab_wbin_fc.
    Each input element becomes three bf16 pieces, so a binary MAC costs three bf16 MACs (6 FLOP)."""
    import ctypes as ct
    out = {}
    total_ms, total_macs = 0.0, 0
    for s in states:
        L = s.L
        nbytes = (dab.lib().dab_wbin_fc_workspace_bytes(s.B, L.C, L.F) if L.is_fc
                  else dab.lib().dab_wbin_conv2d_workspace_bytes(ct.byref(s.desc)))
        ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=s.X.device)
        Y = torch.empty_like(s.Y)

        def run():
            if L.is_fc:
                dab.dab_wbin_fc(s.X.view(s.B, -1), s.EW[0], s.est["alpha"], s.est["beta"], out=Y, ws=ws)
            else:
                dab.dab_wbin_conv2d(s.desc, s.X, s.EW[0], s.est["alpha"], s.est["beta"], out=Y, ws=ws)

        for _ in range(args.warmup):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(1, min(args.steps, 20))
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        total_ms += ms
        total_macs += s.macs
        out[L.name] = {"ms": round(ms, 4), "bf16_tflops": round(6 * s.macs / (ms * 1e-3) / 1e12, 1),
                       "frac_of_mfma_bf16_peak": round(6 * s.macs / (ms * 1e-3) / MFMA_BF16_FLOPS, 4)}
        del ws, Y
    return {"what": "dab_wbin_conv2d / dab_wbin_fc (prepare + product) per layer, fp32 inputs as three bf16 pieces, "
                    "one stream",
            "ms_per_step": round(total_ms, 4), "macs_per_s": total_macs / (total_ms * 1e-3), "per_layer": out}


def cpu_oracle_baseline(batch, wl):
    """The float64 CPU oracle, as it stands, on a small slice of the same workload."""
    import numpy as np
    import torch
    from oracle import estimate as oest
    from oracle import layers as olay
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    imgs = wl.sketch_images(batch)
    w1, ws = wl.config3_weights()
    x0 = wl.config3_conv1_features(imgs, w1).numpy()
    macs = 0
    passes = 3                                                   # about a dozen seconds on the GPU machine's host cores
    t0 = time.perf_counter()
    for _ in range(passes):
        x = x0
        for L, W in zip(wl.CFG3_LAYERS, ws):
            if L.is_fc:
                x = x.reshape(batch, -1)
            x4 = x if x.ndim == 4 else x[:, :, None, None]
            tau = x4.mean(axis=(0, 2, 3)).astype(np.float32)
            r = oest.estimate_alpha_beta(W)
            a = olay.binarize_activations(x4, tau)
            y = olay.conv2d(a, olay.two_valued_filters(r["e"], r["alpha"], r["beta"]), (L.pad, L.pad),
                            (L.stride, L.stride))
            macs += L.macs(batch)
            y = torch.from_numpy(y.astype(np.float32)).permute(0, 3, 1, 2)
            if L.pool_after:
                y = torch.nn.functional.max_pool2d(y, 3, 2)
            x = y.numpy()
    dt = time.perf_counter() - t0
    return {"value": macs / dt, "unit": "binary MAC/s", "cores": int(threads), "kind": "oracle",
            "sample": f"config 3, all six layers incl. alpha/beta estimation, batch {batch} of 256, {passes} passes, {dt:.1f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every layer is computed whole on one MI355X); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1804_02941_amd import binding as dab
    from paper_1804_02941_amd import workloads as wl
    if not os.path.exists(dab.LIB_PATH):
        from paper_1804_02941_amd import build
        build.build()
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    torch.cuda.set_device(0)

    states = build_states(args.batch, dab, torch, wl)
    total_macs = sum(s.macs for s in states)
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # Kernel timing pass: every layer launched eagerly on one stream with a HIP event pair around its
    # binary product (events cannot be recorded inside a captured graph on this platform, and with
    # several streams the eager launches are host-bound, which would put launch gaps between the
    # product's kernels).  In the schedule the products have the chip to themselves, as they do here.
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in states]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    for _ in range(min(args.warmup, 3)):
        for s in states:
            run_layer(s, dab)
    for k in range(args.steps):
        for s, e in zip(states, ev[k]):
            run_layer(s, dab, e)
    torch.cuda.synchronize()
    product_ms = [sum(ev[k][i][0].elapsed_time(ev[k][i][1]) for k in range(args.steps)) / args.steps
                  for i in range(len(states))]

    sched = Schedule(states, args.side_streams, torch, per_layer=not args.wait_all, n_product=args.product_streams,
                     product_ms=product_ms)
    for _ in range(args.warmup):
        sched.step(dab)
    torch.cuda.synchronize()

    # The schedule launched eagerly (host-bound with side streams; reported for comparison)
    t0 = time.perf_counter()
    for k in range(args.steps):
        sched.step(dab)
    t_enqueued = time.perf_counter() - t0
    torch.cuda.synchronize()
    dt_eager = time.perf_counter() - t0

    # Timed region: exactly `steps` steps, each one launch of the captured HIP graph
    if args.no_graph:
        dt = dt_eager
    else:
        graph = sched.capture(dab)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0

    ms_per_step = 1e3 * dt / args.steps
    value = total_macs * args.steps / dt
    # binary product: per layer and aggregate, from the events of the kernel timing pass.  With fp32
    # outputs every large layer sits below the ridge of the fp4 matrix cores (conv2: 784 FLOP per
    # algorithmic byte against 10.1e15 / 8e12 = 1262), so the bound that applies is HBM; the MFMA view
    # is printed beside it.  Algorithmic bytes of a call = fp32 outputs + activation bits + weight bits
    # + alpha and beta.
    per_layer = {}
    conv_ms = 0.0
    algo_bytes = 0
    for i, s in enumerate(states):
        ms = product_ms[i]
        conv_ms += ms
        nbytes = s.Y.numel() * 4 + s.A.numel() * 4 + s.EW[0].numel() * 4 + 8 * s.L.F
        algo_bytes += nbytes
        per_layer[s.L.name] = {"ms": round(ms, 4), "gmacs": round(s.macs / 1e9, 3),
                               "algorithmic_bytes": nbytes,
                               "gb_per_s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                               "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / HBM_BYTES_PER_S, 4),
                               "tflops": round(2 * s.macs / (ms * 1e-3) / 1e12, 1),
                               "frac_of_mfma_fp4_peak": round(2 * s.macs / (ms * 1e-3) / MFMA_FP4_FLOPS, 4)}
    dom = max(per_layer, key=lambda k: per_layer[k]["ms"])         # the dominant call (conv2 at batch 256)
    d = per_layer[dom]
    traffic = CONV2_CALL_HBM_BYTES if (dom == "conv2" and args.batch == 256) else None
    roofline = {"bound": "hbm",
                "kernel": "dab_binconv2d of %s: binconv_prepare_kernel + binconv_mfma_kernel, bracketed by HIP events "
                          "on the launch stream" % dom,
                "achieved": d["gb_per_s"], "peak": HBM_BYTES_PER_S / 1e9, "unit": "GB/s",
                "frac": d["frac_of_hbm_peak"], "traffic": traffic,
                "algorithmic_bytes": d["algorithmic_bytes"], "launch_ms": d["ms"],
                "mfma_view": {"achieved": d["tflops"], "peak": MFMA_FP4_FLOPS / 1e12, "unit": "TFLOP/s",
                              "frac": d["frac_of_mfma_fp4_peak"]},
                "all_layers": {"kernel_ms_per_step": round(conv_ms, 4), "algorithmic_bytes": algo_bytes,
                               "gb_per_s": round(algo_bytes / (conv_ms * 1e-3) / 1e9, 1),
                               "frac_of_hbm_peak": round(algo_bytes / (conv_ms * 1e-3) / HBM_BYTES_PER_S, 4),
                               "tflops": round(2 * total_macs / (conv_ms * 1e-3) / 1e12, 1),
                               "frac_of_mfma_fp4_peak": round(2 * total_macs / (conv_ms * 1e-3) / MFMA_FP4_FLOPS, 4),
                               "binary_macs_per_s": total_macs / (conv_ms * 1e-3),
                               "vs_valu_popcount_peak": round(total_macs / (conv_ms * 1e-3) / VALU_PAIR_MACS, 3)},
                "kernel_ms_per_step": round(conv_ms, 4),
                "per_layer": per_layer}

    # The next row of the scope table, measured beside the headline: the fused chain
    fused = None
    if args.side_streams > 0 and not args.no_fused:
        # its products form one dependent chain, so one side stream (weight sides in layer order) delivers
        # every layer's weights in time, and every further branch of the graph only costs launch overhead
        chain = FusedChain(states, Schedule(states, 1, torch), dab, torch)
        for _ in range(args.warmup):
            chain.step(dab)
        torch.cuda.synchronize()
        fev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in states]
               for _ in range(args.steps)]
        for k in range(args.steps):
            chain.step(dab, fev[k])
        torch.cuda.synchronize()
        fgraph = chain.capture(dab)
        for _ in range(args.warmup):
            fgraph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            fgraph.replay()
        torch.cuda.synchronize()
        fdt = time.perf_counter() - t0
        fused = {"what": "same layers, bits handed from layer to layer by dab_binconv2d_bits / dab_pool_bits "
                         "(fp32 only into conv2 and out of fc7); one HIP graph per step",
                 "ms_per_step": round(1e3 * fdt / args.steps, 4),
                 "binary_macs_per_s": total_macs * args.steps / fdt,
                 "product_ms_per_layer": {s.L.name: round(sum(fev[k][i][0].elapsed_time(fev[k][i][1])
                                                              for k in range(args.steps)) / args.steps, 4)
                                          for i, s in enumerate(states)}}

    training = None if args.no_fused else training_weight_side(states, dab, torch, args)
    wbin = None if args.no_fused else weights_only_products(states, dab, torch, args)
    cpu = cpu_oracle_baseline(args.cpu_batch, wl) if args.cpu_batch > 0 else None
    line = {
        "metric": "effective binary MACs/s on Sketch-A-Net binarized layers",
        "value": value, "unit": "binary MAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4 (e2m1) operands expanded from 1-bit, fp32 MFMA accumulate (exact integers), fp32 epilogue, fp64 estimation", "data": "synthetic",
        "config": {"workload": "config 3: Sketch-A-Net binarized trunk (conv2-conv6, fc7), batch %d, "
                               "estimate + pack weights + pack activations + binary product per layer" % args.batch,
                   "batch": args.batch, "binary_macs_per_step": total_macs,
                   "streams": 1 + args.side_streams + (max(args.product_streams, 1) - 1 if args.side_streams else 0),
                   "launch": "eager" if args.no_graph else "one captured HIP graph per step",
                   "product_stream_of_layer": sched.product_on,
                   "eager_ms_per_step": round(1e3 * dt_eager / args.steps, 4),
                   "eager_host_enqueue_ms_per_step": round(1e3 * t_enqueued / args.steps, 4)},
        "roofline": roofline, "cpu_baseline": cpu, "rebinarized_chain": fused,
        "training_weight_side": training, "weights_only_layers": wbin,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
