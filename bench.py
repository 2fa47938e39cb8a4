"""Benchmark of the binarized-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload: the binarized layers of the Sketch-A-Net trunk at batch 256 (config 3 of
the benchmark spec: conv2..conv6 + fc7 on synthetic sketches).  One step is one pass of the whole
path over the batch: for every layer, alpha/beta estimation of its filters, weight bit
packing, activation bit packing and the binary convolution / fully-connected product.  The
fp32 inputs of all layers and the fp32 weights are resident in HBM before the timed region.

A step is seven calls on one stream, captured as one HIP graph: dab_prepare_layers does the weight
sides of all six layers (estimation + mask packing: one launch for the five layers with short
filters, one for conv6 with its 12544-element filters, one behind it for rows handed to the sort)
and, inside the same launches, packs the activations of all six layers; each binary product is a
single launch that reads the packed bits and writes fp32.  The timed region is K graph launches.

Prints one JSON line: the metric (effective binary MACs/s), the roofline of the dominant
kernel (the binary product of the largest layer), a table of every stage against the HBM
roofline, and the CPU oracle timed on the same workload.  Device times of single calls are
taken from graphs that hold the call several times back to back on one stream, the replay
bracketed by HIP events on that stream: the host cannot enqueue small kernels as fast as the
chip runs them, so an event pair around eager launches would time the host.
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
#   Vector ALU popcount form, for comparison: 256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-ops/s;
#   P_bcnt counts the popcount alone (32 MACs per lane-op), P_pair the AND + popcount a product needs (16).
#   HBM: 8 TB/s; a layer writes 4 bytes per output and reads its packed operands.
MFMA_FP4_FLOPS = 10.1e15
MFMA_BF16_FLOPS = 2.5e15
VALU_LANE_OPS = 256 * 64 * 2.4e9
P_BCNT_SPEC = VALU_LANE_OPS * 32
P_PAIR_SPEC = VALU_LANE_OPS * 16
HBM_BYTES_PER_S = 8.0e12
# HBM byte counters of the dominant kernel (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file,
# scaled by a copy of known size); the file records the commit it was measured at.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=256, help="images per step (the metric is quoted at 256)")
    ap.add_argument("--cpu-batch", type=int, default=256, help="images of the CPU-oracle sample (0 = skip)")
    ap.add_argument("--no-graph", action="store_true",
                    help="time eager launches instead of one captured HIP graph per step")
    ap.add_argument("--separate", action="store_true",
                    help="weight sides and activation packing as two calls instead of dab_prepare_layers")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the measurements beside the headline (stage table, other configs, fused chain, "
                         "training side, weights-only layers, small batch)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three 256 MiB device-to-device copies (a known-size kernel that scales the "
                         "HBM byte counters of a rocprofv3 --pmc run)")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------
# device timing
def device_us(torch, fn, reps=10, replays=5):
    """Average device time of one fn() in microseconds: `reps` calls captured back to back on one stream,
    the graph replayed `replays` times, each replay bracketed by HIP events on the replaying stream."""
    q = torch.cuda.Stream()
    with torch.cuda.stream(q):
        fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=q):
        for _ in range(reps):
            fn()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total = 0.0
    for _ in range(replays):
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        total += e0.elapsed_time(e1)
    return 1e3 * total / (replays * reps)


def hbm_row(us, nbytes, launches):
    return {"us": round(us, 2), "launches": launches, "algorithmic_bytes": int(nbytes),
            "gb_per_s": round(nbytes / (us * 1e-6) / 1e9, 1),
            "frac_of_hbm_peak": round(nbytes / (us * 1e-6) / HBM_BYTES_PER_S, 4)}


# ------------------------------------------------------------------------------------------------
# one binarized layer and the calls on it
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
        self.ws_bytes = nbytes
        self.ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=dev)
        self.est = dab.estimate_outputs(L.F, dev)
        self.EW = dab.pack_weights_outputs(L.F, W.shape[1], W.shape[2], W.shape[3], dev)
        self.est_ws = torch.empty(max(dab.lib().dab_estimate_workspace_bytes(L.F, self.W2.shape[1]), 1),
                                  dtype=torch.uint8, device=dev)

    # algorithmic bytes of the three stages
    def pack_bytes(self):
        return self.X.numel() * 4 + self.A.numel() * 4 + (self.tau.numel() * 4 if self.tau is not None else 0)

    def weight_bytes(self):
        return self.W.numel() * 4 + self.EW[0].numel() * 4 + 8 * self.L.F

    def product_bytes(self):
        return self.Y.numel() * 4 + self.A.numel() * 4 + self.EW[0].numel() * 4 + 8 * self.L.F


def weight_side(s, dab):
    """alpha/beta estimation and weight bit packing of one layer as two calls."""
    est = dab.dab_estimate_alpha_beta(s.W2, out=s.est, ws=s.est_ws)
    dab.dab_pack_weights(s.W, est["thr_val"], est["thr_idx"], est["alpha_is_upper"], out=s.EW)


def activation_side(s, dab):
    dab.dab_pack_activations(s.X, dab.DAB_LAYOUT_NHWC, s.tau, out=s.A)


def product(s, dab):
    if s.desc is None:
        dab.dab_binfc(s.A.view(s.B, -1), s.EW[0], s.est["alpha"], s.est["beta"], s.L.C, out=s.Y, ws=s.ws)
    else:
        dab.dab_binconv2d(s.desc, s.A, s.EW[0], s.est["alpha"], s.est["beta"], out=s.Y, ws=s.ws)


def run_layer(s, dab):
    weight_side(s, dab)
    activation_side(s, dab)
    product(s, dab)
    return s.Y


class GroupedStep:
    """One step of a set of independent layers through the grouped entry points, on one stream:
    dab_prepare_layers (the weight sides of all layers and, in the same launches, the activation
    packing of all layers), then the binary products in layer order.  `separate` issues the weight
    sides and the packing as two calls instead (for comparison)."""

    def __init__(self, states, dab, torch, separate=False):
        self.states, self.torch, self.dab, self.separate = states, torch, dab, separate
        self.pack = dab.pack_jobs([(s.X, s.tau, s.A) for s in states])
        self.jobs = dab.weight_jobs([dict(W=s.W, est=s.est, packed=s.EW) for s in states])
        nbytes = dab.lib().dab_binarize_weights_multi_workspace_bytes(self.jobs, len(self.jobs))
        self.ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=states[0].X.device)

    def weights(self):
        self.dab.dab_binarize_weights_multi(self.jobs, ws=self.ws)

    def pack_all(self):
        self.dab.dab_pack_activations_multi(self.pack)

    def prepare(self):
        self.dab.dab_prepare_layers(self.jobs, self.pack, ws=self.ws)

    def step(self):
        if self.separate:
            self.weights()
            self.pack_all()
        else:
            self.prepare()
        for s in self.states:
            product(s, self.dab)

    def capture(self):
        torch = self.torch
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
            self.step()
        return graph


class FusedChain:
    """The same six layers with the re-binarizing epilogue: bits are handed from layer to layer
    (3/2 max-pooling as an OR on the bits after conv2 and conv5), so between conv2 and fc7 no fp32
    activation is written or read.  conv2 packs its fp32 input (in the launches of the weight sides,
    as in the plain step) and fc7 writes fp32.  Thresholds of the hand-over are the per-channel
    means the plain step uses.  One stream."""

    def __init__(self, states, grouped, dab, torch):
        self.states, self.grouped, self.torch = states, grouped, torch
        self.pack_first = dab.pack_jobs([(states[0].X, states[0].tau, states[0].A)])
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

    def product(self, i, A, dab):
        """Layer i on packed input A; returns the packed input of the next layer."""
        s = self.states[i]
        if s.desc is None:
            dab.dab_binfc(A.view(s.B, -1), s.EW[0], s.est["alpha"], s.est["beta"], s.L.C, out=s.Y, ws=s.ws)
            return None
        out, pooled = self.bits[i]
        dab.dab_binconv2d_bits(s.desc, A, s.EW[0], s.est["alpha"], s.est["beta"], self.states[i + 1].tau, out=out,
                               ws=s.ws)
        if pooled is None:
            return out
        dab.dab_pool_bits(out, s.L.F, 3, 3, 2, 2, out=pooled)
        return pooled

    def inputs(self, dab):
        """The packed input of every layer of the chain (for timing one layer alone)."""
        A, res = self.states[0].A, []
        for i in range(len(self.states)):
            res.append(A)
            A = self.product(i, A, dab)
        return res

    def step(self, dab):
        g = self.grouped
        dab.dab_prepare_layers(g.jobs, self.pack_first, ws=g.ws)
        A = self.states[0].A
        for i in range(len(self.states)):
            A = self.product(i, A, dab)

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


def time_graph(torch, graph, steps, warmup):
    for _ in range(warmup):
        graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


# ------------------------------------------------------------------------------------------------
# measurements beside the headline
def stage_table(states, grouped, dab, torch):
    """Every stage of the step alone on the chip, against the HBM roofline (algorithmic bytes: what the
    stage must read and write once)."""
    rows = {}
    rows["prepare_layers: weight sides and activation packing of all layers, one call"] = hbm_row(
        device_us(torch, grouped.prepare), sum(s.pack_bytes() + s.weight_bytes() for s in states), 3)
    rows["pack_activations: all layers, one launch"] = hbm_row(
        device_us(torch, grouped.pack_all), sum(s.pack_bytes() for s in states), 1)
    rows["estimate + pack_weights: all layers, one grouped call"] = hbm_row(
        device_us(torch, grouped.weights), sum(s.weight_bytes() for s in states), 3)
    for s in states:
        rows[f"pack_activations: {s.L.name}"] = hbm_row(device_us(torch, lambda s=s: activation_side(s, dab)),
                                                        s.pack_bytes(), 1)
        rows[f"estimate: {s.L.name}"] = hbm_row(
            device_us(torch, lambda s=s: dab.dab_estimate_alpha_beta(s.W2, out=s.est, ws=s.est_ws)),
            s.W.numel() * 4 + 24 * s.L.F, None)
        rows[f"pack_weights: {s.L.name}"] = hbm_row(
            device_us(torch, lambda s=s: dab.dab_pack_weights(s.W, s.est["thr_val"], s.est["thr_idx"],
                                                              s.est["alpha_is_upper"], out=s.EW)),
            s.W.numel() * 4 + s.EW[0].numel() * 4 + 9 * s.L.F, 1)
    return rows


def product_rows(states, dab, torch):
    rows = {}
    for s in states:
        us = device_us(torch, lambda s=s: product(s, dab))
        r = hbm_row(us, s.product_bytes(), 1 if s.ws_bytes == 0 else None)
        r.update({"ms": round(us * 1e-3, 5), "gmacs": round(s.macs / 1e9, 3),
                  "tflops": round(2 * s.macs / (us * 1e-6) / 1e12, 1),
                  "frac_of_mfma_fp4_peak": round(2 * s.macs / (us * 1e-6) / MFMA_FP4_FLOPS, 4)})
        rows[s.L.name] = r
    return rows


def popcount_ceiling(dab, torch):
    """P_bcnt and P_pair of the vector-ALU form of the product (Section 3.2) from the measured issue rate
    of the popcount instruction and the shader clock sustained under that load."""
    grid, iters = 256 * 16, 512
    out = torch.empty(grid * 256, dtype=torch.int32, device="cuda:0")
    clocks = torch.zeros(grid * 2, dtype=torch.int64, device="cuda:0")
    res = {}
    for pair, key in ((0, "bcnt"), (1, "and_bcnt_pair")):
        ops, khz = dab.dab_probe_popcount(pair, iters, grid, out, clocks)
        us = device_us(torch, lambda pair=pair: dab.dab_probe_popcount(pair, iters, grid, out, clocks), reps=4)
        c = clocks.view(grid, 2).double()
        mhz = float((c[:, 0] / c[:, 1]).median()) * khz / 1e3
        res[key] = {"lane_ops_per_s": ops / (us * 1e-6), "sustained_shader_mhz": round(mhz, 1)}
    rate = res["bcnt"]["lane_ops_per_s"]
    pair_rate = res["and_bcnt_pair"]["lane_ops_per_s"]
    return {"spec": {"P_bcnt": P_BCNT_SPEC, "P_pair": P_PAIR_SPEC, "clock_mhz": 2400},
            "measured": {"P_bcnt": rate * 32, "P_pair": pair_rate * 32,
                         "popcounts_per_lane_per_clock": round(rate / (256 * 64 * res["bcnt"]["sustained_shader_mhz"] * 1e6), 3),
                         "sustained_shader_mhz": res["bcnt"]["sustained_shader_mhz"],
                         "sustained_shader_mhz_pair": res["and_bcnt_pair"]["sustained_shader_mhz"]},
            "what": "P_bcnt = lane-popcounts/s x 32 MACs; P_pair = AND+popcount pairs/s x 32 MACs (spec: half of P_bcnt); "
                    "measured with %d workgroups x 256 lanes x %d x 64 back-to-back instructions" % (grid, iters)}


def other_configs(dab, torch, wl):
    """Per-call device times of the other workload configurations of the benchmark spec (2: one Sketch-A-Net
    conv2 at batch 128; 4: the four ResNet-18-style 3x3 stages at batch 64; 5: the two wide
    fully-connected layers at batch 1024).  Every stage alone on the chip."""
    dev = torch.device("cuda:0")
    cases = [("config2", wl.config2(128))]
    cases += [(f"config4/{wl.CFG4_LAYERS[i].name}", wl.config4(i, 64)) for i in range(4)]
    cases += [(f"config5/{wl.CFG5_LAYERS[i].name}", wl.config5(i, 1024)) for i in range(2)]
    res = {}
    for name, (L, x, w) in cases:
        if L.is_fc:
            X = torch.from_numpy(x).to(dev)
        else:
            X = torch.from_numpy(wl.nchw_to_nhwc(x)).to(dev)
        s = LayerState(L, torch.from_numpy(w).to(dev), X, None, dab, torch)
        jobs = dab.weight_jobs([dict(W=s.W, est=s.est, packed=s.EW)])
        wsb = dab.lib().dab_binarize_weights_multi_workspace_bytes(jobs, 1)
        wws = torch.empty(max(wsb, 1), dtype=torch.uint8, device=dev)
        rows = {"pack_activations": hbm_row(device_us(torch, lambda: activation_side(s, dab)), s.pack_bytes(), 1),
                "estimate + pack_weights (grouped call)": hbm_row(
                    device_us(torch, lambda: dab.dab_binarize_weights_multi(jobs, ws=wws)), s.weight_bytes(), None)}
        us = device_us(torch, lambda: product(s, dab))
        r = hbm_row(us, s.product_bytes(), 1 if s.ws_bytes == 0 else None)
        r.update({"gmacs": round(s.macs / 1e9, 3), "tflops": round(2 * s.macs / (us * 1e-6) / 1e12, 1),
                  "frac_of_mfma_fp4_peak": round(2 * s.macs / (us * 1e-6) / MFMA_FP4_FLOPS, 4),
                  "vs_P_pair_spec": round(s.macs / (us * 1e-6) / P_PAIR_SPEC, 3)})
        rows["binary product"] = r
        rows["sum_us"] = round(sum(v["us"] for v in rows.values() if isinstance(v, dict)), 2)
        res[name] = rows
        del s, X, jobs, wws
        torch.cuda.empty_cache()
    return res


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

    for _ in range(min(args.warmup, 3)):
        step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
        step()
    dt = time_graph(torch, graph, args.steps, args.warmup)
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


def weights_only_products(states, dab, torch):
    """The six layers as weights-only binarized layers (WBin of Section 5.1) on their real-valued inputs,
    each call alone on the chip.  Each input element becomes three bf16 pieces, so a binary MAC costs
    three bf16 MACs (6 FLOP)."""
    out = {}
    total_us, total_macs = 0.0, 0
    for s in states:
        L = s.L
        nbytes = (dab.lib().dab_wbin_fc_workspace_bytes(s.B, L.C, L.F) if L.is_fc
                  else dab.lib().dab_wbin_conv2d_workspace_bytes(ctypes.byref(s.desc)))
        ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=s.X.device)
        Y = torch.empty_like(s.Y)

        def run():
            if L.is_fc:
                dab.dab_wbin_fc(s.X.view(s.B, -1), s.EW[0], s.est["alpha"], s.est["beta"], out=Y, ws=ws)
            else:
                dab.dab_wbin_conv2d(s.desc, s.X, s.EW[0], s.est["alpha"], s.est["beta"], out=Y, ws=ws)

        us = device_us(torch, run, reps=5)
        total_us += us
        total_macs += s.macs
        out[L.name] = {"ms": round(us * 1e-3, 4), "bf16_tflops": round(6 * s.macs / (us * 1e-6) / 1e12, 1),
                       "frac_of_mfma_bf16_peak": round(6 * s.macs / (us * 1e-6) / MFMA_BF16_FLOPS, 4)}
        del ws, Y
    return {"what": "dab_wbin_conv2d / dab_wbin_fc (prepare + product) per layer, fp32 inputs as three bf16 pieces, "
                    "each call alone on the chip",
            "ms_per_step": round(total_us * 1e-3, 4), "macs_per_s": total_macs / (total_us * 1e-6), "per_layer": out}


def cpu_oracle_baseline(batch, wl):
    """The float64 CPU oracle, as it stands, on the same workload: all six layers incl. estimation.
    Timed twice: with the host's default thread count, then (one pass over a smaller batch) on one thread."""
    import numpy as np
    import torch
    from oracle import estimate as oest
    from oracle import layers as olay
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits = None
        threads = os.cpu_count() or 1
    w1, ws = wl.config3_weights()

    def run(n, passes):
        imgs = wl.sketch_images(n)
        x0 = wl.config3_conv1_features(imgs, w1).numpy()
        macs = 0
        t0 = time.perf_counter()
        for _ in range(passes):
            x = x0
            for L, W in zip(wl.CFG3_LAYERS, ws):
                if L.is_fc:
                    x = x.reshape(n, -1)
                x4 = x if x.ndim == 4 else x[:, :, None, None]
                tau = x4.mean(axis=(0, 2, 3)).astype(np.float32)
                r = oest.estimate_alpha_beta(W)
                a = olay.binarize_activations(x4, tau)
                y = olay.conv2d(a, olay.two_valued_filters(r["e"], r["alpha"], r["beta"]), (L.pad, L.pad),
                                (L.stride, L.stride))
                macs += L.macs(n)
                y = torch.from_numpy(y.astype(np.float32)).permute(0, 3, 1, 2)
                if L.pool_after:
                    y = torch.nn.functional.max_pool2d(y, 3, 2)
                x = y.numpy()
        return macs, time.perf_counter() - t0

    passes = 2
    macs, dt = run(batch, passes)
    res = {"value": macs / dt, "unit": "binary MAC/s", "cores": int(threads), "kind": "oracle",
           "sample": f"config 3, all six layers incl. alpha/beta estimation, batch {batch} of 256, {passes} passes, {dt:.1f} s"}
    if threadpool_limits is not None:
        n1 = max(1, batch // 16)
        old = torch.get_num_threads()
        torch.set_num_threads(1)
        try:
            with threadpool_limits(limits=1):
                macs1, dt1 = run(n1, 1)
        finally:
            torch.set_num_threads(old)
        res["single_thread"] = {"value": macs1 / dt1, "cores": 1,
                                "sample": f"same path, batch {n1}, one pass, {dt1:.1f} s"}
    return res


def load_traffic(layer, batch):
    """HBM bytes per launch of the dominant kernel from the tracked counter summary, or None."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None, None
    if t.get("layer") != layer or t.get("batch") != batch:
        return None, None
    return t.get("traffic_bytes"), {k: t.get(k) for k in ("commit", "kernel", "fetch_bytes", "write_bytes", "source")}


# ------------------------------------------------------------------------------------------------
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
    dab.dab_init()

    states = build_states(args.batch, dab, torch, wl)
    total_macs = sum(s.macs for s in states)
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    grouped = GroupedStep(states, dab, torch, separate=args.separate)
    for _ in range(min(args.warmup, 3)):
        grouped.step()
    torch.cuda.synchronize()

    # The step launched eagerly (host-bound: the host needs longer to enqueue a step than the chip to run it)
    t0 = time.perf_counter()
    for k in range(args.steps):
        grouped.step()
    torch.cuda.synchronize()
    dt_eager = time.perf_counter() - t0

    # Timed region: exactly `steps` steps, each one launch of the captured HIP graph
    if args.no_graph:
        dt = dt_eager
    else:
        graph = grouped.capture()
        dt = time_graph(torch, graph, args.steps, args.warmup)

    ms_per_step = 1e3 * dt / args.steps
    value = total_macs * args.steps / dt

    # Roofline of the dominant kernel: the binary product of the layer with the longest launch.  With
    # fp32 outputs every large layer sits below the ridge of the fp4 matrix cores (conv2: 784 FLOP per
    # algorithmic byte against 10.1e15 / 8e12 = 1262), so the bound that applies is HBM; the MFMA view is
    # printed beside it.  Algorithmic bytes of a launch = fp32 outputs + activation bits + weight bits +
    # alpha and beta.
    per_layer = product_rows(states, dab, torch)
    conv_us = sum(r["us"] for r in per_layer.values())
    algo_bytes = sum(r["algorithmic_bytes"] for r in per_layer.values())
    dom = max(per_layer, key=lambda k: per_layer[k]["us"])
    d = per_layer[dom]
    traffic, traffic_src = load_traffic(dom, args.batch)
    roofline = {"bound": "hbm",
                "kernel": "binconv_direct_kernel (the one launch of dab_binconv2d) of %s; average over graphs of 10 "
                          "back-to-back launches on one stream, each replay bracketed by HIP events on that stream" % dom,
                "achieved": d["gb_per_s"], "peak": HBM_BYTES_PER_S / 1e9, "unit": "GB/s",
                "frac": d["frac_of_hbm_peak"], "traffic": traffic, "traffic_source": traffic_src,
                "algorithmic_bytes": d["algorithmic_bytes"], "launch_ms": d["ms"],
                "mfma_view": {"achieved": d["tflops"], "peak": MFMA_FP4_FLOPS / 1e12, "unit": "TFLOP/s",
                              "frac": d["frac_of_mfma_fp4_peak"]},
                "all_layers": {"kernel_ms_per_step": round(conv_us * 1e-3, 4), "algorithmic_bytes": algo_bytes,
                               "gb_per_s": round(algo_bytes / (conv_us * 1e-6) / 1e9, 1),
                               "frac_of_hbm_peak": round(algo_bytes / (conv_us * 1e-6) / HBM_BYTES_PER_S, 4),
                               "tflops": round(2 * total_macs / (conv_us * 1e-6) / 1e12, 1),
                               "frac_of_mfma_fp4_peak": round(2 * total_macs / (conv_us * 1e-6) / MFMA_FP4_FLOPS, 4),
                               "binary_macs_per_s": total_macs / (conv_us * 1e-6)},
                "per_layer": per_layer}

    extras = {}
    if not args.headline_only:
        pc = popcount_ceiling(dab, torch)
        rate = total_macs / (conv_us * 1e-6)
        pc["products_alone"] = {"vs_P_pair_spec": round(rate / P_PAIR_SPEC, 3), "vs_P_bcnt_spec": round(rate / P_BCNT_SPEC, 3),
                                "vs_P_pair_measured": round(rate / pc["measured"]["P_pair"], 3),
                                "vs_P_bcnt_measured": round(rate / pc["measured"]["P_bcnt"], 3)}
        pc["whole_step"] = {"vs_P_pair_spec": round(value / P_PAIR_SPEC, 3), "vs_P_bcnt_spec": round(value / P_BCNT_SPEC, 3),
                            "vs_P_pair_measured": round(value / pc["measured"]["P_pair"], 3),
                            "vs_P_bcnt_measured": round(value / pc["measured"]["P_bcnt"], 3)}
        extras["valu_popcount_ceiling"] = pc
        extras["stages"] = stage_table(states, grouped, dab, torch)

        # the next row of the scope table: the chain that hands bits from layer to layer
        chain = FusedChain(states, grouped, dab, torch)
        chain.step(dab)
        torch.cuda.synchronize()
        fdt = time_graph(torch, chain.capture(dab), args.steps, args.warmup)
        ins = chain.inputs(dab)
        extras["rebinarized_chain"] = {
            "what": "same layers, bits handed from layer to layer by dab_binconv2d_bits / dab_pool_bits "
                    "(fp32 only into conv2 and out of fc7); one HIP graph per step",
            "ms_per_step": round(1e3 * fdt / args.steps, 4), "binary_macs_per_s": total_macs * args.steps / fdt,
            "product_us_per_layer": {s.L.name: round(device_us(torch, lambda i=i: chain.product(i, ins[i], dab)), 2)
                                     for i, s in enumerate(states)}}
        for s in states:                                          # the chain's fc7 wrote Y from the chain's bits
            product(s, dab)
        extras["training_weight_side"] = training_weight_side(states, dab, torch, args)
        extras["weights_only_layers"] = weights_only_products(states, dab, torch)
        extras["other_configs"] = other_configs(dab, torch, wl)
        if args.batch != 32:
            small = build_states(32, dab, torch, wl)
            g32 = GroupedStep(small, dab, torch)
            g32.step()
            torch.cuda.synchronize()
            dt32 = time_graph(torch, g32.capture(), args.steps, args.warmup)
            extras["batch_32"] = {"ms_per_step": round(1e3 * dt32 / args.steps, 4),
                                  "binary_macs_per_s": sum(s.macs for s in small) * args.steps / dt32}

    cpu = cpu_oracle_baseline(args.cpu_batch, wl) if args.cpu_batch > 0 else None
    line = {
        "metric": "effective binary MACs/s on Sketch-A-Net binarized layers",
        "value": value, "unit": "binary MAC/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp4 (e2m1) operands expanded from 1-bit, fp32 MFMA accumulate (exact integers), fp32 epilogue, fp64 estimation", "data": "synthetic",
        "config": {"workload": "config 3: Sketch-A-Net binarized trunk (conv2-conv6, fc7), batch %d, "
                               "estimate + pack weights + pack activations + binary product per layer" % args.batch,
                   "batch": args.batch, "binary_macs_per_step": total_macs,
                   "streams": 1,
                   "launch": "eager" if args.no_graph else "one captured HIP graph per step",
                   "calls_per_step": (2 if args.separate else 1) + len(states),
                   "eager_ms_per_step": round(1e3 * dt_eager / args.steps, 4)},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    line.update(extras)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
