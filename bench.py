#!/usr/bin/env python3
"""Benchmark of the W4A8 linear-layer hot path on one MI355X.

A step is one pass of the hot path over the decode sweep of Llama-3-8B layer shapes (M in {1, 4, 16} x the four
(K, N) pairs): for each of the 12 cases, FP8 activation quantization (Eq. 13) followed by the fused
INT4 -> E4M3 -> FP8-MFMA linear layer (Eq. 10, 4, 11) with bf16 output.  Weights are packed once before timing
(offline with respect to inference).  Inputs are resident in HBM when timing starts.  Several distinct weight sets
rotate between cases and steps so that weights come from HBM, not from the 256 MB last-level cache.  Steps are
replayed as HIP graphs so that the host's launch cost does not bound microsecond-scale kernels.

`value` = algorithmic bytes of the 12 linear layers / step time, where per layer
bytes = N*K/2 (codes) + 4*N*K/G (scales) + M*K (FP8 activations) + 2*M*N (bf16 output).
Every timed leg is repeated REPEATS times; the median is reported, with the minimum and the maximum next to it.

Also reported: `roofline` for the dominant kernel (the skinny linear kernel, timed alone with HIP events on the
launch stream), `prefill` (TFLOP/s of the MFMA-tiled kernel over the prefill sweep, with its own roofline), and
`cpu_baseline` (the CPU oracle timed on a bounded sample of the same workload); `block` (decoder-block latency),
`weight_modes` (the other weight formats on one layer) and `calibration` (the offline DPQ + GAR step) are short extra legs.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np
import torch

from paper_2505_14638_amd import binding as B
from paper_2505_14638_amd import synthetic as syn

REPEATS = 5                    # timed repetitions per leg: the median is the figure, min and max its spread
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
FP8_PEAK_TFLOPS = 5000.0       # MI355X dense FP8 MFMA
G = 128
# HBM traffic per launch of the dominant kernel on the default workload, from two hardware-counter runs of this file
# (profiles/linear_skinny_decode_sweep_hbm_traffic.txt): FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the factors that make the
# same counters read 1 GiB + 1 GiB for a plain 1 GiB device-to-device copy.  Counters cannot be read from inside a
# timed run, so the figure is carried here and reported only for the workload it was measured on.
SKINNY_TRAFFIC_BYTES_PER_LAUNCH = {4: 29.589e6}          # by --copies
# same for the prefill sweep (profiles/linear_mfma_prefill_sweep_hbm_traffic.txt): mean over its 12 shapes, one launch each
PREFILL_TRAFFIC_BYTES_PER_LAUNCH = 299.9e6


def alg_bytes(m, k, n, out_bytes=2):
    return n * k // 2 + 4 * n * k // G + m * k + out_bytes * m * n


class Layer:
    """One (K, N) layer shape with `copies` independently drawn, packed weight sets."""

    def __init__(self, cfg_id, idx, k, n, copies, dev):
        self.k, self.n = k, n
        self.sets = []
        for c in range(copies):
            w = syn.make_weights(syn.rng_for(cfg_id, idx, k, n, c), n, k)
            self.sets.append(B.pack_weights(torch.from_numpy(w).to(dev), G, B.LAYOUT_TILED))
            del w
        torch.cuda.synchronize()


class Case:
    def __init__(self, cfg_id, layer, m, dev, frac, mult):
        self.layer, self.m = layer, m
        x = syn.make_activations(syn.rng_for(cfg_id, m, layer.k, layer.n, 99), m, layer.k, frac, mult)
        self.s_x = torch.tensor([syn.static_act_scale(x)], dtype=torch.float32, device=dev)
        self.x = torch.from_numpy(x).to(dev)
        self.x8 = torch.empty((m, layer.k), dtype=torch.uint8, device=dev)
        self.y = torch.empty((m, layer.n), dtype=torch.bfloat16, device=dev)
        need = B.linear_workspace_bytes(m, layer.k, layer.n, G)          # scratch for K ranges across workgroups, where asked for
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev) if need else None

    def quantize(self):
        B.quantize_act(self.x, self.s_x, out=self.x8)

    def linear(self, s):
        packed, scales = self.layer.sets[s % len(self.layer.sets)]
        B.linear(self.x8, self.s_x, packed, scales, self.layer.n, G, B.LAYOUT_TILED, out=self.y, workspace=self.ws)

    def fusable(self):
        """Where folding the activation quantization into the layer (w4a8_linear_quantize_in) pays.  Every workgroup
        quantizes all of X, so the work grows with tokens x workgroups per compute unit: measured faster at one token on
        every layer, and up to four tokens on the layers that run one workgroup per compute unit (QKV 8.4 -> 7.9 us, O
        projection 7.4 -> 6.6); slower on gate|up from two tokens on and on the down projection from four."""
        return self.m == 1 or (self.m <= 4 and self.layer.k <= 4096 and self.layer.n <= 6144)

    def quantize_and_linear(self, s):
        """One pass of the path for this case: the fused launch where the library has one, else the two kernels."""
        if self.fusable():
            packed, scales = self.layer.sets[s % len(self.layer.sets)]
            B.linear_quantize_in(self.x, self.s_x, packed, scales, self.layer.n, G, out=self.y)
        else:
            self.quantize()
            self.linear(s)


def capture(fn):
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g


class Eager:
    """Stand-in for a captured graph that launches its kernels one by one."""

    def __init__(self, fn):
        self.replay = fn


class Steps:
    """The steps fn(0) .. fn(copies - 1) (one per weight set) as `copies` single-step graphs plus ONE graph that holds them
    all in a row: a graph replay's own start-up (3-5 us here) is then paid once per `copies` steps.  run(n) replays
    exactly n steps."""

    def __init__(self, fn, copies, eager=False):
        self.copies = copies
        if eager:
            self.singles = [Eager(lambda i=i: fn(i)) for i in range(copies)]
            self.all = Eager(lambda: [fn(i) for i in range(copies)])
        else:
            self.singles = [capture(lambda i=i: fn(i)) for i in range(copies)]
            self.all = capture(lambda: [fn(i) for i in range(copies)])

    def run(self, n):
        for _ in range(n // self.copies):
            self.all.replay()
        for i in range(n % self.copies):
            self.singles[i].replay()


def time_graphs_once(graphs, reps, warmup):
    """Replay graphs round-robin `reps` times after `warmup` (a Steps object: exactly that many steps); returns seconds
    for the timed replays."""
    if isinstance(graphs, Steps):
        replay = graphs.run
    else:
        def replay(n):
            for i in range(n):
                graphs[i % len(graphs)].replay()
    replay(warmup)
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    replay(reps)
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) * 1e-3


def spread(vals):
    """(median, min, max) of the repetitions of one leg."""
    v = sorted(vals)
    return v[len(v) // 2], v[0], v[-1]


def time_graphs(graphs, reps, warmup, repeats=REPEATS):
    """REPEATS timed regions of `reps` replays each (warm-up before the first); seconds of the median region."""
    vals = [time_graphs_once(graphs, reps, warmup if r == 0 else 0) for r in range(repeats)]
    return spread(vals)[0]


def time_graphs_spread(graphs, reps, warmup, repeats=REPEATS):
    return spread([time_graphs_once(graphs, reps, warmup if r == 0 else 0) for r in range(repeats)])


def time_launches(run, reps, repeats=REPEATS):
    """Eager launches: `reps` untimed ones first, then REPEATS timed regions of `reps`; (median, min, max) seconds per launch."""
    for i in range(max(2, reps)):
        run(i)
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    vals = []
    for _ in range(repeats):
        t0.record()
        for i in range(reps):
            run(i)
        t1.record()
        torch.cuda.synchronize()
        vals.append(t0.elapsed_time(t1) * 1e-3 / reps)
    return spread(vals)


def cpu_baseline(min_seconds=10.0):
    """The oracle as it stands, timed on this host: quantize + linear for the decode sweep's layer shapes (the four
    (K, N) pairs at M = 1, 4, 16, in sweep order), repeated until at least `min_seconds` of oracle time."""
    from oracle import w4a8_oracle as o
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    cases = []
    for idx, (k, n) in enumerate(syn.LLAMA3_8B.values()):
        rng = syn.rng_for(2, idx, 1234)
        q = rng.integers(-7, 8, size=(n, k)).astype(np.int8)           # codes with the range of RTN output
        s_w = rng.uniform(0.005, 0.02, size=(n, k // G)).astype(np.float32)
        for m in (1, 4, 16):
            x = syn.make_activations(rng, m, k, 0.01, 20.0)
            cases.append((m, k, n, q, s_w, x, syn.static_act_scale(x)))
    total_bytes, total_t, done = 0, 0.0, 0
    while total_t < min_seconds:
        m, k, n, q, s_w, x, s_x = cases[done % len(cases)]
        t = time.perf_counter()
        x8 = o.quantize_act(x, s_x)
        o.linear_ref(x8, s_x, q, s_w, G)
        total_t += time.perf_counter() - t
        total_bytes += alg_bytes(m, k, n)
        done += 1
    return {"value": round(total_bytes / total_t / 1e9, 4), "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "sample": f"oracle quantize_act + linear_ref (fp64, numpy) over {done} layer passes of the decode sweep "
                      f"(12 cases in order, wrapping around), {total_t:.1f} s of oracle time; same algorithmic-byte count "
                      "as the GPU metric", "seconds": round(total_t, 2)}


def measured_ceilings(dev):
    """Achievable HBM read bandwidth and FP8 MFMA rate of this device, from the library's probe kernels."""
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    B.probe_stream_read(buf, sink)
    torch.cuda.synchronize()
    t0.record()
    for _ in range(5):
        B.probe_stream_read(buf, sink)
    t1.record()
    torch.cuda.synchronize()
    gbs = 5 * buf.numel() / (t0.elapsed_time(t1) * 1e-3) / 1e9
    # a plain device-to-device copy of known size (1 GiB read + 1 GiB written): the reference the FETCH_SIZE and
    # WRITE_SIZE counters of a profiling run are scaled by
    dst = torch.empty_like(buf)
    dst.copy_(buf)
    torch.cuda.synchronize()
    t0.record()
    for _ in range(3):
        dst.copy_(buf)
    t1.record()
    torch.cuda.synchronize()
    copy_gbs = 3 * 2 * buf.numel() / (t0.elapsed_time(t1) * 1e-3) / 1e9
    del buf, dst
    flop = B.probe_mfma(2000, sink)
    torch.cuda.synchronize()
    t0.record()
    for _ in range(3):
        B.probe_mfma(2000, sink)
    t1.record()
    torch.cuda.synchronize()
    tfl = 3 * flop / (t0.elapsed_time(t1) * 1e-3) / 1e12
    return round(gbs, 1), round(copy_gbs, 1), round(tfl, 1)


def library_fp8_gemm_seconds(x8, n, reps):  # noqa: C901
    """Seconds per call of the vendor library's FP8 GEMM (through torch._scaled_mm) for activations x8 [M, K] (E4M3 bytes)
    against random FP8 weights [N, K], bf16 output; None where this torch build has no such GEMM.  A measured reference
    for what a dense FP8 contraction reaches on this machine -- it is not part of the W4A8 path."""
    try:
        a = x8.view(torch.float8_e4m3fn)
        w = torch.randint(0, 120, (n, x8.shape[1]), dtype=torch.uint8, device=x8.device).view(torch.float8_e4m3fn)
        one = torch.ones((), dtype=torch.float32, device=x8.device)
        run = lambda: torch._scaled_mm(a, w.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16)
        for _ in range(max(2, reps)):
            run()
        torch.cuda.synchronize()
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record()
        for _ in range(reps):
            run()
        t1.record()
        torch.cuda.synchronize()
        return t0.elapsed_time(t1) * 1e-3 / reps
    except Exception:                                                    # noqa: BLE001 - any refusal means "not available"
        return None


def plain_read_same_sizes(dev, sizes, copies, steps, warmup):
    """What a kernel that only reads reaches on buffers of the decode sweep's sizes: the library's streaming-read probe
    launched once per case on `sizes[j]` bytes, the same number of launches per HIP graph as the linear kernels, over
    sixteen 64 MiB slots of a 1 GiB pool visited in turn.  Returns microseconds per launch."""
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    pool = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
    slot = 64 << 20

    def reads(i):
        for j, nb in enumerate(sizes):
            at = ((i * len(sizes) + j) % 16) * slot
            B.probe_stream_read(pool[at:at + min(slot, int(nb) // 256 * 256)], sink)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        reads(0)
        torch.cuda.synchronize()
        graphs = Steps(reads, copies)
        sec = time_graphs(graphs, steps, warmup)
    torch.cuda.current_stream().wait_stream(side)
    del graphs, pool
    return sec / steps / len(sizes) * 1e6


class WeightViews:
    """One packed [n_total, K] weight matrix that layers of N rows are sliced from: in the tiled format the bands of 16
    rows are contiguous, so rows [i N, (i + 1) N) of the big matrix are the packed codes and scales of a layer of their
    own.  Enough slices to keep the weights of consecutive launches out of the 256 MB last-level cache."""

    def __init__(self, k, n_total, dev, seed):
        self.k, self.n_total = k, n_total
        gen = torch.Generator(device=dev).manual_seed(seed)
        packed, scales = [], []
        step = 16384
        for r0 in range(0, n_total, step):                               # packed in pieces: the float32 source of one piece at a time
            w = torch.randn((min(step, n_total - r0), k), generator=gen, device=dev) * 0.02
            p_, s_ = B.pack_weights(w, G, B.LAYOUT_TILED)
            packed.append(p_)
            scales.append(s_)
            del w
        self.packed, self.scales = torch.cat(packed), torch.cat(scales)
        torch.cuda.synchronize()

    def count(self, n):
        return self.n_total // n

    def view(self, i, n):
        pb, sc = n * self.k // 2, n * self.k // G
        return self.packed[i * pb:(i + 1) * pb], self.scales[i * sc:(i + 1) * sc]


def decode_cases(dev):
    """Per-case rows of the decode shapes (configs[1]: Llama-3-8B, configs[3]: Llama-3-70B at M = 1 and 16): the linear
    kernel alone on weights that come from HBM (a HIP graph of one launch per weight slice, >= 500 MB of distinct
    weights per case), the launch shape the library chooses, and the best of the built launch shapes timed the same way."""
    pools = [(4096, 286720, [6144, 4096, 28672], (1, 4, 16), "8B"), (14336, 81920, [4096], (1, 4, 16), "8B"),
             (8192, 172032, [10240, 8192, 57344], (1, 16), "70B"), (28672, 40960, [8192], (1, 16), "70B")]
    rows = []
    sx = torch.tensor([0.05], dtype=torch.float32, device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for (k, n_total, ns, ms, model) in pools:
        pool = WeightViews(k, n_total, dev, seed=k)
        for n in ns:
            views = [pool.view(i, n) for i in range(pool.count(n))]
            layer_bytes = n * k // 2 + 4 * n * k // G
            for m in ms:
                x8 = torch.randint(0, 120, (m, k), dtype=torch.uint8, device=dev)
                y = torch.empty((m, n), dtype=torch.bfloat16, device=dev)
                reps = max(2, int(2e-3 / (len(views) * layer_bytes / 4e12)))      # about 2 ms per timed region

                def timed(launch):
                    with torch.cuda.stream(side):
                        launch(*views[0])
                        torch.cuda.synchronize()
                        g = capture(lambda: [launch(p_, s_) for (p_, s_) in views])
                        med, lo, hi = time_graphs_spread([g], reps, reps)            # one untimed region first: clocks ramp up under load
                    del g
                    return [t / (reps * len(views)) for t in (med, lo, hi)]

                shape = B.linear_launch_shape(m, k, n, G)
                best, best_shape, best_args = None, None, None
                for nt in (1, 2, 4):
                    for waves in (2, 4, 8, 16):
                        for depth in (0, 4):
                            p1 = waves | (depth << 8)
                            if depth == 4 and nt > 1:
                                continue                                     # the deeper ring is built for one band and one token block
                            try:
                                t = timed(lambda p_, s_: B.linear_variant(x8, sx, p_, s_, n, G, y, 0, nt, p1))[0]
                            except B.W4A8Error:
                                continue                                     # a combination that is not built
                            if best is None or t < best:
                                best, best_shape, best_args = t, [0, nt, waves | ((depth or 2) << 8)], (nt, p1)
                # the winner of the sweep once more (the smallest of two dozen noisy figures flatters it), then the library's
                # own choice, like the variants after untimed launches of the same kind
                best = timed(lambda p_, s_: B.linear_variant(x8, sx, p_, s_, n, G, y, 0, *best_args))[0]
                med, lo, hi = timed(lambda p_, s_: B.linear(x8, sx, p_, s_, n, G, B.LAYOUT_TILED, out=y))
                if med < best:
                    best, best_shape = med, list(shape[:3])
                nbytes = alg_bytes(m, k, n)
                rows.append({"model": model, "M": m, "K": k, "N": n, "us": round(med * 1e6, 2), "us_min": round(lo * 1e6, 2),
                             "us_max": round(hi * 1e6, 2), "GBps": round(nbytes / med / 1e9, 1),
                             "frac_of_peak": round(nbytes / med / 1e9 / HBM_PEAK_GBS, 4), "launch_shape": list(shape[:3]),
                             "best_variant": best_shape, "best_variant_us": round(best * 1e6, 2),
                             "default_over_best": round(med / best, 3), "weight_slices": len(views)})
                del x8, y
        del pool, views
        torch.cuda.empty_cache()
    torch.cuda.current_stream().wait_stream(side)
    worst = max(r["default_over_best"] for r in rows)
    tot_b = sum(alg_bytes(r["M"], r["K"], r["N"]) for r in rows)
    tot_t = sum(r["us"] for r in rows) * 1e-6
    return {"metric": "the few-token linear kernel per decode case, weights from HBM (one launch per weight slice in a HIP "
                      "graph, >= 500 MB of distinct weights per case); launch_shape / best_variant = (path, param0, param1) "
                      "of w4a8_linear_variant, param1 = wavefronts + 256 * chunks in flight",
            "rows": rows, "worst_default_over_best": worst, "byte_weighted_GBps": round(tot_b / tot_t / 1e9, 1),
            "byte_weighted_frac_of_peak": round(tot_b / tot_t / 1e9 / HBM_PEAK_GBS, 4), "repeats": REPEATS}


def block_latency(dev, steps, warmup, sets=4, stack=12):
    """Config 5: latency of the decoder-block linear stack per batch size, HIP graph replay over `sets` rotating weight
    sets (4 x 116 MB: beyond the 256 MB last-level cache, so the weights come from HBM); the figure with one weight set
    (partly served by that cache) is kept next to it, labelled.  `stack` consecutive blocks in ONE graph (as the blocks
    of a model are replayed) give the per-block figure without a graph replay's own start-up."""
    from paper_2505_14638_amd.block import LAYERS, DecoderBlockLinears
    cfg = syn.CONFIGS[5]
    blocks, fused_blocks = [], []
    for c in range(sets):
        blk = DecoderBlockLinears(cfg["hidden"], cfg["ffn"], syn.LLAMA3_8B["qkv"][1], cfg["group"], dev)
        for idx, name in enumerate(LAYERS):
            k, n = blk.dims[name]
            blk.load_layer(name, torch.from_numpy(syn.make_weights(syn.rng_for(5, idx, c), n, k)))
        for name, s in zip(LAYERS, (0.19, 0.012, 0.004, 0.0006)):      # typical static scales of this block
            blk.set_act_scale(name, s)
        fused = DecoderBlockLinears(cfg["hidden"], cfg["ffn"], syn.LLAMA3_8B["qkv"][1], cfg["group"], dev, fused=True)
        fused.weights, fused.scales_x = blk.weights, blk.scales_x
        blocks.append(blk)
        fused_blocks.append(fused)
    out = {"by_batch": {}, "fused_by_batch": {}, "fused_spread": {}, "fused_in_a_stack_by_batch": {},
           "one_weight_set_by_batch": {}, "one_weight_set_fused_by_batch": {}}
    for m in cfg["batches"]:
        x = syn.make_activations(syn.rng_for(5, 200 + m), m, cfg["hidden"], cfg["frac"], cfg["mult"])
        x_d = torch.from_numpy(x).to(dev).to(torch.bfloat16)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for group, key, key1 in ((blocks, "by_batch", "one_weight_set_by_batch"),
                                     (fused_blocks, "fused_by_batch", "one_weight_set_fused_by_batch")):
                graphs = []
                for blk in group:
                    blk.forward(x_d)
                    torch.cuda.synchronize()
                    graphs.append(capture(lambda blk=blk: blk.forward(x_d)))
                med, lo, hi = time_graphs_spread(graphs, steps, warmup)
                out[key][str(m)] = round(med / steps * 1e6, 2)
                if key == "fused_by_batch":
                    out["fused_spread"][str(m)] = [round(lo / steps * 1e6, 2), round(hi / steps * 1e6, 2)]
                out[key1][str(m)] = round(time_graphs(graphs[:1], steps, warmup) / steps * 1e6, 2)
                del graphs
            g = capture(lambda: [fused_blocks[i % sets].forward(x_d) for i in range(stack)])
            reps = max(3, steps // stack)
            out["fused_in_a_stack_by_batch"][str(m)] = round(time_graphs_spread([g], reps, 2)[0] / (reps * stack) * 1e6, 2)
            del g
        torch.cuda.current_stream().wait_stream(side)
    return {"metric": "decoder-block linear stack latency (config 5: QKV, O, gate|up, SiLU*mul, down; hidden 4096, "
                      "FFN 14336)", "unit": "us per block", "weight_sets": sets, "repeats": REPEATS, **out,
            "fused": "same outputs with each intermediate's FP8 quantization folded into the kernel that produces it "
                     "and, up to 8 tokens, the quantization of the block input into the QKV layer (4 or 5 launches instead of 9)",
            "note": "by_batch / fused_by_batch: one block per graph replay, rotating over the weight sets (weights from "
                    "HBM); fused_in_a_stack_by_batch: %d consecutive fused blocks in one graph over the same rotating weight "
                    "sets, per block (no graph start-up per block); one_weight_set_*: one set replayed, part of whose "
                    "116 MB is then served by the 256 MB last-level cache" % stack}


def weight_modes(dev):
    """The other weight formats of the library on two shapes (gate|up at M = 1 and M = 8192), every buffer made by the
    library's packers from seeded float32 weights, so the timed launches compute the layer: eager launches over six
    rotating weight sets (decode: 6 x 62 MB) or one (prefill); median of REPEATS."""
    k, n = syn.LLAMA3_8B["gate_up"]
    out = {}
    gen = torch.Generator(device=dev).manual_seed(20250514)
    for m in (1, 8192):
        sets = 6 if m == 1 else 1
        x8 = torch.randint(0, 120, (m, k), dtype=torch.uint8, device=dev)
        sx = torch.tensor([0.1], dtype=torch.float32, device=dev)
        y = torch.empty((m, n), dtype=torch.bfloat16, device=dev)
        sym, p2, asym, two = [], [], [], []
        for _ in range(sets):
            w = torch.randn((n, k), generator=gen, device=dev) * 0.02
            sym.append(B.pack_weights(w, G, B.LAYOUT_TILED))                  # signed codes, float32 group scales (Eq. 1 symmetric)
            p2.append(B.pack_weights(w, G, B.LAYOUT_TILED, pow2=True))        # the same with power-of-two scales (Sec. 2.2)
            asym.append(B.pack_weights_asym(w, G))                            # unsigned codes, zero-points (Eq. 8-9)
            packed, scales = sym[-1]
            two.append((packed, scales.abs() * 400.0))                        # FP8-domain group scales (Eq. 8): products up to ~56
            del w
        w_out = torch.rand(n, generator=gen, dtype=torch.float32, device=dev) * 1e-3
        calls = {
            "code_exact": lambda i: B.linear(x8, sx, *sym[i % sets], n, G, B.LAYOUT_TILED, out=y),
            "two_level": lambda i: B.linear_two_level(x8, sx, *two[i % sets], w_out, n, G, out=y),
            "asym": lambda i: B.linear_asym(x8, sx, *asym[i % sets], n, G, out=y),
            "pow2": lambda i: B.linear_pow2(x8, sx, *p2[i % sets], n, G, out=y),
        }
        reps = 60 if m == 1 else 10
        row = {}
        for name, fn in calls.items():
            sec = time_launches(fn, reps)[0]
            extra = n * k // G if name == "asym" else 0                   # zero-point bytes
            row[name] = round((alg_bytes(m, k, n) + extra) / sec / 1e9, 1) if m == 1 else round(2.0 * m * k * n / sec / 1e12, 1)
        out[f"M={m}"] = {"unit": "GB/s" if m == 1 else "TFLOP/s", **row}
        del sym, p2, asym, two
        torch.cuda.empty_cache()
    return {"metric": "weight formats on the gate|up layer (K = 4096, N = 28672), weights packed by the library", "repeats": REPEATS,
            "by_case": out}


def llama70b(dev, steps, warmup):
    """Config 4 (Llama-3-70B shapes): the decode cases (M = 1 and 16) as one HIP graph per weight set, two rotating sets
    (428 MB each) packed by the library from seeded float32 weights; the prefill cases (M = 4096) as eager launches.
    Per-case rows of the decode cases, with weights from HBM for every single case, are in `decode_cases`."""
    shapes = list(syn.LLAMA3_70B.values())
    gen = torch.Generator(device=dev).manual_seed(70)
    sets = []
    for _ in range(2):
        one = []
        for (k, n) in shapes:
            parts = [B.pack_weights(torch.randn((min(16384, n - r0), k), generator=gen, device=dev) * 0.02, G, B.LAYOUT_TILED)
                     for r0 in range(0, n, 16384)]                          # in pieces: 16-row bands are contiguous in the tiled format
            one.append((torch.cat([p_ for (p_, _) in parts]), torch.cat([s_ for (_, s_) in parts])))
            del parts
        sets.append(one)
    sx = torch.tensor([0.05], dtype=torch.float32, device=dev)
    cases = []
    for j, (k, n) in enumerate(shapes):
        for m in (1, 16):
            cases.append((j, m, k, n, torch.randint(0, 120, (m, k), dtype=torch.uint8, device=dev),
                          torch.empty((m, n), dtype=torch.bfloat16, device=dev)))
    total = sum(alg_bytes(m, k, n) for (_, m, k, n, _, _) in cases)

    def run(i):
        for (j, m, k, n, x8, y) in cases:
            B.linear(x8, sx, sets[i % 2][j][0], sets[i % 2][j][1], n, G, B.LAYOUT_TILED, out=y)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(0)
        torch.cuda.synchronize()
        graphs = [capture(lambda i=i: run(i)) for i in range(2)]
        med, lo, hi = [t / steps for t in time_graphs_spread(graphs, steps, warmup)]
    torch.cuda.current_stream().wait_stream(side)
    gbs = total / med / 1e9
    # the prefill cases of the same config (M = 4096), eager launches after untimed ones
    flop, psec, per_shape = 0.0, 0.0, []
    x8 = torch.randint(0, 120, (4096, max(k for (k, _) in shapes)), dtype=torch.uint8, device=dev)
    for j, (k, n) in enumerate(shapes):
        y = torch.empty((4096, n), dtype=torch.bfloat16, device=dev)
        xs = x8[:, :k]
        sec = time_launches(lambda i: B.linear(xs, sx, sets[i % 2][j][0], sets[i % 2][j][1], n, G, B.LAYOUT_TILED, out=y), 3)[0]
        psec += sec
        flop += 2.0 * 4096 * k * n
        per_shape.append({"M": 4096, "K": k, "N": n, "us": round(sec * 1e6, 1), "tflops": round(2.0 * 4096 * k * n / sec / 1e12, 1)})
        del y
    tfl = flop / psec / 1e12
    return {"metric": "W4A8 linear on configs[3] (Llama-3-70B shapes): effective HBM GB/s of the decode cases (M in {1, 16}) "
                      "and TFLOP/s of the prefill cases (M = 4096)",
            "value": round(gbs, 1), "unit": "GB/s", "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4), "repeats": REPEATS,
            "GBps_min_max": [round(total / hi / 1e9, 1), round(total / lo / 1e9, 1)],
            "us_per_launch": round(med / len(cases) * 1e6, 2), "alg_bytes_per_launch": total // len(cases),
            "prefill_tflops": round(tfl, 1), "prefill_frac_of_peak": round(tfl / FP8_PEAK_TFLOPS, 4), "prefill_shapes": per_shape}


def calibration(dev):
    """Offline calibration on one Llama-3-8B-shaped layer (the O projection, 4096 x 4096): Group-Aware Reordering and
    DPQ (Alg. 1) timed on the GPU, and the layer error of the calibrated weights against the same double quantization
    without error compensation, both run through packing and the literal inference layer on 512 calibration tokens.
    The Hessian comes from w4a8_hessian_accumulate, the factor U of Eq. 12 from w4a8_hessian_inverse_factor."""
    n = k = 4096
    t = 8192
    rng = syn.rng_for(9, n, k)
    w = torch.from_numpy(syn.make_weights(rng, n, k)).to(dev)
    x = torch.from_numpy(syn.make_activations(rng, t, k, 0.01, 20.0)).to(dev)
    x = x * torch.exp(torch.from_numpy(rng.uniform(-1.0, 1.0, size=k).astype(np.float32)).to(dev))[None, :]
    s_x = (x.abs().max() / 448.0).reshape(1).to(torch.float32)
    x8 = B.quantize_act(x, s_x)
    s_w = (w.abs().amax(dim=1) / 448.0).to(torch.float32)
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    B.hessian_accumulate(x[:64])                                         # untimed first launch
    torch.cuda.synchronize()
    t0.record()
    h32 = B.hessian_accumulate(x)
    t1.record()
    torch.cuda.synchronize()
    hessian_ms = t0.elapsed_time(t1)
    h_diag = torch.diagonal(h32).contiguous()
    perm = B.gar_permutation(h_diag, G)
    B.hessian_inverse_factor(h32, 0.01, perm)                            # untimed first run
    torch.cuda.synchronize()
    t0.record()
    u, info = B.hessian_inverse_factor(h32, 0.01, perm)
    t1.record()
    torch.cuda.synchronize()
    factor_ms = t0.elapsed_time(t1)
    if int(info.item()) != 0:
        raise RuntimeError(f"calibration: the dampened Hessian is not positive definite (info = {int(info.item())})")
    B.dpq_calibrate(w, u, s_w, G, perm)                                  # untimed first run
    torch.cuda.synchronize()
    t0.record()
    perm = B.gar_permutation(h_diag, G)
    cal = B.dpq_calibrate(w, u, s_w, G, perm)
    t1.record()
    torch.cuda.synchronize()
    ms = t0.elapsed_time(t1)
    t0.record()
    cal_mse = B.dpq_calibrate(w, u, s_w, G, perm, mse_grid=20, mse_max_shrink=0.8)   # with the scale search of Sec. 3.3
    t1.record()
    torch.cuda.synchronize()
    ms_mse = t0.elapsed_time(t1)
    plain = B.dpq_calibrate(w, torch.eye(k, device=dev), s_w, G)         # identity factor: no error reaches another weight
    rows = x8[:512]
    ref = (x[:512].double() @ w.double().T)
    err = {}
    for name, (codes, scales, zeros) in {"dpq_gar": cal, "dpq_gar_mse": cal_mse, "uncompensated": plain}.items():
        packed, params = B.pack_weights_asym(codes, G, scales, zeros)
        y = B.linear_asym_two_level(rows, s_x, packed, params, s_w, n, G, out_dtype=torch.float32)
        err[name] = float(((y.double() - ref) ** 2).sum())
    return {"metric": "Hessian X^T X, its factor U, then GAR + DPQ (Alg. 1), on a 4096 x 4096 layer with 8192 calibration tokens",
            "hessian_ms": round(hessian_ms, 2), "hessian_tflops_f32": round(2.0 * t * k * k / hessian_ms / 1e9, 1),
            "factor_ms": round(factor_ms, 2),
            "calibrate_ms": round(ms, 2),
            "calibrate_with_scale_search_ms": round(ms_mse, 2),
            "layer_error_ratio_vs_uncompensated": round(err["dpq_gar"] / err["uncompensated"], 4),
            "layer_error_ratio_with_scale_search": round(err["dpq_gar_mse"] / err["uncompensated"], 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--copies", type=int, default=4, help="distinct weight sets per layer shape (cache defeat)")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-block", action="store_true")
    ap.add_argument("--no-pow2", action="store_true", help="profiling aid: leave the power-of-two leg out of the prefill sweep")
    ap.add_argument("--prefill-only", action="store_true", help="profiling aid: run only the prefill sweep")
    ap.add_argument("--eager", action="store_true", help="profiling aid: launch the decode sweep kernel by kernel "
                    "instead of replaying HIP graphs (for hardware-counter runs)")
    ap.add_argument("--calibration-only", action="store_true", help="profiling aid: run only the offline-calibration leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibration_only:
        print(json.dumps({"calibration": calibration(dev)}))
        return
    cfg = syn.CONFIGS[2]
    layers = [Layer(2, i, k, n, args.copies, dev) for i, (k, n) in enumerate(syn.LLAMA3_8B.values())]
    result = {}

    if not args.prefill_only:
        cases = [Case(2, L, m, dev, cfg["frac"], cfg["mult"]) for L in layers for m in (1, 4, 16)]
        case_bytes = [alg_bytes(c.m, c.layer.k, c.layer.n) for c in cases]
        step_bytes = sum(case_bytes)

        def step(i):
            for j, c in enumerate(cases):
                c.quantize()
                c.linear(i + j)

        def linears_only(i):
            for j, c in enumerate(cases):
                c.linear(i + j)

        def step_fused(i):
            for j, c in enumerate(cases):
                c.quantize_and_linear(i + j)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)                                                     # eager run before capture
            torch.cuda.synchronize()
            step_graphs = Steps(step, args.copies, args.eager)
            lin_graphs = Steps(linears_only, args.copies, args.eager)
            repeats = 1 if args.eager else REPEATS                      # counter runs: one pass
            sec, sec_lo, sec_hi = time_graphs_spread(step_graphs, args.steps, args.warmup, repeats)
            lin_sec, lin_lo, lin_hi = time_graphs_spread(lin_graphs, args.steps, args.warmup, repeats)
            # the same launches over ONE weight set (109 MB: partly served by the 256 MB last-level cache), labelled as such
            one_set_graphs = Steps(lambda i: [c.linear(0) for c in cases], args.copies, args.eager)
            one_set_sec = time_graphs_spread(one_set_graphs, args.steps, args.warmup, repeats)[0]
            del one_set_graphs
            fused_sec = None
            if not args.eager:
                step_fused(0)
                torch.cuda.synchronize()
                fused_graphs = Steps(step_fused, args.copies)
                fused_sec, f_lo, f_hi = time_graphs_spread(fused_graphs, args.steps, args.warmup)
                del fused_graphs
        two_kernel_gbs = step_bytes / (sec / args.steps) / 1e9
        if fused_sec is not None and fused_sec < sec:
            sec, sec_lo, sec_hi = fused_sec, f_lo, f_hi                  # the step as the library runs it fastest
        ms_per_step = sec / args.steps * 1e3
        value = step_bytes / (sec / args.steps) / 1e9
        lin_gbs = step_bytes / (lin_sec / args.steps) / 1e9
        result.update({
            "metric": "W4A8 linear effective HBM GB/s (decode sweep)", "value": round(value, 1), "unit": "GB/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
            "repeats": repeats, "ms_per_step_min": round(sec_lo / args.steps * 1e3, 5),
            "ms_per_step_max": round(sec_hi / args.steps * 1e3, 5),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp8_e4m3", "data": "synthetic",
            "config": {"workload": "configs[1]: decode sweep, Llama-3-8B shapes, M in {1,4,16} x 4 (K,N), INT4 g128 "
                                   "weights, FP8 e4m3 activations, bf16 out; step = activation quantization + linear for each of the 12 cases",
                       "weight_sets": args.copies, "launch": "eager" if args.eager else "HIP graph replay, %d steps (one per weight set) per graph" % args.copies,
                       "step_form": "w4a8_linear_quantize_in for the single-token cases and for four tokens on QKV and O, quantize_act + linear for the others"
                                    if fused_sec is not None and fused_sec <= sec else "12 x (quantize_act + linear)",
                       "two_kernel_step_GBps": round(two_kernel_gbs, 1)},
            "roofline": {"bound": "hbm", "achieved": round(lin_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(lin_gbs / HBM_PEAK_GBS, 4),
                         "traffic": SKINNY_TRAFFIC_BYTES_PER_LAUNCH.get(args.copies),
                         "kernel": "linear_skinny_kernel", "launches_per_step": len(cases),
                         "avg_launch_us": round(lin_sec / args.steps / len(cases) * 1e6, 3),
                         "avg_launch_us_min_max": [round(lin_lo / args.steps / len(cases) * 1e6, 3),
                                                   round(lin_hi / args.steps / len(cases) * 1e6, 3)],
                         "alg_bytes_per_launch": step_bytes // len(cases),
                         "one_weight_set_GBps": round(step_bytes / (one_set_sec / args.steps) / 1e9, 1),
                         "one_weight_set_note": "the same 12 launches replayed over one weight set, part of which the "
                                                "last-level cache serves; `achieved` rotates over the weight sets (HBM)"},
        })
        del cases, step_graphs, lin_graphs

    if not args.no_prefill:
        pcfg = syn.CONFIGS[3]
        per_shape, tot_flop, tot_sec, tot_sec_p2, tot_bytes = [], 0.0, 0.0, 0.0, 0
        tot_sec_lib = 0.0                                                # None once the library GEMM is unavailable
        for L in layers:
            # the same codes with every group scale rounded up to a power of two, for the block-scaled variant
            p2 = [torch.exp2(torch.ceil(torch.log2(sc.abs()))) for (_, sc) in L.sets]
            for m in (512, 2048, 8192):
                c = Case(3, L, m, dev, pcfg["frac"], pcfg["mult"])
                c.quantize()
                reps = max(3, min(50, int(2e13 / (2.0 * m * L.k * L.n))))
                # untimed launches first, as many as one timed region holds: building the inputs on the host leaves the
                # GPU idle for seconds, and its clocks take some milliseconds of load to come back up
                rep_count = 1 if args.no_pow2 else REPEATS               # counter runs (--no-pow2): one timed region
                s, s_lo, s_hi = time_launches(lambda i: c.linear(i), reps, rep_count)
                flop = 2.0 * m * L.k * L.n

                def pow2(i):
                    B.linear_pow2(c.x8, c.s_x, L.sets[i % len(L.sets)][0], p2[i % len(p2)], L.n, G, out=c.y)
                s2 = s
                if not args.no_pow2:
                    s2 = time_launches(pow2, reps)[0]
                per_shape.append({"M": m, "K": L.k, "N": L.n, "us": round(s * 1e6, 2), "tflops": round(flop / s / 1e12, 1),
                                  "tflops_min_max": [round(flop / s_hi / 1e12, 1), round(flop / s_lo / 1e12, 1)],
                                  "launch_shape": list(B.linear_launch_shape(m, L.k, L.n, G, c.ws is not None))})
                if not args.no_pow2:
                    per_shape[-1]["pow2_tflops"] = round(flop / s2 / 1e12, 1)
                if tot_sec_lib is not None and not args.no_pow2:
                    s3 = library_fp8_gemm_seconds(c.x8, L.n, reps)
                    tot_sec_lib = None if s3 is None else tot_sec_lib + s3
                    if s3 is not None:
                        per_shape[-1]["library_fp8_gemm_tflops"] = round(flop / s3 / 1e12, 1)
                tot_flop += flop
                tot_sec += s
                tot_sec_p2 += 0.0 if args.no_pow2 else s2
                tot_bytes += alg_bytes(m, L.k, L.n)
                del c
            del p2
        tfl = tot_flop / tot_sec / 1e12
        tfl2 = tot_flop / tot_sec_p2 / 1e12 if tot_sec_p2 > 0 else 0.0
        result["prefill"] = {"metric": "W4A8 linear TFLOP/s (prefill sweep, configs[2])", "value": round(tfl, 1),
                             "unit": "TFLOP/s", "repeats": REPEATS, "shapes": per_shape,
                             "roofline": {"bound": "mfma", "achieved": round(tfl, 1), "peak": FP8_PEAK_TFLOPS,
                                          "unit": "TFLOP/s", "frac": round(tfl / FP8_PEAK_TFLOPS, 4),
                                          "traffic": PREFILL_TRAFFIC_BYTES_PER_LAUNCH,
                                          "alg_bytes_per_launch": tot_bytes // len(per_shape),
                                          "kernel": "linear_mfma2d_kernel (the 2048- and 8192-token shapes and gate|up at 512); "
                                                    "linear_mfma_kernel (the other 512-token shapes)"}}
        if not args.no_pow2:
            result["prefill"]["pow2_scales"] = {"metric": "the same sweep through w4a8_linear_pow2 (group scales rounded up "
                                                       "to powers of two and applied by the block-scaled MFMA)",
                                             "value": round(tfl2, 1), "unit": "TFLOP/s",
                                             "frac": round(tfl2 / FP8_PEAK_TFLOPS, 4)}

        if not args.no_pow2 and tot_sec_lib:
            tfl3 = tot_flop / tot_sec_lib / 1e12
            result["prefill"]["library_fp8_gemm"] = {
                "metric": "context, not the product path: the vendor library's dense FP8 x FP8 GEMM (torch._scaled_mm) on "
                          "the same shapes and activations, weights already expanded to FP8 in HBM, one output scale",
                "value": round(tfl3, 1), "unit": "TFLOP/s", "w4a8_linear_frac_of_it": round(tfl / tfl3, 4),
                "w4a8_linear_pow2_frac_of_it": round(tfl2 / tfl3, 4)}

    if not args.prefill_only:
        hbm, copy, mfma = measured_ceilings(dev)
        result["measured_ceilings"] = {"stream_read_GBps": hbm, "copy_read_plus_write_GBps": copy,
                                       "mfma_e4m3_TFLOPs": mfma}
        result["roofline"]["frac_of_measured"] = round(result["roofline"]["achieved"] / hbm, 4)
        if not args.eager and not args.prefill_only:
            # the same comparison at the sizes of the sweep's layers (8.9-63 MB), where launch and ramp-up weigh as much
            # as the transfer: time of the linear kernel against a kernel that only reads as many bytes
            us = plain_read_same_sizes(dev, case_bytes, args.copies, args.steps, args.warmup)
            result["roofline"]["plain_read_same_sizes_us_per_launch"] = round(us, 3)
            result["roofline"]["frac_of_plain_read_same_sizes"] = round(us / result["roofline"]["avg_launch_us"], 4)
        if "prefill" in result:
            result["prefill"]["roofline"]["frac_of_measured"] = round(result["prefill"]["roofline"]["achieved"] / mfma, 4)
        del layers
        torch.cuda.empty_cache()
        if not args.no_block:
            result["decode_cases"] = decode_cases(dev)
            result["block"] = block_latency(dev, 50, 5)
            result["weight_modes"] = weight_modes(dev)
            result["calibration"] = calibration(dev)
            result["llama70b"] = llama70b(dev, 20, 3)
            result["llama70b"]["frac_of_measured"] = round(result["llama70b"]["value"] / hbm, 4)
    if not args.no_cpu and not args.prefill_only:
        result["cpu_baseline"] = cpu_baseline()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
