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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
FP8_PEAK_TFLOPS = 5000.0       # MI355X dense FP8 MFMA
G = 128
# HBM traffic per launch of the dominant kernel on the default workload, from two hardware-counter runs of this file
# (profiles/linear_skinny_decode_sweep_hbm_traffic.txt): FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0, the factors that make the
# same counters read 1 GiB + 1 GiB for a plain 1 GiB device-to-device copy.  Counters cannot be read from inside a
# timed run, so the figure is carried here and reported only for the workload it was measured on.
SKINNY_TRAFFIC_BYTES_PER_LAUNCH = {4: 29.586e6}          # by --copies
# same for the prefill sweep (profiles/linear_mfma_prefill_sweep_hbm_traffic.txt): mean over its 12 shapes, one launch each
PREFILL_TRAFFIC_BYTES_PER_LAUNCH = 369.8e6


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

    def quantize(self):
        B.quantize_act(self.x, self.s_x, out=self.x8)

    def linear(self, s):
        packed, scales = self.layer.sets[s % len(self.layer.sets)]
        B.linear(self.x8, self.s_x, packed, scales, self.layer.n, G, B.LAYOUT_TILED, out=self.y)

    def fusable(self):
        """Where folding the activation quantization into the layer (w4a8_linear_quantize_in) pays: a single token.  Every
        workgroup quantizes all of X, so from four tokens on the separate kernel is the faster form (measured)."""
        return self.m == 1

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


def time_graphs(graphs, reps, warmup):
    """Replay graphs round-robin `reps` times after `warmup`; returns seconds for the timed replays."""
    for i in range(warmup):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for i in range(reps):
        graphs[i % len(graphs)].replay()
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) * 1e-3


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


def library_fp8_gemm_seconds(x8, n, reps):
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
        graphs = [capture(lambda i=i: reads(i)) for i in range(copies)]
        sec = time_graphs(graphs, steps, warmup)
    torch.cuda.current_stream().wait_stream(side)
    del graphs, pool
    return sec / steps / len(sizes) * 1e6


def block_latency(dev, steps, warmup):
    """Config 5: latency of the decoder-block linear stack per batch size, HIP graph replay."""
    from paper_2505_14638_amd.block import LAYERS, DecoderBlockLinears
    cfg = syn.CONFIGS[5]
    blk = DecoderBlockLinears(cfg["hidden"], cfg["ffn"], syn.LLAMA3_8B["qkv"][1], cfg["group"], dev)
    for idx, name in enumerate(LAYERS):
        k, n = blk.dims[name]
        blk.load_layer(name, torch.from_numpy(syn.make_weights(syn.rng_for(5, idx), n, k)))
    for name, s in zip(LAYERS, (0.19, 0.012, 0.004, 0.0006)):          # typical static scales of this block
        blk.set_act_scale(name, s)
    fused = DecoderBlockLinears(cfg["hidden"], cfg["ffn"], syn.LLAMA3_8B["qkv"][1], cfg["group"], dev, fused=True)
    fused.weights, fused.scales_x = blk.weights, blk.scales_x
    out, out_fused = {}, {}
    for m in cfg["batches"]:
        x = syn.make_activations(syn.rng_for(5, 200 + m), m, cfg["hidden"], cfg["frac"], cfg["mult"])
        x_d = torch.from_numpy(x).to(dev).to(torch.bfloat16)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            blk.forward(x_d)
            torch.cuda.synchronize()
            g = capture(lambda: blk.forward(x_d))
            sec = time_graphs([g], steps, warmup)
            fused.forward(x_d)
            torch.cuda.synchronize()
            gf = capture(lambda: fused.forward(x_d))
            sec_f = time_graphs([gf], steps, warmup)
        out[str(m)] = round(sec / steps * 1e6, 2)
        out_fused[str(m)] = round(sec_f / steps * 1e6, 2)
    return {"metric": "decoder-block linear stack latency (config 5: QKV, O, gate|up, SiLU*mul, down; hidden 4096, "
                      "FFN 14336)", "unit": "us per block", "by_batch": out, "fused_by_batch": out_fused,
            "fused": "same outputs with each intermediate's FP8 quantization folded into the kernel that produces it "
                     "(6 launches instead of 9)",
            "note": "one weight set, so at small batch part of the 116 MB of weights is served by the 256 MB cache"}


def weight_modes(dev):
    """The other weight formats of the library on two shapes (gate|up at M = 1 and M = 8192): same measurement as the
    main legs, eager launches over six rotating weight sets (decode) or one (prefill)."""
    k, n = syn.LLAMA3_8B["gate_up"]
    nt = (n + 15) // 16
    out = {}
    for m in (1, 8192):
        sets = 6 if m == 1 else 1
        x8 = torch.randint(0, 120, (m, k), dtype=torch.uint8, device=dev)
        sx = torch.tensor([0.1], dtype=torch.float32, device=dev)
        y = torch.empty((m, n), dtype=torch.bfloat16, device=dev)
        packed = [torch.randint(0, 256, (n * k // 2,), dtype=torch.uint8, device=dev) for _ in range(sets)]
        s32 = [torch.rand(nt * 16 * k // G, dtype=torch.float32, device=dev) * 0.01 + 0.005 for _ in range(sets)]
        s8 = [sc * 400.0 for sc in s32]                                    # FP8-domain group scales, products up to ~56
        sp2 = [torch.exp2(torch.ceil(torch.log2(sc))) for sc in s32]
        w_out = torch.rand(n, dtype=torch.float32, device=dev) * 1e-3
        params = []
        for i in range(sets):
            rec = torch.zeros((nt * (k // G), 80), dtype=torch.uint8, device=dev)
            rec[:, :64] = s32[i].view(-1, 16).view(torch.uint8)
            rec[:, 64:] = torch.randint(0, 16, (nt * (k // G), 16), dtype=torch.uint8, device=dev)
            params.append(rec.reshape(-1))
        calls = {
            "code_exact": lambda i: B.linear(x8, sx, packed[i], s32[i], n, G, B.LAYOUT_TILED, out=y),
            "two_level": lambda i: B.linear_two_level(x8, sx, packed[i], s8[i], w_out, n, G, out=y),
            "asym": lambda i: B.linear_asym(x8, sx, packed[i], params[i], n, G, out=y),
            "pow2": lambda i: B.linear_pow2(x8, sx, packed[i], sp2[i], n, G, out=y),
        }
        reps = 60 if m == 1 else 10
        row = {}
        for name, fn in calls.items():
            for i in range(reps):
                fn(i % sets)
            torch.cuda.synchronize()
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0.record()
            for i in range(reps):
                fn(i % sets)
            t1.record()
            torch.cuda.synchronize()
            sec = t0.elapsed_time(t1) * 1e-3 / reps
            extra = n * k // G if name == "asym" else 0                   # zero-point bytes
            row[name] = round((alg_bytes(m, k, n) + extra) / sec / 1e9, 1) if m == 1 else round(2.0 * m * k * n / sec / 1e12, 1)
        out[f"M={m}"] = {"unit": "GB/s" if m == 1 else "TFLOP/s", **row}
    return {"metric": "weight formats on the gate|up layer (K = 4096, N = 28672), random codes", "by_case": out}


def llama70b(dev, steps, warmup):
    """Config 4's decode cases (Llama-3-70B shapes, M = 1 and 16): the linear kernel alone, HIP graph replay over two
    rotating weight sets of random codes (428 MB each).  Layers of 34-235 MB, where launch and ramp-up weigh less."""
    shapes = list(syn.LLAMA3_70B.values())
    sets = []
    for _ in range(2):
        one = []
        for (k, n) in shapes:
            one.append((torch.randint(0, 256, (n * k // 2,), dtype=torch.uint8, device=dev),
                        torch.rand(n * k // G, dtype=torch.float32, device=dev) * 0.01 + 0.001))
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
        sec = time_graphs(graphs, steps, warmup) / steps
    torch.cuda.current_stream().wait_stream(side)
    gbs = total / sec / 1e9
    # the prefill cases of the same config (M = 4096), eager launches after untimed ones
    flop, psec = 0.0, 0.0
    x8 = torch.randint(0, 120, (4096, max(k for (k, _) in shapes)), dtype=torch.uint8, device=dev)
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for j, (k, n) in enumerate(shapes):
        y = torch.empty((4096, n), dtype=torch.bfloat16, device=dev)
        xs = x8[:, :k]
        for i in range(3):
            B.linear(xs, sx, sets[i % 2][j][0], sets[i % 2][j][1], n, G, B.LAYOUT_TILED, out=y)
        torch.cuda.synchronize()
        t0.record()
        for i in range(3):
            B.linear(xs, sx, sets[i % 2][j][0], sets[i % 2][j][1], n, G, B.LAYOUT_TILED, out=y)
        t1.record()
        torch.cuda.synchronize()
        psec += t0.elapsed_time(t1) * 1e-3 / 3
        flop += 2.0 * 4096 * k * n
        del y
    tfl = flop / psec / 1e12
    return {"metric": "W4A8 linear on configs[3] (Llama-3-70B shapes): effective HBM GB/s of the decode cases (M in {1, 16}) "
                      "and TFLOP/s of the prefill cases (M = 4096)",
            "value": round(gbs, 1), "unit": "GB/s", "frac_of_peak": round(gbs / HBM_PEAK_GBS, 4),
            "us_per_launch": round(sec / len(cases) * 1e6, 2), "alg_bytes_per_launch": total // len(cases),
            "prefill_tflops": round(tfl, 1), "prefill_frac_of_peak": round(tfl / FP8_PEAK_TFLOPS, 4)}


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
            if args.eager:
                step_graphs = [Eager(lambda i=i: step(i)) for i in range(args.copies)]
                lin_graphs = [Eager(lambda i=i: linears_only(i)) for i in range(args.copies)]
            else:
                step_graphs = [capture(lambda i=i: step(i)) for i in range(args.copies)]
                lin_graphs = [capture(lambda i=i: linears_only(i)) for i in range(args.copies)]
            sec = time_graphs(step_graphs, args.steps, args.warmup)
            lin_sec = time_graphs(lin_graphs, args.steps, args.warmup)
            fused_sec = None
            if not args.eager:
                step_fused(0)
                torch.cuda.synchronize()
                fused_graphs = [capture(lambda i=i: step_fused(i)) for i in range(args.copies)]
                fused_sec = time_graphs(fused_graphs, args.steps, args.warmup)
                del fused_graphs
        two_kernel_gbs = step_bytes / (sec / args.steps) / 1e9
        if fused_sec is not None and fused_sec < sec:
            sec = fused_sec                                              # the step as the library runs it fastest
        ms_per_step = sec / args.steps * 1e3
        value = step_bytes / (sec / args.steps) / 1e9
        lin_gbs = step_bytes / (lin_sec / args.steps) / 1e9
        result.update({
            "metric": "W4A8 linear effective HBM GB/s (decode sweep)", "value": round(value, 1), "unit": "GB/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp8_e4m3", "data": "synthetic",
            "config": {"workload": "configs[1]: decode sweep, Llama-3-8B shapes, M in {1,4,16} x 4 (K,N), INT4 g128 "
                                   "weights, FP8 e4m3 activations, bf16 out; step = activation quantization + linear for each of the 12 cases",
                       "weight_sets": args.copies, "launch": "eager" if args.eager else "HIP graph replay",
                       "step_form": "w4a8_linear_quantize_in for the single-token cases, quantize_act + linear for the others"
                                    if fused_sec is not None and fused_sec <= sec else "12 x (quantize_act + linear)",
                       "two_kernel_step_GBps": round(two_kernel_gbs, 1)},
            "roofline": {"bound": "hbm", "achieved": round(lin_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(lin_gbs / HBM_PEAK_GBS, 4),
                         "traffic": SKINNY_TRAFFIC_BYTES_PER_LAUNCH.get(args.copies),
                         "kernel": "linear_skinny_kernel", "launches_per_step": len(cases),
                         "avg_launch_us": round(lin_sec / args.steps / len(cases) * 1e6, 3),
                         "alg_bytes_per_launch": step_bytes // len(cases)},
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
                # untimed launches first, about as many as will be timed: building the inputs on the host leaves the GPU
                # idle for seconds, and its clocks take some milliseconds of load to come back up
                for i in range(max(2, reps)):
                    c.linear(i)
                torch.cuda.synchronize()
                t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                t0.record()
                for i in range(reps):
                    c.linear(i)
                t1.record()
                torch.cuda.synchronize()
                s = t0.elapsed_time(t1) * 1e-3 / reps
                flop = 2.0 * m * L.k * L.n

                def pow2(i):
                    B.linear_pow2(c.x8, c.s_x, L.sets[i % len(L.sets)][0], p2[i % len(p2)], L.n, G, out=c.y)
                s2 = s
                if not args.no_pow2:
                    for i in range(max(2, reps)):
                        pow2(i)
                    torch.cuda.synchronize()
                    t0.record()
                    for i in range(reps):
                        pow2(i)
                    t1.record()
                    torch.cuda.synchronize()
                    s2 = t0.elapsed_time(t1) * 1e-3 / reps
                per_shape.append({"M": m, "K": L.k, "N": L.n, "us": round(s * 1e6, 2), "tflops": round(flop / s / 1e12, 1)})
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
                             "unit": "TFLOP/s", "shapes": per_shape,
                             "roofline": {"bound": "mfma", "achieved": round(tfl, 1), "peak": FP8_PEAK_TFLOPS,
                                          "unit": "TFLOP/s", "frac": round(tfl / FP8_PEAK_TFLOPS, 4),
                                          "traffic": PREFILL_TRAFFIC_BYTES_PER_LAUNCH,
                                          "alg_bytes_per_launch": tot_bytes // len(per_shape),
                                          "kernel": "linear_mfma_kernel"}}
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
