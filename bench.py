#!/usr/bin/env python3
"""Benchmark of the bit-packed merged-expert MoE FFN on one MI355X.

A step is one pzl_moe_ffn call (route -> gate/up decode-GEMM + SwiGLU -> down decode-GEMM ->
combine) over one batch of synthetic tokens on a Mixtral-8x7B-shaped layer whose 8 experts are
merged into 4 packed pairs (the decode-time configuration the metric is quoted on).  Inputs
and weights are resident in HBM before the timed region.  Prints one JSON line.
"""
import argparse
import ctypes
import glob
import json
import os
import sys
import threading
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2511_04805_amd import binding, synth  # noqa: E402

HBM_PEAK_GBS = 8000.0
# Bytes between L2 and memory per launch of the gate/up kernels (streaming at T = 64, tiled at
# T = 4096), from rocprofv3 --pmc runs (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, calibrated on the
# copy below) summarised under profiles/.  Counters cannot be read inside this process.
MEASURED_TRAFFIC_BYTES = {"mixtral_decode_T64": 951.0e6, "mixtral_decode_T64_quantised": 429.2e6,
                          "mixtral_prefill_T4096": 3.339e9}
TRAFFIC_FROM = ("separate rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script, summarised under profiles/ "
                "(stream_kernels_mixtral_decode_T64.md, tile_kernels_mixtral_prefill_T4096.md); not read in this process")
W3 = (synth.GATE, synth.UP, synth.DOWN)


class Hip:
    """The few HIP runtime calls the benchmark needs for its own event timing."""

    def __init__(self):
        self.lib = ctypes.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.lib.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def event(self):
        e = ctypes.c_void_p()
        assert self.lib.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def record(self, e, stream):
        assert self.lib.hipEventRecord(e, ctypes.c_void_p(stream)) == 0

    def elapsed_ms(self, a, b):
        assert self.lib.hipEventSynchronize(b) == 0
        ms = ctypes.c_float()
        assert self.lib.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value


def build_layer(cfg, keep_planes_for=None):
    """Generate on the GPU, pack with the library.  Optionally hand each matrix's pack inputs
    (host copies) to ``keep_planes_for(pair, which, planes)`` for the CPU baseline."""
    packed = {}
    n_bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    for p in range(cfg.n_pairs):
        for which in W3:
            pl = synth.pair_matrix_t(cfg, p, which, device="cuda")
            packed[p, which] = binding.pzl_pack(pl["merged"], pl["mask0"], pl["mask1"], pl["sign0"],
                                                pl["sign1"], n_out_of_range=n_bad)
            if keep_planes_for is not None:
                keep_planes_for(p, which, {k: synth._np_bits(v) for k, v in pl.items()})
            del pl
    shared = []
    for s, fs in enumerate(cfg.shared_d_ffn):
        shared.append(tuple(binding.pzl_tile_dense(synth.shared_matrix_t(cfg, s, w, device="cuda"))
                            for w in W3) + (fs,))
    emap = synth.expert_map(cfg)
    P = cfg.n_pairs
    layer = binding.Layer(cfg.d_model, cfg.d_ffn, emap[0], emap[1],
                          [packed[p, synth.GATE] for p in range(P)], [packed[p, synth.UP] for p in range(P)],
                          [packed[p, synth.DOWN] for p in range(P)], shared=shared)
    torch.cuda.synchronize()
    assert int(n_bad.item()) == 0
    return layer, emap


def build_quantised_layer(cfg):
    """The same synthetic pairs in the quantised format (3-bit codes, group scales, base-3 masks)."""
    q = {}
    for p in range(cfg.n_pairs):
        for which in W3:
            pl = synth.pair_matrix_t(cfg, p, which, device="cuda")
            q[p, which] = binding.pzl_q_pack(pl["merged"], pl["mask0"], pl["mask1"], pl["sign0"], pl["sign1"])
            del pl
    emap = synth.expert_map(cfg)
    P = cfg.n_pairs
    layer = binding.Layer(cfg.d_model, cfg.d_ffn, emap[0], emap[1],
                          [q[p, synth.GATE] for p in range(P)], [q[p, synth.UP] for p in range(P)],
                          [q[p, synth.DOWN] for p in range(P)], quantised=True)
    torch.cuda.synchronize()
    return layer


def batch(cfg, T):
    x = synth.tokens(cfg, T)
    ids, w = synth.routing(cfg, T)
    return (x, ids, w, torch.from_numpy(x.view(np.int16)).cuda(), torch.from_numpy(ids).cuda(),
            torch.from_numpy(w).cuda())


WARM_SECONDS = 0.5      # floor of the warm-up, whatever --warmup says: clocks and caches settle in about that time
REPEATS = 5             # timed regions of K steps each; the median is reported


def _warm(call, warmup):
    """At least `warmup` calls and WARM_SECONDS of them, then on until three batches of 20 calls in a
    row agree within 2 % (at most 3 s in all): a run right after start-up, before the clocks have
    settled, measures up to 20 % slow."""
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    t_end = time.perf_counter() + WARM_SECONDS
    while time.perf_counter() < t_end:
        for _ in range(20):
            call()
        torch.cuda.synchronize()
    last, t_stop = [], time.perf_counter() + 2.5
    while time.perf_counter() < t_stop:
        t0 = time.perf_counter()
        for _ in range(20):
            call()
        torch.cuda.synchronize()
        last = (last + [time.perf_counter() - t0])[-3:]
        if len(last) == 3 and max(last) <= 1.02 * min(last):
            break


def time_plain(hip, layer, xt, idt, wt, steps, warmup):
    """pzl_moe_ffn as a caller makes it (shared experts on the layer's second stream): REPEATS timed
    regions of exactly `steps` calls, each bracketed by synchronisation, HIP events on the stream the
    calls are queued on.  Returns (median ms per step over the regions, all regions' ms per step, y)."""
    y = torch.empty(xt.shape[0], layer.d_model, dtype=torch.bfloat16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    call = lambda: layer.pzl_moe_ffn(xt, idt, wt, y=y)
    _warm(call, warmup)
    t0, t1 = hip.event(), hip.event()
    regions = []
    for _ in range(REPEATS):
        torch.cuda.synchronize()
        hip.record(t0, stream)
        for _ in range(steps):
            call()
        hip.record(t1, stream)
        torch.cuda.synchronize()
        regions.append(hip.elapsed_ms(t0, t1) / steps)
    return float(np.median(regions)), regions, y


def time_cold(hip, layer, xt, idt, wt, calls=15):
    """One call at a time with the caches flushed in front of it: a 1 GiB fill (four times the
    memory-side cache, far more than the L2s) goes through the same stream before every timed
    call, the events bracket the call alone.  Returns the median ms of `calls` such calls."""
    y = torch.empty(xt.shape[0], layer.d_model, dtype=torch.bfloat16, device="cuda")
    flush = torch.empty(1 << 28, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    t0, t1 = hip.event(), hip.event()
    ms = []
    for i in range(calls):
        flush.fill_(i)
        hip.record(t0, stream)
        layer.pzl_moe_ffn(xt, idt, wt, y=y)
        hip.record(t1, stream)
        torch.cuda.synchronize()
        ms.append(hip.elapsed_ms(t0, t1))
    del flush
    return float(np.median(ms))


def time_router(hip, cfg, xt, steps=50, warmup=5):
    """The on-device router in front of the layer (random router weights), on its own: ms per call."""
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    wr = (torch.randn(cfg.n_experts, cfg.d_model, generator=g, device="cuda") * 0.05).to(torch.bfloat16)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(warmup):
        binding.pzl_router_topk(xt, wr, cfg.top_k)
    t0, t1 = hip.event(), hip.event()
    torch.cuda.synchronize()
    hip.record(t0, stream)
    for _ in range(steps):
        binding.pzl_router_topk(xt, wr, cfg.top_k)
    hip.record(t1, stream)
    torch.cuda.synchronize()
    return hip.elapsed_ms(t0, t1) / steps


def touched_pairs(ids, emap):
    return len(set(int(emap[0][e]) for e in np.unique(ids)))


def time_stage(hip, layer, xt, idt, wt, steps, warmup, stage="gateup"):
    """Average duration of one stage's launch: HIP events recorded by the library around that stage
    (pzl_moe_ffn_staged) on the stream it runs on, in every one of `steps` calls after the warm-up.
    Returns (median, mean) in ms."""
    y = torch.empty(xt.shape[0], layer.d_model, dtype=torch.bfloat16, device="cuda")
    si = binding.STAGES.index(stage)
    evs = []
    for _ in range(steps):
        arr = (ctypes.c_void_p * (2 * len(binding.STAGES)))()
        a, b = hip.event(), hip.event()
        arr[2 * si], arr[2 * si + 1] = a, b
        evs.append((arr, a, b))
    _warm(lambda: layer.pzl_moe_ffn(xt, idt, wt, y=y), warmup)
    for arr, _, _ in evs:
        layer.pzl_moe_ffn(xt, idt, wt, y=y, stage_events=arr)
    torch.cuda.synchronize()
    stage_ms = [hip.elapsed_ms(a, b) for _, a, b in evs]
    for _, a, b in evs:
        hip.lib.hipEventDestroy(a); hip.lib.hipEventDestroy(b)
    return float(np.median(stage_ms)), float(np.mean(stage_ms))


class PowerSampler:
    """Board power while a loop runs: the driver's hwmon reading (microwatts), sampled every 20 ms by
    a host thread; None where the files cannot be read.  The reading is the driver's own running
    average, so only loops of a second or more say anything."""

    def __init__(self):
        self.files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input") +
                            glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average"))[:1]
        caps = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap"))[:1]
        self.cap_w = None
        try:
            self.cap_w = int(open(caps[0]).read()) / 1e6 if caps else None
        except (OSError, ValueError):
            pass

    def _read(self):
        try:
            return int(open(self.files[0]).read()) / 1e6
        except (OSError, ValueError, IndexError):
            return None

    def measure(self, call, seconds=2.0):
        """Runs `call` in batches for `seconds`; returns the mean reading over the second half."""
        if self._read() is None:
            return None
        samples, stop = [], [False]

        def loop():
            while not stop[0]:
                samples.append(self._read())
                time.sleep(0.02)
        th = threading.Thread(target=loop)
        th.start()
        t_end = time.perf_counter() + seconds
        while time.perf_counter() < t_end:
            for _ in range(10):
                call()
            torch.cuda.synchronize()
        stop[0] = True
        th.join()
        tail = [v for v in samples[len(samples) // 2:] if v is not None]
        return float(np.mean(tail)) if tail else None


def vendor_gemm_tflops(m, k, n, masked):
    """Context only: the vendor library's plain bf16 GEMM (torch.matmul) of the gate/up contraction's
    shape on operands of the same distribution (x ~ N(0,1), w ~ N(0,0.02), half of w zero if
    `masked`), weights already decoded in memory.  What the matrix cores deliver on this board at
    its power limit when nothing is decoded or gathered."""
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    a = torch.randn(m, k, generator=g, device="cuda").to(torch.bfloat16)
    b = torch.randn(n, k, generator=g, device="cuda") * 0.02
    if masked:
        b = b * (torch.rand(n, k, generator=g, device="cuda") < 0.5)
    b = b.to(torch.bfloat16)
    c = torch.empty(m, n, dtype=torch.bfloat16, device="cuda")
    t_end = time.perf_counter() + 1.0
    while time.perf_counter() < t_end:
        for _ in range(10):
            torch.matmul(a, b.t(), out=c)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ms = []
    for _ in range(REPEATS):
        e0.record()
        for _ in range(20):
            torch.matmul(a, b.t(), out=c)
        e1.record()
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1) / 20)
    return 2.0 * m * k * n / (float(np.median(ms)) * 1e-3) / 1e12


def uniform_routing(T):
    """Top-2 ids over 8 experts that give every expert exactly T/4 tokens (T a multiple of 8)."""
    t = np.arange(T)
    return np.stack([t % 8, (t % 8 + 1 + (t // 8) % 7) % 8], axis=1).astype(np.int32)


def tile_curve(hip, cfg, layer, sizes):
    """Duration of the tiled launches against the tile size: every expert of the Mixtral-shaped layer
    gets exactly n tokens (one tile of n up to 288, else equal tiles), for each n in `sizes`."""
    out = []
    for n in sizes:
        T = 4 * n
        ids = uniform_routing(T)
        x = synth.tokens(cfg, T)
        xt, idt = torch.from_numpy(x.view(np.int16)).cuda(), torch.from_numpy(ids).cuda()
        wt = torch.full((T, 2), 0.5, dtype=torch.float32, device="cuda")
        gu, _ = time_stage(hip, layer, xt, idt, wt, 20, 3, "gateup")
        dn, _ = time_stage(hip, layer, xt, idt, wt, 20, 0, "down")
        tiles = -(-n // 288)
        out.append({"tokens_per_expert": n, "tiles_per_expert": tiles, "fragments_per_tile": -(-(-(-n // tiles)) // 16),
                    "gateup_ms": gu, "down_ms": dn,
                    "gateup_mfma_frac": 2 * 2.0 * T * cfg.top_k * cfg.d_model * cfg.d_ffn / (gu * 1e-3) / 2.5e15})
    return out


PLAN_ALTERNATIVES = (("auto", (-1, -1, -1)), ("stream_only", (0, -1, -1)), ("tiled_one_shot", (1, 0, 0)),
                     ("tiled_one_shot_own_stream", (1, 0, 1)), ("tiled_persistent", (1, 1, 0)),
                     ("tiled_persistent_own_stream", (1, 1, 1)))


def plan_study(hip, names, token_counts):
    """The library's launch plan against the alternatives it could have chosen (pzl_layer_force_plan),
    whole step, on layer shapes that its rules were not fitted on: ms per step for each alternative,
    and how far the library's own choice is from the best of them."""
    out = {}
    for name in names:
        cfg = synth.CONFIGS[name]
        layer, _ = build_layer(cfg)
        rows = {}
        for T in token_counts:
            _, _, _, xt, idt, wt = batch(cfg, T)
            per_expert = T * cfg.top_k / cfg.n_experts
            ms = {}
            for label, force in PLAN_ALTERNATIVES:
                if label == "stream_only" and per_expert > 128:
                    continue                                  # dozens of sweeps over the weights: not a candidate
                layer.pzl_layer_force_plan(*force)
                ms[label], _, _ = time_plain(hip, layer, xt, idt, wt, 20, 3)
            layer.pzl_layer_force_plan(-1, -1, -1)
            pl = binding.pzl_moe_ffn_plan(cfg.n_experts, cfg.d_model, cfg.d_ffn, T, cfg.top_k, shared_d_ffn=cfg.shared_d_ffn)
            best = min(ms, key=ms.get)
            rows[str(T)] = {"ms": ms, "library_plan": {k: pl[k] for k in ("hybrid", "persistent", "tile_stream")},
                            "best": best, "library_over_best": ms["auto"] / ms[best]}
        out[name] = rows
        del layer
        torch.cuda.empty_cache()
    return out


def decode_point(hip, cfg, layer, emap, T, steps, warmup):
    """One decode batch size: the whole step and its two weight-streaming kernels."""
    x, ids, w, xt, idt, wt = batch(cfg, T)
    ms_step, regions, y = time_plain(hip, layer, xt, idt, wt, steps, warmup)
    gu_med, gu_mean = time_stage(hip, layer, xt, idt, wt, steps, 0, "gateup")
    dn_med, dn_mean = time_stage(hip, layer, xt, idt, wt, steps, 0, "down")
    nt = touched_pairs(ids, emap)
    d, f, k = cfg.d_model, cfg.d_ffn, cfg.top_k
    # packed gate+up once, x, H (one 16-bit plane) / packed down once, H, fp32 partial sums out
    gu_bytes = nt * 2 * f * d * 2 + T * d * 2 + T * k * f * 2
    dn_bytes = nt * f * d * 2 + T * k * f * 2
    path_bytes = nt * 3 * f * d * 2
    return {"tokens": T, "touched_pairs": nt, "ms_per_step": ms_step, "ms_per_step_regions": regions,
            "tokens_per_s": T / (ms_step * 1e-3),
            "gateup_ms": gu_mean, "gateup_ms_median": gu_med, "gateup_bytes": gu_bytes,
            "gateup_GBs": gu_bytes / (gu_mean * 1e-3) / 1e9,
            "down_ms": dn_mean, "down_ms_median": dn_med, "down_bytes": dn_bytes,
            "down_GBs": dn_bytes / (dn_mean * 1e-3) / 1e9,
            "path_GBs": path_bytes / (ms_step * 1e-3) / 1e9,
            "path_hbm_frac": path_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS}, (x, ids, w, xt, idt, wt, y)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--tokens", type=int, default=64, help="decode batch size (1, 8, 32 or 64)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-quant", action="store_true")
    ap.add_argument("--no-other-shapes", action="store_true")
    ap.add_argument("--shapes", type=str, default="qwen15_moe,deepseek_moe", metavar="NAME,NAME",
                    help="the other layer shapes to time (a profiler run may want one alone)")
    ap.add_argument("--no-context", action="store_true", help="skip the board-power readings and the vendor GEMM of the prefill shape")
    ap.add_argument("--plan-study", type=str, default="", metavar="SHAPE,SHAPE,...",
                    help="only time the library's launch plan against forced alternatives on these synth.CONFIGS shapes")
    ap.add_argument("--plan-tokens", type=str, default="16,64,128,256,512,1024,2048,4096")
    ap.add_argument("--tile-curve", type=str, default="", metavar="N,N,...",
                    help="only time the tiled launches with exactly N tokens per expert (Mixtral-shaped layer) and print that")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs an MI355X; no GPU is visible", file=sys.stderr)
        sys.exit(2)
    binding.load()
    hip = Hip()
    if args.plan_study:
        print(json.dumps({"plan_study": plan_study(hip, args.plan_study.split(","), [int(v) for v in args.plan_tokens.split(",")])}))
        return
    cfg = synth.CONFIGS["mixtral_decode"]
    T = args.tokens

    want_cpu = not args.no_cpu_baseline
    cpu_packed = {}
    if want_cpu:
        import oracle  # CPU-baseline leg only

        def keep(p, which, planes):
            cpu_packed[p, which] = oracle.pack(planes["merged"], planes["mask0"], planes["mask1"],
                                               planes["sign0"], planes["sign1"])[0]
    layer, emap = build_layer(cfg, keep if want_cpu else None)

    if args.tile_curve:
        print(json.dumps({"tile_curve": tile_curve(hip, cfg, layer, [int(v) for v in args.tile_curve.split(",")])}))
        return

    # A plain copy of known size (256 MiB in, 256 MiB out), outside the timed region: under
    # `rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE` its reading calibrates the HBM byte counters.
    cal = torch.zeros(16384, 8192, dtype=torch.int16, device="cuda")
    binding.pzl_tile_dense(cal)
    torch.cuda.synchronize()
    del cal

    # The sweep first and the headline batch last, each after its own warm-up (time-based, see
    # _warm): what is measured first would otherwise carry the start-up of the process.
    sweep = {}
    if not args.no_sweep:
        for Ts in (1, 8, 32, 64):
            if Ts != T:
                sweep[str(Ts)], _ = decode_point(hip, cfg, layer, emap, Ts, args.steps, args.warmup)
    head, (x, ids, w, xt, idt, wt, y) = decode_point(hip, cfg, layer, emap, T, args.steps, args.warmup)
    sweep[str(T)] = head
    n_touched = head["touched_pairs"]
    d, f, k = cfg.d_model, cfg.d_ffn, cfg.top_k
    pair_bytes_gateup = 2 * f * d * 2
    ms_step = head["ms_per_step"]

    out = {
        "metric": "MoE-FFN tokens/sec at 1 MI355X; achieved HBM GB/s (decode)",
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "ms_per_step_regions": head["ms_per_step_regions"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "mixtral_decode_T%d" % T, "layer": "Mixtral-8x7B-shaped, 8 experts -> 4 packed pairs",
                   "d_model": d, "d_ffn": f, "top_k": k, "tokens": T, "touched_pairs": n_touched},
        "timing": "median of %d timed regions of --steps calls each, after --warmup calls plus a warm-up of at least "
                  "%.1f s that runs until three batches of 20 calls agree within 2 %%" % (REPEATS, WARM_SECONDS),
        "roofline": {"bound": "hbm", "kernel": "stream_kernel<gate/up + SwiGLU>", "achieved": head["gateup_GBs"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head["gateup_GBs"] / HBM_PEAK_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get("mixtral_decode_T%d" % T),
                     "traffic_from": TRAFFIC_FROM if MEASURED_TRAFFIC_BYTES.get("mixtral_decode_T%d" % T) else None,
                     "algorithmic_bytes": head["gateup_bytes"], "avg_launch_ms": head["gateup_ms"],
                     "median_launch_ms": head["gateup_ms_median"]},
        "down_kernel": {"kernel": "stream_kernel<down>", "achieved": head["down_GBs"], "unit": "GB/s",
                        "frac": head["down_GBs"] / HBM_PEAK_GBS, "algorithmic_bytes": head["down_bytes"],
                        "avg_launch_ms": head["down_ms"]},
        "path_hbm_frac": head["path_hbm_frac"],
    }
    power = PowerSampler()
    if not args.no_context:
        out["board_power_W"] = power.measure(lambda: layer.pzl_moe_ffn(xt, idt, wt, y=y), seconds=1.5)
        out["board_power_cap_W"] = power.cap_w
    # the on-device router in front of the layer, on its own (not part of the timed step: ids and
    # weights are inputs of the path)
    out["router_ms"] = time_router(hip, cfg, xt)
    if not args.no_context:
        # the same step with the caches flushed in front of every call (context: the timed loop
        # above does not flush, and the layer's 1.4 GB of packed words do not fit any cache anyway)
        cold_ms = time_cold(hip, layer, xt, idt, wt)
        out["cold_cache"] = {"ms_per_step": cold_ms, "tokens_per_s": T / (cold_ms * 1e-3),
                             "flush": "1 GiB fill on the same stream before each timed call; median of 15 calls"}
    if not args.no_sweep:
        out["sweep"] = {t: {kk: v[kk] for kk in ("tokens_per_s", "ms_per_step", "touched_pairs", "gateup_GBs",
                                                  "down_GBs", "path_GBs", "path_hbm_frac")}
                        for t, v in sorted(sweep.items(), key=lambda kv: int(kv[0]))}

    if not args.no_prefill:
        # Same layer, prefill-sized batch (4096 tokens): the tiled decode-GEMM path on the matrix
        # cores.  Useful flops only: 3 projections x 2*d*f per (token, choice).
        Tp = 4096
        xs, ids_p, ws, xtp, idtp, wtp = batch(cfg, Tp)
        ms_p, _, _ = time_plain(hip, layer, xtp, idtp, wtp, 10, 3)
        _, ms_gu = time_stage(hip, layer, xtp, idtp, wtp, 20, 0, "gateup")
        _, ms_dn = time_stage(hip, layer, xtp, idtp, wtp, 20, 0, "down")
        fl_proj = 2.0 * Tp * k * d * f
        out["prefill"] = {
            "workload": "mixtral_prefill_T4096", "tokens_per_s": Tp / (ms_p * 1e-3), "ms_per_step": ms_p,
            "roofline": {"bound": "mfma", "kernel": "tile_kernel<gate/up + SwiGLU>",
                         "achieved": 2 * fl_proj / (ms_gu * 1e-3) / 1e12, "peak": 2500.0, "unit": "TFLOP/s",
                         "frac": 2 * fl_proj / (ms_gu * 1e-3) / 2.5e15,
                         "traffic": MEASURED_TRAFFIC_BYTES.get("mixtral_prefill_T%d" % Tp),
                         "traffic_from": TRAFFIC_FROM, "avg_launch_ms": ms_gu},
            "down_kernel": {"avg_launch_ms": ms_dn, "useful_TFLOPs": fl_proj / (ms_dn * 1e-3) / 1e12,
                            "frac": fl_proj / (ms_dn * 1e-3) / 2.5e15},
            "path_useful_mfma_frac": 3 * fl_proj / (ms_p * 1e-3) / 2.5e15}
        if not args.no_context:
            # What bounds this path on the board: the power drawn while it loops, against the cap
            # (at the cap the core clock drops well below the 2.4 GHz that the peak assumes), and
            # what the vendor's plain bf16 GEMM of the same shape reaches under the same cap.
            yp = torch.empty(Tp, d, dtype=torch.bfloat16, device="cuda")
            watts = power.measure(lambda: layer.pzl_moe_ffn(xtp, idtp, wtp, y=yp))
            vend = vendor_gemm_tflops(Tp * k, d, 2 * f, masked=True)
            out["prefill"]["context"] = {
                "board_power_W": watts, "board_power_cap_W": power.cap_w,
                "vendor_bf16_gemm_TFLOPs": vend, "vendor_bf16_gemm_frac_of_peak": vend / 2500.0,
                "gateup_vs_vendor_gemm": out["prefill"]["roofline"]["achieved"] / vend,
                "note": "vendor GEMM = torch.matmul on decoded weights of the same distribution resident in HBM, "
                        "shape [T*k, d] x [d, 2f]; context, not part of the path"}

    if not args.no_quant:
        # Same layer and batch with the pairs in the quantised format (the paper's appendix on
        # combining the method with quantisation): 424 bytes per 16x32 tile plus the group scales.
        qlayer = build_quantised_layer(cfg)
        ms_q, _, _ = time_plain(hip, qlayer, xt, idt, wt, max(20, args.steps // 2), 5)
        _, ms_qgu = time_stage(hip, qlayer, xt, idt, wt, max(20, args.steps // 2), 0, "gateup")
        q_pair_bytes_gateup = 2 * (f * d // 512 * 424 + f * d // 128 * 2)
        q_alg = n_touched * q_pair_bytes_gateup + T * d * 2 + T * k * f * 2
        out["quantised"] = {
            "workload": "mixtral_decode_T%d, quantised pairs (3.375 bits per weight)" % T,
            "tokens_per_s": T / (ms_q * 1e-3), "ms_per_step": ms_q,
            "roofline": {"bound": "hbm", "kernel": "stream_kernel<gate/up + SwiGLU, quantised>",
                         "achieved": q_alg / (ms_qgu * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": q_alg / (ms_qgu * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "traffic": MEASURED_TRAFFIC_BYTES.get("mixtral_decode_T%d_quantised" % T),
                         "traffic_from": TRAFFIC_FROM,
                         "algorithmic_bytes": q_alg, "avg_launch_ms": ms_qgu},
            "weight_bytes_vs_16bit": q_pair_bytes_gateup / pair_bytes_gateup}
        del qlayer

    if not args.no_other_shapes:
        # The other two layer shapes at their batch sizes, whole step.  Both roofline fractions are
        # given: bytes = the packed weights of the touched pairs and the shared experts' weights,
        # read once; flops = 3 projections x 2*d*f per (token, choice) and per (token, shared expert).
        del layer
        torch.cuda.empty_cache()
        out["other_shapes"] = {}
        for name in [n for n in args.shapes.split(",") if n]:
            c2 = synth.CONFIGS[name]
            T2 = c2.n_tokens[0]
            l2, emap2 = build_layer(c2)
            x2, ids2, w2, xt2, idt2, wt2 = batch(c2, T2)
            ms2, _, _ = time_plain(hip, l2, xt2, idt2, wt2, 50, 10)
            nt2 = touched_pairs(ids2, emap2)
            w_bytes = nt2 * 3 * c2.d_ffn * c2.d_model * 2 + sum(3 * fs * c2.d_model * 2 for fs in c2.shared_d_ffn)
            flops = 2.0 * 3 * c2.d_model * (T2 * c2.top_k * c2.d_ffn + T2 * sum(c2.shared_d_ffn))
            out["other_shapes"][name] = {
                "tokens": T2, "experts": c2.n_experts, "top_k": c2.top_k, "touched_pairs": nt2,
                "ms_per_step": ms2, "tokens_per_s": T2 / (ms2 * 1e-3), "router_ms": time_router(hip, c2, xt2),
                "hbm_frac": w_bytes / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBS,
                "useful_mfma_frac": flops / (ms2 * 1e-3) / 2.5e15}
            del l2
            torch.cuda.empty_cache()

    if want_cpu:
        import oracle
        P = cfg.n_pairs
        n_sample = min(T, 64)
        # the oracle as it stands on the host cores: whole passes over the batch until about 10 s
        # of CPU work have been timed (the batch is one step's worth: 64 tokens take about 6 s)
        passes, dt = 0, 0.0
        while dt < 10.0 and passes < 8:
            t0 = time.perf_counter()
            y64, _ = oracle.moe_ffn(x[:n_sample], ids[:n_sample], w[:n_sample], emap[0], emap[1],
                                    [cpu_packed[p, synth.GATE] for p in range(P)],
                                    [cpu_packed[p, synth.UP] for p in range(P)],
                                    [cpu_packed[p, synth.DOWN] for p in range(P)])
            dt += time.perf_counter() - t0
            passes += 1
        out["cpu_baseline"] = {"value": passes * n_sample / dt, "unit": "tokens/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
                               "kind": "oracle",
                               "sample": "%d passes over the first %d tokens of the same batch, fp64 oracle, %.1f s"
                                         % (passes, n_sample, dt)}
        # the same bound as the parity tests: every element within 1e-2 of max(|y_ref|, rms of its token's row)
        yg = y[:n_sample].float().cpu().numpy().astype(np.float64)
        rms = np.sqrt(np.mean(y64 ** 2, axis=1, keepdims=True))
        out["parity_sample"] = {"rows": n_sample, "worst_err_over_bound":
                                float((np.abs(yg - y64) / (1e-2 * np.maximum(np.abs(y64), rms))).max())}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
