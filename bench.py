#!/usr/bin/env python3
"""Benchmark of the DSTG+DCRP W4A4 linear hot path on one MI355X.

A step is one pass of the whole hot path over one batch of the ViT-L-shaped
stress workload (config 4: batch 32, 4096 tokens, fc1 1024->4096 and fc2
4096->1024, 32 token groups per image): for each of the two linears
tdq_calibrate_groups -> tdq_quantize_act -> tdq_w4a4_linear.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--heavy 10] [--small]

Around the timed steps the same run also reports (each leg can be switched off): the
heavy-tail sweep of the workload (2 / 25 %), the small configurations 0-3, the
paper-literal per-block path, the 6-bit-format contraction, device probes (what a plain
read, a plain copy, the int8 matrix instruction and the vector unit sustain on this
device in this run), quality figures of the synthetic input, and the CPU oracle.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
PEAK_INT8_TOPS = 5000.0        # MI355X dense int8 MFMA, published (5.0 POP/s)
# Vector lane operations per second.  The published fp32 vector peak, 157.3 TFLOP/s, is
# 256 CUs x 4 SIMDs x 32 lanes x 2 flops x 2.4 GHz: 32 binary32 lane-operations per clock
# and SIMD.  The `probes` leg measures what unpacked v_fma_f32 reaches on this device (four
# wavefronts per SIMD reach about 0.7 of it, two about 0.5, one about 0.27).
PEAK_VALU_TLOPS = 256 * 4 * 32 * 2.4e9 / 1e12
# HBM bytes per launch of the fc1 contraction on the default workload: NOT measured by this
# run but imported from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this same
# command (scaled on the 1 GiB copy of the probes leg), profiles/bench_cfg4_hbm_traffic_pmc.txt
GEMM_FC1_TRAFFIC_BYTES = 1159044046
GEMM_FC1_TRAFFIC_SOURCE = "profiles/bench_cfg4_hbm_traffic_pmc.txt"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5, help="untimed steps right before the timed ones")
    ap.add_argument("--preroll", type=int, default=40,
                    help="untimed steps before the warm-up, the run's own: the clocks take about 20 "
                         "steps (35 ms) to settle under the contraction's load, whatever --warmup is")
    ap.add_argument("--heavy", type=int, default=10, choices=(2, 10, 25),
                    help="heavy-tailed token fraction of config 4, percent")
    ap.add_argument("--small", action="store_true",
                    help="4 images instead of 32 (quick functional run, not the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true",
                    help="skip the device probes (1 GiB read and copy, matrix-instruction and vector rates)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the heavy-tail sweep (2 / 25 %%)")
    ap.add_argument("--no-small", action="store_true", help="skip the small configurations 0-3")
    ap.add_argument("--no-quality", action="store_true")
    ap.add_argument("--no-blocks", action="store_true",
                    help="skip the paper-literal (token, 32-channel block) leg")
    return ap.parse_args()


class Layer:
    """Device-resident state of one quantized linear."""

    def __init__(self, lc, out_dtype, torch, tdq, I, dev):
        self.lc = lc
        X, cls = I.make_activations(lc, workers=16)
        self.X_host, self.cls = X, cls
        self.X = torch.from_numpy(X).to(dev)
        W = torch.from_numpy(I.make_weight(lc)).to(dev)
        self.Qw, self.w_scale = tdq.tdq_quantize_weight(W)      # offline, not timed
        self.p = tdq.default_params(lc.G)
        dt = tdq.TDQ_F16 if lc.dtype == "f16" else tdq.TDQ_F32
        self.ws = tdq.alloc_workspace(lc.B, lc.T, lc.C, dt, self.p, dev)
        self.gid = torch.empty((lc.B, lc.T), dtype=torch.int32, device=dev)
        self.clip = torch.empty((lc.B, lc.G), dtype=torch.float32, device=dev)
        self.scale = torch.empty((lc.B, lc.G), dtype=torch.float32, device=dev)
        self.Q = torch.zeros((lc.M, tdq.packed_row_bytes(lc.C)), dtype=torch.uint8, device=dev)
        self.Y = torch.empty((lc.M, lc.N), dtype=out_dtype, device=dev)
        e = lc.M * lc.C
        s = 2 if lc.dtype == "f16" else 4
        # sweeps of X inside tdq_calibrate_groups: the statistics sweep plus the rank
        # select (one sweep for binary16, four radix levels for binary32)
        sweeps_cal = 2 if lc.dtype == "f16" else 1 + 4
        self.bytes = {
            "calibrate": sweeps_cal * e * s + lc.M * 20,
            "quantize": e * s + lc.M * 4 + e // 2,
            "compulsory": e * s + e // 2,
        }
        ob = 2 if out_dtype == torch.float16 else 4
        self.gemm_ops = 2 * lc.M * lc.N * lc.C
        self.gemm_bytes = lc.M * lc.C // 2 + lc.N * lc.C // 2 + lc.M * lc.N * ob + 4 * (lc.M + lc.N)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (images are independent, so a larger job "
              "would shard the batch with no exchange); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2604_16855_amd import inputs as I
    from paper_2604_16855_amd import tdq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    tdq.lib()        # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    over = dict(B=4) if args.small else {}
    t0 = time.time()
    fc1 = Layer(I.case(f"cfg4_fc1_h{args.heavy}", **over), torch.float16, torch, tdq, I, dev)
    fc2 = Layer(I.case(f"cfg4_fc2_h{args.heavy}", **over), torch.float32, torch, tdq, I, dev)
    layers = [fc1, fc2]
    torch.cuda.synchronize()
    print(f"[bench] inputs ready in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    seg_names = ["calibrate", "quantize", "linear"]

    def step(events=None):
        """One pass of the hot path.  `events`: 3 * len(layers) + 1 HIP events, one at every
        boundary between entry points (the end of one segment is the start of the next, and
        the last event of a step is the first of the following one)."""
        k = 0
        for L in layers:
            lc = L.lc
            if events is not None and k == 0 and events[0] is not None:
                events[0].record()
            tdq.tdq_calibrate_groups(L.X, L.p, L.ws, out=(L.gid, L.clip, L.scale))
            if events is not None:
                events[k + 1].record()
            tdq.tdq_quantize_act(L.X, L.p, L.gid, L.clip, L.scale, out=L.Q)
            if events is not None:
                events[k + 2].record()
            tdq.tdq_w4a4_linear(L.Q, L.gid, L.scale, lc.B, lc.T, lc.C, L.Qw, L.w_scale, None,
                                out=L.Y)
            if events is not None:
                events[k + 3].record()
            k += 3

    for _ in range(args.preroll):           # the run's own clock pre-roll, then the asked-for warm-up
        step()
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    nseg = 3 * len(layers)
    flat = [torch.cuda.Event(enable_timing=True) for _ in range(nseg * args.steps + 1)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        ev = flat[k * nseg:(k + 1) * nseg + 1]
        if k > 0:
            ev = [None] + ev[1:]          # already recorded as the previous step's last event
        step(ev)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps

    seg_ms = np.zeros((len(layers), 3))
    for k in range(args.steps):
        for li in range(len(layers)):
            for sgm in range(3):
                i = k * nseg + 3 * li + sgm
                seg_ms[li, sgm] += flat[i].elapsed_time(flat[i + 1])
    seg_ms /= args.steps

    act_ms = seg_ms[:, 0].sum() + seg_ms[:, 1].sum()
    gemm_ms = seg_ms[:, 2].sum()
    compulsory = sum(L.bytes["compulsory"] for L in layers)
    sweeps = sum(L.bytes["calibrate"] + L.bytes["quantize"] for L in layers)
    act_gbs = compulsory / (act_ms * 1e-3) / 1e9
    act_sweep_gbs = sweeps / (act_ms * 1e-3) / 1e9
    gemm_tops = sum(L.gemm_ops for L in layers) / (gemm_ms * 1e-3) / 1e12

    rooflines = []
    for li, L in enumerate(layers):
        nm = L.lc.name
        for s, key in ((0, "calibrate"), (1, "quantize")):
            a = L.bytes[key] / (seg_ms[li, s] * 1e-3) / 1e9
            rooflines.append({"kernel": f"{key}:{nm}", "bound": "hbm", "achieved": round(a, 1),
                              "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(a / PEAK_HBM_GBS, 4),
                              "ms": round(float(seg_ms[li, s]), 4)})
        ai = L.gemm_ops / L.gemm_bytes
        t = L.gemm_ops / (seg_ms[li, 2] * 1e-3) / 1e12
        rooflines.append({"kernel": f"w4a4_linear:{nm}", "bound": "mfma", "achieved": round(t, 1),
                          "peak": PEAK_INT8_TOPS, "unit": "TOP/s", "frac": round(t / PEAK_INT8_TOPS, 4),
                          "ms": round(float(seg_ms[li, 2]), 4), "ops_per_byte": round(ai, 1),
                          "hbm_gbs": round(L.gemm_bytes / (seg_ms[li, 2] * 1e-3) / 1e9, 1)})

    # The dominant kernel of a step: the fc1 contraction, k_w4a4_gemm_roll<_Float16>,
    # one launch per step (tdq_w4a4_linear launches nothing else), timed by the HIP
    # events around that entry point on the stream it runs on.  Algorithmic work per
    # launch = 2 M N K integer operations.  `traffic` is the HBM bytes per launch
    # measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled on a 1 GiB copy)
    # for exactly this workload in a separate run of this command (`traffic_source`);
    # it is not known for other --heavy / --small settings.
    fc1_ms = float(seg_ms[0, 2])
    fc1_tops = fc1.gemm_ops / (fc1_ms * 1e-3) / 1e12
    traffic = GEMM_FC1_TRAFFIC_BYTES if (fc1.lc.B == 32 and args.heavy == 10) else None
    roofline = {"kernel": "k_w4a4_gemm_roll<_Float16> (fc1 contraction, M=131072 K=1024 N=4096)",
                "bound": "mfma", "achieved": round(fc1_tops, 1), "peak": PEAK_INT8_TOPS,
                "unit": "TOP/s", "frac": round(fc1_tops / PEAK_INT8_TOPS, 4), "traffic": traffic,
                "traffic_source": GEMM_FC1_TRAFFIC_SOURCE if traffic else None,
                "avg_launch_ms": round(fc1_ms, 4), "ops_per_launch": fc1.gemm_ops,
                "algorithmic_bytes": fc1.gemm_bytes}

    out = {
        "metric": "DSTG+DCRP act-quant GB/s + W4A4 linear TOPS (% of HBM / int8 MFMA peak)",
        "value": round(act_gbs, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_preroll_steps": args.preroll,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8 MFMA / int32 acc; fp32 statistics (fp64 merge)",
        "data": "synthetic",
        "config": {"workload": f"config 4 (ViT-L-shaped stress): B={fc1.lc.B} x T=4096, "
                               f"fc1 1024->4096 (fp16 out) + fc2 4096->1024 (fp32 out), "
                               f"G=32, heavy {args.heavy}%, fp16 activations",
                   "value_definition": "bytes of X read once + packed codes written, "
                                       "divided by the time of calibrate+quantize of both linears"},
        "act_quant_gbs": round(act_gbs, 1),
        "act_quant_frac_hbm": round(act_gbs / PEAK_HBM_GBS, 4),
        "act_sweep_gbs": round(act_sweep_gbs, 1),
        "act_sweep_frac_hbm": round(act_sweep_gbs / PEAK_HBM_GBS, 4),
        "linear_tops": round(gemm_tops, 1),
        "linear_frac_mfma": round(gemm_tops / PEAK_INT8_TOPS, 4),
        "act_ms": round(float(act_ms), 4), "linear_ms": round(float(gemm_ms), 4),
        "roofline": roofline,
        "rooflines": rooflines,
    }
    out["rank_select_missed_sets"] = [tdq.exact_select_sets(L.ws) for L in layers]
    if not args.no_probes:
        out["probes"] = probes_leg(torch, tdq, dev)
    if not args.no_sweep and not args.small:
        out["heavy_sweep"] = heavy_sweep(layers, args.heavy, seg_ms, step, torch, tdq, I)
    if not args.no_small:
        out["small_configs"] = small_configs(torch, tdq, I, dev)
    if not args.no_blocks:
        out["paper_literal_blocks"] = blocks_leg(layers, torch, tdq)
        out["f6_contraction"] = f6_leg(layers, torch, tdq)
    if not args.no_quality:
        out["quality"] = quality(fc1, torch, tdq)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layers, np, I)
    print(json.dumps(out), flush=True)


def _time_events(torch, fn, iters, warm):
    """Mean milliseconds of fn() over `iters` launches after `warm` untimed ones (HIP events
    on the launching stream)."""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def probes_leg(torch, tdq, dev):
    """What this device sustains in this run, from kernels inside libtdq (tdq_probe): a plain
    read and a plain copy of 1 GiB (the achievable-bandwidth denominators beside the 8 TB/s
    peak), a register-only stream of the contraction's matrix instruction in the contraction's
    4 x 4 operand pattern on all-zero operands, on random bytes and on random int4 codes in
    the kernels' operand encoding (the data-dependent ceilings beside the 5.0 POP/s peak), and
    register-only v_fma_f32 streams with one and with two wavefronts per SIMD (lanes per
    clock of the vector unit)."""
    res = {}
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    buf = torch.zeros((2 << 30) + 4096, dtype=torch.uint8, device=dev)
    gib = 1 << 30
    rd = buf[:gib + 4096]
    ms = _time_events(torch, lambda: tdq.tdq_probe(tdq.PROBE_READ, rd), 10, 3)
    res["read_1gib"] = {"ms": round(ms, 4), "gbs": round(gib / (ms * 1e-3) / 1e9, 1)}
    cp = buf[:2 * gib]
    ms = _time_events(torch, lambda: tdq.tdq_probe(tdq.PROBE_COPY, cp), 10, 3)
    res["copy_1gib"] = {"ms": round(ms, 4), "gbs_read_plus_write": round(2 * gib / (ms * 1e-3) / 1e9, 1)}
    del rd, cp
    grid, iters = 4 * cus, 4000
    small = buf[:grid * 32768 + 4096]
    ops = grid * 4 * iters * 16 * 65536
    ms = _time_events(torch, lambda: tdq.tdq_probe(tdq.PROBE_MFMA_I8, small, iters, grid), 5, 20)
    res["mfma_i8_zeros"] = {"ms": round(ms, 4), "tops": round(ops / (ms * 1e-3) / 1e12, 1),
                            "frac_of_peak": round(ops / (ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 4)}
    g = torch.Generator(device=dev).manual_seed(7)
    small.copy_(torch.randint(0, 256, (small.numel(),), dtype=torch.uint8, device=dev, generator=g))
    ms = _time_events(torch, lambda: tdq.tdq_probe(tdq.PROBE_MFMA_I8, small, iters, grid), 5, 20)
    res["mfma_i8_random_bytes"] = {"ms": round(ms, 4), "tops": round(ops / (ms * 1e-3) / 1e12, 1),
                                   "frac_of_peak": round(ops / (ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 4)}
    # uniformly random int4 codes as the contraction feeds them: the code in the high
    # nibble of the byte (16 x code), low nibble zero
    small.copy_(torch.randint(0, 16, (small.numel(),), dtype=torch.uint8, device=dev, generator=g) * 16)
    ms = _time_events(torch, lambda: tdq.tdq_probe(tdq.PROBE_MFMA_I8, small, iters, grid), 5, 20)
    res["mfma_i8_random_codes"] = {"ms": round(ms, 4), "tops": round(ops / (ms * 1e-3) / 1e12, 1),
                                   "frac_of_peak": round(ops / (ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 4)}
    fb = buf[:8192].view(torch.float32)
    fb[:64] = 0.999
    fb[64:128] = 0.001
    for key, kind, tpw in (("fma_f32_1_wave_per_simd", tdq.PROBE_FMA_1WAVE, 256),
                           ("fma_f32_2_waves_per_simd", tdq.PROBE_FMA_2WAVES, 512),
                           ("fma_f32_4_waves_per_simd", tdq.PROBE_FMA_4WAVES, 1024)):
        it2 = 20000
        ms = _time_events(torch, lambda: tdq.tdq_probe(kind, buf[:8192], it2, cus), 5, 5)
        lane_ops = cus * tpw * it2 * 16
        t = lane_ops / (ms * 1e-3) / 1e12
        res[key] = {"ms": round(ms, 4), "t_lane_ops": round(t, 2),
                    "lanes_per_clock_per_simd_at_2.4ghz": round(t * 1e12 / (cus * 4 * 2.4e9), 1),
                    "frac_of_peak": round(t / PEAK_VALU_TLOPS, 4)}
    res["compute_units"] = cus
    del buf
    return res


def heavy_sweep(layers, heavy_main, seg_main, step, torch, tdq, I, iters=20, warm=20):
    """The heavy-tail sweep of the workload: the timed step's entry points on inputs with 2,
    10 and 25 % heavy tokens (the --heavy setting is the timed run itself), per layer
    calibrate / quantize / linear milliseconds and the count of token sets whose sampled key
    interval missed the rank.  The device buffers of the timed run are reused."""
    res = {}
    keep = [L.X for L in layers]
    for h in (2, 10, 25):
        if h == heavy_main:
            res[f"h{h}"] = {L.lc.name: {"calibrate_ms": round(float(seg_main[li, 0]), 4),
                                        "quantize_ms": round(float(seg_main[li, 1]), 4),
                                        "linear_ms": round(float(seg_main[li, 2]), 4),
                                        "rank_select_missed_sets": tdq.exact_select_sets(L.ws)}
                            for li, L in enumerate(layers)}
            res[f"h{h}"]["source"] = "the timed steps"
            continue
        entry = {}
        for li, L in enumerate(layers):
            lc = I.case(L.lc.name.rsplit("_h", 1)[0] + f"_h{h}")
            X, _ = I.make_activations(lc, workers=16)
            L.X.copy_(torch.from_numpy(X))
            del X
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(iters)]
            for it in range(warm + iters):           # back to back, as in the timed steps
                ev = evs[it - warm] if it >= warm else None
                if ev:
                    ev[0].record()
                tdq.tdq_calibrate_groups(L.X, L.p, L.ws, out=(L.gid, L.clip, L.scale))
                if ev:
                    ev[1].record()
                tdq.tdq_quantize_act(L.X, L.p, L.gid, L.clip, L.scale, out=L.Q)
                if ev:
                    ev[2].record()
                tdq.tdq_w4a4_linear(L.Q, L.gid, L.scale, lc.B, lc.T, lc.C, L.Qw, L.w_scale, None, out=L.Y)
                if ev:
                    ev[3].record()
            torch.cuda.synchronize()
            t = [sum(ev[s].elapsed_time(ev[s + 1]) for ev in evs) for s in range(3)]
            assert tdq.device_status(L.ws) == 0
            entry[lc.name] = {"calibrate_ms": round(t[0] / iters, 4), "quantize_ms": round(t[1] / iters, 4),
                              "linear_ms": round(t[2] / iters, 4),
                              "rank_select_missed_sets": tdq.exact_select_sets(L.ws)}
        res[f"h{h}"] = entry
    # the timed run's inputs back in place (the legs after this one use them)
    for L in layers:
        L.X.copy_(torch.from_numpy(L.X_host))
        tdq.tdq_calibrate_groups(L.X, L.p, L.ws, out=(L.gid, L.clip, L.scale))
        tdq.tdq_quantize_act(L.X, L.p, L.gid, L.clip, L.scale, out=L.Q)
    torch.cuda.synchronize()
    return res


def small_configs(torch, tdq, I, dev, iters=30, warm=10):
    """Configurations 0-3 (single linears up to the 80 linears of the 4-stage encoder at
    batch 8): per linear the microseconds of the activation path by the multi-kernel route
    (tdq_calibrate_groups + tdq_quantize_act) and by the single-launch route
    (tdq_calibrate_quantize_fused), of the contraction, and the bandwidth of the whole linear
    on its algorithmic bytes (X read once, codes written and read, weights, Y written).
    These shapes are launch- or HBM-bound: the figures are microseconds first, rates second."""
    names = ["cfg0", "cfg1", "cfg2_qkv", "cfg2_proj", "cfg2_fc1", "cfg2_fc2"]
    names += sorted(n for n in I.CASES if n.startswith("cfg3_"))
    rows, tot3_multi, tot3_best, n3 = [], 0.0, 0.0, 0
    for name in names:
        lc = I.case(name)
        X, _ = I.make_activations(lc, workers=16)
        Xd = torch.from_numpy(X).to(dev)
        Qw, sw = tdq.tdq_quantize_weight(torch.from_numpy(I.make_weight(lc)).to(dev))
        p = tdq.default_params(lc.G)
        dt = tdq.TDQ_F16 if lc.dtype == "f16" else tdq.TDQ_F32
        ws = tdq.alloc_workspace(lc.B, lc.T, lc.C, dt, p, dev)
        gid = torch.empty((lc.B, lc.T), dtype=torch.int32, device=dev)
        clip = torch.empty((lc.B, lc.G), dtype=torch.float32, device=dev)
        scale = torch.empty((lc.B, lc.G), dtype=torch.float32, device=dev)
        flags = torch.empty((lc.B,), dtype=torch.int32, device=dev)
        Q = torch.zeros((lc.M, tdq.packed_row_bytes(lc.C)), dtype=torch.uint8, device=dev)
        Y = torch.empty((lc.M, lc.N), dtype=torch.float32, device=dev)

        def multi():
            tdq.tdq_calibrate_groups(Xd, p, ws, out=(gid, clip, scale))
            tdq.tdq_quantize_act(Xd, p, gid, clip, scale, out=Q)

        def fused():
            tdq.tdq_calibrate_quantize_fused(Xd, p, ws, out=(gid, clip, scale, flags, Q))

        def linear():
            tdq.tdq_w4a4_linear(Q, gid, scale, lc.B, lc.T, lc.C, Qw, sw, None, out=Y)

        t_multi = _time_events(torch, multi, iters, warm) * 1e3
        t_fused = _time_events(torch, fused, iters, warm) * 1e3
        multi()
        t_lin = _time_events(torch, linear, iters, warm) * 1e3
        e = lc.M * lc.C
        sz = 2 if lc.dtype == "f16" else 4
        byt = e * sz + e + lc.N * lc.C // 2 + lc.M * lc.N * 4 + 4 * (lc.M + lc.N)
        best = min(t_multi, t_fused)
        rows.append({"linear": name, "shape": [lc.B, lc.T, lc.C, lc.N], "act_multi_kernel_us": round(t_multi, 1),
                     "act_single_launch_us": round(t_fused, 1), "contraction_us": round(t_lin, 1),
                     "linear_gbs": round(byt / ((best + t_lin) * 1e-6) / 1e9, 1),
                     "contraction_tops": round(2.0 * lc.M * lc.N * lc.C / (t_lin * 1e-6) / 1e12, 2)})
        if name.startswith("cfg3_"):
            depth = I.CFG3_DEPTH[int(name[6])]
            tot3_multi += depth * (t_multi + t_lin)
            tot3_best += depth * (best + t_lin)
            n3 += depth
        del Xd, Q, Y, ws
    return {"linears": rows,
            "cfg3_all_linears": {"count": n3, "ms_multi_kernel_route": round(tot3_multi * 1e-3, 4),
                                 "ms_faster_route_per_linear": round(tot3_best * 1e-3, 4)}}


def blocks_leg(layers, torch, tdq, iters=10, warm=5):
    """The paper's own granularity (one group per token and block of 32 channels) on the
    same inputs, outside the timed steps: tdq_quantize_act_blocks -> tdq_w4a4_linear_blocks
    per linear, HIP events on the launching stream.  The quantizer is one sweep of X (bytes:
    X read, codes and steps written); the contraction rescales every 32-wide block of K in
    binary32, 2 vector operations (convert, fused multiply-add) per output element and
    block, which bounds it by the vector unit rather than by the matrix cores."""
    res = {"layers": []}
    tot = tot6 = 0.0
    for L in layers:
        lc = L.lc
        p = tdq.block_params()
        KB = (lc.C + 31) // 32
        bs = torch.empty((lc.M, KB), dtype=torch.float32, device=L.X.device)
        Q = torch.zeros_like(L.Q)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        tq = tl = 0.0
        for it in range(warm + iters):
            ev[0].record()
            tdq.tdq_quantize_act_blocks(L.X, p, out=(Q, bs))
            ev[1].record()
            tdq.tdq_w4a4_linear_blocks(Q, bs, lc.C, L.Qw, L.w_scale, None, out=L.Y)
            ev[2].record()
            torch.cuda.synchronize()
            if it >= warm:
                tq += ev[0].elapsed_time(ev[1])
                tl += ev[1].elapsed_time(ev[2])
        tq, tl = tq / iters, tl / iters
        e = lc.M * lc.C
        qbytes = e * (2 if lc.dtype == "f16" else 4) + e // 2 + lc.M * KB * 4
        lane_ops = 2.0 * lc.M * lc.N * KB
        res["layers"].append({
            "layer": lc.name, "quantize_ms": round(tq, 4), "linear_ms": round(tl, 4),
            "quantize": {"bound": "hbm", "achieved": round(qbytes / (tq * 1e-3) / 1e9, 1),
                         "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(qbytes / (tq * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
            "linear": {"bound": "alu", "achieved": round(lane_ops / (tl * 1e-3) / 1e12, 2),
                       "peak": round(PEAK_VALU_TLOPS, 1), "unit": "T vector lane-ops/s",
                       "frac": round(lane_ops / (tl * 1e-3) / 1e12 / PEAK_VALU_TLOPS, 4),
                       "tops_int8": round(L.gemm_ops / (tl * 1e-3) / 1e12, 1)}})
        tot += tq + tl
        # the same granularity with the codes as bf6 operands of the 6-bit matrix instruction
        # (tdq_quantize_act_blocks_f6 -> tdq_w4a4_linear_blocks_f6): the same bits of Y,
        # 16 instead of 38 vector instructions per matrix instruction
        F = torch.empty((tdq.f6_bytes(lc.M, lc.C),), dtype=torch.uint8, device=L.X.device)
        W6 = tdq.tdq_pack_codes_f6(L.Qw, lc.C)                       # offline
        tq6 = tl6 = 0.0
        for it in range(warm + iters):
            ev[0].record()
            tdq.tdq_quantize_act_blocks_f6(L.X, p, out=(F, bs))
            ev[1].record()
            tdq.tdq_w4a4_linear_blocks_f6(F, bs, lc.C, W6, lc.N, L.w_scale, None, out=L.Y)
            ev[2].record()
            torch.cuda.synchronize()
            if it >= warm:
                tq6 += ev[0].elapsed_time(ev[1])
                tl6 += ev[1].elapsed_time(ev[2])
        tq6, tl6 = tq6 / iters, tl6 / iters
        q6bytes = e * (2 if lc.dtype == "f16" else 4) + tdq.f6_bytes(lc.M, lc.C) + lc.M * KB * 4
        res["layers"][-1]["f6_route"] = {
            "quantize_ms": round(tq6, 4), "linear_ms": round(tl6, 4),
            "quantize_gbs": round(q6bytes / (tq6 * 1e-3) / 1e9, 1),
            "linear_lane_tops": round(lane_ops / 2.0 / (tl6 * 1e-3) / 1e12, 2),
            "tops_int8": round(L.gemm_ops / (tl6 * 1e-3) / 1e12, 1)}
        tot6 += tq6 + tl6
        del F, W6
        # the same buffer read as a feature map [B, C, 64, 64] (the 4-D branch): re-layout
        # alone, and the per-block sweep reading the map in place
        Xc = L.X.reshape(lc.B, lc.C, 64, lc.T // 64)
        Xt = torch.empty_like(L.X)
        tt = tc = 0.0
        for it in range(warm + iters):
            ev[0].record()
            tdq.tdq_tokenize_chw(Xc, out=Xt)
            ev[1].record()
            tdq.tdq_quantize_act_blocks_chw(Xc, p, out=(Q, bs))
            ev[2].record()
            torch.cuda.synchronize()
            if it >= warm:
                tt += ev[0].elapsed_time(ev[1])
                tc += ev[1].elapsed_time(ev[2])
        tt, tc = tt / iters, tc / iters
        xb = e * (2 if lc.dtype == "f16" else 4)
        res["layers"][-1]["conv_layout"] = {
            "tokenize_ms": round(tt, 4), "tokenize_gbs": round(2 * xb / (tt * 1e-3) / 1e9, 1),
            "quantize_blocks_chw_ms": round(tc, 4),
            "quantize_blocks_chw_gbs": round(qbytes / (tc * 1e-3) / 1e9, 1)}
        del bs, Q, Xt
    res["ms_per_pass"] = round(tot, 4)
    res["ms_per_pass_f6_route"] = round(tot6, 4)
    # the token-set path overwrote nothing it needs: L.Y is rewritten by the next step
    return res


def f6_leg(layers, torch, tdq, iters=10, warm=5):
    """The same token-set path with the codes carried as bf6 operands of the 6-bit matrix
    instruction (tdq_quantize_act_f6 -> tdq_w4a4_linear_f6, bit-identical Y), outside the
    timed steps: the instruction runs at twice the int8 rate and needs no nibble expansion,
    but the operands are 0.75 instead of 0.5 bytes per code."""
    res = []
    for L in layers:
        lc = L.lc
        F = torch.empty((tdq.f6_bytes(lc.M, lc.C),), dtype=torch.uint8, device=L.X.device)
        W6 = tdq.tdq_pack_codes_f6(L.Qw, lc.C)                       # offline
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        tq = tl = 0.0
        for it in range(warm + iters):
            ev[0].record()
            tdq.tdq_quantize_act_f6(L.X, L.p, L.gid, L.clip, L.scale, out=F)
            ev[1].record()
            tdq.tdq_w4a4_linear_f6(F, L.gid, L.scale, lc.B, lc.T, lc.C, W6, lc.N, L.w_scale, None,
                                   out=L.Y)
            ev[2].record()
            torch.cuda.synchronize()
            if it >= warm:
                tq += ev[0].elapsed_time(ev[1])
                tl += ev[1].elapsed_time(ev[2])
        tq, tl = tq / iters, tl / iters
        res.append({"layer": lc.name, "quantize_f6_ms": round(tq, 4), "linear_f6_ms": round(tl, 4),
                    "linear_f6_tops": round(L.gemm_ops / (tl * 1e-3) / 1e12, 1),
                    "frac_of_fp6_peak": round(L.gemm_ops / (tl * 1e-3) / 1e12 / 10100.0, 4)})
        del F, W6
    return res


def quality(L, torch, tdq):
    """SQNR and zero-bin mass of the synthetic fc1 input under token-group DCRP and
    under naive per-image abs-max (one group, DCRP off), from the GPU's own codes."""
    lc = L.lc

    def measure(gid, scale, Q):
        lo = (Q[:, :lc.C // 2] & 0xF).to(torch.int8)
        hi = (Q[:, :lc.C // 2] >> 4).to(torch.int8)
        lo = torch.where(lo > 7, lo - 16, lo)
        hi = torch.where(hi > 7, hi - 16, hi)
        q = torch.stack((lo, hi), dim=-1).reshape(lc.M, lc.C)
        rs = scale.reshape(lc.B, -1).gather(1, gid.reshape(lc.B, -1).long()).reshape(lc.M, 1)
        x = L.X.reshape(lc.M, lc.C).float()
        err = x - q.float() * rs
        weak = torch.from_numpy(L.cls.reshape(-1) == 2).to(x.device)
        res = {}
        for nm, m in (("all", slice(None)), ("weak_tokens", weak)):
            sx = (x[m].double() ** 2).sum()
            se = (err[m].double() ** 2).sum()
            res["sqnr_db_" + nm] = round(float(10 * torch.log10(sx / se)), 2)
            res["rho0_" + nm] = round(float((q[m] == 0).float().mean()), 4)
        return res

    out = {"tdq": measure(L.gid, L.scale, L.Q)}
    # which term of the projection set each token set's radius (Eq. dcrp), and the
    # step-to-dispersion ratio eta = Delta / sigma of the sets (Eq. cg_Delta_eta)
    _, _, _, stats, _ = tdq.tdq_calibrate_groups(L.X, L.p, want_stats=True)
    st = tdq.stats_to_numpy(stats)
    names = ("base", "c1_tau", "c2_zr", "eps_floor", "empty")
    out["tdq"]["bind_counts"] = {n: int((st["bind"] == i).sum()) for i, n in enumerate(names)}
    used = st["n"] > 0
    out["tdq"]["eta_max"] = round(float((st["scale"][used] / st["sigma"][used]).max()), 4)
    # range disparity D(X) = max |x| / median_t median_c |x| (Eq. range_disparity) of every
    # image, on the device; reported: the median and the largest over the batch
    D, _, _ = tdq.tdq_range_disparity(L.X)
    out["range_disparity"] = {"median_over_images": round(float(D.median()), 1),
                              "max_over_images": round(float(D.max()), 1)}
    p1 = tdq.default_params(1, flags=0)
    gid1, clip1, scale1, _, _ = tdq.tdq_calibrate_groups(L.X, p1)
    Q1 = tdq.tdq_quantize_act(L.X, p1, gid1, clip1, scale1)
    out["per_image_absmax"] = measure(gid1, scale1, Q1)
    torch.cuda.synchronize()
    return out


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _oracle_stages(O, X, W, G, np):
    """The oracle's steps on X[B, T, C] (and W[N, C] or None), timed one by one: per-token
    ranges + assignment, per-set moments + rank select + projection, quantize, and the
    integer contraction with its epilogue.  Only calls into oracle/; the loop over images and
    sets is the one of `calibrate_groups`, opened up so that the stages can be timed apart."""
    p = O.Params(n_groups=G)
    B, T, C = X.shape
    t = [0.0, 0.0, 0.0, 0.0]
    gid = np.zeros((B, T), np.int32)
    clip = np.zeros((B, G), np.float32)
    scale = np.zeros((B, G), np.float32)
    for b in range(B):
        t0 = time.perf_counter()
        gid[b] = O.assign_groups(O.token_range(X[b]), G)
        t1 = time.perf_counter()
        for j in range(G):
            s = O.dcrp_group(X[b][gid[b] == j], p)
            clip[b, j], scale[b, j] = s["clip"], s["scale"]
        t[0] += t1 - t0
        t[1] += time.perf_counter() - t1
    t0 = time.perf_counter()
    q = O.quantize_act(X, gid, clip, scale, p)
    t[2] = time.perf_counter() - t0
    if W is not None:
        qw, sw = O.quantize_weight(W)
        t0 = time.perf_counter()
        O.w4a4_linear(q.reshape(B * T, C), O.row_scales(gid, scale), qw, sw)
        t[3] = time.perf_counter() - t0
    return t, q


def cpu_baseline(layers, np, I, budget_s=14.0):
    """The CPU oracle, as it stands, on the host cores of this machine (numpy runs these loops and
    its integer matmul on one thread): configurations 0 and 1 in full, and a bounded sample
    of the timed workload -- the activation path (calibrate + quantize) of the first images
    of both linears' inputs, and the contraction of the first rows of fc1 -- each sized from a
    small probe so that the whole leg takes about budget_s seconds.  Seconds per stage:
    ranges + assignment / moments + rank select + projection / quantize / contraction."""
    from oracle import tdq_oracle as O

    names = ("stats_assign_s", "select_project_s", "quantize_s", "contraction_s")
    full = {}
    for name in ("cfg0", "cfg1"):
        lc = I.case(name)
        X, _ = I.make_activations(lc)
        t, _ = _oracle_stages(O, X, I.make_weight(lc), lc.G, np)
        e = lc.M * lc.C
        full[name] = dict(zip(names, (round(v, 5) for v in t)))
        full[name]["act_gbs"] = round(e * ((2 if lc.dtype == "f16" else 4) + 0.5) / sum(t[:3]) / 1e9, 4)
        full[name]["linear_tops"] = round(2.0 * lc.M * lc.N * lc.C / t[3] / 1e12, 6)

    t_act, e_act, parts, q1 = [0.0, 0.0, 0.0], 0, [], None
    for L in layers:
        t1, _ = _oracle_stages(O, L.X_host[:1], None, L.lc.G, np)
        nimg = int(max(1, min(L.lc.B, round(budget_s / 4 / max(sum(t1), 1e-3)))))
        t, q = _oracle_stages(O, L.X_host[:nimg], None, L.lc.G, np)
        for s in range(3):
            t_act[s] += t[s]
        e = nimg * L.lc.T * L.lc.C
        e_act += e
        parts.append(f"{nimg} of {L.lc.B} images of {L.lc.name} ({e} elements, {sum(t):.2f} s)")
        if q1 is None:
            q1 = q
    lc = layers[0].lc
    qw = np.random.Generator(np.random.PCG64(1)).integers(-7, 8, (lc.N, lc.C), dtype=np.int8)
    q2 = q1.reshape(-1, lc.C)
    ones_n = np.ones(lc.N, np.float32)

    def mm(rows):
        t0 = time.perf_counter()
        O.w4a4_linear(q2[:rows], np.ones(rows, np.float32), qw, ones_n)
        return time.perf_counter() - t0

    t16 = mm(16)
    rows = int(max(16, min(q2.shape[0], round(16 * budget_s / 2 / max(t16, 1e-3)))))
    t_mm = mm(rows)
    return {"value": round(e_act * 2.5 / sum(t_act) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "activation path (calibrate+quantize) of " + " and ".join(parts) +
                      f"; contraction of {rows} rows x {lc.N} x {lc.C}: {t_mm:.2f} s",
            "stage_seconds_of_sample": dict(zip(names, (round(v, 3) for v in (*t_act, t_mm)))),
            "linear_tops": round(2 * rows * lc.N * lc.C / t_mm / 1e12, 6),
            "configs_in_full": full,
            "cpu_model": _cpu_model(), "host_cpus_visible": os.cpu_count()}


if __name__ == "__main__":
    main()
