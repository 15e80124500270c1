#!/usr/bin/env python3
"""Benchmark of the DSTG+DCRP W4A4 linear hot path on one MI355X.

A step is one pass of the whole hot path over one batch of the ViT-L-shaped
stress workload (config 4: batch 32, 4096 tokens, fc1 1024->4096 and fc2
4096->1024, 32 token groups per image): for each of the two linears
tdq_calibrate_groups -> tdq_quantize_act -> tdq_w4a4_linear.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--heavy 10] [--small]
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
# vector lane operations per second: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz (one fp32
# FMA per lane per clock is the published 78.6 TFLOP/s of unpacked fp32)
PEAK_VALU_TLOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# HBM bytes per launch of the fc1 contraction on the default workload, from the
# FETCH_SIZE + WRITE_SIZE counters (see profiles/bench_cfg4_hbm_traffic_pmc.txt)
GEMM_FC1_TRAFFIC_BYTES = 1182249898


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps first; the clocks take about 20 steps to settle")
    ap.add_argument("--heavy", type=int, default=10, choices=(2, 10, 25),
                    help="heavy-tailed token fraction of config 4, percent")
    ap.add_argument("--small", action="store_true",
                    help="4 images instead of 32 (quick functional run, not the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain device copy of 1 GiB (a kernel of known traffic, "
                         "used to scale the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
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
        for li, L in enumerate(layers):
            lc = L.lc
            if events is not None:
                events[li][0].record()
            tdq.tdq_calibrate_groups(L.X, L.p, L.ws, out=(L.gid, L.clip, L.scale))
            if events is not None:
                events[li][1].record()
            tdq.tdq_quantize_act(L.X, L.p, L.gid, L.clip, L.scale, out=L.Q)
            if events is not None:
                events[li][2].record()
            tdq.tdq_w4a4_linear(L.Q, L.gid, L.scale, lc.B, lc.T, lc.C, L.Qw, L.w_scale, None,
                                out=L.Y)
            if events is not None:
                events[li][3].record()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    all_events = [[[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in layers]
                  for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(args.steps):
        step(all_events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps

    seg_ms = np.zeros((len(layers), 3))
    for ev in all_events:
        for li in range(len(layers)):
            for s in range(3):
                seg_ms[li, s] += ev[li][s].elapsed_time(ev[li][s + 1])
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

    # The dominant kernel of a step: the fc1 contraction, k_w4a4_gemm_wide<_Float16>,
    # one launch per step (tdq_w4a4_linear launches nothing else), timed by the HIP
    # events around that entry point on the stream it runs on.  Algorithmic work per
    # launch = 2 M N K integer operations.  `traffic` is the HBM bytes per launch
    # measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled on a 1 GiB copy)
    # for exactly this workload; it is not known for other --heavy / --small settings.
    fc1_ms = float(seg_ms[0, 2])
    fc1_tops = fc1.gemm_ops / (fc1_ms * 1e-3) / 1e12
    traffic = GEMM_FC1_TRAFFIC_BYTES if (fc1.lc.B == 32 and args.heavy == 10) else None
    roofline = {"kernel": "k_w4a4_gemm_wide<_Float16> (fc1 contraction, M=131072 K=1024 N=4096)",
                "bound": "mfma", "achieved": round(fc1_tops, 1), "peak": PEAK_INT8_TOPS,
                "unit": "TOP/s", "frac": round(fc1_tops / PEAK_INT8_TOPS, 4), "traffic": traffic,
                "avg_launch_ms": round(fc1_ms, 4), "ops_per_launch": fc1.gemm_ops,
                "algorithmic_bytes": fc1.gemm_bytes}

    out = {
        "metric": "DSTG+DCRP act-quant GB/s + W4A4 linear TOPS (% of HBM / int8 MFMA peak)",
        "value": round(act_gbs, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
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
    if not args.no_blocks:
        out["paper_literal_blocks"] = blocks_leg(layers, torch, tdq)
        out["f6_contraction"] = f6_leg(layers, torch, tdq)
    if not args.no_quality:
        out["quality"] = quality(fc1, torch, tdq)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layers, np)
    print(json.dumps(out), flush=True)


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
        F = torch.empty((tdq.f6_bytes(lc.M, lc.C),), dtype=torch.uint8, device=L.X.device)
        tc6 = 0.0
        for it in range(warm + iters):
            ev[0].record()
            tdq.tdq_quantize_act_blocks_chw_f6(Xc, p, out=(F, bs))
            ev[1].record()
            torch.cuda.synchronize()
            if it >= warm:
                tc6 += ev[0].elapsed_time(ev[1])
        tc6 /= iters
        xb = e * (2 if lc.dtype == "f16" else 4)
        res["layers"][-1]["conv_layout"] = {
            "tokenize_ms": round(tt, 4), "tokenize_gbs": round(2 * xb / (tt * 1e-3) / 1e9, 1),
            "quantize_blocks_chw_ms": round(tc, 4),
            "quantize_blocks_chw_gbs": round(qbytes / (tc * 1e-3) / 1e9, 1),
            "quantize_blocks_chw_f6_ms": round(tc6, 4),
            "quantize_blocks_chw_f6_gbs": round(q6bytes / (tc6 * 1e-3) / 1e9, 1)}
        del bs, Q, Xt, F
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


def cpu_baseline(layers, np, budget_s=16.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the
    activation path (calibrate + quantize) of the first images of both linears'
    inputs, and the contraction of the first rows of fc1, each sized from a small
    probe so that the whole leg takes about budget_s seconds.  Host cores of this machine;
    numpy runs these loops and its integer matmul on one thread."""
    from oracle import tdq_oracle as O

    def act(L, n):
        X = L.X_host[:n]
        p = O.Params(n_groups=L.lc.G)
        t0 = time.perf_counter()
        gid, clip, scale, _ = O.calibrate_groups(X, p)
        q = O.quantize_act(X, gid, clip, scale, p)
        return time.perf_counter() - t0, X.size, q

    t_act, e_act, parts, q1 = 0.0, 0, [], None
    for L in layers:
        t1, e1, _ = act(L, 1)
        nimg = int(max(1, min(L.lc.B, round(budget_s / 4 / max(t1, 1e-3)))))
        t, e, q = act(L, nimg)
        t_act += t
        e_act += e
        parts.append(f"{nimg} of {L.lc.B} images of {L.lc.name} ({e} elements, {t:.2f} s)")
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
    return {"value": round(e_act * 2.5 / t_act / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "activation path (calibrate+quantize) of " + " and ".join(parts) +
                      f"; contraction of {rows} rows x {lc.N} x {lc.C}: {t_mm:.2f} s",
            "linear_tops": round(2 * rows * lc.N * lc.C / t_mm / 1e12, 6),
            "host_cpus_visible": os.cpu_count()}


if __name__ == "__main__":
    main()
