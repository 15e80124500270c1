"""GPU parity on seeded random VALID draws for the entry points beside the token-set
path of test_gpu_random_shapes.py: the per-(token, block) quantizer and its contraction
(nibble and 6-bit storage), the single-launch path, the conv-layout readers, the set
diagnostics and the range disparity.  Every draw is checked with the bars of the
hand-picked cases (the helpers are theirs); the draws combine what those keep apart:
ragged shapes with padded rows, both input types, every flag combination, the percentile
base radius, offset data, constant and all-zero tokens."""
import numpy as np
import pytest
import torch

from oracle import tdq_oracle as O
from paper_2604_16855_amd import inputs as I
from paper_2604_16855_amd import tdq

import parity_util as U
import test_gpu_blocks as TB
import test_gpu_fused as TF
from test_gpu_f6 import f6_fragments

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _activations(rng, B, T, C, dtype, kind, case):
    if kind == "offset":
        return I.offset_activations(B, T, C, dtype, float(rng.choice([10, 100, 1000])), seed=case,
                                    token_jitter=0.05, outlier_head=bool(rng.integers(0, 2)))
    X = rng.laplace(0, 1, (B, T, C)) * rng.lognormal(0, 1.5, (B, T, 1))
    if kind == "outliers":
        X[rng.random((B, T, C)) < 0.02] *= 30.0
    if kind == "const":
        X[:, ::3, :] = 0.75
    if kind == "zeros_some":
        X[:, 1::2, :] = 0.0
        X[:, :, C // 2:] *= (rng.random((B, T, C - C // 2)) < 0.3)
    return np.clip(X, -60000.0, 60000.0).astype(np.float16 if dtype == "f16" else np.float32)


def _kind(rng):
    return str(rng.choice(["mix", "outliers", "offset", "const", "zeros_some"]))


# ------------------------------------------------------------- per-(token, block) quantizer
@pytest.mark.parametrize("seed", [21, 22, 23])
def test_random_block_quantizer(seed):
    """tdq_quantize_act_blocks against Algorithm 1 steps 1-9 of the oracle; the 6-bit
    variant writes the same steps and radii and the fragments of the same codes."""
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(16):
        B = int(rng.integers(1, 4))
        T = int(rng.choice([1, 2, 7, 63, 64, 65, 121, 300]))
        C = int(rng.choice([1, 3, 31, 32, 33, 64, 70, 100, 320, 544, 1000, 1024, 2056, 4096]))
        if B * T * -(-C // 32) > 12000:
            T = max(1, 12000 // (B * -(-C // 32)))
        dtype = str(rng.choice(["f16", "f32"]))
        kind = _kind(rng)
        X = _activations(rng, B, T, C, dtype, kind, 100 * seed + case)
        p = tdq.block_params(tau=float(rng.choice([0.3, 1.0, 2.0])), zr=float(rng.choice([0.05, 0.2, 0.3, 0.5, 0.9])),
                             flags=int(rng.integers(0, 4)), base_pct=float(rng.choice([0.0, 0.0, 0.9, 0.5])))
        ld_pad = int(rng.choice([0, 0, 3, 8]))
        _say(f"[random blocks {seed}.{case}] {kind}")
        Q, bs, q_gpu, _ = TB._check_block_quantizer(X, p, ld_pad)
        Xd = U.to_device(X, ld_pad)
        bc = tdq.tdq_quantize_act_blocks(Xd, p, want_clip=True)[2]
        F = torch.full((tdq.f6_bytes(B * T, C),), 0xA5, dtype=torch.uint8, device=U.dev())
        F, bs6, bc6 = tdq.tdq_quantize_act_blocks_f6(Xd, p, want_clip=True,
                                                     out=(F, torch.full_like(bs, float("nan"))))
        torch.cuda.synchronize()
        assert torch.equal(bs6, bs) and torch.equal(bc6, bc)
        assert np.array_equal(F.cpu().numpy(), f6_fragments(q_gpu))


@pytest.mark.parametrize("seed", [31, 32])
def test_random_block_quantizer_conv_layout(seed):
    """tdq_quantize_act_blocks_chw on a strided view of a feature map: the bits of the
    token-major sweep on the tokenized map, which the oracle checks."""
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(12):
        B, C = int(rng.integers(1, 4)), int(rng.choice([1, 7, 32, 40, 72, 100, 128, 130, 256, 320, 1024]))
        H, W = int(rng.choice([1, 3, 5, 8, 12, 16, 22])), int(rng.choice([1, 3, 5, 8, 12, 16, 22]))
        dtype = str(rng.choice(["f16", "f32"]))
        oc, oh = int(rng.integers(0, 3)), int(rng.integers(0, 2))
        Xf = _activations(rng, B, H + oh, (C + oc) * W, dtype, _kind(rng), 100 * seed + case)
        Xf = np.ascontiguousarray(Xf.reshape(B, H + oh, C + oc, W).transpose(0, 2, 1, 3))
        p = tdq.block_params(tau=float(rng.choice([0.3, 1.0])), zr=float(rng.choice([0.05, 0.2, 0.3])),
                             flags=int(rng.integers(0, 4)), base_pct=float(rng.choice([0.0, 0.0, 0.9])))
        _say(f"[random blocks-chw {seed}.{case}] B={B} C={C} H={H} W={W} {dtype} view +{oc} channels +{oh} rows "
             f"flags={p.flags} tau={p.tau} zr={p.zr} pct={p.base_pct}")
        Xd = torch.from_numpy(Xf).to(U.dev())[:, oc:oc + C, :H, :]
        Q, bs, bc = tdq.tdq_quantize_act_blocks_chw(Xd, p, want_clip=True)
        Xt = tdq.tdq_tokenize_chw(Xd)
        Q2, bs2, bc2 = tdq.tdq_quantize_act_blocks(Xt, p, want_clip=True)
        torch.cuda.synchronize()
        Xt_ref = O.tokenize_chw(Xf[:, oc:oc + C, :H, :])
        assert np.array_equal(Xt.cpu().numpy().view(np.uint8), Xt_ref.view(np.uint8))
        assert torch.equal(Q, Q2) and torch.equal(bs, bs2) and torch.equal(bc, bc2)
        if B * H * W * -(-C // 32) <= 12000:
            TB._check_block_quantizer(Xt_ref, p)


# ---------------------------------------------------------------- block-scaled contraction
@pytest.mark.parametrize("seed", [41, 42])
def test_random_block_scaled_linear(seed):
    """tdq_w4a4_linear_blocks within the bound of the binary32 evaluation of Algorithm 1
    step 10; tdq_w4a4_linear_blocks_f6 gives the same bits."""
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(14):
        M = int(rng.choice([1, 5, 31, 64, 129, 200, 256, 300, 513]))
        K = int(rng.choice([1, 31, 32, 33, 64, 96, 128, 320, 1000, 1280, 2048, 4100]))
        N = int(rng.choice([1, 3, 64, 129, 130, 200, 256, 320]))
        out_dtype = torch.float16 if rng.integers(0, 3) == 0 else torch.float32
        ld_s_pad = int(rng.choice([0, 0, 1, 4]))
        codes, bscale, qw, w_scale, bias = TB._random_block_operands(
            M, K, N, 100 * seed + case, spread=1.0 if out_dtype == torch.float16 else 5.0)
        if rng.integers(0, 2):
            bias = None
        _say(f"[random blocks-linear {seed}.{case}]")
        Y = TB._check_blocks_linear(codes, bscale, qw, w_scale, bias, out_dtype, ld_s_pad)
        KB = -(-K // 32)
        bs_buf = torch.full((M, KB + ld_s_pad), float("nan"), dtype=torch.float32)
        bs_buf[:, :KB] = torch.from_numpy(bscale)
        Y6 = tdq.tdq_w4a4_linear_blocks_f6(
            torch.from_numpy(f6_fragments(codes)).to(U.dev()), bs_buf.to(U.dev())[:, :KB], K,
            torch.from_numpy(f6_fragments(qw)).to(U.dev()), N, torch.from_numpy(w_scale).to(U.dev()),
            None if bias is None else torch.from_numpy(bias).to(U.dev()), out_dtype)
        torch.cuda.synchronize()
        assert np.array_equal(Y6.cpu().numpy().astype(np.float64), Y)


# --------------------------------------------------------------------- single-launch path
@pytest.mark.parametrize("seed", [51, 52])
def test_random_single_launch_path(seed):
    """tdq_calibrate_quantize_fused with the bars of the multi-kernel path, and the same
    set ids, thresholds and base radii as that path."""
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(16):
        B = int(rng.integers(1, 5))
        T = int(rng.choice([1, 2, 7, 63, 64, 65, 121, 300, 484, 1500]))
        C = int(rng.choice([1, 3, 8, 31, 33, 64, 70, 128, 320, 520, 1024, 2050]))
        if B * T * C > 600_000:
            T = max(1, 600_000 // (B * C))
        G = int(rng.choice([1, 2, 3, 5, 8, 16, 32, 64]))
        dtype = str(rng.choice(["f16", "f32"]))
        kind = _kind(rng)
        X = _activations(rng, B, T, C, dtype, kind, 100 * seed + case)
        p = tdq.default_params(G, tau=float(rng.choice([0.3, 1.0, 2.0])),
                               zr=float(rng.choice([0.01, 0.2, 0.5, 0.9])), flags=int(rng.integers(0, 4)))
        p.base_pct = float(rng.choice([0.0, 0.0, 0.99, 0.5]))
        ld_pad = int(rng.choice([0, 0, 3, 8]))
        _say(f"[random fused {seed}.{case}] {kind} tau={p.tau} zr={p.zr}")
        g = TF._check(X, p, ld_pad)
        h = U.gpu_calibrate(X, p, ld_pad)
        assert np.array_equal(g["gid"], h["gid"])
        assert np.array_equal(g["stats"]["thr"], h["stats"]["thr"])
        assert np.array_equal(g["stats"]["c_base"], h["stats"]["c_base"])


# ----------------------------------------------------- token sets read from the conv layout
@pytest.mark.parametrize("seed", [61, 62])
def test_random_token_sets_conv_layout(seed):
    """tdq_calibrate_groups_chw on a strided view: an exact token-major copy, and the
    oracle's ids, thresholds, radii and steps on the oracle's tokens."""
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(12):
        B, C = int(rng.integers(1, 4)), int(rng.choice([1, 7, 32, 64, 72, 100, 130, 320, 1024]))
        H, W = int(rng.choice([1, 3, 7, 8, 12, 16, 22, 32])), int(rng.choice([1, 3, 7, 8, 12, 16, 22, 32]))
        G = int(rng.choice([1, 2, 3, 5, 8, 16, 32, 65, 129]))
        dtype = str(rng.choice(["f16", "f32"]))
        oc, oh = int(rng.integers(0, 3)), int(rng.integers(0, 2))
        Xf = _activations(rng, B, H + oh, (C + oc) * W, dtype, _kind(rng), 100 * seed + case)
        Xf = np.ascontiguousarray(Xf.reshape(B, H + oh, C + oc, W).transpose(0, 2, 1, 3))
        p = tdq.default_params(G, tau=float(rng.choice([0.3, 1.0])), zr=float(rng.choice([0.05, 0.2, 0.5])),
                               flags=int(rng.integers(0, 4)))
        p.base_pct = float(rng.choice([0.0, 0.0, 0.99]))
        _say(f"[random calibrate-chw {seed}.{case}] B={B} C={C} H={H} W={W} G={G} {dtype} view +{oc} channels "
             f"+{oh} rows flags={p.flags} tau={p.tau} zr={p.zr} pct={p.base_pct}")
        Xd = torch.from_numpy(Xf).to(U.dev())[:, oc:oc + C, :H, :]
        Xt, gid, clip, scale, stats, ws = tdq.tdq_calibrate_groups_chw(Xd, p, want_stats=True)
        torch.cuda.synchronize()
        Xt_ref = O.tokenize_chw(Xf[:, oc:oc + C, :H, :])
        assert np.array_equal(Xt.cpu().numpy().view(np.uint8), Xt_ref.view(np.uint8))
        assert tdq.device_status(ws) == 0
        g = dict(gid=gid.cpu().numpy(), clip=clip.cpu().numpy(), scale=scale.cpu().numpy(),
                 stats=tdq.stats_to_numpy(stats))
        U.assert_calibration_matches(g, Xt_ref, p)


# ---------------------------------------------------------- diagnostics and range disparity
@pytest.mark.parametrize("seed", [71, 72])
def test_random_diagnostics_and_disparity(seed):
    """Zero-bin and clipped counts per set (Eq. rho0_def) with user radii of any size,
    exactly; D(X) of Eq. (range_disparity) with its medians and maxima, exactly."""
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(14):
        B = int(rng.integers(1, 4))
        T = int(rng.choice([1, 2, 7, 64, 65, 121, 300, 1000]))
        C = int(rng.choice([1, 2, 3, 8, 9, 31, 33, 64, 70, 320, 1000, 1024, 2050, 4096]))
        if B * T * C > 1_000_000:
            T = max(1, 1_000_000 // (B * C))
        G = int(rng.choice([1, 2, 3, 8, 32, 64, 100]))
        dtype = str(rng.choice(["f16", "f32"]))
        kind = _kind(rng)
        ld_pad = int(rng.choice([0, 0, 4, 7]))
        X = _activations(rng, B, T, C, dtype, kind, 100 * seed + case)
        _say(f"[random diag {seed}.{case}] B={B} T={T} C={C} G={G} {dtype} {kind} ld_pad={ld_pad}")
        Xd = U.to_device(X, ld_pad)
        D, med, mx = tdq.tdq_range_disparity(Xd)
        torch.cuda.synchronize()
        Dr, medr, mxr = O.range_disparity(X)
        assert np.array_equal(med.cpu().numpy(), medr)
        assert np.array_equal(mx.cpu().numpy(), mxr)
        assert np.array_equal(D.cpu().numpy(), Dr, equal_nan=True)
        # radii and steps of the caller's choosing, unrelated to the data's own
        p = tdq.default_params(G)
        gid = rng.integers(0, G, (B, T)).astype(np.int32)
        scale = np.exp(rng.normal(-2, 2, (B, G))).astype(np.float32)
        clip = (scale * np.float32(7.5) * rng.choice([0.25, 1.0, 1.0, 4.0], (B, G))).astype(np.float32)
        gid_d = torch.from_numpy(gid).to(U.dev())
        zero, clipped = tdq.tdq_group_diagnostics(Xd, p, gid_d if G > 1 else None,
                                                  torch.from_numpy(clip).to(U.dev()),
                                                  torch.from_numpy(scale).to(U.dev()))
        torch.cuda.synchronize()
        if G == 1:
            gid[:] = 0
        q = O.quantize_act(X, gid, clip, scale, U.oracle_params(p))
        zr = np.zeros((B, G), np.int64)
        cr = np.zeros((B, G), np.int64)
        for b in range(B):
            for j in range(G):
                m = gid[b] == j
                zr[b, j] = int((q[b][m] == 0).sum())
                cr[b, j] = int((np.abs(X[b][m].astype(np.float32)) > clip[b, j]).sum())
        assert np.array_equal(zero.cpu().numpy(), zr)
        assert np.array_equal(clipped.cpu().numpy(), cr)
