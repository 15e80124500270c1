"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on the same seeded inputs.  Stage-wise protocol: every stage is
checked (i) end to end from X and (ii) in isolation, fed the oracle's upstream
outputs, where group ids, codes and accumulators must be bit-exact."""
import numpy as np
import pytest
import torch

from oracle import tdq_oracle as O
from paper_2604_16855_amd import inputs as I
from paper_2604_16855_amd import tdq

import parity_util as U

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _full_path(lc, p, X, W, bias=None, ld_pad=0, out_dtype=torch.float32):
    """Runs calibrate -> quantize -> linear on the GPU and checks every stage."""
    B, T, C = X.shape
    N = W.shape[0]
    _say(f"[case] {lc} B={B} T={T} C={C} N={N} G={p.n_groups} dtype={X.dtype} ld_pad={ld_pad}")
    g = U.gpu_calibrate(X, p, ld_pad)
    assert g["status"] == 0
    gid, clip, scale, st = U.assert_calibration_matches(g, X, p)
    op = U.oracle_params(p)

    # (ii) quantizer in isolation: oracle gid / clip / step in, codes bit-exact out
    gid_d = torch.from_numpy(gid).to(U.dev())
    clip_d = torch.from_numpy(clip).to(U.dev())
    scale_d = torch.from_numpy(scale).to(U.dev())
    Q_iso = tdq.tdq_quantize_act(g["Xd"], p, gid_d, clip_d, scale_d)
    q_ref = O.quantize_act(X, gid, clip, scale, op).reshape(B * T, C)
    q_iso = U.unpack_device_codes(Q_iso, C)
    assert np.array_equal(q_iso, q_ref), "codes differ given identical scales"
    if C % 2:      # the pad nibble of an odd row is zero
        assert not (Q_iso.cpu().numpy()[:, C // 2] >> 4).any()

    # (i) quantizer end to end: GPU's own calibration
    Q_e2e = tdq.tdq_quantize_act(g["Xd"], p, g["gid_d"], g["clip_d"], g["scale_d"])
    q_e2e = U.unpack_device_codes(Q_e2e, C)
    rows = np.arange(B)[:, None]
    c_row = clip[rows, gid].reshape(-1)
    d_row = scale[rows, gid].reshape(-1)
    exact = np.array_equal(g["scale"], scale) and np.array_equal(g["clip"], clip)
    flips = U.assert_codes_match(q_e2e, q_ref, X, c_row, d_row, exact)
    _say(f"  scales bit-identical: {exact}; code flips end-to-end: {flips}")

    # weights: offline quantizer parity
    Wd = torch.from_numpy(W).to(U.dev())
    Qw_d, ws_d = tdq.tdq_quantize_weight(Wd)
    qw_ref, sw_ref = O.quantize_weight(W)
    assert np.array_equal(U.unpack_device_codes(Qw_d, C), qw_ref)
    assert np.array_equal(ws_d.cpu().numpy(), sw_ref)

    # (ii) contraction in isolation: oracle codes and scales in
    bias_d = None if bias is None else torch.from_numpy(bias).to(U.dev())
    acc, Y = U.gpu_linear(Q_iso, gid_d, scale_d, B, T, C, Qw_d, ws_d, bias_d, out_dtype)
    acc_ref, Y_ref = O.w4a4_linear(q_ref, O.row_scales(gid, scale), qw_ref, sw_ref, bias)
    assert np.array_equal(acc, acc_ref), "int32 accumulators differ"
    if out_dtype == torch.float16:
        assert np.array_equal(Y, Y_ref.astype(np.float16))
    else:
        assert np.array_equal(Y, Y_ref), "fp32 epilogue differs given identical inputs"

    # (i) contraction end to end; the oracle contraction re-run on the GPU's codes
    acc2, Y2 = U.gpu_linear(Q_e2e, g["gid_d"], g["scale_d"], B, T, C, Qw_d, ws_d, bias_d, out_dtype)
    acc2_ref, Y2_ref = O.w4a4_linear(q_e2e, O.row_scales(g["gid"], g["scale"]), qw_ref, sw_ref,
                                     bias)
    assert np.array_equal(acc2, acc2_ref)
    if out_dtype == torch.float32:
        assert np.array_equal(Y2, Y2_ref)
        if flips == 0:
            floor = 0 if bias is None else np.abs(bias)[None, :]
            err = np.abs(Y2.astype(np.float64) - Y_ref)
            assert (err <= U.OUT_RTOL * (np.abs(Y_ref) + floor) + 1e-30).all()
    return g


# --------------------------------------------------------------- named configs
def test_cfg0_fp32_full_path():
    lc = I.case("cfg0")
    X, _ = I.make_activations(lc)
    _full_path("cfg0", tdq.default_params(lc.G), X, I.make_weight(lc), I.make_bias(lc))


def test_cfg1_fp16_full_path():
    lc = I.case("cfg1")
    X, _ = I.make_activations(lc)
    _full_path("cfg1", tdq.default_params(lc.G), X, I.make_weight(lc))


@pytest.mark.parametrize("name", ["cfg2_qkv", "cfg2_proj", "cfg2_fc2"])
def test_cfg2_linears(name):
    lc = I.case(name, B=4)          # 4 of the 16 images keep the oracle's GEMM to seconds
    X, _ = I.make_activations(lc)
    _full_path(name, tdq.default_params(lc.G), X, I.make_weight(lc))


def test_cfg2_activation_path_full_batch():
    lc = I.case("cfg2_fc1")
    X, _ = I.make_activations(lc)
    p = tdq.default_params(lc.G)
    g = U.gpu_calibrate(X, p)
    U.assert_calibration_matches(g, X, p)


@pytest.mark.parametrize("name", sorted(n for n in I.CASES if n.startswith("cfg3_")))
def test_cfg3_shapes(name):
    """Every distinct linear of the 4-stage encoder set (20 shapes), two images each."""
    lc = I.case(name, B=2)
    X, _ = I.make_activations(lc)
    _full_path(name, tdq.default_params(lc.G), X, I.make_weight(lc), I.make_bias(lc))


# --------------------------------------------------- ragged / unaligned shapes
@pytest.mark.parametrize("B,T,C,N,G,dtype,ld_pad", [
    (3, 37, 70, 19, 5, "f16", 0),      # C not a multiple of 8
    (2, 50, 33, 7, 4, "f16", 0),       # odd C: pad nibble
    (2, 41, 64, 130, 8, "f16", 3),     # row stride not a multiple of 8: scalar loads
    (1, 1, 8, 1, 4, "f32", 0),         # a single token
    (2, 3, 24, 5, 16, "f16", 0),       # more token sets than tokens
    (2, 129, 100, 257, 32, "f32", 1),  # tile tails everywhere
    (1, 300, 520, 96, 1, "f16", 0),    # one token set = per-image quantization
    (1, 64, 2050, 40, 8, "f16", 0),    # many K stages plus a ragged last one
])
def test_ragged_shapes(B, T, C, N, G, dtype, ld_pad):
    lc = I.LinearCase("ragged", B, T, C, N, G, dtype, 0.1, 0.1, False, (T, 1), 500 + C)
    X, _ = I.make_activations(lc)
    _full_path("ragged", tdq.default_params(G), X, I.make_weight(lc), I.make_bias(lc), ld_pad)


@pytest.mark.parametrize("flags,tau,zr", [(0, 1.0, 0.2), (1, 0.3, 0.2), (2, 1.0, 0.05),
                                          (3, 0.5, 0.5), (3, 2.0, 0.9)])
def test_dcrp_variants(flags, tau, zr):
    lc = I.case("cfg1", grid=(40, 40))
    X, _ = I.make_activations(lc)
    p = tdq.default_params(lc.G, tau=tau, zr=zr, flags=flags)
    g = _full_path(f"variants flags={flags}", p, X, I.make_weight(lc))
    binds = set(int(b) for b in g["stats"]["bind"])
    if flags == 0:
        assert binds <= {0, 4}
    if flags == 1:
        assert 2 not in binds
    if flags == 2:
        assert 1 not in binds


def test_fp16_output():
    lc = I.case("cfg2_proj", B=2)
    X, _ = I.make_activations(lc)
    _full_path("fp16 out", tdq.default_params(lc.G), X, I.make_weight(lc), I.make_bias(lc),
               out_dtype=torch.float16)


# ------------------------------------------------------------ degenerate input
def test_degenerate_groups():
    rng = np.random.Generator(np.random.PCG64(9))
    X = rng.laplace(0, 1, (4, 40, 32)).astype(np.float16)
    X[0] = 0                      # an all-zero image: every clip on the eps floor
    X[1] = np.float16(2.5)        # a constant image: sigma = 1e-12, codes +1
    X[2, :20] = 0                 # zero tokens beside normal ones (24-octave floor)
    X[3, :, ::2] = 0              # half the elements exactly zero: thr = 0
    p = tdq.default_params(4)
    g = U.gpu_calibrate(X, p)
    gid, clip, scale, st = U.assert_calibration_matches(g, X, p)
    assert (g["clip"][0] == np.float32(1e-8)).all() and (g["clip"][1] == np.float32(1e-8)).all()
    Q = tdq.tdq_quantize_act(g["Xd"], p, g["gid_d"], g["clip_d"], g["scale_d"])
    q = U.unpack_device_codes(Q, 32)
    q_ref = O.quantize_act(X, gid, clip, scale, U.oracle_params(p)).reshape(-1, 32)
    exact = np.array_equal(g["scale"], scale)
    U.assert_codes_match(q, q_ref, X, clip[np.arange(4)[:, None], gid].reshape(-1),
                         scale[np.arange(4)[:, None], gid].reshape(-1), exact)
    assert not q[:40].any() and (q[40:80] == 1).all()


def test_nonfinite_flag():
    X = np.ones((2, 16, 16), dtype=np.float16)
    p = tdq.default_params(2)
    assert U.gpu_calibrate(X, p)["status"] == 0
    X[1, 3, 5] = np.inf
    assert U.gpu_calibrate(X, p)["status"] == tdq.DEV_NONFINITE
    X[1, 3, 5] = np.nan
    assert U.gpu_calibrate(X, p)["status"] == tdq.DEV_NONFINITE
    Xf = np.ones((1, 8, 8), dtype=np.float32)
    Xf[0, 0, 0] = -np.inf
    assert U.gpu_calibrate(Xf, p)["status"] == tdq.DEV_NONFINITE


def test_user_supplied_radii_are_clamped():
    """tdq_quantize_act with radii that are not a projection's (clip >> 7 step):
    codes clamp to [-8, 7] as the definition says."""
    rng = np.random.Generator(np.random.PCG64(10))
    X = (rng.laplace(0, 4, (1, 32, 64))).astype(np.float32)
    gid = np.zeros((1, 32), np.int32)
    clip = np.array([[100.0]], np.float32)
    scale = np.array([[0.37]], np.float32)
    p = tdq.default_params(1)
    Q = tdq.tdq_quantize_act(U.to_device(X), p, None, torch.from_numpy(clip).to(U.dev()),
                             torch.from_numpy(scale).to(U.dev()))
    q = U.unpack_device_codes(Q, 64)
    q_ref = O.quantize_act(X, gid, clip, scale, U.oracle_params(p)).reshape(-1, 64)
    assert np.array_equal(q, q_ref) and q.min() == -8 and q.max() == 7


# --------------------------------------------------- contraction on raw codes
@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (5, 31, 3), (64, 33, 64), (129, 64, 130),
                                   (300, 100, 17), (128, 257, 128), (257, 1024, 200),
                                   (100, 4100, 50)])
def test_contraction_full_code_range(M, K, N):
    """Codes drawn from the whole nibble range, -8 included; ragged M, N, K."""
    _say(f"[gemm] M={M} K={K} N={N}")
    qx = I.random_codes((M, K), 11 * M + K)
    qw = I.random_codes((N, K), 13 * N + K)
    rng = np.random.Generator(np.random.PCG64(M + K + N))
    B, T = (1, M) if M % 3 else (3, M // 3)
    G = 4
    gid = rng.integers(0, G, (B, T)).astype(np.int32)
    scale = rng.uniform(0.01, 2.0, (B, G)).astype(np.float32)
    sw = rng.uniform(0.001, 0.01, N).astype(np.float32)
    bias = rng.normal(0, 0.02, N).astype(np.float32)
    acc, Y = U.gpu_linear(U.pack_to_device(qx), torch.from_numpy(gid).to(U.dev()),
                          torch.from_numpy(scale).to(U.dev()), B, T, K, U.pack_to_device(qw),
                          torch.from_numpy(sw).to(U.dev()), torch.from_numpy(bias).to(U.dev()))
    acc_ref, Y_ref = O.w4a4_linear(qx, O.row_scales(gid, scale), qw, sw, bias)
    assert np.array_equal(acc, acc_ref)
    assert np.array_equal(Y, Y_ref)


def test_contraction_extreme_accumulator():
    """Every product at its largest magnitude: |acc| = 64 K."""
    M, K, N = 40, 4096, 36
    qx = np.full((M, K), -8, np.int8)
    qw = np.full((N, K), -8, np.int8)
    qw[::2] = 7
    scale = np.ones((1, 1), np.float32)
    sw = np.ones(N, np.float32)
    acc, Y = U.gpu_linear(U.pack_to_device(qx), None, torch.from_numpy(scale).to(U.dev()), 1, M,
                          K, U.pack_to_device(qw), torch.from_numpy(sw).to(U.dev()))
    acc_ref, Y_ref = O.w4a4_linear(qx, np.ones(M, np.float32), qw, sw)
    assert np.array_equal(acc, acc_ref) and acc.max() == 64 * K and acc.min() == -56 * K
    assert np.array_equal(Y, Y_ref)


def test_junk_past_row_end_is_ignored():
    """Bytes between ceil(K/2) and the leading dimension must not reach the result."""
    M, K, N = 33, 40, 20          # 20 packed bytes per row, ld = 32
    qx = I.random_codes((M, K), 1)
    qw = I.random_codes((N, K), 2)
    A = U.pack_to_device(qx)
    Bm = U.pack_to_device(qw)
    A[:, 20:] = 0xAB
    Bm[:, 20:] = 0xCD
    scale = np.ones((1, 1), np.float32)
    sw = np.ones(N, np.float32)
    acc, _ = U.gpu_linear(A, None, torch.from_numpy(scale).to(U.dev()), 1, M, K, Bm,
                          torch.from_numpy(sw).to(U.dev()))
    assert np.array_equal(acc, O.int_accumulate(qx, qw))


# ------------------------------------------------------------------ invariants
def test_repeatable_bitwise():
    lc = I.case("cfg2_qkv", B=3)
    X, _ = I.make_activations(lc)
    p = tdq.default_params(lc.G)
    a = U.gpu_calibrate(X, p)
    b = U.gpu_calibrate(X, p)
    for k in ("gid", "clip", "scale"):
        assert np.array_equal(a[k], b[k])
    assert a["stats"].tobytes() == b["stats"].tobytes()


def test_token_permutation_invariance_on_gpu():
    lc = I.case("cfg1", grid=(48, 48))
    X, _ = I.make_activations(lc)
    p = tdq.default_params(lc.G)
    a = U.gpu_calibrate(X, p)
    perm = np.random.Generator(np.random.PCG64(5)).permutation(lc.T)
    b = U.gpu_calibrate(X[:, perm], p)
    assert np.array_equal(a["gid"][:, perm], b["gid"])
    for k in ("n", "k", "thr", "c_base", "c_zr"):
        assert np.array_equal(a["stats"][k], b["stats"][k])
    assert np.allclose(a["scale"], b["scale"], rtol=1e-6, atol=0)


# ------------------------------------------------- full size, sampled checks
@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,out_dtype", [("cfg4_fc1_h10", torch.float16), ("cfg4_fc2_h10", torch.float32)])
def test_cfg4_full_size_sampled(name, out_dtype):
    """ViT-L-shaped stress at its full size, both linears, in the launch configuration the
    benchmark times (fc1 with binary16 output, fc2 with binary32 output; the same kernels:
    statistics sweep, single-sweep rank select, quantizer, wide-stage contraction); the
    oracle checks two whole images of the calibration and sampled rows of codes and
    outputs."""
    lc = I.case(name)
    _say(f"[cfg4] {name}: generating inputs")
    X, _ = I.make_activations(lc, workers=16)
    W = I.make_weight(lc)
    p = tdq.default_params(lc.G)
    B, T, C, N, G = lc.B, lc.T, lc.C, lc.N, lc.G
    _say("[cfg4] GPU path")
    Xd = torch.from_numpy(X).to(U.dev())
    gid_d, clip_d, scale_d, stats_d, ws = tdq.tdq_calibrate_groups(Xd, p, want_stats=True)
    Q = tdq.tdq_quantize_act(Xd, p, gid_d, clip_d, scale_d)
    Qw_d, ws_d = tdq.tdq_quantize_weight(torch.from_numpy(W).to(U.dev()))
    Y = tdq.tdq_w4a4_linear(Q, gid_d, scale_d, B, T, C, Qw_d, ws_d, None, out_dtype)
    torch.cuda.synchronize()
    assert tdq.device_status(ws) == 0
    _say(f"[cfg4] sets resolved by the per-set radix select: {tdq.exact_select_sets(ws)}")
    gid, clip, scale = gid_d.cpu().numpy(), clip_d.cpu().numpy(), scale_d.cpu().numpy()
    stats = tdq.stats_to_numpy(stats_d).reshape(B, G)
    op = U.oracle_params(p)
    qw_ref, sw_ref = O.quantize_weight(W)
    assert np.array_equal(ws_d.cpu().numpy(), sw_ref)
    # properties that hold at any size
    assert int(stats["n"].sum()) == B * T * C
    used = stats["n"] > 0
    assert (stats["scale"][used] <= stats["sigma"][used] * (1 + 1e-6)).all()         # C1
    assert (stats["scale"][used] / 2 <= stats["thr"][used] * (1 + 1e-6)).all()       # C2
    for b in (0, B - 1):
        _say(f"[cfg4] oracle calibration of image {b}")
        g1, c1, s1, st1 = O.calibrate_groups(X[b:b + 1], op)
        assert np.array_equal(gid[b], g1[0])
        for j in range(G):
            assert stats[b, j]["n"] == st1[0][j]["n"]
            if st1[0][j]["n"]:
                assert stats[b, j]["thr"] == st1[0][j]["thr"]
                assert stats[b, j]["k"] == st1[0][j]["k"]
                assert stats[b, j]["c_base"] == st1[0][j]["c_base"]
                assert abs(float(stats[b, j]["sigma"]) - float(st1[0][j]["sigma"])) \
                    <= U.SCALE_RTOL * float(st1[0][j]["sigma"])
        assert np.allclose(clip[b], c1[0], rtol=1e-6, atol=0)
        assert np.allclose(scale[b], s1[0], rtol=1e-6, atol=0)
        rows = np.random.Generator(np.random.PCG64(b)).choice(T, 48, replace=False)
        q_ref = O.quantize_codes(X[b, rows], c1[0][g1[0][rows]][:, None],
                                 s1[0][g1[0][rows]][:, None], op)
        q_gpu = O.unpack_nibbles(Q[b * T + torch.from_numpy(rows).to(U.dev())].cpu().numpy(), C)
        exact = np.array_equal(scale[b], s1[0]) and np.array_equal(clip[b], c1[0])
        U.assert_codes_match(q_gpu, q_ref, X[b, rows], c1[0][g1[0][rows]], s1[0][g1[0][rows]],
                             exact)
        acc_ref, Y_ref = O.w4a4_linear(q_gpu, scale[b][gid[b, rows]], qw_ref, sw_ref)
        Y_gpu = Y[b * T + torch.from_numpy(rows).to(U.dev())].cpu().numpy()
        if out_dtype == torch.float16:
            Y_ref = Y_ref.astype(np.float16)
        assert np.array_equal(Y_gpu, Y_ref)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["cfg4_fc1_h2", "cfg4_fc1_h25", "cfg4_fc2_h2", "cfg4_fc2_h25"])
def test_cfg4_heavy_sweep_calibration(name):
    """The heavy-tail sweep of the stress configuration (2 % and 25 % heavy tokens; 10 % is
    the case above): calibration of the whole batch on the GPU, two images against the
    oracle; the count of sets whose sampled key interval missed is reported."""
    lc = I.case(name)
    _say(f"[cfg4-sweep] {name}: generating inputs")
    X, _ = I.make_activations(lc, workers=16)
    p = tdq.default_params(lc.G)
    B, T, C, G = lc.B, lc.T, lc.C, lc.G
    Xd = torch.from_numpy(X).to(U.dev())
    gid_d, clip_d, scale_d, stats_d, ws = tdq.tdq_calibrate_groups(Xd, p, want_stats=True)
    torch.cuda.synchronize()
    assert tdq.device_status(ws) == 0
    _say(f"[cfg4-sweep] {name}: sets resolved by the per-set radix select: {tdq.exact_select_sets(ws)}")
    stats = tdq.stats_to_numpy(stats_d).reshape(B, G)
    assert int(stats["n"].sum()) == B * T * C
    for b in (1, B - 2):
        g = dict(gid=gid_d[b:b + 1].cpu().numpy(), clip=clip_d[b:b + 1].cpu().numpy(),
                 scale=scale_d[b:b + 1].cpu().numpy(), stats=stats[b:b + 1].reshape(-1))
        U.assert_calibration_matches(g, X[b:b + 1], p)


# ------------------------------------- large-tile contraction, sampled checks
@pytest.mark.parametrize("out_dtype,with_bias,ld_pad,K,N", [(torch.float32, True, 0, 256, 4096),
                                                            (torch.float16, False, 0, 256, 4096),
                                                            (torch.float16, True, 8, 256, 4096),
                                                            (torch.float32, False, 2, 256, 4096),
                                                            (torch.float32, True, 0, 320, 4096),
                                                            (torch.float16, False, 6, 200, 4096),
                                                            (torch.float32, True, 0, 384, 4096),
                                                            (torch.float16, True, 0, 128, 4096),
                                                            (torch.float16, False, 0, 768, 4096),
                                                            (torch.float32, True, 0, 256, 4096 + 40),
                                                            (torch.float16, False, 0, 128, 4096 + 40),
                                                            (torch.float16, True, 2, 320, 4096 + 40),
                                                            (torch.float32, False, 0, 512, 4096 + 200)])
def test_large_tile_contraction_sampled(out_dtype, with_bias, ld_pad, K, N):
    """Shapes that take the large-tile kernels (many 256x256 tiles; K a multiple of
    256 for the wide-stage pipelined one, K = 384 and 128 for the 128-code-stage one,
    K = 320 and 200 for the generic one with its K tail; 768 = three wide stages)
    without the accumulator dump, so interior tiles take the epilogue's fast
    path and the ragged last row of tiles the bounds-checked one; N = 4096 + 40 / + 200
    adds a ragged last COLUMN of tiles.  ld_pad gives Y a padded leading dimension, whose
    padding must stay untouched.  The oracle checks whole tiles' worth of rows plus a
    random sample."""
    M = 8192 + 37
    _say(f"[gemm-large] M={M} K={K} N={N} out={out_dtype} bias={with_bias} ld_pad={ld_pad}")
    qx = I.random_codes((M, K), 101)
    qw = I.random_codes((N, K), 102)
    rng = np.random.Generator(np.random.PCG64(103))
    B, T, G = 1, M, 8
    gid = rng.integers(0, G, (B, T)).astype(np.int32)
    scale = rng.uniform(0.01, 2.0, (B, G)).astype(np.float32)
    sw = rng.uniform(0.001, 0.01, N).astype(np.float32)
    bias = rng.normal(0, 0.5, N).astype(np.float32) if with_bias else None
    Ybuf = torch.full((M, N + ld_pad), -77.0, dtype=out_dtype, device=U.dev())
    Y = tdq.tdq_w4a4_linear(U.pack_to_device(qx), torch.from_numpy(gid).to(U.dev()),
                            torch.from_numpy(scale).to(U.dev()), B, T, K, U.pack_to_device(qw),
                            torch.from_numpy(sw).to(U.dev()),
                            None if bias is None else torch.from_numpy(bias).to(U.dev()),
                            out_dtype, out=Ybuf[:, :N])
    torch.cuda.synchronize()
    if ld_pad:
        assert (Ybuf[:, N:] == -77.0).all(), "wrote past the row end"
    rows = np.unique(np.concatenate([np.arange(0, 256), np.arange(3 * 256 - 8, 3 * 256 + 8),
                                     rng.choice(M, 128, replace=False), np.arange(8192 - 8, M)]))
    _, Y_ref = O.w4a4_linear(qx[rows], O.row_scales(gid, scale)[rows], qw, sw, bias)
    if out_dtype == torch.float16:
        Y_ref = Y_ref.astype(np.float16)
    Y_gpu = Y[torch.from_numpy(rows).to(U.dev())].cpu().numpy()
    assert np.array_equal(Y_gpu, Y_ref)


# ------------------------------------------- the two routes of the rank select
def test_exact_select_route_alone():
    """TDQ_FLAG_EXACT_SELECT resolves every set's zr rank by the per-set radix
    select (the route a set takes when its sampled key interval misses the rank):
    same results as the oracle, and every non-empty set is counted."""
    lc = I.case("cfg2_fc2", B=3)
    X, _ = I.make_activations(lc)
    p = tdq.default_params(lc.G)
    p.flags |= tdq.FLAG_EXACT_SELECT
    g = U.gpu_calibrate(X, p)
    U.assert_calibration_matches(g, X, p)
    assert g["exact_sets"] == int((g["stats"]["n"] > 0).sum())
    p2 = tdq.default_params(lc.G)
    g2 = U.gpu_calibrate(X, p2)
    assert g2["stats"].tobytes() == g["stats"].tobytes()
    assert g2["exact_sets"] == 0, "a sampled interval missed on the benchmark's own input recipe"


def test_sampled_interval_miss_falls_back_exactly():
    """An input built to defeat the sample: nine tokens of 4096 channels, all with
    the same range (so they share one token set although G = 32, which leaves that
    set 512 one-key bins), whose smallest fifth sits in one contiguous run of
    channels, so that the share of it inside a token's sampled channel window depends
    on where the window starts; the rest is spread over ten octaves, which turns the
    sample's rank error into thousands of keys.  The result must still be the exact
    order statistic; the diagnostic counter shows that the radix levels produced it."""
    T, C = 9, 4096
    rng = np.random.Generator(np.random.PCG64(77))
    X = np.exp2(rng.uniform(-9.0, 1.0, (1, T, C))).astype(np.float16)
    X[:, :, 0:819] = rng.uniform(1e-4, 2e-4, (1, T, 819)).astype(np.float16)
    X[:, :, 4000] = 2.0
    X *= rng.choice([-1.0, 1.0], X.shape).astype(np.float16)
    p = tdq.default_params(32)
    g = U.gpu_calibrate(X, p)
    assert (g["gid"] == 0).all()
    U.assert_calibration_matches(g, X, p)
    assert g["exact_sets"] == 1


@pytest.mark.parametrize("T,C,G", [(700, 8, 4), (9, 33, 2), (1500, 48, 256), (64, 4100, 1),
                                   (3000, 40, 64)])
def test_rank_select_shapes(T, C, G):
    """Shapes around the sample geometry: sets smaller than the sample, rows narrower
    than one sampled run, odd and unaligned C, the largest number of sets that the
    single-sweep select takes (64: 256 one-key bins each) and more (radix levels)."""
    rng = np.random.Generator(np.random.PCG64(T + C + G))
    X = (rng.laplace(0, 1, (2, T, C)) * rng.lognormal(0, 1.0, (2, T, 1))).astype(np.float16)
    p = tdq.default_params(G)
    g = U.gpu_calibrate(X, p, ld_pad=3 if C % 2 else 0)
    U.assert_calibration_matches(g, X, p)


@pytest.mark.parametrize("G,exact", [(128, 0), (129, 0), (200, 0), (256, 0), (256, 256)])
def test_radix_levels_many_sets_f32(G, exact):
    """binary32 input with more than 128 sets per image: 2^5 bins per set are all the LDS
    histogram holds, so the 31-bit key takes seven radix levels (six up to 128 sets).
    Orders of magnitude between tokens, so that the digits of every level matter."""
    _say(f"[radix-levels] G={G} exact={exact}")
    rng = np.random.Generator(np.random.PCG64(900 + G))
    X = (rng.laplace(0, 1, (2, 1200, 40)) * rng.lognormal(0, 2.5, (2, 1200, 1))).astype(np.float32)
    p = tdq.default_params(G)
    p.flags |= exact
    g = U.gpu_calibrate(X, p)
    assert g["status"] == 0
    U.assert_calibration_matches(g, X, p)


# ------------------------------------------------- percentile base radius Q_p
@pytest.mark.parametrize("case,pct,flags,extra", [("cfg2_fc2", 0.99, 3, 0), ("cfg2_qkv", 0.5, 0, 0),
                                                  ("cfg0", 0.99, 3, 0), ("cfg0", 0.9, 0, 0),
                                                  ("cfg2_proj", 0.999, 3, 256)])
def test_percentile_base_radius(case, pct, flags, extra):
    """Base radius = the ceil(p n)-th smallest |x| of the set instead of its maximum
    (Eq. DSTG_clip, percentile branch): binary16 input through the single-sweep select
    (twice: base radius, then the zr quantile), binary32 input and the validation
    switch through the radix levels.  flags = 0 makes the base radius the clip itself."""
    lc = I.case(case) if case == "cfg0" else I.case(case, B=3)
    X, _ = I.make_activations(lc)
    p = tdq.default_params(lc.G, flags=flags)
    p.base_pct = pct
    p.flags |= extra
    g = U.gpu_calibrate(X, p)
    assert g["status"] == 0
    gid, clip, scale, st = U.assert_calibration_matches(g, X, p)
    used = g["stats"]["n"] > 0
    if flags == 0:
        assert np.array_equal(g["stats"]["clip"][used], np.maximum(g["stats"]["c_base"][used], 1e-8))
    # quantize with the projected radii: codes match the oracle's
    Q = tdq.tdq_quantize_act(g["Xd"], p, g["gid_d"], g["clip_d"], g["scale_d"])
    q_ref = O.quantize_act(X, gid, clip, scale, U.oracle_params(p)).reshape(lc.M, lc.C)
    rows = np.arange(lc.B)[:, None]
    exact = np.array_equal(g["scale"], scale) and np.array_equal(g["clip"], clip)
    U.assert_codes_match(U.unpack_device_codes(Q, lc.C), q_ref, X, clip[rows, gid].reshape(-1),
                         scale[rows, gid].reshape(-1), exact)


# ------------------------------------------------------- device diagnostics
@pytest.mark.parametrize("case,ld_pad", [("cfg0", 0), ("cfg1", 0), ("cfg2_fc2", 0), ("cfg2_qkv", 4)])
def test_group_diagnostics(case, ld_pad):
    """Zero-bin and clipped counts per token set (Eq. rho0_def) against the oracle's
    codes, exactly; with the projected radii nothing exceeds the base radius, so a
    second call uses halved radii to make the clipped count non-trivial."""
    lc = I.case(case) if case in ("cfg0", "cfg1") else I.case(case, B=3)
    X, _ = I.make_activations(lc)
    p = tdq.default_params(lc.G)
    g = U.gpu_calibrate(X, p, ld_pad)
    gid, clip, scale = g["gid"], g["clip"], g["scale"]
    for shrink in (1.0, 0.5):
        c = (clip * shrink).astype(np.float32)
        cd = torch.from_numpy(c).to(U.dev())
        zero, clipped = tdq.tdq_group_diagnostics(g["Xd"], p, g["gid_d"], cd, g["scale_d"])
        torch.cuda.synchronize()
        q = O.quantize_act(X, gid, c, scale, U.oracle_params(p))
        zr = np.zeros((lc.B, lc.G), np.int64)
        cr = np.zeros((lc.B, lc.G), np.int64)
        for b in range(lc.B):
            for j in range(lc.G):
                m = gid[b] == j
                zr[b, j] = int((q[b][m] == 0).sum())
                cr[b, j] = int((np.abs(X[b][m].astype(np.float32)) > c[b, j]).sum())
        assert np.array_equal(zero.cpu().numpy(), zr)
        assert np.array_equal(clipped.cpu().numpy(), cr)
        if shrink == 0.5:
            assert cr.sum() > 0


@pytest.mark.parametrize("case,over,ld_pad", [("cfg0", {}, 0), ("cfg1", {}, 0), ("cfg2_qkv", dict(B=3), 4),
                                              ("cfg2_fc2", dict(B=2), 0), ("cfg4_fc1_h10", dict(B=1), 0)])
def test_range_disparity(case, over, ld_pad):
    """D(X) of Eq. (range_disparity) on the device: per-token lower medians, their
    median and the maximum are elements of the data, hence bit-exact; D is one binary32
    division."""
    lc = I.case(case, **over)
    X, _ = I.make_activations(lc)
    if case.startswith("cfg4"):
        X = X[:, :300]
    _say(f"[disparity] {case} {X.shape} {X.dtype}")
    D, med, mx = tdq.tdq_range_disparity(U.to_device(X, ld_pad))
    torch.cuda.synchronize()
    Dr, medr, mxr = O.range_disparity(X)
    assert np.array_equal(med.cpu().numpy(), medr)
    assert np.array_equal(mx.cpu().numpy(), mxr)
    assert np.array_equal(D.cpu().numpy(), Dr)


def test_range_disparity_degenerate():
    X = np.zeros((3, 5, 9), dtype=np.float16)
    X[1] = -2.0
    X[2, :, :4] = 1.0          # 4 of 9 channels non-zero: every token's median is 0
    X[2, 0, 8] = 7.0
    D, med, mx = tdq.tdq_range_disparity(U.to_device(X))
    torch.cuda.synchronize()
    Dr, medr, mxr = O.range_disparity(X)
    assert np.array_equal(D.cpu().numpy(), Dr) and np.isinf(Dr[0]) and Dr[1] == 1.0 and np.isinf(Dr[2])
    assert np.array_equal(med.cpu().numpy(), medr) and np.array_equal(mx.cpu().numpy(), mxr)


# ------------------------------------------ the quotient at rounding boundaries
def _ulp_step(a: np.ndarray, j: int) -> np.ndarray:
    """Positive binary32 values moved j units in the last place."""
    return (a.astype(np.float32).view(np.int32) + np.int32(j)).view(np.float32)


def _adversarial_steps(n: int, seed: int) -> np.ndarray:
    """n binary32 steps: all-ones and all-zeros mantissas at several exponents, the
    1e-8 floor and its neighbours, one past a power of two, and random ones."""
    rng = np.random.Generator(np.random.PCG64(seed))
    fixed = []
    for e in (-30, -26, -20, -7, -1, 0, 1, 5, 9):
        fixed += [np.ldexp(1.0, e), np.nextafter(np.float32(np.ldexp(1.0, e)), np.float32(0)),
                  np.nextafter(np.float32(np.ldexp(1.0, e)), np.float32(np.inf)),
                  np.ldexp(1.5, e), np.ldexp(1.0 + 2.0 ** -12, e), np.ldexp(2.0 - 2.0 ** -12, e)]
    fixed += [1e-8, np.nextafter(np.float32(1e-8), np.float32(1)), 3.0 / 7.0, 1.0 / 3.0, 0.1]
    d = np.array(fixed, dtype=np.float32)
    extra = np.exp2(rng.uniform(-20, 8, n - d.size)).astype(np.float32)
    extra[::3] = (extra[::3].view(np.int32) | np.int32(0x7FFFFF)).view(np.float32)   # all-ones mantissas
    return np.concatenate([d, extra])[:n]


@pytest.mark.parametrize("clip_mult", [7.0, 1e6])
def test_quotient_at_rounding_boundaries_f32(clip_mult):
    """The quantizer replaces the division x~ / Delta by a reciprocal and two fused
    multiply-adds; the code must still be that of the correctly rounded quotient
    (Eqs. clipx, dequant; ties to even).  Every token is its own set with an adversarial
    step; its row holds, for every k in -8..7, the binary32 numbers around (k + 1/2) Delta
    (the boundary between codes k and k + 1), and a few tiny and huge values."""
    B, G = 4, 256
    T = G
    d = _adversarial_steps(B * G, 21).reshape(B, G)
    ks = np.arange(-8, 8, dtype=np.float64) + 0.5
    offs = np.arange(-3, 4)
    base = (ks[None, None, :] * d[:, :, None].astype(np.float64)).astype(np.float32)     # [B, G, 16]
    mag = np.abs(base)
    cols = [np.copysign(_ulp_step(mag, int(j)), base) for j in offs]
    X = np.stack(cols, axis=-1).reshape(B, T, -1)
    tail = np.array([0.0, -0.0, 1e-30, -1e-30, 1e-38, 3e38, -3e38, 1.0], dtype=np.float32)
    X = np.concatenate([X, np.broadcast_to(tail, (B, T, tail.size))], axis=-1).astype(np.float32)
    C = X.shape[-1]
    gid = np.broadcast_to(np.arange(T, dtype=np.int32), (B, T)).copy()
    clip = (d * np.float32(clip_mult)).astype(np.float32)
    p = tdq.default_params(G)
    _say(f"[quotient-f32] B={B} T={T} C={C} clip = {clip_mult} * step")
    Q = tdq.tdq_quantize_act(U.to_device(X), p, torch.from_numpy(gid).to(U.dev()),
                             torch.from_numpy(clip).to(U.dev()), torch.from_numpy(d).to(U.dev()))
    torch.cuda.synchronize()
    q_ref = O.quantize_act(X, gid, clip, d, U.oracle_params(p)).reshape(B * T, C)
    q = U.unpack_device_codes(Q, C)
    bad = np.argwhere(q != q_ref)
    assert bad.size == 0, f"{len(bad)} codes differ, first at row {bad[0][0]} (step " \
                          f"{d.reshape(-1)[bad[0][0]]!r}), x = {X.reshape(B * T, C)[tuple(bad[0])]!r}"
    # a radius of 7 steps keeps x~ / Delta inside [-7, 7]; a wide one reaches the clamp at -8
    assert set(np.unique(q_ref)) == set(range(-7 if clip_mult == 7.0 else -8, 8))


def test_quotient_at_rounding_boundaries_f16():
    """The same for binary16 input: x = (2k + 1) a with a small dyadic a is exact in
    binary16, and the step 2a moved by -2..2 units in the last place puts every x of the
    row exactly on, just below or just above a rounding boundary."""
    B, G = 5, 64
    T = G
    rng = np.random.Generator(np.random.PCG64(22))
    a = (rng.integers(1, 64, (B, G)) * np.exp2(rng.integers(-12, 3, (B, G)))).astype(np.float32)
    d = np.empty((B, G), np.float32)
    for b in range(B):
        d[b] = _ulp_step(2.0 * a[b], b - 2)
    k2 = np.arange(-15, 16, 2, dtype=np.float32)                         # 2k + 1, k = -8..7
    X = (a[:, :, None] * k2[None, None, :]).astype(np.float16)
    assert np.array_equal(X.astype(np.float32), a[:, :, None] * k2[None, None, :])
    X = np.concatenate([X, np.zeros((B, T, 16), np.float16)], axis=-1)   # 32 channels
    C = X.shape[-1]
    gid = np.broadcast_to(np.arange(T, dtype=np.int32), (B, T)).copy()
    clip = (d * np.float32(1e3)).astype(np.float32)
    p = tdq.default_params(G)
    _say(f"[quotient-f16] B={B} T={T} C={C}")
    Q = tdq.tdq_quantize_act(U.to_device(X), p, torch.from_numpy(gid).to(U.dev()),
                             torch.from_numpy(clip).to(U.dev()), torch.from_numpy(d).to(U.dev()))
    torch.cuda.synchronize()
    q_ref = O.quantize_act(X, gid, clip, d, U.oracle_params(p)).reshape(B * T, C)
    assert np.array_equal(U.unpack_device_codes(Q, C), q_ref)
    # image 2 has the unmoved steps: every x is a tie, rounded to the even neighbour
    tie = q_ref.reshape(B, T, C)[2, :, :16]
    assert (tie[:, :15] % 2 == 0).all() and (tie[:, 15] == 7).all()      # 7.5 -> 8, clamped to 7


# ------------------------- persistent (rolling) contraction, sampled checks
@pytest.mark.parametrize("K,out_dtype,with_bias,T,G,ld_pad", [(1024, torch.float32, False, 128, 8, 0),
                                                              (3072, torch.float16, True, 4096, 1, 0),
                                                              (512, torch.float16, True, 4096, 1, 0),
                                                              (1024, torch.float16, False, 2048, 32, 8),
                                                              (1024, torch.float16, True, 2048, 4, 2),
                                                              (1536, torch.float32, True, 256, 5, 4),
                                                              (2048, torch.float16, True, 16384, 3, 0)])
def test_rolling_contraction_sampled(K, out_dtype, with_bias, T, G, ld_pad):
    """Shapes of whole 256 x 256 tiles, at least eight for every CU, an even number of
    256-code stages: the persistent kernel whose stage stream runs across tile boundaries
    (4, 6, 8 and 12 stages per tile; several images per tile and several tiles per image;
    one token set without an id array; K = 512, two stages, is below the kernel's smallest K
    and takes the non-persistent kernel, and so does a leading dimension of Y that is not a
    multiple of 4: the persistent kernel stores four adjacent outputs per lane).  Sampled rows of every kind of tile position
    against the oracle, bit for bit; Y's padding untouched."""
    M, N = 16384, 8192
    _say(f"[gemm-roll] M={M} K={K} N={N} out={out_dtype} bias={with_bias} T={T} G={G} ld_pad={ld_pad}")
    qx = I.random_codes((M, K), 201)
    qw = I.random_codes((N, K), 202)
    rng = np.random.Generator(np.random.PCG64(203))
    B = M // T
    gid = rng.integers(0, G, (B, T)).astype(np.int32)
    scale = rng.uniform(0.01, 2.0, (B, G)).astype(np.float32)
    sw = rng.uniform(0.001, 0.01, N).astype(np.float32)
    bias = rng.normal(0, 0.5, N).astype(np.float32) if with_bias else None
    Ybuf = torch.full((M, N + ld_pad), -77.0, dtype=out_dtype, device=U.dev())
    Y = tdq.tdq_w4a4_linear(U.pack_to_device(qx), None if G == 1 else torch.from_numpy(gid).to(U.dev()),
                            torch.from_numpy(scale).to(U.dev()), B, T, K, U.pack_to_device(qw),
                            torch.from_numpy(sw).to(U.dev()),
                            None if bias is None else torch.from_numpy(bias).to(U.dev()),
                            out_dtype, out=Ybuf[:, :N])
    torch.cuda.synchronize()
    if ld_pad:
        assert (Ybuf[:, N:] == -77.0).all(), "wrote past the row end"
    # every tile row of the first and last workgroup rounds, rows at tile and image borders, and
    # a random sample; all N columns (every tile column)
    rows = np.unique(np.concatenate([np.arange(0, 16), np.arange(250, 262), np.arange(2040, 2056),
                                     np.arange(M - 300, M - 250), np.arange(M - 8, M),
                                     rng.choice(M, 160, replace=False)]))
    _, Y_ref = O.w4a4_linear(qx[rows], O.row_scales(gid, scale)[rows], qw, sw, bias)
    if out_dtype == torch.float16:
        Y_ref = Y_ref.astype(np.float16)
    Y_gpu = Y[torch.from_numpy(rows).to(U.dev())].cpu().numpy()
    assert np.array_equal(Y_gpu, Y_ref)
    # and the whole output against the non-persistent kernels (they take over when an
    # accumulator dump is asked for), bit for bit
    acc = torch.empty((M, N), dtype=torch.int32, device=U.dev())
    Y2 = tdq.tdq_w4a4_linear(U.pack_to_device(qx), None if G == 1 else torch.from_numpy(gid).to(U.dev()),
                             torch.from_numpy(scale).to(U.dev()), B, T, K, U.pack_to_device(qw),
                             torch.from_numpy(sw).to(U.dev()),
                             None if bias is None else torch.from_numpy(bias).to(U.dev()),
                             out_dtype, acc_dump=acc)
    torch.cuda.synchronize()
    assert torch.equal(Y2, Y)
