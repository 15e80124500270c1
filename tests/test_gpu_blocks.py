"""GPU parity of the paper-literal granularity (one group per token and block of 32
channels; Sec. 4.2, Supp. Algorithm 1) against the CPU oracle: the fused block quantizer
and the block-scaled contraction, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import tdq_oracle as O
from paper_2604_16855_amd import inputs as I
from paper_2604_16855_amd import tdq

import parity_util as U

pytestmark = pytest.mark.gpu

G_BLK = 32


def _say(msg):
    print(msg, flush=True)


def _oracle_params(p):
    return O.Params(n_groups=1, flags=p.flags & 3, tau=p.tau, zr=p.zr, base_pct=p.base_pct)


def _blocks_view(a, C):
    """[M, C] -> [M * KB, 32], the channel axis zero-padded to whole blocks."""
    M = a.shape[0]
    KB = -(-C // G_BLK)
    out = np.zeros((M, KB * G_BLK), dtype=a.dtype)
    out[:, :C] = a
    return out.reshape(M * KB, G_BLK)


def _check_block_quantizer(X, p, ld_pad=0):
    """X[B, T, C]: radii, steps and codes of every (token, block) against the oracle."""
    B, T, C = X.shape
    KB = -(-C // G_BLK)
    _say(f"[blocks] B={B} T={T} C={C} dtype={X.dtype} flags={p.flags} tau={p.tau} zr={p.zr} "
         f"base_pct={p.base_pct} ld_pad={ld_pad}")
    Xd = U.to_device(X, ld_pad)
    Q, bs, bc = tdq.tdq_quantize_act_blocks(Xd, p, want_clip=True)
    torch.cuda.synchronize()
    _, q_ref, clip, scale = O.dstg_dcrp_blocks(X.reshape(B * T, C), G_BLK, _oracle_params(p))
    clip_g, scale_g = bc.cpu().numpy(), bs.cpu().numpy()
    assert clip_g.shape == (B * T, KB)
    if not (p.flags & tdq.FLAG_C1):
        # without the dispersion bound every radius is an element of the data times an
        # exact constant: bit-exact, and so are the steps and the codes
        assert np.array_equal(clip_g, clip), "clip radii differ (order statistics)"
        assert np.array_equal(scale_g, scale)
    assert np.allclose(clip_g, clip, rtol=U.SCALE_RTOL, atol=0), "clip radii differ"
    assert np.allclose(scale_g, scale, rtol=U.SCALE_RTOL, atol=0), "steps differ"
    q_gpu = U.unpack_device_codes(Q, C)
    exact = np.array_equal(clip_g, clip) and np.array_equal(scale_g, scale)
    flips = U.assert_codes_match(_blocks_view(q_gpu, C), _blocks_view(q_ref, C),
                                 _blocks_view(X.reshape(B * T, C).astype(np.float32), C),
                                 clip.reshape(-1), scale.reshape(-1), exact)
    if C % 2:      # the pad nibble of an odd row is zero
        assert not (Q.cpu().numpy()[:, C // 2] >> 4).any()
    _say(f"  scales bit-identical: {exact}; code flips: {flips}")
    return Q, bs, q_gpu, scale_g


def _acts(name, B, T, C=None, dtype=None):
    """Activations of a named workload cut to [B, T, C]."""
    kw = dict(B=B)
    if dtype:
        kw["dtype"] = dtype
    lc = I.case(name, **kw)
    X, _ = I.make_activations(lc)
    C = C or lc.C
    return np.ascontiguousarray(X[:, :T, :C])


@pytest.mark.parametrize("name,B,T,C", [("cfg2_fc2", 2, 300, None), ("cfg2_qkv", 1, 484, None),
                                        ("cfg4_fc1_h10", 1, 150, 1024), ("cfg4_fc2_h10", 1, 40, 4096)])
def test_block_quantizer_on_workloads(name, B, T, C):
    _check_block_quantizer(_acts(name, B, T, C), tdq.block_params())


@pytest.mark.parametrize("B,T,C,dtype,ld_pad", [
    (1, 77, 80, np.float16, 0),      # last block half padding
    (1, 1000, 33, np.float16, 0),    # odd C, one real channel in the last block
    (1, 5, 7, np.float16, 0),        # less than one lane's share
    (3, 50, 4100, np.float16, 0),    # rows not a multiple of 16 bytes apart -> scalar loads
    (2, 64, 1024, np.float16, 8),    # padded row stride, still aligned
    (2, 33, 96, np.float16, 3),      # padded row stride, unaligned
    (1, 1, 32, np.float16, 0),       # one block
    (1, 200, 96, np.float32, 0),
    (2, 64, 1000, np.float32, 0),
    (1, 31, 45, np.float32, 5),
])
def test_block_quantizer_ragged_shapes(B, T, C, dtype, ld_pad):
    rng = np.random.Generator(np.random.PCG64([B, T, C, 5]))
    # heavy-tailed rows: Gaussian bulk, a few large channels, per-token range spread
    X = rng.standard_normal((B, T, C)) * np.exp(rng.normal(0, 1.5, (B, T, 1)))
    X[rng.random((B, T, C)) < 0.02] *= 30.0
    _check_block_quantizer(X.astype(dtype), tdq.block_params(), ld_pad)


@pytest.mark.parametrize("flags,tau,zr,base_pct", [
    (0, 1.0, 0.2, 0.0),       # DSTG only: max-abs radii
    (1, 0.3, 0.2, 0.0),       # C1 only
    (2, 1.0, 0.2, 0.0),       # C2 only: every radius an order statistic (rank 7)
    (2, 1.0, 0.01, 0.0),      # rank 1: the block minimum
    (2, 1.0, 0.25, 0.0),      # rank 8: last rank of the sorting-network route
    (2, 1.0, 0.26, 0.0),      # rank 9: first rank of the bisection route
    (2, 1.0, 0.6, 0.0),       # rank 20
    (2, 1.0, 0.99, 0.0),      # rank 32: the maximum
    (3, 2.0, 0.1, 0.0),
    (0, 1.0, 0.2, 0.9),       # percentile base radius, rank 29
    (3, 1.0, 0.2, 0.5),       # rank 16 base with both bounds
])
@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_block_quantizer_variants(flags, tau, zr, base_pct, dtype):
    X = _acts("cfg2_fc2", 1, 160).astype(dtype)
    _check_block_quantizer(X, tdq.block_params(tau, zr, flags, base_pct))


@pytest.mark.parametrize("dtype,ratio", [("f16", 10.0), ("f16", 100.0), ("f16", 1000.0),
                                         ("f32", 10.0), ("f32", 1000.0)])
def test_block_quantizer_on_offset_data(dtype, ratio):
    """Blocks far from zero mean (mean / sigma up to 1000) with C1 only: every step is
    tau * sigma of its 32 values (Eq. tau_constraint), so the block dispersion must hold
    the 1e-6 bar where a one-pass variance in binary32 would not."""
    X = I.offset_activations(2, 70, 200, dtype, ratio, seed=11 + int(ratio), token_jitter=0.05)
    _check_block_quantizer(X, tdq.block_params(1.0, 0.2, tdq.FLAG_C1, 0.0), ld_pad=8)


@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_block_quantizer_degenerate_blocks(dtype):
    """All-zero blocks (eps floors), constant blocks (sigma = eps_std), ties at the rank,
    a single non-zero, subnormal magnitudes, the largest finite values."""
    rng = np.random.Generator(np.random.PCG64(11))
    T, C = 64, 256
    X = rng.standard_normal((1, T, C)).astype(np.float32)
    X[0, 0] = 0.0
    X[0, 1] = 3.25
    X[0, 2] = 0.0
    X[0, 2, 5::32] = -2.5                                  # one non-zero per block
    X[0, 3] = np.where(rng.random(C) < 0.5, 1.0, -1.0)     # all magnitudes tie
    X[0, 4] = rng.integers(-2, 3, C)                       # many ties around the rank
    tiny = 6e-8 if dtype == np.float16 else 1e-40
    X[0, 5] = tiny * rng.integers(-5, 6, C)                # subnormals
    big = 65504.0 if dtype == np.float16 else 1.0e37
    X[0, 6, ::7] = big
    X[0, 7, :32] = 0.0
    X[0, 7, 31] = 1.0
    for flags in (3, 2, 0):
        _check_block_quantizer(X.astype(dtype), tdq.block_params(flags=flags))


def test_block_quantizer_repeatable_and_order_free():
    """Bitwise repeatable, and a block's result does not depend on where the block sits:
    permuting tokens permutes the outputs."""
    X = _acts("cfg2_fc2", 2, 200)
    p = tdq.block_params()
    Xd = U.to_device(X)
    Q1, s1, _ = tdq.tdq_quantize_act_blocks(Xd, p)
    Q2, s2, _ = tdq.tdq_quantize_act_blocks(Xd, p)
    perm = torch.randperm(X.shape[1], generator=torch.Generator().manual_seed(3)).to(U.dev())
    Q3, s3, _ = tdq.tdq_quantize_act_blocks(Xd[:, perm].contiguous(), p)
    torch.cuda.synchronize()
    assert torch.equal(Q1, Q2) and torch.equal(s1, s2)
    T = X.shape[1]
    idx = torch.cat([perm + b * T for b in range(X.shape[0])])
    assert torch.equal(Q1[idx], Q3) and torch.equal(s1[idx], s3)


# ---------------------------------------------------------------- block-scaled contraction
def _blocks_linear_bound(codes, bscale, qw, w_scale, bias, KB):
    """Error bound of the binary32 evaluation: one rounding per block and three in the
    epilogue, each relative to sum_kb |acc_kb Delta| s_n (+ |bias|); plus the rounding of
    the oracle's own binary64 sum, relative to the sum of the magnitudes of its terms
    (a block sum can cancel to exactly 0 where the binary64 sum leaves 1e-18)."""
    M, K = codes.shape
    S = np.zeros((M, qw.shape[0]))
    A = np.zeros((M, qw.shape[0]))
    for kb in range(KB):
        sl = slice(kb * G_BLK, min((kb + 1) * G_BLK, K))
        acc = codes[:, sl].astype(np.int64) @ qw[:, sl].astype(np.int64).T
        S += np.abs(acc) * bscale[:, kb].astype(np.float64)[:, None]
        A += (np.abs(codes[:, sl].astype(np.int64)) @ np.abs(qw[:, sl].astype(np.int64)).T) * \
            bscale[:, kb].astype(np.float64)[:, None]
    S *= w_scale.astype(np.float64)[None, :]
    A *= w_scale.astype(np.float64)[None, :]
    if bias is not None:
        S += np.abs(bias.astype(np.float64))[None, :]
    return (KB + 3) * 2.0 ** -24 * S + 2.0 ** -44 * A + 1e-37


def _check_blocks_linear(codes, bscale, qw, w_scale, bias, out_dtype=torch.float32, ld_s_pad=0):
    M, K = codes.shape
    N = qw.shape[0]
    KB = -(-K // G_BLK)
    _say(f"[blocks-linear] M={M} K={K} N={N} bias={bias is not None} out={out_dtype} "
         f"ld_s_pad={ld_s_pad}")
    Qx_d = U.pack_to_device(codes)
    Qw_d = U.pack_to_device(qw)
    bs_buf = torch.full((M, KB + ld_s_pad), float("nan"), dtype=torch.float32)
    bs_buf[:, :KB] = torch.from_numpy(bscale)
    bs_d = bs_buf.to(U.dev())[:, :KB]
    ws_d = torch.from_numpy(w_scale).to(U.dev())
    bias_d = None if bias is None else torch.from_numpy(bias).to(U.dev())
    Y = tdq.tdq_w4a4_linear_blocks(Qx_d, bs_d, K, Qw_d, ws_d, bias_d, out_dtype)
    Y2 = tdq.tdq_w4a4_linear_blocks(Qx_d, bs_d, K, Qw_d, ws_d, bias_d, out_dtype)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2), "not repeatable"
    Y = Y.cpu().numpy().astype(np.float64)
    Yref = O.blocks_linear(codes, bscale, G_BLK, qw, w_scale, bias)
    tol = _blocks_linear_bound(codes, bscale, qw, w_scale, bias, KB)
    assert KB > 160 or (KB + 3) * 2.0 ** -24 <= U.OUT_RTOL
    if out_dtype == torch.float16:
        tol = tol * 1.001 + 2.0 ** -11 * 1.001 * np.abs(Yref) + 2.0 ** -24   # + half an ulp of binary16
    err = np.abs(Y - Yref)
    assert (err <= tol).all(), f"worst error / bound = {(err / tol).max()}"
    return Y


def _random_block_operands(M, K, N, seed, spread=6.0):
    rng = np.random.Generator(np.random.PCG64([seed, M, K, N]))
    KB = -(-K // G_BLK)
    codes = I.random_codes((M, K), seed)
    qw = I.random_codes((N, K), seed + 1)
    # steps over many octaves within one row, as outlier channels make them
    bscale = np.exp(rng.normal(-3.0, spread, (M, KB))).astype(np.float32)
    w_scale = np.exp(rng.normal(-6.0, 0.5, N)).astype(np.float32)
    bias = rng.normal(0, 0.02, N).astype(np.float32)
    return codes, bscale, qw, w_scale, bias


@pytest.mark.parametrize("M,K,N,with_bias,ld_s_pad", [
    (1, 1, 1, False, 0), (5, 31, 3, True, 0), (64, 33, 64, False, 1), (129, 64, 130, True, 0),
    (300, 320, 200, False, 0), (256, 1280, 320, True, 0), (130, 4100, 140, False, 3),
    (200, 128, 129, True, 4), (77, 96, 300, False, 0)])
def test_blocks_linear_shapes(M, K, N, with_bias, ld_s_pad):
    codes, bscale, qw, w_scale, bias = _random_block_operands(M, K, N, 21)
    _check_blocks_linear(codes, bscale, qw, w_scale, bias if with_bias else None,
                         ld_s_pad=ld_s_pad)


def test_blocks_linear_fp16_output():
    codes, bscale, qw, w_scale, bias = _random_block_operands(140, 256, 150, 22, spread=1.0)
    _check_blocks_linear(codes, bscale, qw, w_scale, bias, out_dtype=torch.float16)


def test_blocks_linear_extreme_codes():
    """Every product at its largest magnitude, alternating block signs: block sums of
    +-2048 with steps that differ by 2^20 between neighbours."""
    M, K, N = 64, 512, 64
    codes = np.full((M, K), -8, dtype=np.int8)
    qw = np.full((N, K), -8, dtype=np.int8)
    qw[:, 32:64] = 7
    qw[1::2] = -qw[1::2] - 1
    KB = K // G_BLK
    bscale = np.where(np.arange(KB) % 2 == 0, 1.0, 2.0 ** -20).astype(np.float32)[None, :].repeat(M, 0)
    w_scale = np.full(N, 0.5, dtype=np.float32)
    _check_blocks_linear(codes, bscale, qw, w_scale, None)


def test_blocks_linear_equal_steps_reduces_to_the_token_set_linear():
    """With one step for all blocks of a row and sums that stay exact in binary32 the
    result is the whole-K contraction's, bit for bit."""
    M, K, N = 96, 256, 80
    codes = I.random_codes((M, K), 31)
    qw = I.random_codes((N, K), 32)
    rng = np.random.Generator(np.random.PCG64(33))
    row = (2.0 ** rng.integers(-12, 4, M)).astype(np.float32)        # powers of two: exact
    KB = K // G_BLK
    bscale = np.repeat(row[:, None], KB, axis=1)
    w_scale = np.exp(rng.normal(-6.0, 0.5, N)).astype(np.float32)
    Y = _check_blocks_linear(codes, bscale, qw, w_scale, None)
    _, Yt = O.w4a4_linear(codes, row, qw, w_scale)
    assert np.array_equal(Y.astype(np.float32), Yt)


@pytest.mark.parametrize("name,B,T", [("cfg2_fc2", 1, 300), ("cfg2_qkv", 2, 200)])
def test_blocks_path_end_to_end(name, B, T):
    """X -> block quantizer -> block-scaled linear on the GPU against the oracle's
    Algorithm 1 (steps 1-10)."""
    lc = I.case(name, B=B)
    X = _acts(name, B, T)
    W = I.make_weight(lc)
    bias = I.make_bias(lc)
    p = tdq.block_params()
    Q, bs, q_gpu, scale_g = _check_block_quantizer(X, p)
    Wd = torch.from_numpy(W).to(U.dev())
    Qw_d, ws_d = tdq.tdq_quantize_weight(Wd)
    Y = tdq.tdq_w4a4_linear_blocks(Q, bs, lc.C, Qw_d, ws_d, torch.from_numpy(bias).to(U.dev()))
    torch.cuda.synchronize()
    Y = Y.cpu().numpy().astype(np.float64)
    qw, sw = O.quantize_weight(W)
    # the GPU contraction on the GPU's own codes and steps
    KB = -(-lc.C // G_BLK)
    Yself = O.blocks_linear(q_gpu, scale_g, G_BLK, qw, sw, bias)
    tol = _blocks_linear_bound(q_gpu, scale_g, qw, sw, bias, KB)
    assert (np.abs(Y - Yself) <= tol).all()
    # and the whole path against the oracle's own codes and steps
    _, q_ref, _, scale = O.dstg_dcrp_blocks(X.reshape(B * T, lc.C), G_BLK, _oracle_params(p))
    if np.array_equal(q_ref, q_gpu):
        Yref = O.blocks_linear(q_ref, scale, G_BLK, qw, sw, bias)
        tol = _blocks_linear_bound(q_ref, scale, qw, sw, bias, KB) + \
            2 * U.SCALE_RTOL * (tol / ((KB + 3) * 2.0 ** -24))
        assert (np.abs(Y - Yref) <= tol).all()


@pytest.mark.timeout(600)
def test_blocks_linear_full_size_sampled():
    """The 131072 x 1024 -> 4096 shape of the largest configuration in the launch that the
    measurement times, checked on sampled rows."""
    M, K, N = 131072, 1024, 4096
    codes, bscale, qw, w_scale, bias = _random_block_operands(M, K, N, 41, spread=2.0)
    _say(f"[blocks-linear] full size M={M} K={K} N={N}")
    Qx_d = U.pack_to_device(codes)
    Qw_d = U.pack_to_device(qw)
    Y = tdq.tdq_w4a4_linear_blocks(Qx_d, torch.from_numpy(bscale).to(U.dev()), K, Qw_d,
                                   torch.from_numpy(w_scale).to(U.dev()), None, torch.float16)
    torch.cuda.synchronize()
    rows = np.concatenate([np.arange(0, 130), np.arange(M - 130, M),
                           np.random.Generator(np.random.PCG64(5)).integers(0, M, 256)])
    Ys = Y[torch.from_numpy(rows).to(U.dev())].cpu().numpy().astype(np.float64)
    Yref = O.blocks_linear(codes[rows], bscale[rows], G_BLK, qw, w_scale, None)
    tol = _blocks_linear_bound(codes[rows], bscale[rows], qw, w_scale, None, K // G_BLK)
    tol = tol * 1.001 + 2.0 ** -11 * 1.001 * np.abs(Yref) + 2.0 ** -24   # + half an ulp of binary16
    assert (np.abs(Ys - Yref) <= tol).all()


@pytest.mark.timeout(600)
def test_blocks_path_full_size_sampled():
    """The fc2 input of the largest configuration (32 x 4096 tokens x 4096 channels) through
    the per-block quantizer and the block-scaled linear in the launches the measurement
    times; sampled rows against the oracle (every block is local to its row), and sums
    that hold at any size."""
    lc = I.case("cfg4_fc2_h10")
    _say("[blocks full size] generating inputs")
    X, _ = I.make_activations(lc, workers=16)
    W = I.make_weight(lc)
    p = tdq.block_params()
    B, T, C, N = lc.B, lc.T, lc.C, lc.N
    KB = C // G_BLK
    Xd = torch.from_numpy(X).to(U.dev())
    Q, bs, bc = tdq.tdq_quantize_act_blocks(Xd, p, want_clip=True)
    Qw_d, ws_d = tdq.tdq_quantize_weight(torch.from_numpy(W).to(U.dev()))
    Y = tdq.tdq_w4a4_linear_blocks(Q, bs, C, Qw_d, ws_d)
    torch.cuda.synchronize()
    # any size: radius = 7 steps (or the eps floor), no radius above the block maximum
    assert bool(((bc <= bs * 7 * (1 + 1e-6)) & (bs > 0)).all())
    xmax = Xd.reshape(B * T, KB, G_BLK).abs().amax(dim=2).float()
    assert bool((bc <= torch.clamp(xmax, min=1e-8)).all())
    del xmax
    rows = np.concatenate([np.arange(40), np.arange(B * T - 40, B * T),
                           np.random.Generator(np.random.PCG64(8)).integers(0, B * T, 120)])
    rd = torch.from_numpy(rows).to(U.dev())
    Xs = X.reshape(B * T, C)[rows]
    _say("[blocks full size] oracle on sampled rows")
    _, q_ref, clip, scale = O.dstg_dcrp_blocks(Xs, G_BLK, _oracle_params(p))
    cg, sg = bc[rd].cpu().numpy(), bs[rd].cpu().numpy()
    assert np.allclose(cg, clip, rtol=U.SCALE_RTOL, atol=0) and np.allclose(sg, scale, rtol=U.SCALE_RTOL, atol=0)
    q_gpu = O.unpack_nibbles(Q[rd].cpu().numpy()[:, :C // 2], C)
    exact = np.array_equal(cg, clip) and np.array_equal(sg, scale)
    U.assert_codes_match(_blocks_view(q_gpu, C), _blocks_view(q_ref, C),
                         _blocks_view(Xs.astype(np.float32), C), clip.reshape(-1),
                         scale.reshape(-1), exact)
    qw, sw = O.quantize_weight(W)
    Yref = O.blocks_linear(q_gpu, sg, G_BLK, qw, sw, None)
    tol = _blocks_linear_bound(q_gpu, sg, qw, sw, None, KB)
    assert (np.abs(Y[rd].cpu().numpy().astype(np.float64) - Yref) <= tol).all()
    # the same launch shapes on the 6-bit format: the whole of its operand and of its output
    # against the nibble route just checked
    _say("[blocks full size] the 6-bit route")
    F, bs6, bc6 = tdq.tdq_quantize_act_blocks_f6(Xd, p, want_clip=True)
    assert torch.equal(bs6, bs) and torch.equal(bc6, bc)
    assert torch.equal(F, tdq.tdq_pack_codes_f6(Q, C))
    Y6 = tdq.tdq_w4a4_linear_blocks_f6(F, bs6, C, tdq.tdq_pack_codes_f6(Qw_d, C), N, ws_d)
    torch.cuda.synchronize()
    assert torch.equal(Y6, Y)
