"""GPU parity of the 6-bit-format contraction (int4 codes carried exactly as bf6 operands
of the matrix instruction) against the CPU oracle and against the int8 contraction."""
import numpy as np
import pytest
import torch

from oracle import tdq_oracle as O
from paper_2604_16855_amd import inputs as I
from paper_2604_16855_amd import tdq

import parity_util as U
from test_gpu_blocks import _blocks_linear_bound

pytestmark = pytest.mark.gpu

BF6 = np.array([0x00, 0x0C, 0x10, 0x12, 0x14, 0x15, 0x16, 0x17,
                0x38, 0x37, 0x36, 0x35, 0x34, 0x32, 0x30, 0x2C], dtype=np.uint64)


def _say(msg):
    print(msg, flush=True)


def bf6_value(p):
    """Value of a 6-bit e3m2 pattern (1 sign, 3 exponent bits with bias 3, 2 mantissa bits)."""
    s, e, m = (p >> 5) & 1, (p >> 2) & 7, p & 3
    v = (m / 4.0) * 2.0 ** -2 if e == 0 else (1 + m / 4.0) * 2.0 ** (e - 3)
    return -v if s else v


def f6_fragments(codes):
    """Reference of the storage format, written from its definition in the header: int8
    codes [R, K] -> bytes."""
    R, K = codes.shape
    KB = 2 * ((K + 127) // 128)
    RB = (R + 31) // 32
    pad = np.zeros((RB * 32, KB * 64), dtype=np.int64)
    pad[:R, :K] = codes
    pat = BF6[pad & 15]                                   # [rows, k] 6-bit patterns
    # block (rb, kb), lane l = row % 32 + 32 * ((k % 64) // 32), code j = k % 32
    pat = pat.reshape(RB, 32, KB, 2, 32).transpose(0, 2, 3, 1, 4)     # rb, kb, half, row, j
    pat = pat.reshape(RB, KB, 64, 32)
    out = np.zeros((RB, KB, 64, 24), dtype=np.uint8)
    for j in range(32):
        bit = 6 * j
        v = pat[..., j] << np.uint64(bit % 8)             # at most 13 bits
        out[..., bit // 8] |= (v & np.uint64(0xFF)).astype(np.uint8)
        if bit % 8 > 2:
            out[..., bit // 8 + 1] |= (v >> np.uint64(8)).astype(np.uint8)
    return out.reshape(-1)


def test_bf6_patterns_are_the_sixteen_codes():
    for n in range(16):
        code = n if n < 8 else n - 16
        assert bf6_value(int(BF6[n])) == float(code)


@pytest.mark.parametrize("R,K", [(1, 1), (33, 70), (64, 128), (100, 129), (257, 1000), (32, 4096)])
def test_pack_codes_f6_matches_the_format(R, K):
    codes = I.random_codes((R, K), 50 + R)
    F = tdq.tdq_pack_codes_f6(U.pack_to_device(codes), K)
    torch.cuda.synchronize()
    ref = f6_fragments(codes)
    assert F.numel() == ref.size == tdq.f6_bytes(R, K)
    assert np.array_equal(F.cpu().numpy(), ref)


@pytest.mark.parametrize("R,K,ld_pad,off", [(70, 200, 5, 0), (33, 129, 0, 3), (64, 256, 16, 0), (40, 63, 1, 1)])
def test_pack_codes_f6_unaligned_rows_and_junk_pad_nibble(R, K, ld_pad, off):
    """Rows that do not start on 16-byte boundaries (a view into a wider buffer) take the
    byte loads; whatever stands in the unused high nibble of an odd row's last byte and in
    the bytes behind a row is not read as codes."""
    codes = I.random_codes((R, K), 90 + R)
    packed = O.pack_nibbles(codes)                                   # [R, ceil(K / 2)]
    nb = packed.shape[1]
    wide = np.full((R, off + nb + ld_pad), 0xEE, dtype=np.uint8)
    wide[:, off:off + nb] = packed
    if K % 2:
        wide[:, off + nb - 1] |= 0xF0                               # junk in the pad nibble
    Qd = torch.from_numpy(wide).to(U.dev())[:, off:off + nb]
    F = tdq.tdq_pack_codes_f6(Qd, K)
    torch.cuda.synchronize()
    assert np.array_equal(F.cpu().numpy(), f6_fragments(codes))


def _f6_linear(codes, qw, gid, scale, B, T, bias=None, out_dtype=torch.float32):
    M, K = codes.shape
    N = qw.shape[0]
    A6 = torch.from_numpy(f6_fragments(codes)).to(U.dev())
    B6 = torch.from_numpy(f6_fragments(qw)).to(U.dev())
    acc = torch.empty((M, N), dtype=torch.int32, device=U.dev())
    Y = tdq.tdq_w4a4_linear_f6(A6, None if gid is None else torch.from_numpy(gid).to(U.dev()),
                               torch.from_numpy(scale).to(U.dev()), B, T, K, B6, N,
                               torch.from_numpy(np.ones(N, np.float32) if False else WS[:N]).to(U.dev()),
                               None if bias is None else torch.from_numpy(bias).to(U.dev()), out_dtype,
                               acc_dump=acc)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), Y.cpu().numpy()


WS = np.exp(np.random.Generator(np.random.PCG64(77)).normal(-6.0, 0.5, 8192)).astype(np.float32)


@pytest.mark.parametrize("B,T,K,N,G,with_bias,out_dtype", [
    (1, 1, 1, 1, 1, False, torch.float32), (1, 5, 31, 3, 2, True, torch.float32),
    (2, 32, 64, 64, 4, False, torch.float32), (1, 129, 130, 130, 3, True, torch.float32),
    (3, 100, 320, 200, 8, False, torch.float16), (1, 300, 1280, 320, 16, True, torch.float32),
    (2, 256, 4100, 140, 5, False, torch.float32), (1, 512, 256, 512, 1, True, torch.float16)])
def test_f6_contraction_bit_exact(B, T, K, N, G, with_bias, out_dtype):
    _say(f"[f6] B={B} T={T} K={K} N={N} G={G} bias={with_bias} out={out_dtype}")
    M = B * T
    rng = np.random.Generator(np.random.PCG64([B, T, K, N]))
    codes = I.random_codes((M, K), 60)
    qw = I.random_codes((N, K), 61)
    gid = rng.integers(0, G, (B, T)).astype(np.int32)
    scale = np.exp(rng.normal(-3, 1, (B, G))).astype(np.float32)
    bias = rng.normal(0, 0.02, N).astype(np.float32) if with_bias else None
    acc, Y = _f6_linear(codes, qw, gid if G > 1 else None, scale, B, T, bias, out_dtype)
    acc_ref, Y_ref = O.w4a4_linear(codes, O.row_scales(gid if G > 1 else np.zeros_like(gid), scale),
                                   qw, WS[:N], bias)
    assert np.array_equal(acc, acc_ref), "accumulators differ"
    if out_dtype == torch.float16:
        assert np.array_equal(Y, Y_ref.astype(np.float16))
    else:
        assert np.array_equal(Y, Y_ref)


def test_f6_contraction_extreme_accumulator():
    """All codes -8 on both sides and K = 4096: the largest sum, 4096 * 64 = 2^18, and its
    negative with codes 7 against -8."""
    M, K, N = 64, 4096, 64
    codes = np.full((M, K), -8, dtype=np.int8)
    qw = np.full((N, K), -8, dtype=np.int8)
    qw[1::2] = 7
    scale = np.ones((1, 1), np.float32)
    acc, _ = _f6_linear(codes, qw, None, scale, 1, M)
    assert (acc[:, 0::2] == 64 * K).all() and (acc[:, 1::2] == -56 * K).all()


@pytest.mark.timeout(600)
def test_f6_contraction_full_size_sampled():
    """131072 x 1024 -> 4096 in the launch the measurement times; sampled rows bit-exact."""
    M, K, N = 131072, 1024, 4096
    codes = I.random_codes((M, K), 62)
    qw = I.random_codes((N, K), 63)
    B, T, G = 32, 4096, 32
    rng = np.random.Generator(np.random.PCG64(64))
    gid = rng.integers(0, G, (B, T)).astype(np.int32)
    scale = np.exp(rng.normal(-3, 1, (B, G))).astype(np.float32)
    A6 = tdq.tdq_pack_codes_f6(U.pack_to_device(codes), K)
    B6 = tdq.tdq_pack_codes_f6(U.pack_to_device(qw), K)
    Y = tdq.tdq_w4a4_linear_f6(A6, torch.from_numpy(gid).to(U.dev()), torch.from_numpy(scale).to(U.dev()),
                               B, T, K, B6, N, torch.from_numpy(WS[:N]).to(U.dev()), None, torch.float16)
    torch.cuda.synchronize()
    rows = np.concatenate([np.arange(130), np.arange(M - 130, M),
                           np.random.Generator(np.random.PCG64(5)).integers(0, M, 256)])
    _, Y_ref = O.w4a4_linear(codes[rows], O.row_scales(gid, scale)[rows], qw, WS[:N])
    Ys = Y[torch.from_numpy(rows).to(U.dev())].cpu().numpy()
    assert np.array_equal(Ys, Y_ref.astype(np.float16))


@pytest.mark.parametrize("B,T,C,G,dtype,ld_pad", [
    (2, 484, 320, 16, "f16", 0), (3, 37, 70, 5, "f16", 0), (2, 50, 33, 4, "f16", 0),
    (2, 41, 64, 8, "f16", 3), (1, 1, 8, 1, "f32", 0), (2, 129, 100, 32, "f32", 1),
    (1, 300, 520, 1, "f16", 0), (1, 64, 2050, 8, "f16", 0)])
def test_quantizer_writes_f6_fragments(B, T, C, G, dtype, ld_pad):
    """tdq_quantize_act_f6: the fragments of the oracle's codes (given the oracle's radii),
    and the same bytes as packing the nibble quantizer's output."""
    _say(f"[quantize-f6] B={B} T={T} C={C} G={G} {dtype} ld_pad={ld_pad}")
    lc = I.LinearCase("f6", B, T, C, 8, G, dtype, 0.1, 0.1, False, (T, 1), 900 + C)
    X, _ = I.make_activations(lc)
    p = tdq.default_params(G)
    gid, clip, scale, _ = O.calibrate_groups(X, U.oracle_params(p))
    q_ref = O.quantize_act(X, gid, clip, scale, U.oracle_params(p)).reshape(B * T, C)
    Xd = U.to_device(X, ld_pad)
    gid_d = None if G == 1 else torch.from_numpy(gid).to(U.dev())
    clip_d, scale_d = torch.from_numpy(clip).to(U.dev()), torch.from_numpy(scale).to(U.dev())
    F = tdq.tdq_quantize_act_f6(Xd, p, gid_d, clip_d, scale_d)
    Q = tdq.tdq_quantize_act(Xd, p, gid_d, clip_d, scale_d)
    F2 = tdq.tdq_pack_codes_f6(Q, C)
    torch.cuda.synchronize()
    assert np.array_equal(F.cpu().numpy(), f6_fragments(q_ref))
    assert torch.equal(F, F2)


def test_quantizer_f6_clamps_user_radii():
    rng = np.random.Generator(np.random.PCG64(10))
    X = (rng.laplace(0, 4, (1, 40, 64))).astype(np.float32)
    gid = np.zeros((1, 40), np.int32)
    clip = np.array([[100.0]], np.float32)
    scale = np.array([[0.37]], np.float32)
    p = tdq.default_params(1)
    q_ref = O.quantize_act(X, gid, clip, scale, U.oracle_params(p)).reshape(40, 64)
    assert q_ref.min() == -8 and q_ref.max() == 7
    F = tdq.tdq_quantize_act_f6(torch.from_numpy(X).to(U.dev()), p, None,
                                torch.from_numpy(clip).to(U.dev()), torch.from_numpy(scale).to(U.dev()))
    torch.cuda.synchronize()
    assert np.array_equal(F.cpu().numpy(), f6_fragments(q_ref))


def test_f6_path_end_to_end():
    """calibrate -> quantize_f6 -> linear_f6 equals calibrate -> quantize -> linear, bit for bit."""
    lc = I.case("cfg2_fc2", B=3)
    X, _ = I.make_activations(lc)
    W = I.make_weight(lc)
    p = tdq.default_params(lc.G)
    Xd = torch.from_numpy(X).to(U.dev())
    gid, clip, scale, _, ws = tdq.tdq_calibrate_groups(Xd, p)
    Qw, sw = tdq.tdq_quantize_weight(torch.from_numpy(W).to(U.dev()))
    Y1 = tdq.tdq_w4a4_linear(tdq.tdq_quantize_act(Xd, p, gid, clip, scale), gid, scale, lc.B, lc.T,
                             lc.C, Qw, sw)
    Y2 = tdq.tdq_w4a4_linear_f6(tdq.tdq_quantize_act_f6(Xd, p, gid, clip, scale), gid, scale, lc.B,
                                lc.T, lc.C, tdq.tdq_pack_codes_f6(Qw, lc.C), lc.N, sw)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
    ref = O.tdq_linear_forward(X, W, O.Params(n_groups=lc.G))
    if np.array_equal(scale.cpu().numpy(), ref["scale"]):
        assert np.array_equal(Y2.cpu().numpy(), ref["Y"])


@pytest.mark.parametrize("M,K,N,with_bias,out_dtype", [
    (1, 1, 1, False, torch.float32), (5, 31, 3, True, torch.float32), (64, 33, 64, False, torch.float32),
    (129, 64, 130, True, torch.float32), (300, 320, 200, False, torch.float16),
    (256, 1280, 320, True, torch.float32), (130, 4100, 140, False, torch.float32),
    (200, 128, 129, True, torch.float16)])
def test_f6_block_scaled_linear_equals_the_int8_one(M, K, N, with_bias, out_dtype):
    """tdq_w4a4_linear_blocks_f6: the same bits as tdq_w4a4_linear_blocks, and within the
    bound of the binary32 evaluation of the oracle's Algorithm 1 linear."""
    _say(f"[f6-blocks] M={M} K={K} N={N} bias={with_bias} out={out_dtype}")
    rng = np.random.Generator(np.random.PCG64([M, K, N, 3]))
    KB = -(-K // 32)
    codes = I.random_codes((M, K), 70)
    qw = I.random_codes((N, K), 71)
    spread = 1.0 if out_dtype == torch.float16 else 4.0        # keep binary16 outputs finite
    bscale = np.exp(rng.normal(-3.0, spread, (M, KB))).astype(np.float32)
    bias = rng.normal(0, 0.02, N).astype(np.float32) if with_bias else None
    bs_d = torch.from_numpy(bscale).to(U.dev())
    ws_d = torch.from_numpy(WS[:N]).to(U.dev())
    bias_d = None if bias is None else torch.from_numpy(bias).to(U.dev())
    A6 = torch.from_numpy(f6_fragments(codes)).to(U.dev())
    B6 = torch.from_numpy(f6_fragments(qw)).to(U.dev())
    Y6 = tdq.tdq_w4a4_linear_blocks_f6(A6, bs_d, K, B6, N, ws_d, bias_d, out_dtype)
    Y8 = tdq.tdq_w4a4_linear_blocks(U.pack_to_device(codes), bs_d, K, U.pack_to_device(qw), ws_d, bias_d,
                                    out_dtype)
    torch.cuda.synchronize()
    assert torch.equal(Y6, Y8)
    Yref = O.blocks_linear(codes, bscale, 32, qw, WS[:N], bias)
    tol = _blocks_linear_bound(codes, bscale, qw, WS[:N], bias, KB)
    if out_dtype == torch.float16:
        tol = tol * 1.001 + 2.0 ** -11 * 1.001 * np.abs(Yref) + 2.0 ** -24   # + half an ulp of binary16
    assert (np.abs(Y6.cpu().numpy().astype(np.float64) - Yref) <= tol).all()


@pytest.mark.parametrize("M,K,N,with_bias,out_dtype", [
    (16500, 200, 1030, True, torch.float32), (33000, 96, 520, False, torch.float16)])
def test_f6_block_scaled_linear_many_tiles(M, K, N, with_bias, out_dtype):
    """Several workgroups per CU, ragged in M, K and N: the same bits as
    tdq_w4a4_linear_blocks everywhere, and sampled rows within the bound of the oracle's
    Algorithm 1 linear."""
    _say(f"[f6-blocks-many] M={M} K={K} N={N} bias={with_bias} out={out_dtype}")
    rng = np.random.Generator(np.random.PCG64([M, K, N, 5]))
    KB = -(-K // 32)
    codes = I.random_codes((M, K), 72)
    qw = I.random_codes((N, K), 73)
    bscale = np.exp(rng.normal(-3.0, 1.0, (M, KB))).astype(np.float32)
    wsc = np.exp(rng.normal(-4.0, 0.5, N)).astype(np.float32)
    bias = rng.normal(0, 0.02, N).astype(np.float32) if with_bias else None
    bs_d = torch.from_numpy(bscale).to(U.dev())
    ws_d = torch.from_numpy(wsc).to(U.dev())
    bias_d = None if bias is None else torch.from_numpy(bias).to(U.dev())
    A6 = tdq.tdq_pack_codes_f6(U.pack_to_device(codes), K)
    B6 = tdq.tdq_pack_codes_f6(U.pack_to_device(qw), K)
    Y6 = tdq.tdq_w4a4_linear_blocks_f6(A6, bs_d, K, B6, N, ws_d, bias_d, out_dtype)
    Y8 = tdq.tdq_w4a4_linear_blocks(U.pack_to_device(codes), bs_d, K, U.pack_to_device(qw), ws_d, bias_d,
                                    out_dtype)
    torch.cuda.synchronize()
    assert torch.equal(Y6, Y8)
    rows = np.unique(np.concatenate([np.arange(0, 300), np.arange(M - 300, M),
                                     rng.integers(0, M, 200)]))
    Yref = O.blocks_linear(codes[rows], bscale[rows], 32, qw, wsc, bias)
    tol = _blocks_linear_bound(codes[rows], bscale[rows], qw, wsc, bias, KB)
    if out_dtype == torch.float16:
        tol = tol * 1.001 + 2.0 ** -11 * 1.001 * np.abs(Yref) + 2.0 ** -24
    got = Y6[torch.from_numpy(rows).to(U.dev())].cpu().numpy().astype(np.float64)
    assert (np.abs(got - Yref) <= tol).all()


@pytest.mark.parametrize("B,T,C,dtype,ld_pad,variant", [
    (1, 77, 80, np.float16, 0, (3, 1.0, 0.2, 0.0)),      # last block half padding, one K tile
    (1, 1000, 33, np.float16, 0, (3, 1.0, 0.2, 0.0)),    # odd C
    (1, 5, 7, np.float16, 0, (3, 1.0, 0.2, 0.0)),
    (3, 50, 4100, np.float16, 0, (3, 1.0, 0.2, 0.0)),    # scalar loads, many K tiles, ragged last
    (2, 64, 1024, np.float16, 8, (3, 1.0, 0.2, 0.0)),    # whole tiles
    (2, 33, 96, np.float16, 3, (2, 1.0, 0.6, 0.0)),      # unaligned rows, bisection rank
    (1, 200, 96, np.float32, 0, (3, 2.0, 0.1, 0.0)),
    (2, 64, 1000, np.float32, 0, (0, 1.0, 0.2, 0.9)),    # percentile base radius
    (1, 31, 45, np.float32, 5, (1, 0.3, 0.2, 0.0)),
    (1, 300, 544, np.float16, 0, (3, 1.0, 0.2, 0.5)),    # 17 blocks: second K tile holds one
])
def test_block_quantizer_f6_equals_the_nibble_one(B, T, C, dtype, ld_pad, variant):
    """tdq_quantize_act_blocks_f6: steps and radii bit for bit those of
    tdq_quantize_act_blocks (checked against the oracle in test_gpu_blocks.py), and the
    fragments are its codes in the storage format written out above, padding zero."""
    flags, tau, zr, base_pct = variant
    _say(f"[f6-blockquant] B={B} T={T} C={C} dtype={dtype.__name__} ld_pad={ld_pad} variant={variant}")
    rng = np.random.Generator(np.random.PCG64([B, T, C, 9]))
    X = rng.standard_normal((B, T, C)) * np.exp(rng.normal(0, 1.5, (B, T, 1)))
    X[rng.random((B, T, C)) < 0.02] *= 30.0
    X = X.astype(dtype)
    p = tdq.block_params(tau, zr, flags, base_pct)
    Xd = U.to_device(X, ld_pad)
    Q, bs, bc = tdq.tdq_quantize_act_blocks(Xd, p, want_clip=True)
    F = torch.full((tdq.f6_bytes(B * T, C),), 0xA5, dtype=torch.uint8, device=U.dev())   # all must be written
    bs6 = torch.full_like(bs, float("nan"))
    F, bs6, bc6 = tdq.tdq_quantize_act_blocks_f6(Xd, p, want_clip=True, out=(F, bs6))
    torch.cuda.synchronize()
    assert torch.equal(bs6, bs) and torch.equal(bc6, bc)
    codes = U.unpack_device_codes(Q, C)
    assert np.array_equal(F.cpu().numpy(), f6_fragments(codes))


def test_blocks_f6_path_end_to_end():
    """Activations -> tdq_quantize_act_blocks_f6 -> tdq_w4a4_linear_blocks_f6: the bits of
    the nibble route (tdq_quantize_act_blocks -> tdq_w4a4_linear_blocks)."""
    lc = I.case("cfg2_fc2", B=2)
    X, _ = I.make_activations(lc)
    X = np.ascontiguousarray(X[:, :300])
    W = I.make_weight(lc)
    _say(f"[f6-blocks-e2e] {lc.name} X={X.shape} W={W.shape}")
    p = tdq.block_params()
    Xd = U.to_device(X)
    Wd = torch.from_numpy(W).to(U.dev())
    Qw, sw = tdq.tdq_quantize_weight(Wd)
    Q, bs, _ = tdq.tdq_quantize_act_blocks(Xd, p)
    Y8 = tdq.tdq_w4a4_linear_blocks(Q, bs, lc.C, Qw, sw)
    F, bs6, _ = tdq.tdq_quantize_act_blocks_f6(Xd, p)
    Y6 = tdq.tdq_w4a4_linear_blocks_f6(F, bs6, lc.C, tdq.tdq_pack_codes_f6(Qw, lc.C), lc.N, sw)
    torch.cuda.synchronize()
    assert torch.equal(Y6, Y8)


@pytest.mark.parametrize("out_dtype,ld_y_pad,ld_s_pad", [
    (torch.float32, 5, 3), (torch.float16, 3, 1), (torch.float32, 4, 0), (torch.float16, 8, 2)])
def test_f6_block_scaled_linear_strided_outputs_and_steps(out_dtype, ld_y_pad, ld_s_pad):
    """Rows of Y and of the steps longer than their data (views of wider buffers): rows of
    Y that do not start on 16-byte boundaries take the element-wise stores; the padding
    is left alone."""
    M, K, N = 300, 200, 260
    _say(f"[f6-blocks-strided] out={out_dtype} ld_y_pad={ld_y_pad} ld_s_pad={ld_s_pad}")
    rng = np.random.Generator(np.random.PCG64([ld_y_pad, ld_s_pad, 11]))
    KB = -(-K // 32)
    codes = I.random_codes((M, K), 74)
    qw = I.random_codes((N, K), 75)
    bscale = np.exp(rng.normal(-3.0, 1.0, (M, KB))).astype(np.float32)
    bias = rng.normal(0, 0.02, N).astype(np.float32)
    wide = torch.full((M, KB + ld_s_pad), float("nan"), dtype=torch.float32, device=U.dev())
    wide[:, :KB] = torch.from_numpy(bscale).to(U.dev())
    bs_d = wide[:, :KB]
    ws_d = torch.from_numpy(WS[:N]).to(U.dev())
    bias_d = torch.from_numpy(bias).to(U.dev())
    A6 = tdq.tdq_pack_codes_f6(U.pack_to_device(codes), K)
    B6 = tdq.tdq_pack_codes_f6(U.pack_to_device(qw), K)
    Ybuf = torch.full((M, N + ld_y_pad), -77.0, dtype=out_dtype, device=U.dev())
    Y6 = tdq.tdq_w4a4_linear_blocks_f6(A6, bs_d, K, B6, N, ws_d, bias_d, out=Ybuf[:, :N])
    Y8 = tdq.tdq_w4a4_linear_blocks(U.pack_to_device(codes), bs_d.contiguous(), K, U.pack_to_device(qw),
                                    ws_d, bias_d, out_dtype)
    torch.cuda.synchronize()
    assert torch.equal(Y6, Y8)
    assert bool((Ybuf[:, N:] == -77.0).all())


def test_block_scaled_linears_at_the_largest_k():
    """K = 131072, the largest the block-scaled entry points accept (4096 blocks, 1024
    stages of the 6-bit kernel): both routes against the oracle, and equal to each other."""
    M, K, N = 40, 131072, 24
    _say(f"[blocks-max-K] M={M} K={K} N={N}")
    rng = np.random.Generator(np.random.PCG64([M, K, N, 13]))
    KB = K // 32
    codes = I.random_codes((M, K), 76)
    qw = I.random_codes((N, K), 77)
    bscale = np.exp(rng.normal(-3.0, 1.0, (M, KB))).astype(np.float32)
    bs_d = torch.from_numpy(bscale).to(U.dev())
    ws_d = torch.from_numpy(WS[:N]).to(U.dev())
    Qx, Qw = U.pack_to_device(codes), U.pack_to_device(qw)
    Y8 = tdq.tdq_w4a4_linear_blocks(Qx, bs_d, K, Qw, ws_d)
    Y6 = tdq.tdq_w4a4_linear_blocks_f6(tdq.tdq_pack_codes_f6(Qx, K), bs_d, K, tdq.tdq_pack_codes_f6(Qw, K),
                                       N, ws_d)
    torch.cuda.synchronize()
    assert torch.equal(Y6, Y8)
    Yref = O.blocks_linear(codes, bscale, 32, qw, WS[:N], None)
    tol = _blocks_linear_bound(codes, bscale, qw, WS[:N], None, KB)
    assert (np.abs(Y6.cpu().numpy().astype(np.float64) - Yref) <= tol).all()
    # one more code than the limit is refused
    L = tdq.lib()
    assert L.tdq_w4a4_linear_blocks_f6(Qx.data_ptr(), bs_d.data_ptr(), KB + 1, M, K + 1, N, Qw.data_ptr(),
                                       ws_d.data_ptr(), None, Y6.data_ptr(), tdq.TDQ_F32, N, None) == tdq.ERR_SHAPE
