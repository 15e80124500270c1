"""CPU oracle for the DSTG + DCRP W4A4 quantized linear path (COD-TDQ).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, obviously-correct numpy
implementation of what the hot path computes.  It shares no code with the HIP
library and must never be imported by the product path: only the tests, the
smoke check and the CPU-baseline leg of the benchmark may call it.

Every function follows a passage of the paper step by step, with statistics in
binary64 and the final scale / rounding arithmetic in binary32 (so that the
rounding boundaries are those of an fp32 device):

  * symmetric a-bit uniform quantizer ........ Sec. 3.1 "Preliminaries",
                                               Sec. 4.1, Eqs. (clipx), (dequant)
  * direct-sum token-group decomposition ..... Sec. 4.2, Eq. (direct_sum)
  * base radius (max-abs or rank quantile) ... Eq. (DSTG_clip), Supp. "Quantile
                                               Implementation"
  * constraint C1 (step-to-dispersion) ....... Eq. (tau_constraint)
  * constraint C2 (zero-bin mass) ............ Eq. (zr_constraint)
  * projection ............................... Eq. (dcrp), Lemma 1
  * forward of the quantized linear .......... Supp. Algorithm 1
  * static per-output-channel weight quant ... Eq. (weight_quant)
  * numerical conventions (eps, rounding) .... Supp. "Reproducibility
                                               Checklist", numerical conventions

A *quantization group* is a multiset of activation elements that shares one
clip radius.  The paper's formulas are stated per group and do not depend on
how a group is formed, so one routine (`dcrp_group`) serves both settings:

  hot-path setting   group = (image, token set S_j), channel block = whole row;
                     tokens are assigned to G sets per image by `assign_groups`
  paper-literal      group = (token, block of g contiguous channels) after
                     zero-padding C to a multiple of g (Algorithm 1, steps 1-2)

Parity status of the pieces the paper does not fix ("parity unpinned"):
  * `assign_groups` — the token -> token-set rule is this build's reading (the
    paper's groups are positional); pinned only by hand-computed cases, the
    G = 1 special case and scale/permutation equivariance.
  * `quantize_weight` scale rule (abs-max / q_max) and the nibble order of
    `pack_nibbles` — the paper calls both implementation details.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

F32 = np.float32

FLAG_C1 = 1   # step-to-dispersion bound active
FLAG_C2 = 2   # zero-bin mass bound active


@dataclass(frozen=True)
class Params:
    """Hyper-parameters (Supp. "Default Hyperparameters": g=32, tau=1, zr=0.2)."""

    n_groups: int = 8          # G token sets per image (hot-path setting)
    act_bits: int = 4
    flags: int = FLAG_C1 | FLAG_C2
    tau: float = 1.0
    zr: float = 0.2
    base_pct: float = 0.0      # 0 or 1: max-abs base radius; (0,1): rank quantile
    eps_scale: float = 1e-8    # floor of the clip radius and of the step
    eps_std: float = 1e-12     # added to the population standard deviation

    @property
    def q_max(self) -> int:
        return 2 ** (self.act_bits - 1) - 1

    @property
    def q_min(self) -> int:
        return -(2 ** (self.act_bits - 1))


# --------------------------------------------------------------------------
# rank rule (Supp. "Quantile Implementation"): k = ceil(p * n), 1-indexed
# --------------------------------------------------------------------------
def quantile_rank(p: float, n: int) -> int:
    """1-indexed rank of the empirical p-quantile of n values, k = ceil(p*n),
    with the product taken in binary64 and the result kept inside [1, n]."""
    k = int(math.ceil(float(p) * float(n)))
    return min(max(k, 1), n)


def kth_smallest(values: np.ndarray, k: int) -> float:
    """k-th smallest value (1-indexed), no interpolation."""
    return np.partition(values, k - 1)[k - 1]


# --------------------------------------------------------------------------
# DCRP on one group (Eqs. DSTG_clip, tau_constraint, zr_constraint, dcrp)
# --------------------------------------------------------------------------
def dcrp_group(values: np.ndarray, p: Params) -> Dict[str, object]:
    """Clip radius and step of ONE quantization group.

    `values` holds every element of the group (any shape, fp16/fp32/fp64).
    Returns n, c_base, sigma, k, thr, c_tau, c_zr, clip, scale, rho0 with the
    floating-point entries as binary32.
    """
    v = np.asarray(values, dtype=np.float64).ravel()
    n = int(v.size)
    eps = F32(p.eps_scale)
    qmax = F32(p.q_max)
    if n == 0:      # paper silent: an empty group gets the floor values
        z = F32(0)
        return dict(n=0, c_base=z, sigma=z, k=0, thr=z, c_tau=z, c_zr=z,
                    clip=eps, scale=eps, rho0=z)
    mag = np.abs(v)
    # base radius: max-abs, or the k = ceil(p n)-th smallest magnitude
    if 0.0 < p.base_pct < 1.0:
        c_base = F32(kth_smallest(mag, quantile_rank(p.base_pct, n)))
    else:
        c_base = F32(mag.max())
    # population standard deviation (two-pass, binary64) plus the stabiliser
    mu = v.sum() / n
    var = ((v - mu) ** 2).sum() / n
    sigma = F32(math.sqrt(var) + p.eps_std)
    # zr rank quantile of the magnitudes
    k = quantile_rank(p.zr, n)
    thr = F32(kth_smallest(mag, k))
    # the two upper bounds, in binary32:  q_max*tau*sigma  and  2*q_max*thr
    c_tau = (qmax * F32(p.tau)) * sigma
    c_zr = (F32(2) * qmax) * thr
    c = c_base
    if p.flags & FLAG_C1:
        c = min(c, c_tau)
    if p.flags & FLAG_C2:
        c = min(c, c_zr)
    c = F32(max(c, eps))                      # c <- max(c, eps)
    scale = F32(max(F32(c / qmax), eps))      # Delta = max(c / q_max, eps)
    rho0 = F32(np.count_nonzero(mag <= float(scale) / 2.0) / n)
    return dict(n=n, c_base=c_base, sigma=sigma, k=k, thr=thr, c_tau=F32(c_tau),
                c_zr=F32(c_zr), clip=c, scale=scale, rho0=rho0)


# --------------------------------------------------------------------------
# hot-path setting: per-token range, token -> token-set assignment
# --------------------------------------------------------------------------
def token_range(X: np.ndarray) -> np.ndarray:
    """r_t = max_c |x_{t,c}| for X[..., C] (the per-token infinity norm of
    Eq. DSTG_clip taken over the whole row), binary32."""
    return np.abs(np.asarray(X, dtype=np.float32)).max(axis=-1)


OCTAVE_FLOOR = 24   # keys more than 24 octaves below the image maximum share bin 0


def assign_groups(r: np.ndarray, G: int) -> np.ndarray:
    """Token-set id of every token of ONE image from its range r[T].

    The key of a token is the bit pattern of its non-negative binary32 range,
    which orders like the value and is roughly linear in log2(r).  Tokens are
    put in G equal-width key bins between the image's smallest and largest key
    (the lower end is raised to at most 24 octaves below the top so a zero
    token cannot stretch the bins).  Integer arithmetic only.
    """
    key = np.ascontiguousarray(r, dtype=np.float32).view(np.uint32).astype(np.int64)
    T = key.size
    gid = np.zeros(T, dtype=np.int32)
    if T == 0 or G == 1:
        return gid
    hi = int(key.max())
    lo = max(int(key.min()), hi - (OCTAVE_FLOOR << 23))
    if hi == lo:
        return gid
    width = hi - lo + 1
    gid[:] = np.where(key <= lo, 0, ((key - lo) * G) // width)
    return gid


def calibrate_groups(X: np.ndarray, p: Params
                     ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, list]:
    """Hot-path calibration for X[B, T, C].

    Returns (gid[B, T] int32, clip[B, G] f32, scale[B, G] f32, stats) where
    stats[b][j] is the dict of `dcrp_group` for token set j of image b.
    """
    X = np.asarray(X)
    B, T, C = X.shape
    G = p.n_groups
    gid = np.zeros((B, T), dtype=np.int32)
    clip = np.zeros((B, G), dtype=np.float32)
    scale = np.zeros((B, G), dtype=np.float32)
    stats = []
    for b in range(B):
        gid[b] = assign_groups(token_range(X[b]), G)
        row = []
        for j in range(G):
            s = dcrp_group(X[b][gid[b] == j], p)
            clip[b, j] = s["clip"]
            scale[b, j] = s["scale"]
            row.append(s)
        stats.append(row)
    return gid, clip, scale, stats


# --------------------------------------------------------------------------
# quantizer (Eqs. clipx, dequant): clip, divide, round-to-nearest-even, clamp
# --------------------------------------------------------------------------
def quantize_codes(x: np.ndarray, clip, scale, p: Params = Params()) -> np.ndarray:
    """Integer codes of x for (broadcastable) clip radius and step, binary32
    arithmetic: q = clamp(rint(clip(x, -c, c) / Delta), q_min, q_max)."""
    x = np.asarray(x, dtype=np.float32)
    c = np.asarray(clip, dtype=np.float32)
    d = np.asarray(scale, dtype=np.float32)
    xt = np.minimum(np.maximum(x, -c), c)
    y = (xt / d).astype(np.float32)           # IEEE binary32 division
    q = np.rint(y)                            # ties to even
    return np.clip(q, p.q_min, p.q_max).astype(np.int8)


def quantize_act(X: np.ndarray, gid: np.ndarray, clip: np.ndarray,
                 scale: np.ndarray, p: Params = Params()) -> np.ndarray:
    """codes[B, T, C] int8 of X[B, T, C] with one (clip, step) per (image,
    token set): row t of image b uses clip[b, gid[b, t]]."""
    B, T, C = X.shape
    rows = np.arange(B)[:, None]
    c_row = clip[rows, gid][..., None]
    d_row = scale[rows, gid][..., None]
    return quantize_codes(X, c_row, d_row, p)


def dequantize(codes: np.ndarray, scale) -> np.ndarray:
    """x_hat = Delta * q in binary32."""
    return codes.astype(np.float32) * np.asarray(scale, dtype=np.float32)


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """Two's-complement int4 codes [..., C] -> bytes [..., ceil(C/2)]: element
    2i in bits 0-3, element 2i+1 in bits 4-7; an odd C pads one zero nibble."""
    q = np.asarray(codes, dtype=np.int8)
    C = q.shape[-1]
    if C % 2:
        q = np.concatenate([q, np.zeros(q.shape[:-1] + (1,), np.int8)], axis=-1)
    u = (q.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed: np.ndarray, C: int) -> np.ndarray:
    """Inverse of `pack_nibbles` (sign-extends each nibble)."""
    b = np.asarray(packed, dtype=np.uint8)
    lo = (b & 0xF).astype(np.int8)
    hi = (b >> 4).astype(np.int8)
    lo = np.where(lo > 7, lo - 16, lo).astype(np.int8)
    hi = np.where(hi > 7, hi - 16, hi).astype(np.int8)
    out = np.empty(b.shape[:-1] + (2 * b.shape[-1],), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out[..., :C]


# --------------------------------------------------------------------------
# paper-literal setting: Algorithm 1 on (token, g-channel block) groups
# --------------------------------------------------------------------------
def dstg_dcrp_blocks(X: np.ndarray, g: int, p: Params):
    """Algorithm 1 steps 1-9 for X[..., C]: zero-pad the channel axis to a
    multiple of g, view as blocks of g channels, one `dcrp_group` per block
    (padding zeros are part of the block), quantize, dequantize, unpad.

    Returns (x_hat[..., C] f32, codes[..., C] int8, clip[..., K] f32,
    scale[..., K] f32)."""
    X = np.asarray(X, dtype=np.float32)
    lead, C = X.shape[:-1], X.shape[-1]
    K = -(-C // g)
    Xp = np.zeros(lead + (K * g,), dtype=np.float32)
    Xp[..., :C] = X
    blocks = Xp.reshape(-1, K, g)
    clip = np.zeros(blocks.shape[:2], dtype=np.float32)
    scale = np.zeros(blocks.shape[:2], dtype=np.float32)
    for m in range(blocks.shape[0]):
        for k in range(K):
            s = dcrp_group(blocks[m, k], p)
            clip[m, k], scale[m, k] = s["clip"], s["scale"]
    codes = quantize_codes(blocks, clip[..., None], scale[..., None], p)
    xhat = dequantize(codes, scale[..., None])
    codes = codes.reshape(lead + (K * g,))[..., :C]
    xhat = xhat.reshape(lead + (K * g,))[..., :C]
    return xhat, codes, clip.reshape(lead + (K,)), scale.reshape(lead + (K,))


def tokenize_chw(X: np.ndarray) -> np.ndarray:
    """The 4-D branch of the dynamic activation path (Supp. "Implementation details"):
    a feature map X[B, C, H, W] becomes tokens X'[B, H*W, C], token t = h*W + w, and
    DSTG + DCRP then run along the channel axis of X'."""
    X = np.asarray(X)
    B, C = X.shape[0], X.shape[1]
    return np.ascontiguousarray(X.reshape(B, C, -1).transpose(0, 2, 1))


# --------------------------------------------------------------------------
# weights (Eq. weight_quant) and the quantized linear (Algorithm 1, step 10)
# --------------------------------------------------------------------------
def quantize_weight(W: np.ndarray, bits: int = 4, eps: float = 1e-8
                    ) -> Tuple[np.ndarray, np.ndarray]:
    """Static symmetric per-output-channel weight quantization of W[O, I]:
    s_o = max(max_i |W_oi|, eps) / q_max,  Q = clamp(rint(W / s_o)).
    Returns (codes[O, I] int8, s[O] f32)."""
    W = np.asarray(W, dtype=np.float32)
    qmax = F32(2 ** (bits - 1) - 1)
    amax = np.maximum(np.abs(W).max(axis=1), F32(eps)).astype(np.float32)
    s = (amax / qmax).astype(np.float32)
    q = np.rint((W / s[:, None]).astype(np.float32))
    q = np.clip(q, -(2 ** (bits - 1)), 2 ** (bits - 1) - 1).astype(np.int8)
    return q, s


def int_accumulate(qx: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """acc[m, n] = sum_i qx[m, i] * qw[n, i], exact integers (int32 result)."""
    acc = qx.astype(np.int64) @ qw.astype(np.int64).T
    assert np.abs(acc).max(initial=0) < 2 ** 31
    return acc.astype(np.int32)


def w4a4_linear(qx: np.ndarray, row_scale: np.ndarray, qw: np.ndarray,
                w_scale: np.ndarray, bias: Optional[np.ndarray] = None
                ) -> Tuple[np.ndarray, np.ndarray]:
    """y = Linear(x_hat, W_hat) written on the integer codes:
    sum_i (Delta q_x)(s q_w) = Delta s sum_i q_x q_w.

    qx[M, K] int8 codes, row_scale[M] f32 (step of each row's token set),
    qw[N, K] int8, w_scale[N] f32.  Returns (acc[M, N] int32, Y[M, N] f32) with
    Y = (f32(acc) * Delta_m) * s_n (+ bias_n), each product rounded to binary32.
    """
    acc = int_accumulate(qx, qw)
    d = np.asarray(row_scale, dtype=np.float32)[:, None]
    s = np.asarray(w_scale, dtype=np.float32)[None, :]
    Y = ((acc.astype(np.float32) * d).astype(np.float32) * s).astype(np.float32)
    if bias is not None:
        Y = (Y + np.asarray(bias, dtype=np.float32)[None, :]).astype(np.float32)
    return acc, Y


def blocks_linear(codes: np.ndarray, block_scale: np.ndarray, g: int, qw: np.ndarray,
                  w_scale: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """Algorithm 1, step 10, in the paper-literal setting: y = Linear(x_hat, W_hat)
    with x_hat[m, i] = Delta[m, i // g] * q_x[m, i] (Eq. dequant, one step per block of
    g channels of every token) and W_hat[n, i] = s_n * q_w[n, i] (Eq. weight_quant),
    evaluated in binary64.

    codes[M, K] int8, block_scale[M, ceil(K/g)] f32, qw[N, K] int8, w_scale[N] f32.
    Returns Y[M, N] float64."""
    codes = np.asarray(codes)
    M, K = codes.shape
    d = np.repeat(np.asarray(block_scale, dtype=np.float64), g, axis=1)[:, :K]
    xhat = d * codes.astype(np.float64)
    what = np.asarray(w_scale, dtype=np.float64)[:, None] * np.asarray(qw).astype(np.float64)
    Y = xhat @ what.T
    if bias is not None:
        Y = Y + np.asarray(bias, dtype=np.float64)[None, :]
    return Y


def row_scales(gid: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Step of every row: scale[b, gid[b, t]] flattened to [B*T]."""
    B = gid.shape[0]
    return scale[np.arange(B)[:, None], gid].reshape(-1)


def tdq_linear_forward(X: np.ndarray, W: np.ndarray, p: Params,
                       bias: Optional[np.ndarray] = None) -> Dict[str, object]:
    """Whole hot path for X[B, T, C], W[N, C] in the hot-path setting."""
    B, T, C = X.shape
    gid, clip, scale, stats = calibrate_groups(X, p)
    qx = quantize_act(X, gid, clip, scale, p)
    qw, sw = quantize_weight(W)
    acc, Y = w4a4_linear(qx.reshape(B * T, C), row_scales(gid, scale), qw, sw, bias)
    return dict(gid=gid, clip=clip, scale=scale, stats=stats, qx=qx, qw=qw,
                w_scale=sw, acc=acc, Y=Y)


# --------------------------------------------------------------------------
# diagnostics (Sec. 3.1: zero-bin mass; SQNR is this build's addition)
# --------------------------------------------------------------------------
def zero_bin_mass(x: np.ndarray, scale) -> float:
    """rho_0 = fraction of elements with |x| <= Delta / 2 (Eq. rho0_def)."""
    x = np.asarray(x, dtype=np.float64)
    return float(np.count_nonzero(np.abs(x) <= np.asarray(scale, np.float64) / 2) / x.size)


def range_disparity(X: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Range disparity of Eq. (range_disparity), per image of X[B, T, C]:
    D = max |x| / median_t median_c |x|.  The paper does not say which median it takes for
    an even count; here it is the lower one, the ceil(n/2)-th smallest, i.e. the paper's
    own rank rule k = ceil(p n) at p = 1/2 (and what `torch.median` returns).
    Returns (D[B] f32 (inf where the denominator is 0), token_median[B, T] f32,
    max_abs[B] f32)."""
    A = np.abs(np.asarray(X, dtype=np.float32))
    B, T, C = A.shape
    tok = np.empty((B, T), dtype=np.float32)
    for b in range(B):
        for t in range(T):
            tok[b, t] = kth_smallest(A[b, t], quantile_rank(0.5, C))
    den = np.array([kth_smallest(tok[b], quantile_rank(0.5, T)) for b in range(B)], dtype=np.float32)
    mx = A.reshape(B, -1).max(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        D = np.where(den > 0, mx / den, np.float32(np.inf)).astype(np.float32)
    return D, tok, mx


def sqnr_db(x: np.ndarray, xhat: np.ndarray) -> float:
    x = np.asarray(x, dtype=np.float64)
    e = x - np.asarray(xhat, dtype=np.float64)
    return float(10.0 * np.log10((x * x).sum() / max((e * e).sum(), 1e-300)))
