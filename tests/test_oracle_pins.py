"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP path.  Each one checks the oracle against
something other than itself: the paper's printed rank example, a group worked
by hand, Lemma 1 / Proposition 1, closed-form population quantiles, special
cases that reduce to a textbook routine, brute-force search on tiny inputs and
exact symmetries.
"""
import math
import os

import numpy as np
import pytest

from oracle import tdq_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
P0 = O.Params()


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _groups(seed, count=40):
    """A zoo of groups: different laws, sizes, offsets, exact zeros, ties."""
    rng = _rng(seed)
    out = []
    for i in range(count):
        n = int(rng.integers(5, 3000))
        kind = i % 6
        if kind == 0:
            v = rng.laplace(0, 1, n)
        elif kind == 1:
            v = 20 * rng.standard_t(2, n)
        elif kind == 2:
            v = 0.05 * np.sin(np.arange(n) * 0.3) + rng.normal(0, 0.01, n)
        elif kind == 3:
            v = rng.normal(3.0, 0.2, n)                     # offset: C1 binds
        elif kind == 4:
            v = np.round(rng.normal(0, 2, n))               # many ties and zeros
        else:
            v = rng.uniform(-1, 1, n)
        out.append(v.astype(np.float32))
    return out


# ---------------------------------------------------------------- rank rule
def test_rank_rule_golden():
    """Supp. 'Quantile Implementation': k = ceil(p n); 32 values at p = 0.99
    give rank 32, the group maximum."""
    for line in open(os.path.join(GOLD, "rank_rule.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n, p, k, _ = line.split()
        assert O.quantile_rank(float(p), int(n)) == int(k), line
    v = _rng(1).normal(size=32)
    assert O.kth_smallest(np.abs(v), O.quantile_rank(0.99, 32)) == np.abs(v).max()


def test_kth_smallest_is_sorted_element():
    rng = _rng(2)
    for _ in range(50):
        n = int(rng.integers(1, 200))
        v = np.round(rng.normal(0, 3, n), 1)                # ties on purpose
        k = int(rng.integers(1, n + 1))
        assert O.kth_smallest(v, k) == np.sort(v)[k - 1]


def test_percentile_base_radius():
    """Eq. (DSTG_clip), percentile branch: base radius is the ceil(p n)-th
    smallest magnitude; p = 0.99 on 32 values is the maximum."""
    v = _rng(3).laplace(size=32).astype(np.float32)
    s_max = O.dcrp_group(v, O.Params(flags=0))
    s_p99 = O.dcrp_group(v, O.Params(flags=0, base_pct=0.99))
    assert s_p99["c_base"] == s_max["c_base"] == np.abs(v).max()
    s_p50 = O.dcrp_group(v, O.Params(flags=0, base_pct=0.5))
    assert s_p50["c_base"] == np.sort(np.abs(v))[15]


# --------------------------------------------------- hand-worked DCRP group
def _read_example():
    d = {}
    for line in open(os.path.join(GOLD, "dcrp_worked_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *vals = line.split()
        d[k] = [float(x) for x in vals]
    return d


def test_dcrp_worked_example():
    ex = _read_example()
    v = np.array(ex["values"], dtype=np.float32)
    s = O.dcrp_group(v, P0)
    assert s["n"] == 10 and s["k"] == 2
    assert s["thr"] == np.float32(ex["thr"][0])
    assert s["c_base"] == np.float32(ex["c_base"][0])
    assert s["c_zr"] == np.float32(ex["c_zr"][0])
    assert abs(float(s["sigma"]) - ex["sigma"][0]) <= 1e-7 * ex["sigma"][0]
    assert abs(float(s["c_tau"]) - ex["c_tau"][0]) <= 2e-7 * ex["c_tau"][0]
    assert s["clip"] == np.float32(ex["clip"][0])
    assert s["scale"] == np.float32(ex["scale"][0])
    assert abs(float(s["rho0"]) - ex["rho0"][0]) < 1e-7
    q = O.quantize_codes(v, s["clip"], s["scale"])
    assert q.tolist() == [int(c) for c in ex["codes"]]


def test_assign_examples_golden():
    for line in open(os.path.join(GOLD, "assign_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        G, r, ids = [s.strip() for s in line.split("|")]
        r = np.array([float(x) for x in r.split()], dtype=np.float32)
        got = O.assign_groups(r, int(G))
        assert got.tolist() == [int(x) for x in ids.split()], line


# ---------------------------------------------------------- Lemma 1 (C1, C2)
@pytest.mark.parametrize("seed", [10, 11, 12])
def test_lemma1_both_constraints_hold(seed):
    """After projection Delta <= tau*sigma and Delta/2 <= Q_zr(|x|); the open
    zero-bin count is below zr*n and the closed one is at most the number of
    magnitudes not above the rank threshold (the discrete-rank slack)."""
    for tau, zr in ((1.0, 0.2), (0.3, 0.2), (1.0, 0.05), (2.0, 0.5)):
        p = O.Params(tau=tau, zr=zr)
        for v in _groups(seed):
            s = O.dcrp_group(v, p)
            if s["clip"] <= np.float32(p.eps_scale):
                continue
            d, sig, thr = float(s["scale"]), float(s["sigma"]), float(s["thr"])
            slack = 1 + 4 * 2.0 ** -24
            assert d <= tau * sig * slack
            assert d / 2 <= thr * slack
            mag = np.abs(v.astype(np.float64))
            assert np.count_nonzero(mag < d / 2 * (1 - 2.0 ** -22)) < zr * v.size
            assert (np.count_nonzero(mag <= d / 2 * (1 - 2.0 ** -22))
                    <= np.count_nonzero(mag <= thr))
            # the projected radius never exceeds the base radius
            assert s["clip"] <= s["c_base"]


def test_projection_is_min_of_three_and_flags():
    """Eq. (dcrp): c = min(c_base, c_tau, c_zr); a bound that is switched off
    drops out (Algorithm 1 step 4: without DCRP c = c_base)."""
    for v in _groups(20, 24):
        full = O.dcrp_group(v, P0)
        eps = np.float32(1e-8)
        assert full["clip"] == max(min(full["c_base"], full["c_tau"], full["c_zr"]), eps)
        only1 = O.dcrp_group(v, O.Params(flags=O.FLAG_C1))
        assert only1["clip"] == max(min(full["c_base"], full["c_tau"]), eps)
        only2 = O.dcrp_group(v, O.Params(flags=O.FLAG_C2))
        assert only2["clip"] == max(min(full["c_base"], full["c_zr"]), eps)
        none = O.dcrp_group(v, O.Params(flags=0))
        assert none["clip"] == max(full["c_base"], eps)
        assert none["clip"] >= only1["clip"] >= full["clip"]


def test_sigma_is_population_std():
    """Std with unbiased=False plus 1e-12 (numerical conventions)."""
    for v in _groups(21, 18):
        s = O.dcrp_group(v, P0)
        ref = np.std(v.astype(np.float64), ddof=0) + 1e-12
        assert abs(float(s["sigma"]) - ref) <= 6e-8 * ref + 1e-45
        if v.size > 1:      # and it is NOT the unbiased one
            unb = np.std(v.astype(np.float64), ddof=1)
            if v.size < 500:
                assert abs(float(s["sigma"]) - unb) > 1e-5 * unb


# --------------------------------------------- brute force on tiny inputs
@pytest.mark.parametrize("seed", range(6))
def test_clip_matches_brute_force_grid(seed):
    """The largest radius on a dense grid over (0, c_base] that satisfies both
    constraints as stated (step <= tau*sigma, fewer than zr*n magnitudes
    strictly inside the zero bin) is the oracle's radius, to one grid step."""
    rng = _rng(100 + seed)
    n = int(rng.integers(8, 400))
    v = [rng.laplace(0, 1, n), 20 * rng.standard_t(2, n), rng.normal(1.5, 0.3, n),
         rng.uniform(-2, 2, n), rng.normal(0, 1, n), rng.laplace(0, 0.1, n)][seed]
    v = v.astype(np.float32).astype(np.float64)
    tau, zr = (1.0, 0.2) if seed % 2 == 0 else (0.5, 0.3)
    s = O.dcrp_group(v, O.Params(tau=tau, zr=zr))
    mag = np.abs(v)
    sigma = np.std(v) + 1e-12
    c_base = mag.max()
    grid = np.unique(np.concatenate([
        np.linspace(0, c_base, 2 ** 16 + 1)[1:], 14 * mag[14 * mag <= c_base],
        [min(7 * tau * sigma, c_base)]]))
    srt = np.sort(mag)
    inside = np.searchsorted(srt, grid / 14, side="left")   # #{|x| < c/14}
    ok = (grid / 7 <= tau * sigma * (1 + 1e-12)) & (inside < zr * n)
    best = grid[ok].max()
    step = c_base / 2 ** 16
    assert abs(best - float(s["clip"])) <= step + 1e-6 * best


# ----------------------------------------------- closed forms, large groups
def test_closed_form_laplace_c2_binds():
    """Laplace(0,b): Q_0.2(|x|) = b ln(1/0.8), so c -> 14 b ln 1.25 = 3.1240 b
    (< c_tau = 7 sqrt(2) b = 9.90 b)."""
    n, b = 2_000_000, 0.7
    v = _rng(30).laplace(0, b, n)
    s = O.dcrp_group(v, P0)
    assert abs(float(s["clip"]) / (14 * b * math.log(1.25)) - 1) < 6e-3
    assert abs(float(s["c_tau"]) / (7 * math.sqrt(2) * b) - 1) < 6e-3
    assert s["clip"] == s["c_zr"]


def test_closed_form_normal_c2_binds():
    """N(0,s^2): Q_0.2(|x|) = s * Phi^-1(0.6) = 0.253347 s -> c = 3.54686 s."""
    n, sd = 2_000_000, 1.3
    v = _rng(31).normal(0, sd, n)
    s = O.dcrp_group(v, P0)
    assert abs(float(s["clip"]) / (14 * 0.2533471031357997 * sd) - 1) < 6e-3
    assert s["clip"] == s["c_zr"]


def test_closed_form_uniform_base_binds():
    """Uniform(-a,a): c_zr = 14*0.2a = 2.8a and c_tau = 7a/sqrt(3) = 4.04a both
    exceed max|x| -> a, so the base radius survives."""
    n, a = 1_000_000, 2.0
    v = _rng(32).uniform(-a, a, n)
    s = O.dcrp_group(v, P0)
    assert s["clip"] == s["c_base"] == np.float32(np.abs(v).max())
    assert abs(float(s["c_zr"]) / (2.8 * a) - 1) < 5e-3
    assert abs(float(s["c_tau"]) / (7 * a / math.sqrt(3)) - 1) < 5e-3


def test_closed_form_c1_binds():
    """tau = 0.3 on Laplace: c = 7*0.3*sqrt(2) b = 2.970 b < 3.124 b; and offset
    data mu + N(0,s^2) with mu > 7s: c = 7 s."""
    n, b = 2_000_000, 1.0
    v = _rng(33).laplace(0, b, n)
    s = O.dcrp_group(v, O.Params(tau=0.3))
    assert s["clip"] == s["c_tau"]
    assert abs(float(s["clip"]) / (7 * 0.3 * math.sqrt(2) * b) - 1) < 5e-3
    v = _rng(34).normal(10.0, 0.5, 500_000)
    s = O.dcrp_group(v, P0)
    assert s["clip"] == s["c_tau"]
    assert abs(float(s["clip"]) / 3.5 - 1) < 5e-3


# ------------------------------------------------------------ the quantizer
def test_single_group_no_dcrp_is_per_tensor_absmax():
    """One token set and DCRP off is the textbook per-tensor abs-max int4
    quantizer: c = max|X|, one step c/7 for the whole image."""
    rng = _rng(40)
    X = rng.laplace(0, 1, (2, 50, 24)).astype(np.float32)
    p = O.Params(n_groups=1, flags=0)
    gid, clip, scale, _ = O.calibrate_groups(X, p)
    assert not gid.any()
    for b in range(2):
        c = np.abs(X[b]).max()
        assert clip[b, 0] == c and scale[b, 0] == np.float32(c / np.float32(7))
        ref = np.clip(np.rint(X[b] / scale[b, 0]), -8, 7).astype(np.int8)
        q = O.quantize_act(X[b:b + 1], gid[b:b + 1], clip[b:b + 1], scale[b:b + 1], p)
        assert np.array_equal(q[0], ref)
    # with DCRP on there is still exactly one projected scale per image
    gid, clip, scale, st = O.calibrate_groups(X, O.Params(n_groups=1))
    for b in range(2):
        one = O.dcrp_group(X[b], O.Params(n_groups=1))
        assert clip[b, 0] == one["clip"] and scale[b, 0] == one["scale"]


def test_quantizer_idempotent_on_own_grid():
    rng = _rng(41)
    X = (rng.laplace(0, 1, (3, 64, 40)) * rng.choice([0.01, 1, 30], (3, 64, 1))
         ).astype(np.float32)
    p = O.Params(n_groups=6)
    gid, clip, scale, _ = O.calibrate_groups(X, p)
    q = O.quantize_act(X, gid, clip, scale, p)
    xhat = O.dequantize(q, scale[np.arange(3)[:, None], gid][..., None])
    q2 = O.quantize_act(xhat, gid, clip, scale, p)
    assert np.array_equal(q, q2)


def test_rounding_is_ties_to_even_and_codes_in_range():
    c, d = np.float32(1.75), np.float32(0.25)
    x = np.array([0.125, 0.375, 0.625, 0.875, -0.125, -0.375, -0.625, 9.0, -9.0],
                 dtype=np.float32)
    assert O.quantize_codes(x, c, d).tolist() == [0, 2, 2, 4, 0, -2, -2, 7, -7]


def test_prop1_rounding_error_bound_and_zero_code():
    """Proposition 1: |x_hat - x_tilde| <= Delta/2 elementwise, l2 norm
    <= sqrt(n) Delta/2 <= sqrt(n) tau sigma/2.  And code 0 <=> |x| <= Delta/2
    (away from the boundary); activation codes stay in [-7, 7]."""
    for v in _groups(50, 30):
        s = O.dcrp_group(v, P0)
        if s["clip"] <= np.float32(1e-8):
            continue
        c, d = s["clip"], s["scale"]
        q = O.quantize_codes(v, c, d)
        assert q.min() >= -7 and q.max() <= 7
        xt = np.clip(v.astype(np.float64), -float(c), float(c))
        err = q.astype(np.float64) * float(d) - xt
        assert np.abs(err).max() <= float(d) / 2 * (1 + 1e-6)
        n = v.size
        assert np.linalg.norm(err) <= math.sqrt(n) * float(d) / 2 * (1 + 1e-6)
        assert math.sqrt(n) * float(d) / 2 <= math.sqrt(n) * 1.0 * float(s["sigma"]) / 2 * (1 + 1e-6)
        mag = np.abs(v.astype(np.float64))
        away = np.abs(mag - float(d) / 2) > 1e-5 * float(d)
        assert np.array_equal((q == 0)[away], (mag <= float(d) / 2)[away])
        rho_codes = np.count_nonzero(q == 0) / n
        assert abs(rho_codes - float(s["rho0"])) <= np.count_nonzero(~away) / n + 1e-7


# --------------------------------------------------------------- symmetries
def test_power_of_two_equivariance():
    rng = _rng(60)
    X = (rng.laplace(0, 1, (2, 96, 32)) * rng.choice([0.05, 1, 20], (2, 96, 1))
         ).astype(np.float32)
    p = O.Params(n_groups=8)
    g0, c0, s0, st = O.calibrate_groups(X, p)
    q0 = O.quantize_act(X, g0, c0, s0, p)
    used = np.array([[s["n"] > 0 for s in row] for row in st])   # empty sets sit on the eps floor
    for e in (-7, 5):
        f = np.float32(2.0 ** e)
        g1, c1, s1, _ = O.calibrate_groups(X * f, p)
        q1 = O.quantize_act(X * f, g1, c1, s1, p)
        assert np.array_equal(g0, g1) and np.array_equal(q0, q1)
        assert np.array_equal((c0 * f)[used], c1[used])
        assert np.array_equal((s0 * f)[used], s1[used])


def test_token_and_channel_permutation():
    rng = _rng(61)
    X = (rng.laplace(0, 1, (1, 120, 48)) * rng.choice([0.05, 1, 20], (1, 120, 1))
         ).astype(np.float32)
    p = O.Params(n_groups=8)
    g0, c0, s0, st0 = O.calibrate_groups(X, p)
    q0 = O.quantize_act(X, g0, c0, s0, p)
    pt, pc = rng.permutation(120), rng.permutation(48)
    Xp = X[:, pt][:, :, pc]
    g1, c1, s1, st1 = O.calibrate_groups(Xp, p)
    q1 = O.quantize_act(Xp, g1, c1, s1, p)
    assert np.array_equal(g0[:, pt], g1)
    for j in range(8):
        for key in ("n", "thr", "c_base", "c_zr"):
            assert st0[0][j][key] == st1[0][j][key]
        assert abs(float(st0[0][j]["sigma"]) - float(st1[0][j]["sigma"])) <= \
            2e-7 * float(st0[0][j]["sigma"])
    same = np.isclose(s0, s1, rtol=0, atol=0)
    if same.all():
        assert np.array_equal(q0[:, pt][:, :, pc], q1)


def test_assignment_properties():
    rng = _rng(62)
    r = np.abs(rng.laplace(0, 1, 500)).astype(np.float32) * \
        rng.choice([0.01, 1, 100], 500).astype(np.float32)
    for G in (1, 2, 8, 16, 32):
        gid = O.assign_groups(r, G)
        assert gid.min() >= 0 and gid.max() <= G - 1
        assert gid[np.argmax(r)] == (G - 1 if G > 1 else 0)
        assert gid[np.argmin(r)] == 0
        order = np.argsort(r, kind="stable")      # monotone in the range
        assert (np.diff(gid[order]) >= 0).all()


# ----------------------------------------------------- paper-literal setting
def test_paper_literal_blocks():
    """Algorithm 1 on (token, 32-channel block) groups, checked against a
    direct transcription with library reductions: amax, std, sort."""
    rng = _rng(70)
    X = rng.laplace(0, 1, (7, 80)).astype(np.float32)       # 80 -> pad to 96
    xhat, codes, clip, scale = O.dstg_dcrp_blocks(X, 32, P0)
    assert xhat.shape == X.shape and clip.shape == (7, 3)
    Xp = np.zeros((7, 96)); Xp[:, :80] = X
    blk = Xp.reshape(7, 3, 32)
    base = np.abs(blk).max(-1)
    sig = blk.std(-1) + 1e-12
    thr = np.sort(np.abs(blk), -1)[..., 7 - 1]              # ceil(0.2*32) = 7
    c = np.maximum(np.minimum(np.minimum(base, 7 * sig), 14 * thr), 1e-8)
    assert np.allclose(clip, c, rtol=3e-7, atol=0)
    assert np.allclose(scale, np.maximum(c / 7, 1e-8), rtol=4e-7, atol=0)
    # zero padding is counted: last block has 16 zeros of 32, rank 7 -> thr = 0
    assert (thr[:, 2] == 0).all() and (clip[:, 2] == np.float32(1e-8)).all()
    # max-abs only (no DCRP): every block's radius is its own max
    _, _, clip0, _ = O.dstg_dcrp_blocks(X, 32, O.Params(flags=0))
    assert np.array_equal(clip0, base.astype(np.float32))


def test_blocks_linear_against_scalar_loops_and_float_linear():
    """Paper-literal linear: the vectorised binary64 form against (i) scalar triple loops
    over the integer block sums, y = s_n sum_k Delta_mk sum_{i in k} q_x q_w, and (ii)
    a plain float linear on the dequantized tensors that dstg_dcrp_blocks returns."""
    rng = _rng(71)
    X = rng.laplace(0, 1, (5, 80)).astype(np.float32)
    W = rng.normal(0, 0.02, (6, 80)).astype(np.float32)
    bias = rng.normal(0, 0.1, 6).astype(np.float32)
    xhat, codes, clip, scale = O.dstg_dcrp_blocks(X, 32, P0)
    qw, sw = O.quantize_weight(W)
    Y = O.blocks_linear(codes, scale, 32, qw, sw, bias)
    ref = np.zeros((5, 6))
    for m in range(5):
        for n in range(6):
            tot = 0.0
            for k in range(3):
                acc = 0
                for i in range(32 * k, min(32 * k + 32, 80)):
                    acc += int(codes[m, i]) * int(qw[n, i])
                tot += float(scale[m, k]) * acc
            ref[m, n] = float(sw[n]) * tot + float(bias[n])
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-15)
    what = sw[:, None].astype(np.float64) * qw
    mag = np.abs(xhat).astype(np.float64) @ np.abs(what).T + np.abs(bias)   # x_hat is rounded to binary32
    assert (np.abs(Y - (xhat.astype(np.float64) @ what.T + bias)) <= 2e-7 * mag).all()
    # one block per row and a whole-row step: the hot-path form of the same linear
    X1 = rng.laplace(0, 1, (4, 32)).astype(np.float32)
    _, c1, _, s1 = O.dstg_dcrp_blocks(X1, 32, P0)
    q1, w1 = O.quantize_weight(rng.normal(0, 0.02, (3, 32)).astype(np.float32))
    _, Yhot = O.w4a4_linear(c1, s1[:, 0], q1, w1)
    Yb = O.blocks_linear(c1, s1, 32, q1, w1)
    assert (np.abs(Yb - Yhot) <= 2e-7 * np.abs(Yb) + 1e-30).all()


def test_degenerate_groups():
    z = O.dcrp_group(np.zeros(16, np.float32), P0)
    assert z["clip"] == np.float32(1e-8) and z["scale"] == np.float32(1e-8)
    assert not O.quantize_codes(np.zeros(16, np.float32), z["clip"], z["scale"]).any()
    k = O.dcrp_group(np.full(16, 2.5, np.float32), P0)      # sigma = 1e-12
    assert k["clip"] == np.float32(1e-8)
    assert (O.quantize_codes(np.full(16, 2.5, np.float32), k["clip"], k["scale"]) == 1).all()
    e = O.dcrp_group(np.zeros(0, np.float32), P0)
    assert e["n"] == 0 and e["clip"] == np.float32(1e-8)


# -------------------------------------------------------- weights and linear
def test_weight_quant_roundtrip():
    """Eq. (weight_quant): W_hat = s * Q with per-output-channel s; the abs-max
    entry of each row maps to +-7 and the error is at most s/2."""
    rng = _rng(80)
    W = rng.normal(0, 0.02, (24, 50)).astype(np.float32)
    q, s = O.quantize_weight(W)
    assert q.min() >= -7 and q.max() <= 7
    assert (np.abs(q).max(axis=1) == 7).all()
    err = np.abs(q.astype(np.float64) * s[:, None] - W)
    assert (err <= s[:, None] / 2 * (1 + 1e-6)).all()


def test_pack_unpack_nibbles():
    rng = _rng(81)
    for C in (1, 2, 7, 64, 65):
        q = rng.integers(-8, 8, (5, C), dtype=np.int8)
        pk = O.pack_nibbles(q)
        assert pk.shape == (5, (C + 1) // 2) and pk.dtype == np.uint8
        assert np.array_equal(O.unpack_nibbles(pk, C), q)
    assert O.pack_nibbles(np.array([[-8, 7, 1]], np.int8)).tolist() == [[0x78, 0x01]]


def test_int_accumulate_brute_force():
    rng = _rng(82)
    qx = rng.integers(-8, 8, (9, 37), dtype=np.int8)
    qw = rng.integers(-8, 8, (6, 37), dtype=np.int8)
    acc = O.int_accumulate(qx, qw)
    for m in range(9):
        for n in range(6):
            t = 0
            for i in range(37):
                t += int(qx[m, i]) * int(qw[n, i])
            assert acc[m, n] == t
    assert np.abs(acc).max() <= 64 * 37


def test_linear_equals_float_linear_on_dequantized_operands():
    """Algorithm 1 step 10: y = Linear(x_hat, W_hat).  The integer form with the
    scale epilogue equals it (evaluated in binary64) to 1e-5 relative."""
    rng = _rng(83)
    X = (rng.laplace(0, 1, (2, 60, 48)) * rng.choice([0.05, 1, 20], (2, 60, 1))
         ).astype(np.float32)
    W = rng.normal(0, 0.02, (20, 48)).astype(np.float32)
    bias = rng.normal(0, 0.02, 20).astype(np.float32)
    p = O.Params(n_groups=4)
    out = O.tdq_linear_forward(X, W, p, bias)
    rs = O.row_scales(out["gid"], out["scale"]).astype(np.float64)
    xhat = out["qx"].reshape(120, 48).astype(np.float64) * rs[:, None]
    what = out["qw"].astype(np.float64) * out["w_scale"].astype(np.float64)[:, None]
    ref = xhat @ what.T + bias.astype(np.float64)
    noise = np.abs(xhat) @ np.abs(what).T + np.abs(bias)
    assert (np.abs(out["Y"] - ref) <= 1e-5 * noise + 1e-30).all()
    # and x_hat is the paper's quantize-dequantize of X with those radii (Eqs. clipx,
    # dequant), token by token with the radius and step of the token's own set, looked up
    # here by explicit indexing (not through `row_scales`)
    for b in range(2):
        for t in range(60):
            j = int(out["gid"][b, t])
            c, d = np.float32(out["clip"][b, j]), np.float32(out["scale"][b, j])
            xt = np.clip(X[b, t], -c, c)
            q = np.clip(np.rint((xt / d).astype(np.float32)), -8, 7)
            assert np.array_equal(q, out["qx"][b, t].astype(np.float32)), (b, t)
            assert np.array_equal((q * d).astype(np.float64), xhat[b * 60 + t].astype(np.float32)), (b, t)
            assert (np.abs(xhat[b * 60 + t] - xt) <= d / 2 * (1 + 1e-6)).all()      # Proposition 1
    assert np.abs(out["acc"]).max() <= 56 * 48


def test_row_scales_hand_values():
    """The step of a row is the step of ITS image's token set: two images whose tokens sit
    in different sets, values written out by hand.  A transposed or image-blind lookup
    gives another list."""
    gid = np.array([[0, 2, 1], [1, 1, 0]], dtype=np.int32)
    scale = np.array([[1.0, 2.0, 3.0], [10.0, 20.0, 30.0]], dtype=np.float32)
    assert O.row_scales(gid, scale).tolist() == [1.0, 3.0, 2.0, 20.0, 20.0, 10.0]
    assert O.row_scales(gid, scale).dtype == np.float32
    # one set per image: every row of an image takes that image's single step
    assert O.row_scales(np.zeros((2, 2), np.int32), np.array([[5.0], [7.0]], np.float32)).tolist() \
        == [5.0, 5.0, 7.0, 7.0]


def test_zero_bin_mass_and_sqnr_hand_values():
    """Eq. (rho0_def): the share of elements with |x| <= Delta / 2, boundary included;
    it is the share of zero codes under round-to-nearest (Sec. 3.1), and the value
    `dcrp_group` reports.  SQNR = 10 log10(sum x^2 / sum (x - x_hat)^2) on a 3-4-5 case."""
    x = np.array([0.0, 0.25, -0.5, 0.625, 2.0, -0.375], dtype=np.float32)
    assert O.zero_bin_mass(x, 1.0) == 4 / 6            # 0, 0.25, -0.5 (on the boundary), -0.375
    assert O.zero_bin_mass(x, 0.5) == 2 / 6
    codes = O.quantize_codes(x, 7.0, 1.0)
    assert codes.tolist() == [0, 0, 0, 1, 2, 0] and (codes == 0).mean() == O.zero_bin_mass(x, 1.0)
    rng = _rng(85)
    v = rng.laplace(0, 1, 500).astype(np.float32)
    s = O.dcrp_group(v, O.Params())
    assert s["rho0"] == np.float32(O.zero_bin_mass(v, s["scale"]))
    assert abs(O.sqnr_db(np.array([3.0, 4.0]), np.array([3.0, 3.0])) - 10 * np.log10(25.0)) < 1e-12
    assert abs(O.sqnr_db(np.array([1.0, -1.0]), np.array([0.9, -1.1])) - 20.0) < 1e-9


def test_tokenize_chw_by_explicit_index_loops():
    """X[b, c, h, w] lands at X'[b, h*W + w, c] (the 4-D branch of the supplementary
    implementation details), checked element by element, and the per-block radii of the
    tokenized map are those of each pixel's channel vector."""
    rng = np.random.Generator(np.random.PCG64(71))
    B, C, H, W = 2, 40, 3, 5
    X = rng.standard_normal((B, C, H, W)).astype(np.float32)
    Xt = O.tokenize_chw(X)
    assert Xt.shape == (B, H * W, C)
    for b in range(B):
        for c in range(C):
            for h in range(H):
                for w in range(W):
                    assert Xt[b, h * W + w, c] == X[b, c, h, w]
    _, _, clip, _ = O.dstg_dcrp_blocks(Xt, 32, O.Params(flags=0))
    assert clip[1, 7, 0] == np.abs(X[1, :32, 1, 2]).max()
    assert clip[1, 7, 1] == np.abs(X[1, 32:, 1, 2]).max()


def test_range_disparity_hand_cases_and_invariances():
    """Eq. (range_disparity) on cases worked by hand, scale invariance, and the lower
    median against sorting."""
    # two tokens of three channels: medians 2 and 20 -> lower median of {2, 20} is 2
    X = np.array([[[1.0, -2.0, 3.0], [10.0, 20.0, -400.0]]], dtype=np.float32)
    D, tok, mx = O.range_disparity(X)
    assert tok.tolist() == [[2.0, 20.0]] and mx.tolist() == [400.0] and D.tolist() == [200.0]
    # even counts take the lower middle value
    X = np.array([[[4.0, 1.0, 3.0, 2.0]]], dtype=np.float32)
    assert O.range_disparity(X)[1].tolist() == [[2.0]]
    # a constant tensor has D = 1, an all-zero one D = inf
    assert O.range_disparity(np.full((1, 5, 7), -3.0, np.float32))[0].tolist() == [1.0]
    assert np.isinf(O.range_disparity(np.zeros((1, 4, 4), np.float32))[0][0])
    rng = np.random.Generator(np.random.PCG64(81))
    X = rng.standard_normal((3, 9, 14)).astype(np.float32)
    D, tok, mx = O.range_disparity(X)
    for b in range(3):
        med = [np.sort(np.abs(X[b, t]))[(14 + 1) // 2 - 1] for t in range(9)]
        assert tok[b].tolist() == med
        assert D[b] == np.float32(np.abs(X[b]).max() / np.sort(med)[(9 + 1) // 2 - 1])
    # power-of-two rescaling leaves D unchanged bit for bit; one spike raises it in proportion
    assert np.array_equal(O.range_disparity(X * np.float32(8))[0], D)
    Y = X.copy()
    Y[0, 0, 0] = 1024.0
    den0 = np.sort(O.range_disparity(Y)[1][0])[(9 + 1) // 2 - 1]
    assert O.range_disparity(Y)[0][0] == np.float32(np.float32(1024.0) / den0)
