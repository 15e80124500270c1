"""GPU parity of the dispersion on data far from zero.  The group dispersion of Sec. 4.2
is a population standard deviation, and where the step-to-dispersion bound binds
(Eq. tau_constraint, Lemma 1) the step IS tau * sigma, so sigma's error goes straight into
the step.  With flags = C1 only every step inherits sigma; the bar is the path's own:
sigma, clip and step within 1e-6 of the oracle's two-pass binary64 value, group ids and
thresholds bit-exact — through all three calibration entry points."""
import numpy as np
import pytest
import torch

from oracle import tdq_oracle as O
from paper_2604_16855_amd import inputs as I
from paper_2604_16855_amd import tdq

import parity_util as U

pytestmark = pytest.mark.gpu

# (B, T, C, G): sets of one token of 64 channels up to whole images; rows that take the
# several-rows-per-wavefront sweep (C = 64, 70), one row per wavefront (1024) and one
# row per workgroup (4096); a ragged C
SHAPES = [(2, 1, 64, 1), (3, 33, 64, 8), (2, 50, 70, 5), (1, 300, 1024, 4), (1, 40, 4096, 1),
          (2, 64, 320, 64)]


def _say(msg):
    print(msg, flush=True)


def _check_binds(g, ratio):
    """The step inherits sigma: C1 binds on every set once the offset dwarfs the spread
    (at mu / sigma = 10 a wide token's 7 sigma can still exceed its range)."""
    binds = g["stats"]["bind"][g["stats"]["n"] > 0]
    assert (binds == 1).any(), "C1 was meant to bind"
    if ratio >= 100.0:
        assert (binds == 1).all()


@pytest.mark.parametrize("B,T,C,G", SHAPES)
@pytest.mark.parametrize("ratio", [10.0, 100.0, 1000.0])
@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_sigma_on_offset_data(dtype, ratio, B, T, C, G):
    X = I.offset_activations(B, T, C, dtype, ratio, seed=int(ratio) + C + T)
    p = tdq.default_params(G, flags=tdq.FLAG_C1)
    _say(f"[offset] {dtype} mu/sigma={ratio} B={B} T={T} C={C} G={G}")
    g = U.gpu_calibrate(X, p)
    assert g["status"] == 0
    U.assert_calibration_matches(g, X, p)
    _check_binds(g, ratio)


@pytest.mark.parametrize("dtype,ratio,jitter,head", [("f16", 100.0, 0.02, False), ("f32", 1000.0, 0.01, False),
                                                     ("f16", 0.0, 0.0, True), ("f16", 300.0, 0.0, True),
                                                     ("f32", 50.0, 0.1, True)])
@pytest.mark.parametrize("B,T,C,G", [(2, 130, 64, 4), (1, 64, 1024, 8), (1, 9, 4096, 2)])
def test_sigma_between_token_offsets_and_bad_pivots(dtype, ratio, jitter, head, B, T, C, G):
    """Token means that differ (the between-token part of a set's variance) and rows whose
    first values are outliers (the row's pivot is then far from its mean and the row is
    summed a second time)."""
    X = I.offset_activations(B, T, C, dtype, ratio, seed=7 + C, token_jitter=jitter,
                             outlier_head=head)
    p = tdq.default_params(G, flags=tdq.FLAG_C1 | tdq.FLAG_C2)
    _say(f"[offset] {dtype} mu/sigma={ratio} jitter={jitter} head={head} B={B} T={T} C={C} G={G}")
    g = U.gpu_calibrate(X, p)
    U.assert_calibration_matches(g, X, p)


@pytest.mark.parametrize("dtype,ratio", [("f16", 10.0), ("f16", 1000.0), ("f32", 100.0), ("f32", 1000.0)])
@pytest.mark.parametrize("B,T,C,G", [(2, 1, 64, 1), (3, 33, 64, 8), (2, 50, 70, 5), (1, 128, 1024, 4)])
def test_sigma_on_offset_data_single_launch(dtype, ratio, B, T, C, G):
    X = I.offset_activations(B, T, C, dtype, ratio, seed=11 + C)
    p = tdq.default_params(G, flags=tdq.FLAG_C1)
    _say(f"[offset-fused] {dtype} mu/sigma={ratio} B={B} T={T} C={C} G={G}")
    gid, clip, scale, stats, flags, Q, ws = tdq.tdq_calibrate_quantize_fused(U.to_device(X), p,
                                                                            want_stats=True)
    torch.cuda.synchronize()
    g = dict(gid=gid.cpu().numpy(), clip=clip.cpu().numpy(), scale=scale.cpu().numpy(),
             stats=tdq.stats_to_numpy(stats))
    assert not flags.cpu().numpy().any()
    U.assert_calibration_matches(g, X, p)
    _check_binds(g, ratio)


@pytest.mark.parametrize("dtype,ratio,head", [("f16", 10.0, False), ("f16", 1000.0, False),
                                              ("f32", 100.0, False), ("f32", 1000.0, True),
                                              ("f16", 100.0, True)])
@pytest.mark.parametrize("B,C,H,W,G", [(2, 64, 1, 1, 1), (2, 64, 6, 7, 8), (1, 70, 10, 5, 5),
                                       (1, 1024, 16, 12, 4)])
def test_sigma_on_offset_feature_maps(dtype, ratio, head, B, C, H, W, G):
    """The same through tdq_calibrate_groups_chw: the map X[B, C, H, W] is the transposed
    token matrix."""
    Xt_ref = I.offset_activations(B, H * W, C, dtype, ratio, seed=13 + C, outlier_head=head)
    X = np.ascontiguousarray(Xt_ref.transpose(0, 2, 1)).reshape(B, C, H, W)
    p = tdq.default_params(G, flags=tdq.FLAG_C1)
    _say(f"[offset-chw] {dtype} mu/sigma={ratio} head={head} B={B} C={C} H={H} W={W} G={G}")
    Xt, gid, clip, scale, stats, ws = tdq.tdq_calibrate_groups_chw(torch.from_numpy(X).to(U.dev()), p,
                                                                  want_stats=True)
    torch.cuda.synchronize()
    assert np.array_equal(Xt.cpu().numpy().view(np.uint8), Xt_ref.view(np.uint8))
    assert tdq.device_status(ws) == 0
    g = dict(gid=gid.cpu().numpy(), clip=clip.cpu().numpy(), scale=scale.cpu().numpy(),
             stats=tdq.stats_to_numpy(stats))
    U.assert_calibration_matches(g, Xt_ref, p)


def _constant_sets_input(B, T, C, dtype):
    """Images whose token sets include sets of IDENTICAL values away from everything else:
    every other token all zero (the padding of a masked image), every fifth token a constant
    row, the rest Laplace rows of growing scale; the first token, whatever pivot a kernel
    might take from it, belongs to none of the constant sets."""
    rng = np.random.Generator(np.random.PCG64(B * 1000 + T + C))
    X = rng.laplace(0, 1, (B, T, C)) * (1.0 + 0.05 * np.arange(T))[None, :, None]
    X[:, 0, :] += 3.0
    X[:, 1::2, :] = 0.0
    X[:, 5::10, :] = 40.0 * float(T)          # larger than anything else: the top set, constant
    np.clip(X, -60000.0, 60000.0, out=X)
    return X.astype(np.float16 if dtype == "f16" else np.float32)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
@pytest.mark.parametrize("B,T,C,G", [(2, 64, 64, 8), (1, 300, 1024, 16), (2, 41, 4096, 4), (1, 2100, 40, 32)])
def test_sets_of_identical_values_have_zero_dispersion(dtype, B, T, C, G):
    """A set whose elements are all equal has a population standard deviation of exactly
    zero (Sec. 4.2), so its sigma is eps_std and the projection ends at the eps floor
    (Eq. dcrp with the supplementary numerical conventions): the merge of the per-token
    moments must not leave a rounding residue there.  Through the multi-kernel path, the
    single launch and the conv-layout sweep."""
    X = _constant_sets_input(B, T, C, dtype)
    p = tdq.default_params(G, flags=tdq.FLAG_C1 | tdq.FLAG_C2)
    _say(f"[constant sets] {dtype} B={B} T={T} C={C} G={G}")
    g = U.gpu_calibrate(X, p)
    gid, clip, scale, st = U.assert_calibration_matches(g, X, p)
    sig = g["stats"]["sigma"].reshape(B, G)
    zero_sets = [(b, j) for b in range(B) for j in range(G) if st[b][j]["n"] and st[b][j]["sigma"] == np.float32(1e-12)]
    assert len(zero_sets) >= B, "the input was meant to hold constant sets"
    for b, j in zero_sets:
        assert sig[b, j] == np.float32(1e-12), (b, j, sig[b, j])
    if G <= 64 and T * C <= 400000:      # the single launch takes at most 64 sets; keep the image small
        gid2, clip2, scale2, stats2, flags2, Q2, ws2 = tdq.tdq_calibrate_quantize_fused(U.to_device(X), p,
                                                                                      want_stats=True)
        torch.cuda.synchronize()
        g2 = dict(gid=gid2.cpu().numpy(), clip=clip2.cpu().numpy(), scale=scale2.cpu().numpy(),
                  stats=tdq.stats_to_numpy(stats2))
        U.assert_calibration_matches(g2, X, p)
    Xc = torch.from_numpy(np.ascontiguousarray(X.transpose(0, 2, 1)).reshape(B, C, T, 1)).to(U.dev())
    Xt, gid3, clip3, scale3, stats3, ws3 = tdq.tdq_calibrate_groups_chw(Xc, p, want_stats=True)
    torch.cuda.synchronize()
    g3 = dict(gid=gid3.cpu().numpy(), clip=clip3.cpu().numpy(), scale=scale3.cpu().numpy(),
              stats=tdq.stats_to_numpy(stats3))
    U.assert_calibration_matches(g3, X, p)
