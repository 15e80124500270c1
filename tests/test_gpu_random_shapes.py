"""GPU parity on seeded random VALID shapes and parameters: the token-set path end to end
(calibrate, quantize, contraction) against the oracle, with the path's own bars -- set ids,
ranks, thresholds, base radii, codes given equal scales and int32 accumulators bit for bit,
sigma / clip / step within 1e-6, outputs bit-identical given the device's codes and steps.
The draws cover what the hand-picked cases do not combine: tiny and ragged shapes with many
sets, both input types, every flag combination, the percentile base radius, padded rows,
offset data, constant tokens and all-zero tokens (sets of identical values)."""
import numpy as np
import pytest
import torch

from oracle import tdq_oracle as O
from paper_2604_16855_amd import inputs as I
from paper_2604_16855_amd import tdq

import parity_util as U

pytestmark = pytest.mark.gpu


def _draw(rng, case):
    B = int(rng.integers(1, 5))
    T = int(rng.choice([1, 2, 7, 63, 64, 65, 121, 300, 484, 1000, 2049]))
    C = int(rng.choice([1, 3, 8, 31, 32, 33, 64, 70, 128, 200, 320, 512, 1000, 1024, 2048, 2056, 4096]))
    if B * T * C > 2_000_000:
        T = max(1, 2_000_000 // (B * C))
    G = int(rng.choice([1, 2, 3, 8, 16, 32, 64, 65, 128, 129, 256]))
    dtype = str(rng.choice(["f16", "f32"]))
    flags = int(rng.choice([0, 1, 2, 3, 3, 3])) | int(rng.choice([0, 0, 0, tdq.FLAG_EXACT_SELECT]))
    kind = str(rng.choice(["mix", "offset", "const", "zeros_some"]))
    if kind == "offset":
        X = I.offset_activations(B, T, C, dtype, float(rng.choice([10, 100, 1000])), seed=case,
                                 token_jitter=0.05, outlier_head=bool(rng.integers(0, 2)))
    else:
        X = rng.laplace(0, 1, (B, T, C)) * rng.lognormal(0, 1.5, (B, T, 1))
        if kind == "const":
            X[:, ::3, :] = 0.75
        if kind == "zeros_some":
            X[:, 1::2, :] = 0.0
        X = np.clip(X, -60000.0, 60000.0).astype(np.float16 if dtype == "f16" else np.float32)
    p = tdq.default_params(G, flags=flags)
    p.tau = float(rng.choice([0.3, 1.0, 2.0]))
    p.zr = float(rng.choice([0.01, 0.2, 0.5, 0.9]))
    p.base_pct = float(rng.choice([0.0, 0.0, 0.0, 0.99, 0.5]))
    return X, p, kind, int(rng.choice([0, 0, 3, 8])), int(rng.choice([1, 8, 64, 130, 256, 512]))


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_valid_shapes_end_to_end(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    for case in range(25):
        X, p, kind, ld_pad, N = _draw(rng, 100 * seed + case)
        B, T, C = X.shape
        print(f"[random {seed}.{case}] B={B} T={T} C={C} G={p.n_groups} {X.dtype} flags={p.flags} tau={p.tau} "
              f"zr={p.zr} pct={p.base_pct} {kind} ld_pad={ld_pad} N={N}", flush=True)
        g = U.gpu_calibrate(X, p, ld_pad=ld_pad)
        assert g["status"] == 0
        gid, clip, scale, _ = U.assert_calibration_matches(g, X, p)
        Q = tdq.tdq_quantize_act(g["Xd"], p, g["gid_d"], g["clip_d"], g["scale_d"])
        torch.cuda.synchronize()
        rows = np.arange(B)[:, None]
        q_ref = O.quantize_act(X, gid, clip, scale, U.oracle_params(p)).reshape(B * T, C)
        exact = np.array_equal(g["scale"], scale) and np.array_equal(g["clip"], clip)
        q_gpu = U.unpack_device_codes(Q, C)
        U.assert_codes_match(q_gpu, q_ref, X.reshape(B * T, C).astype(np.float32),
                             clip[rows, gid].reshape(-1), scale[rows, gid].reshape(-1), exact)
        W = rng.normal(0, 0.02, (N, C)).astype(np.float32)
        Qw, ws = tdq.tdq_quantize_weight(torch.from_numpy(W).to(U.dev()))
        qw_ref, sw_ref = O.quantize_weight(W)
        assert np.array_equal(O.unpack_nibbles(Qw.cpu().numpy()[:, :(C + 1) // 2], C), qw_ref)
        assert np.array_equal(ws.cpu().numpy(), sw_ref)
        acc, Y = U.gpu_linear(Q, g["gid_d"], g["scale_d"], B, T, C, Qw, ws)
        acc_ref, Y_ref = O.w4a4_linear(q_gpu, g["scale"][rows, g["gid"]].reshape(-1), qw_ref, sw_ref)
        assert np.array_equal(acc, acc_ref), "accumulators differ"
        assert np.array_equal(Y, Y_ref), "outputs differ"
