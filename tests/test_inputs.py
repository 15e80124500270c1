"""The seeded synthetic generators: shapes, class mix, determinism, finiteness."""
import numpy as np

from paper_2604_16855_amd import inputs as I


def test_cases_cover_baseline_configs():
    assert I.CASES["cfg0"].M == 196 and I.CASES["cfg0"].dtype == "f32"
    assert I.CASES["cfg1"].T == 7744 and I.CASES["cfg1"].N == 512
    assert I.CASES["cfg2_fc2"].C == 1280 and I.CASES["cfg2_qkv"].N == 960
    assert I.CASES["cfg4_fc1_h10"].M == 131072 and I.CASES["cfg4_fc2_h10"].C == 4096
    n3 = sum(I.CFG3_DEPTH[int(k[6])] for k in I.CASES if k.startswith("cfg3_"))
    assert n3 == 80          # 5 linears x (3+4+6+3) blocks


def test_cfg0_mixture_and_determinism():
    lc = I.case("cfg0")
    X, cls = I.make_activations(lc)
    X2, cls2 = I.make_activations(lc)
    assert X.dtype == np.float32 and X.shape == (1, 196, 64)
    assert np.array_equal(X, X2) and np.array_equal(cls, cls2)
    assert (cls == I.HEAVY).sum() == 10 and (cls == I.WEAK).sum() == 10
    r = np.abs(X[0]).max(axis=1)
    assert np.median(r[cls[0] == I.HEAVY]) > 10 * np.median(r[cls[0] == I.BULK])
    assert r[cls[0] == I.WEAK].max() < 0.2
    assert np.isfinite(X).all()


def test_cfg1_clustered_fp16():
    lc = I.case("cfg1")
    X, cls = I.make_activations(lc)
    assert X.dtype == np.float16 and X.shape == (1, 7744, 64)
    assert abs((cls == I.HEAVY).mean() - 0.15) < 1e-3
    assert abs((cls == I.WEAK).mean() - 0.05) < 1e-3
    assert np.isfinite(X.astype(np.float32)).all()
    # clustered: a heavy token's 4-neighbourhood is mostly heavy
    hm = (cls[0] == I.HEAVY).reshape(88, 88)
    nb = hm[1:-1, 1:-1] & hm[:-2, 1:-1] & hm[2:, 1:-1]
    assert nb.sum() > 0.7 * hm.sum()


def test_batched_case_images_differ():
    lc = I.case("cfg2_proj", B=3)
    X, _ = I.make_activations(lc, workers=2)
    assert X.shape == (3, 484, 320)
    assert not np.array_equal(X[0], X[1])
    Xs, _ = I.make_activations(lc, workers=1)
    assert np.array_equal(X, Xs)
    W = I.make_weight(lc)
    assert W.shape == (320, 320) and abs(W.std() - 0.02) < 1e-3
