"""Seeded synthetic inputs for the DSTG+DCRP W4A4 linear path.

This module only draws random numbers and lays them out; it contains none of
the quantization method's arithmetic, so both the CPU oracle's tests and the
HIP path's tests/bench can take their inputs from it without sharing any of
the method itself.

The tensors stand in for the pre-linear activations of hierarchical COD
encoders, which the paper describes qualitatively as a token population
dominated by heavy-tailed background tokens plus a small set of tokens that
carry small-amplitude, spatially structured boundary responses (Sec. 3.2
"Range Domination", Sec. 3.3 "Zero-bin Mass Collapse").  Three token classes:

  bulk   every channel ~ Laplace(0, 1)
  heavy  every channel ~ 20 * Student-t(nu=2)          (background spikes)
  weak   0.05*sin(2*pi*k_t*c/64) + N(0, 0.01^2), k_t = 1 + (t mod 8)
                                                      (weak boundary cues)

Everything is generated on the host with numpy's PCG64 from fixed seeds (one
independent stream per image), so any two callers see the same bits.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np

BULK, HEAVY, WEAK = 0, 1, 2
FP16_MAX = 65504.0


@dataclass(frozen=True)
class LinearCase:
    """One quantized linear: activations X[B, T, C] against W[N, C]."""

    name: str
    B: int            # images
    T: int            # tokens per image
    C: int            # input channels (K of the contraction)
    N: int            # output channels
    G: int            # token groups per image
    dtype: str        # "f16" or "f32"
    heavy: float      # fraction of heavy-tailed tokens
    weak: float       # fraction of weak-cue tokens
    clustered: bool   # heavy tokens in 2-D blobs, weak tokens ringing them
    grid: Tuple[int, int]
    seed: int

    @property
    def M(self) -> int:
        return self.B * self.T


def _case(name, B, grid, C, N, G, dtype, heavy, weak, clustered, seed):
    return LinearCase(name, B, grid[0] * grid[1], C, N, G, dtype, heavy, weak,
                      clustered, grid, seed)


def _build_cases() -> Dict[str, LinearCase]:
    c: Dict[str, LinearCase] = {}
    # config 0: single small linear, fp32 activations, 90/5/5 mixture.
    c["cfg0"] = _case("cfg0", 1, (14, 14), 64, 64, 8, "f32", 0.05, 0.05, False, 0)
    # config 1: stage-1 MLP fc1, 88x88 tokens, 15 % heavy tokens in blobs.
    c["cfg1"] = _case("cfg1", 1, (88, 88), 64, 512, 16, "f16", 0.15, 0.05, True, 1)
    # config 2: stage-3 linears, batch 16, 22x22 tokens, config-0 mixture.
    for nm, C, N in (("qkv", 320, 960), ("proj", 320, 320),
                     ("fc1", 320, 1280), ("fc2", 1280, 320)):
        c["cfg2_" + nm] = _case("cfg2_" + nm, 16, (22, 22), C, N, 16, "f16",
                                0.05, 0.05, False, 1000 + (C == 1280))
    # config 3: 4-stage encoder linear set at 352x352, batch 8 (one entry per
    # distinct shape; depth repeats of a shape differ only in seed).
    stages = ((88, 64, 8, 3), (44, 128, 8, 4), (22, 320, 4, 6), (11, 512, 4, 3))
    for si, (side, C, r, depth) in enumerate(stages, start=1):
        shapes = (("q", side, C, C), ("kv", 11, C, 2 * C), ("proj", side, C, C),
                  ("fc1", side, C, r * C), ("fc2", side, r * C, C))
        for li, (nm, s, cin, cout) in enumerate(shapes):
            key = f"cfg3_s{si}_{nm}"
            c[key] = _case(key, 8, (s, s), cin, cout, 16, "f16", 0.15, 0.05,
                           True, 3000 + 100 * si + li)
    # config 4: ViT-L-shaped stress, batch 32, 64x64 tokens, heavy swept.
    for h in (2, 10, 25):
        c[f"cfg4_fc1_h{h}"] = _case(f"cfg4_fc1_h{h}", 32, (64, 64), 1024, 4096,
                                    32, "f16", h / 100.0, 0.05, False, 4000 + h)
        c[f"cfg4_fc2_h{h}"] = _case(f"cfg4_fc2_h{h}", 32, (64, 64), 4096, 1024,
                                    32, "f16", h / 100.0, 0.05, False, 4100 + h)
    return c


CASES: Dict[str, LinearCase] = _build_cases()

# depth of each config-3 stage (how many times its five linears repeat)
CFG3_DEPTH = {1: 3, 2: 4, 3: 6, 4: 3}


def case(name: str, **overrides) -> LinearCase:
    """Look up a named case, optionally with fields replaced (e.g. B=2)."""
    base = CASES[name]
    if "grid" in overrides:
        g = overrides["grid"]
        overrides["T"] = g[0] * g[1]
    return replace(base, **overrides) if overrides else base


# --------------------------------------------------------------------------
# token classes
# --------------------------------------------------------------------------
def _classes_random(T: int, heavy: float, weak: float,
                    rng: np.random.Generator) -> np.ndarray:
    n_h = int(round(heavy * T))
    n_w = int(round(weak * T))
    cls = np.full(T, BULK, dtype=np.int8)
    perm = rng.permutation(T)
    cls[perm[:n_h]] = HEAVY
    cls[perm[n_h:n_h + n_w]] = WEAK
    return cls


def _classes_clustered(grid: Tuple[int, int], heavy: float, weak: float,
                       rng: np.random.Generator) -> np.ndarray:
    """Heavy tokens = union of Gaussian blobs thresholded to the wanted area;
    weak tokens = a seeded sample of the one-token ring around the blobs."""
    H, W = grid
    T = H * W
    n_h = int(round(heavy * T))
    n_w = int(round(weak * T))
    yy, xx = np.mgrid[0:H, 0:W].astype(np.float64)
    n_blobs = int(rng.integers(3, 7))
    field = np.zeros((H, W))
    for _ in range(n_blobs):
        cy, cx = rng.uniform(0, H), rng.uniform(0, W)
        s = rng.uniform(0.06, 0.18) * max(H, W) + 0.5
        field += np.exp(-((yy - cy) ** 2 + (xx - cx) ** 2) / (2 * s * s))
    field += 1e-9 * rng.random((H, W))           # break ties reproducibly
    cls = np.full(T, BULK, dtype=np.int8)
    order = np.argsort(-field.ravel(), kind="stable")
    heavy_idx = order[:n_h]
    cls[heavy_idx] = HEAVY
    hm = (cls == HEAVY).reshape(H, W)
    ring = np.zeros_like(hm)
    ring[1:, :] |= hm[:-1, :]
    ring[:-1, :] |= hm[1:, :]
    ring[:, 1:] |= hm[:, :-1]
    ring[:, :-1] |= hm[:, 1:]
    ring &= ~hm
    ring_idx = np.flatnonzero(ring.ravel())
    ring_idx = rng.permutation(ring_idx)
    chosen = ring_idx[:n_w]
    if chosen.size < n_w:                        # small grids: top up anywhere
        rest = np.flatnonzero((cls == BULK) & ~ring.ravel())
        rest = rng.permutation(rest)
        chosen = np.concatenate([chosen, rest[:n_w - chosen.size]])
    cls[chosen] = WEAK
    return cls


def _image(lc: LinearCase, b: int) -> Tuple[np.ndarray, np.ndarray]:
    rng = np.random.Generator(np.random.PCG64([lc.seed, b]))
    if lc.clustered:
        cls = _classes_clustered(lc.grid, lc.heavy, lc.weak, rng)
    else:
        cls = _classes_random(lc.T, lc.heavy, lc.weak, rng)
    X = np.empty((lc.T, lc.C), dtype=np.float32)
    idx = np.flatnonzero(cls == BULK)
    X[idx] = rng.laplace(0.0, 1.0, size=(idx.size, lc.C))
    idx = np.flatnonzero(cls == HEAVY)
    X[idx] = 20.0 * rng.standard_t(2.0, size=(idx.size, lc.C))
    idx = np.flatnonzero(cls == WEAK)
    k_t = 1.0 + (idx % 8).astype(np.float64)
    ch = np.arange(lc.C, dtype=np.float64)
    cue = 0.05 * np.sin(2.0 * np.pi * k_t[:, None] * ch[None, :] / 64.0)
    X[idx] = cue + rng.normal(0.0, 0.01, size=(idx.size, lc.C))
    if lc.dtype == "f16":
        np.clip(X, -FP16_MAX, FP16_MAX, out=X)   # saturate, keep finite
        return X.astype(np.float16), cls
    return X, cls


def make_activations(lc: LinearCase, workers: int = 8
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (X[B, T, C] in lc.dtype, token class[B, T] int8)."""
    dt = np.float16 if lc.dtype == "f16" else np.float32
    X = np.empty((lc.B, lc.T, lc.C), dtype=dt)
    cls = np.empty((lc.B, lc.T), dtype=np.int8)

    def job(b):
        X[b], cls[b] = _image(lc, b)

    if lc.B == 1 or workers <= 1:
        for b in range(lc.B):
            job(b)
    else:
        with ThreadPoolExecutor(max_workers=min(workers, lc.B)) as ex:
            list(ex.map(job, range(lc.B)))
    return X, cls


def make_weight(lc: LinearCase) -> np.ndarray:
    """W[N, C] ~ N(0, 0.02^2), fp32."""
    rng = np.random.Generator(np.random.PCG64([lc.seed, 1 << 20]))
    return rng.normal(0.0, 0.02, size=(lc.N, lc.C)).astype(np.float32)


def make_bias(lc: LinearCase) -> np.ndarray:
    """bias[N] ~ N(0, 0.02^2), fp32 (the configs name no bias; used by tests
    of the optional bias term only)."""
    rng = np.random.Generator(np.random.PCG64([lc.seed, (1 << 20) + 1]))
    return rng.normal(0.0, 0.02, size=(lc.N,)).astype(np.float32)


def random_codes(shape, seed: int, lo: int = -8, hi: int = 7) -> np.ndarray:
    """Uniform int8 codes in [lo, hi] — for contraction-only tests."""
    rng = np.random.Generator(np.random.PCG64([seed, 77]))
    return rng.integers(lo, hi + 1, size=shape, dtype=np.int8)


def offset_activations(B: int, T: int, C: int, dtype: str, ratio: float, seed: int,
                       token_jitter: float = 0.0, outlier_head: bool = False) -> np.ndarray:
    """X[B, T, C] whose values sit far from zero: x = mu_t + s_t * N(0, 1) with a per-token
    spread s_t (log-normal around 0.25, so tokens fall into different token sets) and a
    mean mu_t = ratio * 0.25 * (1 + token_jitter * u_t), u_t ~ U(-1, 1).  This is the regime
    where the step-to-dispersion bound of Eq. (tau_constraint) binds and where a variance
    computed from raw sums of squares cancels.  `outlier_head` puts two large values of
    opposite offset at the start of every third token's row."""
    rng = np.random.Generator(np.random.PCG64([seed, 1 << 21]))
    s = 0.25 * rng.lognormal(0.0, 0.5, size=(B, T, 1))
    mu = ratio * 0.25 * (1.0 + token_jitter * rng.uniform(-1.0, 1.0, size=(B, T, 1)))
    X = mu + s * rng.normal(0.0, 1.0, size=(B, T, C))
    if outlier_head and C >= 3:
        X[:, ::3, 0] += 40.0 * s[:, ::3, 0]
        X[:, ::3, 1] += 55.0 * s[:, ::3, 0]
    if dtype == "f16":
        np.clip(X, -FP16_MAX, FP16_MAX, out=X)
        return X.astype(np.float16)
    return X.astype(np.float32)
