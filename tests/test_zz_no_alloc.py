"""tdq_calibrate_groups_static (the entry point for callers that cannot allocate: the
calibration scratch is a static device array inside the library) against
tdq_calibrate_groups with a caller-owned workspace: same kernels, so every output must be
the same bits.  Two calls in a row share the static array, the second on a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_16855_amd import inputs as I
from paper_2604_16855_amd import tdq

pytestmark = pytest.mark.gpu


def _both(X, p):
    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X).to(dev)
    B, T, Cc = X.shape
    G = p.n_groups
    gid, clip, scale, stats, ws = tdq.tdq_calibrate_groups(Xd, p, want_stats=True)
    torch.cuda.synchronize()
    ref = (gid.cpu().numpy(), clip.cpu().numpy(), scale.cpu().numpy(), stats.cpu().numpy(),
           ws[:12].view(torch.int32).cpu().numpy())
    out = (torch.full((B, T), -1, dtype=torch.int32, device=dev),
           torch.full((B, G), -1.0, dtype=torch.float32, device=dev),
           torch.full((B, G), -1.0, dtype=torch.float32, device=dev))
    st = torch.zeros((B * G, C.sizeof(tdq.GroupStats)), dtype=torch.uint8, device=dev)
    status = torch.full((4,), -1, dtype=torch.int32, device=dev)
    print(f"[static] B={B} T={T} C={Cc} G={G} {X.dtype}", flush=True)
    tdq.tdq_calibrate_groups_static(Xd, p, out, st, status)
    torch.cuda.synchronize()
    assert np.array_equal(out[0].cpu().numpy(), ref[0])
    assert np.array_equal(out[1].cpu().numpy(), ref[1])
    assert np.array_equal(out[2].cpu().numpy(), ref[2])
    assert np.array_equal(st.cpu().numpy(), ref[3])
    s = status.cpu().numpy()
    assert np.array_equal(s[:3], ref[4]) and s[3] == 0
    return s


def test_static_scratch_matches_workspace_twice_in_a_row():
    # binary16, single-sweep rank select; then a smaller binary16 input with a forced
    # per-set select; then binary32 (radix levels) smaller still
    lc = I.case("cfg2_fc2", B=3)
    X1, _ = I.make_activations(lc)
    s1 = _both(X1, tdq.default_params(lc.G))
    assert s1[0] == 0
    lc2 = I.case("cfg2_qkv", B=2)
    X2, _ = I.make_activations(lc2)
    p2 = tdq.default_params(8)
    p2.flags |= tdq.FLAG_EXACT_SELECT
    s2 = _both(np.ascontiguousarray(X2[:, :100]), p2)
    assert s2[1] > 0
    X3, _ = I.make_activations(I.case("cfg0"))
    _both(X3, tdq.default_params(4))
    # a non-finite input raises the status word through the static path too
    X4 = X3.copy()
    X4[0, 5, 7] = np.inf
    assert _both(X4, tdq.default_params(4))[0] == tdq.DEV_NONFINITE


def test_static_scratch_rejects_what_does_not_fit():
    p = tdq.default_params(32)
    B, T, Cc = 64, 16384, 64                      # 1 Mi tokens: 20 MB of per-token records
    assert tdq.workspace_bytes(B, T, Cc, tdq.TDQ_F16, p) > tdq.STATIC_SCRATCH_BYTES
    fake = 1 << 20
    rc = tdq.lib().tdq_calibrate_groups_static(fake, tdq.TDQ_F16, B, T, Cc, Cc, C.byref(p), fake, fake,
                                               fake, None, None, None)
    assert rc == tdq.ERR_WORKSPACE
    # and the configuration the benchmark times fits
    assert tdq.workspace_bytes(32, 4096, 4096, tdq.TDQ_F16, p) <= tdq.STATIC_SCRATCH_BYTES
