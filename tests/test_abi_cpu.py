"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before launching."""
import ctypes as C
import os
import re

import pytest

from paper_2604_16855_amd import tdq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tdq.h")

pytestmark = pytest.mark.skipif(not os.path.exists(tdq.LIB_PATH),
                                reason="libtdq.so not built (python -m paper_2604_16855_amd.build)")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tdq_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert {"tdq_calibrate_groups", "tdq_quantize_act", "tdq_w4a4_linear",
            "tdq_quantize_act_blocks", "tdq_w4a4_linear_blocks", "tdq_tokenize_chw", "tdq_quantize_act_blocks_chw",
            "tdq_calibrate_quantize_fused", "tdq_range_disparity",
            "tdq_calibrate_groups_chw", "tdq_calibrate_groups_static", "tdq_w4a4_linear_f6", "tdq_quantize_act_f6",
            "tdq_pack_codes_f6", "tdq_f6_bytes", "tdq_w4a4_linear_blocks_f6",
            "tdq_quantize_act_blocks_f6",
            "tdq_quantize_weight", "tdq_workspace_bytes", "tdq_version",
            "tdq_status_string", "tdq_default_params"} <= set(names)
    L = tdq.lib()
    for n in names:
        assert hasattr(L, n), n


def test_every_declared_entry_point_has_a_binding_of_the_same_name():
    for n in _declared():
        assert callable(getattr(tdq, n, None)), n


def test_version_and_strings():
    assert tdq.version() == 110
    assert tdq.status_string(0) == "ok"
    for s in range(-8, 0):
        assert tdq.status_string(s) != "unknown status"
    assert tdq.status_string(-99) == "unknown status"


def test_struct_sizes_match_header_layout():
    assert C.sizeof(tdq.Params) == 48
    assert C.sizeof(tdq.GroupStats) == 48
    p = tdq.default_params()
    assert (p.n_groups, p.act_bits, p.flags, p.tau, p.zr) == (8, 4, 3, 1.0, 0.2)
    assert abs(p.eps_scale - 1e-8) < 1e-15 and abs(p.eps_std - 1e-12) < 1e-19


def test_workspace_bytes():
    p = tdq.default_params(n_groups=16)
    n = tdq.workspace_bytes(1, 7744, 64, tdq.TDQ_F16, p)
    assert n > 7744 * 20 and n % 256 == 0
    assert tdq.workspace_bytes(32, 4096, 1024, tdq.TDQ_F16, tdq.default_params(32)) > \
        tdq.workspace_bytes(1, 4096, 1024, tdq.TDQ_F16, tdq.default_params(32))
    assert tdq.workspace_bytes(0, 10, 10, tdq.TDQ_F16, p) == 0
    assert tdq.workspace_bytes(65536, 10, 10, tdq.TDQ_F16, p) == 0
    assert tdq.workspace_bytes(65535, 10, 10, tdq.TDQ_F16, p) > 0
    assert tdq.workspace_bytes(1, 10, 10, 7, p) == 0
    bad = tdq.default_params(n_groups=0)
    assert tdq.workspace_bytes(1, 10, 10, tdq.TDQ_F16, bad) == 0


FAKE = 4096   # a non-null, aligned "device pointer"; never dereferenced by a failing call


def _calib(p, X=FAKE, dt=tdq.TDQ_F16, B=1, T=8, Cc=8, ld=8, gid=FAKE, clip=FAKE, scale=FAKE,
           ws=FAKE, wsb=1 << 30):
    return tdq.lib().tdq_calibrate_groups(X, dt, B, T, Cc, ld, C.byref(p), gid, clip, scale, None,
                                          ws, wsb, None)


def test_calibrate_rejects_bad_arguments():
    p = tdq.default_params()
    assert _calib(p, X=None) == tdq.ERR_NULL
    assert _calib(p, gid=None) == tdq.ERR_NULL
    assert _calib(p, ws=None) == tdq.ERR_NULL
    assert _calib(p, dt=5) == tdq.ERR_DTYPE
    assert _calib(p, B=0) == tdq.ERR_SHAPE
    assert _calib(p, B=65536) == tdq.ERR_SHAPE          # images index a 16-bit grid axis
    assert _calib(p, ld=7) == tdq.ERR_SHAPE
    assert _calib(p, wsb=16) == tdq.ERR_WORKSPACE
    assert _calib(p, ws=FAKE + 8) == tdq.ERR_WORKSPACE
    assert _calib(p, X=FAKE + 1) == tdq.ERR_ALIGN
    for field, val, err in (("n_groups", 0, tdq.ERR_PARAM), ("n_groups", 257, tdq.ERR_PARAM),
                            ("tau", 0.0, tdq.ERR_PARAM), ("zr", 0.0, tdq.ERR_PARAM),
                            ("zr", 1.0, tdq.ERR_PARAM), ("flags", 4, tdq.ERR_PARAM),
                            ("act_bits", 3, tdq.ERR_PARAM), ("act_bits", 8, tdq.ERR_UNSUPPORTED),
                            ("chan_group", 32, tdq.ERR_UNSUPPORTED),
                            ("base_pct", 1.5, tdq.ERR_PARAM), ("base_pct", -0.1, tdq.ERR_PARAM),
                            ("eps_scale", 0.0, tdq.ERR_PARAM)):
        q = tdq.default_params()
        setattr(q, field, val)
        assert _calib(q) == err, (field, val)


def test_quantize_and_linear_reject_bad_arguments():
    L = tdq.lib()
    p = tdq.default_params()
    q = L.tdq_quantize_act
    assert q(None, 0, 1, 8, 8, 8, C.byref(p), FAKE, FAKE, FAKE, FAKE, 4, None) == tdq.ERR_NULL
    assert q(FAKE, 0, 1, 8, 8, 8, C.byref(p), None, FAKE, FAKE, FAKE, 4, None) == tdq.ERR_NULL
    assert q(FAKE, 0, 1, 8, 8, 8, C.byref(p), FAKE, FAKE, FAKE, FAKE, 3, None) == tdq.ERR_SHAPE
    assert q(FAKE, 9, 1, 8, 8, 8, C.byref(p), FAKE, FAKE, FAKE, FAKE, 4, None) == tdq.ERR_DTYPE
    g = L.tdq_w4a4_linear
    ok = dict(Qx=FAKE, ld_q=32, gid=FAKE, scale=FAKE, B=1, T=8, K=64, N=8, G=4, Qw=FAKE, ld_w=32,
              ws=FAKE, bias=None, Y=FAKE, ydt=1, ld_y=8, dump=None, st=None)

    def call(**kw):
        a = dict(ok, **kw)
        return g(a["Qx"], a["ld_q"], a["gid"], a["scale"], a["B"], a["T"], a["K"], a["N"], a["G"],
                 a["Qw"], a["ld_w"], a["ws"], a["bias"], a["Y"], a["ydt"], a["ld_y"], a["dump"],
                 a["st"])

    assert call(Qx=None) == tdq.ERR_NULL
    assert call(gid=None) == tdq.ERR_NULL          # G > 1 needs group ids
    assert call(K=0) == tdq.ERR_SHAPE
    assert call(K=200000) == tdq.ERR_SHAPE
    # the int32 accumulator holds 256 * acc and |acc| <= 64 K: K = 2^17 could reach 2^31
    assert call(K=131072, ld_q=65536, ld_w=65536) == tdq.ERR_SHAPE
    assert call(ld_q=16) == tdq.ERR_SHAPE          # 64 codes need 32 bytes
    assert call(ld_q=40) == tdq.ERR_ALIGN
    assert call(Qw=FAKE + 4) == tdq.ERR_ALIGN
    assert call(ld_y=4) == tdq.ERR_SHAPE
    assert call(ydt=3) == tdq.ERR_DTYPE
    assert call(G=0) == tdq.ERR_PARAM
    w = L.tdq_quantize_weight
    assert w(None, 8, 8, 8, FAKE, 4, FAKE, None) == tdq.ERR_NULL
    assert w(FAKE, 8, 8, 4, FAKE, 4, FAKE, None) == tdq.ERR_SHAPE
    assert w(FAKE, 8, 8, 8, FAKE, 3, FAKE, None) == tdq.ERR_SHAPE


def test_static_scratch_entry_point_rejects_bad_arguments():
    """tdq_calibrate_groups_static checks its arguments like tdq_calibrate_groups and refuses,
    before touching the device, a shape whose scratch exceeds the static array."""
    f = tdq.lib().tdq_calibrate_groups_static
    p = tdq.default_params(32)

    def call(X=FAKE, dt=0, B=2, T=64, Cc=64, ld=64, q=None, gid=FAKE, clip=FAKE, scale=FAKE, status=None):
        return f(X, dt, B, T, Cc, ld, C.byref(q or p), gid, clip, scale, None, status, None)

    assert call(X=None) == tdq.ERR_NULL
    assert call(scale=None) == tdq.ERR_NULL
    assert call(dt=7) == tdq.ERR_DTYPE
    assert call(ld=63) == tdq.ERR_SHAPE
    assert call(status=FAKE + 2) == tdq.ERR_ALIGN
    q = tdq.default_params(32)
    q.zr = 1.5
    assert call(q=q) == tdq.ERR_PARAM
    assert tdq.workspace_bytes(64, 16384, 64, tdq.TDQ_F16, p) > tdq.STATIC_SCRATCH_BYTES
    assert call(B=64, T=16384) == tdq.ERR_WORKSPACE
    src = open(HEADER).read()
    assert re.search(r"#define\s+TDQ_STATIC_SCRATCH_BYTES\s+\(16u << 20\)", src)


def test_probe_rejects_bad_arguments():
    f = tdq.lib().tdq_probe
    assert f(0, None, 8192, 1, 1, None) == tdq.ERR_NULL
    assert f(0, FAKE + 4, 8192, 1, 1, None) == tdq.ERR_ALIGN
    assert f(9, FAKE, 8192, 1, 1, None) == tdq.ERR_PARAM
    assert f(tdq.PROBE_READ, FAKE, 1000, 1, 1, None) == tdq.ERR_SHAPE
    assert f(tdq.PROBE_COPY, FAKE, 4096, 1, 1, None) == tdq.ERR_SHAPE
    assert f(tdq.PROBE_MFMA_I8, FAKE, 131072, 1, 4, None) == tdq.ERR_SHAPE    # 4 workgroups need 132 KiB
    assert f(tdq.PROBE_FMA_1WAVE, FAKE, 8192, 0, 1, None) == tdq.ERR_SHAPE


def test_block_quantizer_rejects_bad_arguments():
    L = tdq.lib()
    f = L.tdq_quantize_act_blocks
    p = tdq.block_params()

    def call(q=None, X=FAKE, dt=0, B=1, T=8, Cc=40, ld=40, Q=FAKE, ld_q=20, bs=FAKE, bc=None,
             ld_s=2):
        return f(X, dt, B, T, Cc, ld, C.byref(q or p), Q, ld_q, bs, bc, ld_s, None)

    assert call(X=None) == tdq.ERR_NULL
    assert call(Q=None) == tdq.ERR_NULL
    assert call(bs=None) == tdq.ERR_NULL
    assert call(dt=3) == tdq.ERR_DTYPE
    assert call(T=0) == tdq.ERR_SHAPE
    assert call(ld=39) == tdq.ERR_SHAPE
    assert call(ld_q=19) == tdq.ERR_SHAPE          # 40 codes need 20 bytes
    assert call(ld_s=1) == tdq.ERR_SHAPE           # 40 channels are 2 blocks
    assert call(B=1 << 15, T=1 << 15, Cc=64, ld=64, ld_q=32) == tdq.ERR_SHAPE   # 2^31 blocks
    assert call(X=FAKE + 1) == tdq.ERR_ALIGN
    assert call(bs=FAKE + 2) == tdq.ERR_ALIGN
    assert call(q=tdq.default_params()) == tdq.ERR_UNSUPPORTED       # chan_group 0: the token-set path
    for field, val, err in (("chan_group", 16, tdq.ERR_UNSUPPORTED), ("chan_group", -1, tdq.ERR_PARAM),
                            ("zr", 0.0, tdq.ERR_PARAM), ("tau", -1.0, tdq.ERR_PARAM),
                            ("base_pct", 2.0, tdq.ERR_PARAM), ("act_bits", 8, tdq.ERR_UNSUPPORTED)):
        q = tdq.block_params()
        setattr(q, field, val)
        assert call(q=q) == err, (field, val)


def test_block_linear_rejects_bad_arguments():
    g = tdq.lib().tdq_w4a4_linear_blocks
    ok = dict(Qx=FAKE, ld_q=32, bs=FAKE, ld_s=2, M=8, K=64, N=8, Qw=FAKE, ld_w=32, ws=FAKE,
              bias=None, Y=FAKE, ydt=1, ld_y=8, st=None)

    def call(**kw):
        a = dict(ok, **kw)
        return g(a["Qx"], a["ld_q"], a["bs"], a["ld_s"], a["M"], a["K"], a["N"], a["Qw"], a["ld_w"],
                 a["ws"], a["bias"], a["Y"], a["ydt"], a["ld_y"], a["st"])

    assert call(Qx=None) == tdq.ERR_NULL
    assert call(bs=None) == tdq.ERR_NULL
    assert call(M=0) == tdq.ERR_SHAPE
    assert call(K=200000) == tdq.ERR_SHAPE
    # the int32 accumulator holds 256 * acc and |acc| <= 64 K: K = 2^17 could reach 2^31
    assert call(K=131072, ld_q=65536, ld_w=65536) == tdq.ERR_SHAPE
    assert call(ld_s=1) == tdq.ERR_SHAPE           # 64 codes are 2 blocks
    assert call(ld_q=16) == tdq.ERR_SHAPE
    assert call(ld_w=40) == tdq.ERR_ALIGN
    assert call(bs=FAKE + 2) == tdq.ERR_ALIGN
    assert call(Qx=FAKE + 8) == tdq.ERR_ALIGN
    assert call(ld_y=7) == tdq.ERR_SHAPE
    assert call(ydt=2) == tdq.ERR_DTYPE


def test_tokenize_rejects_bad_arguments():
    f = tdq.lib().tdq_tokenize_chw

    def call(X=FAKE, dt=0, B=2, Cc=8, T=12, ld_c=12, ld_b=96, Xt=FAKE, ld_xt=8):
        return f(X, dt, B, Cc, T, ld_c, ld_b, Xt, ld_xt, None)

    assert call(X=None) == tdq.ERR_NULL
    assert call(Xt=None) == tdq.ERR_NULL
    assert call(dt=2) == tdq.ERR_DTYPE
    assert call(Cc=0) == tdq.ERR_SHAPE
    assert call(B=70000, T=1, ld_c=1, ld_b=8) == tdq.ERR_SHAPE
    assert call(ld_c=11) == tdq.ERR_SHAPE
    assert call(ld_b=95) == tdq.ERR_SHAPE          # (C-1)*ld_c + T = 96
    assert call(ld_xt=7) == tdq.ERR_SHAPE
    assert call(X=FAKE + 1) == tdq.ERR_ALIGN


def test_conv_layout_block_quantizer_rejects_bad_arguments():
    f = tdq.lib().tdq_quantize_act_blocks_chw
    p = tdq.block_params()

    def call(q=None, X=FAKE, dt=0, B=2, Cc=40, T=12, ld_c=12, ld_b=480, Q=FAKE, ld_q=20, bs=FAKE,
             bc=None, ld_s=2):
        return f(X, dt, B, Cc, T, ld_c, ld_b, C.byref(q or p), Q, ld_q, bs, bc, ld_s, None)

    assert call(X=None) == tdq.ERR_NULL
    assert call(bs=None) == tdq.ERR_NULL
    assert call(dt=4) == tdq.ERR_DTYPE
    assert call(T=0) == tdq.ERR_SHAPE
    assert call(ld_c=11) == tdq.ERR_SHAPE
    assert call(ld_b=479) == tdq.ERR_SHAPE         # (C-1)*ld_c + T = 480
    assert call(ld_q=19) == tdq.ERR_SHAPE
    assert call(ld_s=1) == tdq.ERR_SHAPE
    assert call(X=FAKE + 1) == tdq.ERR_ALIGN
    assert call(q=tdq.default_params()) == tdq.ERR_UNSUPPORTED


def test_fused_entry_rejects_bad_arguments():
    f = tdq.lib().tdq_calibrate_quantize_fused
    p = tdq.default_params()

    def call(q=None, X=FAKE, dt=0, B=1, T=8, Cc=8, ld=8, gid=FAKE, clip=FAKE, scale=FAKE, flags=None,
             Q=FAKE, ld_q=4, ws=FAKE, wsb=1 << 30):
        return f(X, dt, B, T, Cc, ld, C.byref(q or p), gid, clip, scale, None, flags, Q, ld_q, ws, wsb,
                 None)

    assert call(X=None) == tdq.ERR_NULL
    assert call(Q=None) == tdq.ERR_NULL
    assert call(ws=None) == tdq.ERR_NULL
    assert call(dt=5) == tdq.ERR_DTYPE
    assert call(T=0) == tdq.ERR_SHAPE
    assert call(ld_q=3) == tdq.ERR_SHAPE
    assert call(wsb=16) == tdq.ERR_WORKSPACE
    assert call(ws=FAKE + 8) == tdq.ERR_WORKSPACE
    assert call(flags=FAKE + 2) == tdq.ERR_ALIGN
    assert call(q=tdq.default_params(n_groups=65)) == tdq.ERR_UNSUPPORTED
    assert call(q=tdq.block_params()) == tdq.ERR_UNSUPPORTED


def test_range_disparity_rejects_bad_arguments():
    f = tdq.lib().tdq_range_disparity

    def call(X=FAKE, dt=0, B=1, T=8, Cc=8, ld=8, med=FAKE, tmax=FAKE, D=FAKE, mx=FAKE):
        return f(X, dt, B, T, Cc, ld, med, tmax, D, mx, None)

    assert call(X=None) == tdq.ERR_NULL
    assert call(D=None) == tdq.ERR_NULL
    assert call(dt=2) == tdq.ERR_DTYPE
    assert call(Cc=0) == tdq.ERR_SHAPE
    assert call(ld=7) == tdq.ERR_SHAPE
    assert call(X=FAKE + 1) == tdq.ERR_ALIGN
    assert call(med=FAKE + 2) == tdq.ERR_ALIGN


def test_conv_layout_calibration_rejects_bad_arguments():
    f = tdq.lib().tdq_calibrate_groups_chw
    p = tdq.default_params()

    def call(q=None, X=FAKE, dt=0, B=2, Cc=8, T=12, ld_c=12, ld_b=96, Xt=FAKE, ld_xt=8, gid=FAKE,
             ws=FAKE, wsb=1 << 30):
        return f(X, dt, B, Cc, T, ld_c, ld_b, C.byref(q or p), Xt, ld_xt, gid, FAKE, FAKE, None, ws,
                 wsb, None)

    assert call(X=None) == tdq.ERR_NULL
    assert call(Xt=None) == tdq.ERR_NULL
    assert call(gid=None) == tdq.ERR_NULL
    assert call(dt=3) == tdq.ERR_DTYPE
    assert call(ld_c=11) == tdq.ERR_SHAPE
    assert call(ld_b=95) == tdq.ERR_SHAPE
    assert call(ld_xt=7) == tdq.ERR_SHAPE
    assert call(wsb=8) == tdq.ERR_WORKSPACE
    assert call(X=FAKE + 1) == tdq.ERR_ALIGN
    assert call(q=tdq.block_params()) == tdq.ERR_UNSUPPORTED


def test_f6_entries_reject_bad_arguments():
    L = tdq.lib()
    assert tdq.f6_bytes(1, 1) == 2 * 1536 and tdq.f6_bytes(33, 129) == 2 * 4 * 1536
    assert tdq.f6_bytes(0, 8) == 0
    pk = L.tdq_pack_codes_f6
    assert pk(None, 4, 8, 8, FAKE, None) == tdq.ERR_NULL
    assert pk(FAKE, 3, 8, 8, FAKE, None) == tdq.ERR_SHAPE
    assert pk(FAKE, 4, 8, 8, FAKE + 8, None) == tdq.ERR_ALIGN
    p = tdq.default_params()
    q = L.tdq_quantize_act_f6
    assert q(FAKE, 0, 1, 8, 8, 8, C.byref(p), None, FAKE, FAKE, FAKE, None) == tdq.ERR_NULL   # G > 1 needs ids
    assert q(FAKE, 0, 1, 8, 8, 8, C.byref(p), FAKE, FAKE, FAKE, None, None) == tdq.ERR_NULL
    assert q(FAKE, 0, 1, 8, 8, 8, C.byref(p), FAKE, FAKE, FAKE, FAKE + 4, None) == tdq.ERR_ALIGN
    assert q(FAKE, 0, 1, 8, 8, 7, C.byref(p), FAKE, FAKE, FAKE, FAKE, None) == tdq.ERR_SHAPE
    g = L.tdq_w4a4_linear_f6
    ok = dict(Qx=FAKE, gid=FAKE, scale=FAKE, B=1, T=8, K=64, N=8, G=4, Qw=FAKE, ws=FAKE, bias=None,
              Y=FAKE, ydt=1, ld_y=8, dump=None)

    def call(**kw):
        a = dict(ok, **kw)
        return g(a["Qx"], a["gid"], a["scale"], a["B"], a["T"], a["K"], a["N"], a["G"], a["Qw"],
                 a["ws"], a["bias"], a["Y"], a["ydt"], a["ld_y"], a["dump"], None)

    assert call(Qx=None) == tdq.ERR_NULL
    assert call(gid=None) == tdq.ERR_NULL
    assert call(K=0) == tdq.ERR_SHAPE
    assert call(ld_y=7) == tdq.ERR_SHAPE
    assert call(G=300) == tdq.ERR_PARAM
    assert call(Qw=FAKE + 8) == tdq.ERR_ALIGN
    assert call(ydt=2) == tdq.ERR_DTYPE
    qb = L.tdq_quantize_act_blocks_f6
    pb = tdq.block_params()
    assert qb(None, 0, 1, 8, 64, 64, C.byref(pb), FAKE, FAKE, None, 2, None) == tdq.ERR_NULL
    assert qb(FAKE, 0, 1, 8, 64, 64, C.byref(pb), FAKE, None, None, 2, None) == tdq.ERR_NULL
    assert qb(FAKE, 0, 1, 8, 64, 64, C.byref(pb), FAKE, FAKE, None, 1, None) == tdq.ERR_SHAPE   # two blocks
    assert qb(FAKE, 0, 1, 8, 64, 64, C.byref(pb), FAKE + 8, FAKE, None, 2, None) == tdq.ERR_ALIGN
    assert qb(FAKE, 5, 1, 8, 64, 64, C.byref(pb), FAKE, FAKE, None, 2, None) == tdq.ERR_DTYPE
    assert qb(FAKE, 0, 1, 8, 64, 64, C.byref(p), FAKE, FAKE, None, 2, None) == tdq.ERR_UNSUPPORTED   # chan_group 0: the token-set path
    gb = L.tdq_w4a4_linear_blocks_f6
    okb = dict(Qx=FAKE, ds=FAKE, ld_s=2, M=8, K=64, N=8, Qw=FAKE, ws=FAKE, bias=None, Y=FAKE, ydt=1, ld_y=8)

    def callb(**kw):
        a = dict(okb, **kw)
        return gb(a["Qx"], a["ds"], a["ld_s"], a["M"], a["K"], a["N"], a["Qw"], a["ws"], a["bias"],
                  a["Y"], a["ydt"], a["ld_y"], None)

    assert callb(ds=None) == tdq.ERR_NULL
    assert callb(ld_s=1) == tdq.ERR_SHAPE          # K = 64 has two blocks of 32
    assert callb(M=0) == tdq.ERR_SHAPE
    assert callb(Qx=FAKE + 8) == tdq.ERR_ALIGN
    assert callb(ds=FAKE + 2) == tdq.ERR_ALIGN
    assert callb(ydt=3) == tdq.ERR_DTYPE


def test_binding_shape_helpers_ignore_strides_of_unit_axes():
    """The marshalling takes leading dimensions from strides; the stride of an axis of
    extent 1 addresses nothing (torch and numpy report whatever is convenient for it), so
    it must neither be rejected nor handed on as a leading dimension."""
    import numpy as np
    import torch
    assert tdq._btc(torch.zeros(2, 5, 12)[:, :, :8]) == (2, 5, 8, 12)
    assert tdq._btc(torch.zeros(3, 1, 10)[:, :, :8]) == (3, 1, 8, 10)       # one token per image
    assert tdq._btc(torch.zeros(1, 1, 8)) == (1, 1, 8, 8)
    assert tdq._btc(torch.zeros(4, 6, 3)[:, :, :1]) == (4, 6, 1, 3)         # one channel
    with pytest.raises(ValueError):
        tdq._btc(torch.zeros(2, 5, 12)[:, :, ::2])
    with pytest.raises(ValueError):
        tdq._btc(torch.zeros(3, 5, 8)[::2])
    a = torch.from_numpy(np.ascontiguousarray(np.zeros((3, 1, 64, 8), np.float16).transpose(0, 2, 1, 3)))
    assert a.shape == (3, 64, 1, 8) and tdq._bct(a) == (3, 64, 8, 8, 512)   # H = 1
    assert tdq._bct(torch.zeros(2, 16, 7, 1)) == (2, 16, 7, 7, 112)         # W = 1
    with pytest.raises(ValueError):
        tdq._bct(torch.zeros(2, 16, 7, 4)[:, :, :, ::2])


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only and says so."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr
