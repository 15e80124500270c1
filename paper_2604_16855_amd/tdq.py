"""Thin binding over the C ABI of libtdq (include/tdq.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch is used for device memory and streams and nothing else.  The
functions carry the names of the C entry points and fail loudly when the
library is missing — there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch  # first: the library resolves libamdhip64 against the copy torch loaded

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtdq.so")

TDQ_F16, TDQ_F32 = 0, 1
FLAG_C1, FLAG_C2 = 1, 2
FLAG_EXACT_SELECT = 256     # validation switch: rank select by the per-set radix select only
DEV_NONFINITE = 1
BIND_NAMES = ("base", "C1", "C2", "eps", "empty")

ERR_NULL, ERR_SHAPE, ERR_PARAM, ERR_WORKSPACE = -1, -2, -3, -4
ERR_DTYPE, ERR_HIP, ERR_UNSUPPORTED, ERR_ALIGN = -5, -6, -7, -8


class Params(C.Structure):
    """Mirror of tdq_params."""

    _fields_ = [("n_groups", C.c_int32), ("chan_group", C.c_int32), ("act_bits", C.c_int32),
                ("flags", C.c_uint32), ("tau", C.c_double), ("zr", C.c_double),
                ("base_pct", C.c_double), ("eps_scale", C.c_float), ("eps_std", C.c_float)]


class GroupStats(C.Structure):
    """Mirror of tdq_group_stats (48 bytes)."""

    _fields_ = [("n", C.c_int64), ("k", C.c_int64), ("c_base", C.c_float), ("sigma", C.c_float),
                ("thr", C.c_float), ("c_tau", C.c_float), ("c_zr", C.c_float), ("clip", C.c_float),
                ("scale", C.c_float), ("bind", C.c_uint32)]


class TdqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """Loads libtdq.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2604_16855_amd.build` "
            "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.tdq_version.restype = C.c_int
    L.tdq_status_string.restype = C.c_char_p
    L.tdq_status_string.argtypes = [C.c_int]
    L.tdq_default_params.restype = None
    L.tdq_default_params.argtypes = [C.POINTER(Params)]
    L.tdq_workspace_bytes.restype = sz
    L.tdq_workspace_bytes.argtypes = [i32, i32, i32, C.c_int, C.POINTER(Params)]
    L.tdq_calibrate_groups.restype = C.c_int
    L.tdq_calibrate_groups.argtypes = [vp, C.c_int, i32, i32, i32, i64, C.POINTER(Params), vp, vp,
                                       vp, vp, vp, sz, vp]
    L.tdq_calibrate_groups_static.restype = C.c_int
    L.tdq_calibrate_groups_static.argtypes = [vp, C.c_int, i32, i32, i32, i64, C.POINTER(Params), vp,
                                              vp, vp, vp, vp, vp]
    L.tdq_quantize_act.restype = C.c_int
    L.tdq_quantize_act.argtypes = [vp, C.c_int, i32, i32, i32, i64, C.POINTER(Params), vp, vp, vp,
                                   vp, i64, vp]
    L.tdq_w4a4_linear.restype = C.c_int
    L.tdq_w4a4_linear.argtypes = [vp, i64, vp, vp, i32, i32, i32, i32, i32, vp, i64, vp, vp, vp,
                                  C.c_int, i64, vp, vp]
    L.tdq_quantize_act_blocks.restype = C.c_int
    L.tdq_quantize_act_blocks.argtypes = [vp, C.c_int, i32, i32, i32, i64, C.POINTER(Params), vp,
                                          i64, vp, vp, i64, vp]
    L.tdq_quantize_act_blocks_f6.restype = C.c_int
    L.tdq_quantize_act_blocks_f6.argtypes = [vp, C.c_int, i32, i32, i32, i64, C.POINTER(Params), vp,
                                             vp, vp, i64, vp]
    L.tdq_w4a4_linear_blocks.restype = C.c_int
    L.tdq_w4a4_linear_blocks.argtypes = [vp, i64, vp, i64, i64, i32, i32, vp, i64, vp, vp, vp,
                                         C.c_int, i64, vp]
    L.tdq_tokenize_chw.restype = C.c_int
    L.tdq_tokenize_chw.argtypes = [vp, C.c_int, i32, i32, i32, i64, i64, vp, i64, vp]
    L.tdq_quantize_act_blocks_chw.restype = C.c_int
    L.tdq_quantize_act_blocks_chw.argtypes = [vp, C.c_int, i32, i32, i32, i64, i64,
                                              C.POINTER(Params), vp, i64, vp, vp, i64, vp]
    L.tdq_calibrate_quantize_fused.restype = C.c_int
    L.tdq_calibrate_quantize_fused.argtypes = [vp, C.c_int, i32, i32, i32, i64, C.POINTER(Params),
                                               vp, vp, vp, vp, vp, vp, i64, vp, sz, vp]
    L.tdq_range_disparity.restype = C.c_int
    L.tdq_range_disparity.argtypes = [vp, C.c_int, i32, i32, i32, i64, vp, vp, vp, vp, vp]
    L.tdq_calibrate_groups_chw.restype = C.c_int
    L.tdq_calibrate_groups_chw.argtypes = [vp, C.c_int, i32, i32, i32, i64, i64, C.POINTER(Params),
                                           vp, i64, vp, vp, vp, vp, vp, sz, vp]
    L.tdq_f6_bytes.restype = sz
    L.tdq_f6_bytes.argtypes = [i64, i32]
    L.tdq_quantize_act_f6.restype = C.c_int
    L.tdq_quantize_act_f6.argtypes = [vp, C.c_int, i32, i32, i32, i64, C.POINTER(Params), vp, vp, vp,
                                      vp, vp]
    L.tdq_w4a4_linear_blocks_f6.restype = C.c_int
    L.tdq_w4a4_linear_blocks_f6.argtypes = [vp, vp, i64, i64, i32, i32, vp, vp, vp, vp, C.c_int, i64,
                                            vp]
    L.tdq_pack_codes_f6.restype = C.c_int
    L.tdq_pack_codes_f6.argtypes = [vp, i64, i64, i32, vp, vp]
    L.tdq_w4a4_linear_f6.restype = C.c_int
    L.tdq_w4a4_linear_f6.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, C.c_int,
                                     i64, vp, vp]
    L.tdq_group_diagnostics.restype = C.c_int
    L.tdq_group_diagnostics.argtypes = [vp, C.c_int, i32, i32, i32, i64, C.POINTER(Params), vp, vp,
                                        vp, vp, vp, vp]
    L.tdq_probe.restype = C.c_int
    L.tdq_probe.argtypes = [C.c_int32, vp, sz, C.c_int32, C.c_int32, vp]
    L.tdq_quantize_weight.restype = C.c_int
    L.tdq_quantize_weight.argtypes = [vp, i32, i32, i64, vp, i64, vp, vp]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().tdq_status_string(int(status)).decode()


def version() -> int:
    return int(lib().tdq_version())


def default_params(n_groups: int = 8, tau: float = 1.0, zr: float = 0.2,
                   flags: int = FLAG_C1 | FLAG_C2) -> Params:
    p = Params()
    lib().tdq_default_params(C.byref(p))
    p.n_groups, p.tau, p.zr, p.flags = n_groups, tau, zr, flags
    return p


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return TDQ_F16
    if t.dtype == torch.float32:
        return TDQ_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != 0:
        raise TdqError(rc, where)


def _btc(X: torch.Tensor) -> Tuple[int, int, int, int]:
    # the stride of an axis of extent 1 is never used to address anything, and torch is
    # free to report any value for it
    if X.dim() != 3 or (X.shape[2] > 1 and X.stride(2) != 1):
        raise ValueError("X must be [B, T, C] with contiguous channels and uniform row stride")
    if X.shape[1] > 1:
        ld = X.stride(1)
    else:
        ld = X.stride(0) if X.shape[0] > 1 else max(X.shape[2], 1)
    if X.shape[0] > 1 and X.stride(0) != X.shape[1] * ld:
        raise ValueError("X must be [B, T, C] with contiguous channels and uniform row stride")
    return X.shape[0], X.shape[1], X.shape[2], ld


def workspace_bytes(B: int, T: int, C_: int, dt: int, p: Params) -> int:
    return int(lib().tdq_workspace_bytes(B, T, C_, dt, C.byref(p)))


def alloc_workspace(B: int, T: int, C_: int, dt: int, p: Params, device) -> torch.Tensor:
    n = workspace_bytes(B, T, C_, dt, p)
    if n == 0:
        raise TdqError(ERR_PARAM, "tdq_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def tdq_calibrate_groups(X: torch.Tensor, p: Params, workspace: Optional[torch.Tensor] = None,
                         want_stats: bool = False, out=None):
    """-> (group_id[B,T] int32, clip[B,G] f32, scale[B,G] f32, stats or None, workspace).
    `stats` is a uint8 tensor [B*G, 48] holding tdq_group_stats records (see
    `stats_to_numpy`).  Asynchronous on the current stream."""
    B, T, Cc, ld = _btc(X)
    G = p.n_groups
    dev = X.device
    if workspace is None:
        workspace = alloc_workspace(B, T, Cc, _dt(X), p, dev)
    if out is None:
        gid = torch.empty((B, T), dtype=torch.int32, device=dev)
        clip = torch.empty((B, G), dtype=torch.float32, device=dev)
        scale = torch.empty((B, G), dtype=torch.float32, device=dev)
    else:
        gid, clip, scale = out
    stats = (torch.empty((B * G, C.sizeof(GroupStats)), dtype=torch.uint8, device=dev)
             if want_stats else None)
    rc = lib().tdq_calibrate_groups(X.data_ptr(), _dt(X), B, T, Cc, ld, C.byref(p), gid.data_ptr(),
                                    clip.data_ptr(), scale.data_ptr(), _ptr(stats),
                                    workspace.data_ptr(), workspace.numel(), _stream())
    _check(rc, "tdq_calibrate_groups")
    return gid, clip, scale, stats, workspace


STATIC_SCRATCH_BYTES = 16 << 20     # TDQ_STATIC_SCRATCH_BYTES


def tdq_calibrate_groups_static(X: torch.Tensor, p: Params, out, stats: Optional[torch.Tensor] = None,
                                status: Optional[torch.Tensor] = None) -> None:
    """tdq_calibrate_groups on the library's static scratch.  Allocates nothing: the caller
    passes every buffer — out = (group_id[B,T] int32, clip[B,G] f32, scale[B,G] f32), stats
    (uint8 [B*G, 48]) or None, status (int32 [4]) or None.  Asynchronous on the current
    stream."""
    B, T, Cc, ld = _btc(X)
    gid, clip, scale = out
    rc = lib().tdq_calibrate_groups_static(X.data_ptr(), _dt(X), B, T, Cc, ld, C.byref(p),
                                           gid.data_ptr(), clip.data_ptr(), scale.data_ptr(),
                                           _ptr(stats), _ptr(status), _stream())
    _check(rc, "tdq_calibrate_groups_static")


def tdq_calibrate_quantize_fused(X: torch.Tensor, p: Params,
                                 workspace: Optional[torch.Tensor] = None,
                                 want_stats: bool = False, out=None):
    """One launch for tdq_calibrate_groups + tdq_quantize_act (small shapes).
    -> (group_id[B,T], clip[B,G], scale[B,G], stats or None, image_flags[B] int32, Qx,
    workspace)."""
    B, T, Cc, ld = _btc(X)
    G = p.n_groups
    dev = X.device
    if workspace is None:
        workspace = alloc_workspace(B, T, Cc, _dt(X), p, dev)
    if out is None:
        gid = torch.empty((B, T), dtype=torch.int32, device=dev)
        clip = torch.empty((B, G), dtype=torch.float32, device=dev)
        scale = torch.empty((B, G), dtype=torch.float32, device=dev)
        flags = torch.empty((B,), dtype=torch.int32, device=dev)
        Qx = torch.zeros((B * T, packed_row_bytes(Cc)), dtype=torch.uint8, device=dev)
    else:
        gid, clip, scale, flags, Qx = out
    stats = (torch.empty((B * G, C.sizeof(GroupStats)), dtype=torch.uint8, device=dev)
             if want_stats else None)
    rc = lib().tdq_calibrate_quantize_fused(X.data_ptr(), _dt(X), B, T, Cc, ld, C.byref(p),
                                            gid.data_ptr(), clip.data_ptr(), scale.data_ptr(),
                                            _ptr(stats), flags.data_ptr(), Qx.data_ptr(),
                                            Qx.stride(0), workspace.data_ptr(), workspace.numel(),
                                            _stream())
    _check(rc, "tdq_calibrate_quantize_fused")
    return gid, clip, scale, stats, flags, Qx, workspace


def device_status(workspace: torch.Tensor) -> int:
    """Status word left by the last tdq_calibrate_groups (synchronises)."""
    return int(workspace[:4].view(torch.int32).item())


def exact_select_sets(workspace: torch.Tensor) -> int:
    """How many token sets the last binary16 tdq_calibrate_groups resolved by the
    per-set radix select because the sampled key interval missed their rank (synchronises)."""
    return int(workspace[4:12].view(torch.int32).sum().item())


def stats_to_numpy(stats: torch.Tensor):
    import numpy as np
    dt = np.dtype([("n", "<i8"), ("k", "<i8"), ("c_base", "<f4"), ("sigma", "<f4"), ("thr", "<f4"),
                   ("c_tau", "<f4"), ("c_zr", "<f4"), ("clip", "<f4"), ("scale", "<f4"),
                   ("bind", "<u4")])
    return stats.cpu().numpy().view(dt).reshape(-1)


def packed_row_bytes(K: int) -> int:
    """Leading dimension (bytes) the contraction wants for K codes per row."""
    return 16 * ((K + 31) // 32)


def tdq_quantize_act(X: torch.Tensor, p: Params, gid: Optional[torch.Tensor],
                     clip: torch.Tensor, scale: torch.Tensor,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """-> Qx[B*T, ld_q] uint8 packed int4 codes (ld_q = 16*ceil(C/32), bytes past
    ceil(C/2) of a row are zero on a fresh buffer)."""
    B, T, Cc, ld = _btc(X)
    if out is None:
        out = torch.zeros((B * T, packed_row_bytes(Cc)), dtype=torch.uint8, device=X.device)
    rc = lib().tdq_quantize_act(X.data_ptr(), _dt(X), B, T, Cc, ld, C.byref(p), _ptr(gid),
                                clip.data_ptr(), scale.data_ptr(), out.data_ptr(), out.stride(0),
                                _stream())
    _check(rc, "tdq_quantize_act")
    return out


def _bct(X: torch.Tensor) -> Tuple[int, int, int, int, int]:
    """(B, C, T, ld_c, ld_b) of a feature map [B, C, H, W] or [B, C, T] with contiguous
    spatial axes."""
    if X.dim() == 4:
        if (X.shape[3] > 1 and X.stride(3) != 1) or (X.shape[2] > 1 and X.stride(2) != X.shape[3]):
            raise ValueError("the spatial axes of X must be contiguous")
        B, Cc, T = X.shape[0], X.shape[1], X.shape[2] * X.shape[3]
    elif X.dim() == 3 and (X.shape[2] == 1 or X.stride(2) == 1):
        B, Cc, T = X.shape
    else:
        raise ValueError("X must be [B, C, H, W] or [B, C, T] with contiguous tokens")
    ld_c = X.stride(1) if Cc > 1 else T
    ld_b = X.stride(0) if B > 1 else max((Cc - 1) * ld_c + T, 1)
    return B, Cc, T, ld_c, ld_b


def tdq_calibrate_groups_chw(X: torch.Tensor, p: Params, workspace: Optional[torch.Tensor] = None,
                             want_stats: bool = False, out=None):
    """tdq_calibrate_groups on a feature map X[B, C, H, W] read in place.
    -> (Xt[B, H*W, C] token-major copy, group_id[B,T], clip[B,G], scale[B,G], stats or None,
    workspace); quantize with tdq_quantize_act(Xt, ...)."""
    B, Cc, T, ld_c, ld_b = _bct(X)
    G = p.n_groups
    dev = X.device
    if workspace is None:
        workspace = alloc_workspace(B, T, Cc, _dt(X), p, dev)
    if out is None:
        Xt = torch.empty((B, T, Cc), dtype=X.dtype, device=dev)
        gid = torch.empty((B, T), dtype=torch.int32, device=dev)
        clip = torch.empty((B, G), dtype=torch.float32, device=dev)
        scale = torch.empty((B, G), dtype=torch.float32, device=dev)
    else:
        Xt, gid, clip, scale = out
    stats = (torch.empty((B * G, C.sizeof(GroupStats)), dtype=torch.uint8, device=dev)
             if want_stats else None)
    rc = lib().tdq_calibrate_groups_chw(X.data_ptr(), _dt(X), B, Cc, T, ld_c, ld_b, C.byref(p),
                                        Xt.data_ptr(), Xt.stride(1), gid.data_ptr(), clip.data_ptr(),
                                        scale.data_ptr(), _ptr(stats), workspace.data_ptr(),
                                        workspace.numel(), _stream())
    _check(rc, "tdq_calibrate_groups_chw")
    return Xt, gid, clip, scale, stats, workspace


def tdq_quantize_act_blocks_chw(X: torch.Tensor, p: Params, want_clip: bool = False,
                                out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None):
    """tdq_quantize_act_blocks on a feature map X[B, C, H, W] read in place:
    -> (Qx[B*H*W, ld_q], block_scale[B*H*W, KB], block_clip or None)."""
    B, Cc, T, ld_c, ld_b = _bct(X)
    KB = (Cc + 31) // 32
    if out is None:
        Qx = torch.zeros((B * T, packed_row_bytes(Cc)), dtype=torch.uint8, device=X.device)
        bs = torch.empty((B * T, KB), dtype=torch.float32, device=X.device)
    else:
        Qx, bs = out
    bc = torch.empty((B * T, KB), dtype=torch.float32, device=X.device) if want_clip else None
    rc = lib().tdq_quantize_act_blocks_chw(X.data_ptr(), _dt(X), B, Cc, T, ld_c, ld_b, C.byref(p),
                                           Qx.data_ptr(), Qx.stride(0), bs.data_ptr(), _ptr(bc),
                                           bs.stride(0), _stream())
    _check(rc, "tdq_quantize_act_blocks_chw")
    return Qx, bs, bc


def tdq_tokenize_chw(X: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """X[B, C, H, W] (or [B, C, T]) with contiguous spatial axes -> Xt[B, H*W, C]."""
    B, Cc, T, ld_c, ld_b = _bct(X)
    if out is None:
        out = torch.empty((B, T, Cc), dtype=X.dtype, device=X.device)
    rc = lib().tdq_tokenize_chw(X.data_ptr(), _dt(X), B, Cc, T, ld_c, ld_b, out.data_ptr(),
                                out.stride(1), _stream())
    _check(rc, "tdq_tokenize_chw")
    return out


BLOCK = 32                  # TDQ_BLOCK: channel block of the per-(token, block) entry points


def block_params(tau: float = 1.0, zr: float = 0.2, flags: int = FLAG_C1 | FLAG_C2,
                 base_pct: float = 0.0) -> Params:
    """tdq_params for the *_blocks entry points (chan_group = TDQ_BLOCK)."""
    p = default_params(1, tau, zr, flags)
    p.chan_group, p.base_pct = BLOCK, base_pct
    return p


def tdq_quantize_act_blocks(X: torch.Tensor, p: Params, want_clip: bool = False,
                            out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None):
    """-> (Qx[B*T, ld_q] uint8 packed codes, block_scale[B*T, KB] f32, block_clip or None),
    KB = ceil(C / 32): one step per (token, 32-channel block)."""
    B, T, Cc, ld = _btc(X)
    KB = (Cc + BLOCK - 1) // BLOCK
    if out is None:
        Qx = torch.zeros((B * T, packed_row_bytes(Cc)), dtype=torch.uint8, device=X.device)
        bs = torch.empty((B * T, KB), dtype=torch.float32, device=X.device)
    else:
        Qx, bs = out
    bc = torch.empty((B * T, KB), dtype=torch.float32, device=X.device) if want_clip else None
    rc = lib().tdq_quantize_act_blocks(X.data_ptr(), _dt(X), B, T, Cc, ld, C.byref(p), Qx.data_ptr(),
                                       Qx.stride(0), bs.data_ptr(), _ptr(bc), bs.stride(0), _stream())
    _check(rc, "tdq_quantize_act_blocks")
    return Qx, bs, bc


def tdq_quantize_act_blocks_f6(X: torch.Tensor, p: Params, want_clip: bool = False,
                               out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None):
    """tdq_quantize_act_blocks writing f6 fragments:
    -> (Qx6[f6_bytes(B*T, C)] uint8, block_scale[B*T, KB] f32, block_clip or None)."""
    B, T, Cc, ld = _btc(X)
    KB = (Cc + BLOCK - 1) // BLOCK
    if out is None:
        Qx6 = torch.empty((f6_bytes(B * T, Cc),), dtype=torch.uint8, device=X.device)
        bs = torch.empty((B * T, KB), dtype=torch.float32, device=X.device)
    else:
        Qx6, bs = out
    if Qx6.numel() < f6_bytes(B * T, Cc):
        raise ValueError("Qx6 is too small")
    bc = torch.empty((B * T, KB), dtype=torch.float32, device=X.device) if want_clip else None
    rc = lib().tdq_quantize_act_blocks_f6(X.data_ptr(), _dt(X), B, T, Cc, ld, C.byref(p), Qx6.data_ptr(),
                                          bs.data_ptr(), _ptr(bc), bs.stride(0), _stream())
    _check(rc, "tdq_quantize_act_blocks_f6")
    return Qx6, bs, bc


def tdq_w4a4_linear_blocks(Qx: torch.Tensor, block_scale: torch.Tensor, K: int, Qw: torch.Tensor,
                           w_scale: torch.Tensor, bias: Optional[torch.Tensor] = None,
                           out_dtype=torch.float32, out: Optional[torch.Tensor] = None
                           ) -> torch.Tensor:
    """-> Y[M, N] from block-quantized activations: one step per (row, 32-code block)."""
    M, N = Qx.shape[0], Qw.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=Qx.device)
    rc = lib().tdq_w4a4_linear_blocks(Qx.data_ptr(), Qx.stride(0), block_scale.data_ptr(),
                                      block_scale.stride(0), M, K, N, Qw.data_ptr(), Qw.stride(0),
                                      w_scale.data_ptr(), _ptr(bias), out.data_ptr(), _dt(out),
                                      out.stride(0), _stream())
    _check(rc, "tdq_w4a4_linear_blocks")
    return out


def tdq_group_diagnostics(X: torch.Tensor, p: Params, gid: Optional[torch.Tensor],
                          clip: torch.Tensor, scale: torch.Tensor
                          ) -> Tuple[torch.Tensor, torch.Tensor]:
    """-> (zero_count[B, G], clipped_count[B, G]) int64: elements of every token set
    whose code is 0, and elements with |x| above the set's clip radius."""
    B, T, Cc, ld = _btc(X)
    G = p.n_groups
    zero = torch.empty((B, G), dtype=torch.int64, device=X.device)
    clipped = torch.empty((B, G), dtype=torch.int64, device=X.device)
    rc = lib().tdq_group_diagnostics(X.data_ptr(), _dt(X), B, T, Cc, ld, C.byref(p), _ptr(gid),
                                     clip.data_ptr(), scale.data_ptr(), zero.data_ptr(),
                                     clipped.data_ptr(), _stream())
    _check(rc, "tdq_group_diagnostics")
    return zero, clipped


def tdq_range_disparity(X: torch.Tensor):
    """-> (D[B], token_median[B, T], max_abs[B]) f32: range disparity per image."""
    B, T, Cc, ld = _btc(X)
    dev = X.device
    med = torch.empty((B, T), dtype=torch.float32, device=dev)
    tmax = torch.empty((B, T), dtype=torch.float32, device=dev)
    D = torch.empty((B,), dtype=torch.float32, device=dev)
    mx = torch.empty((B,), dtype=torch.float32, device=dev)
    rc = lib().tdq_range_disparity(X.data_ptr(), _dt(X), B, T, Cc, ld, med.data_ptr(),
                                   tmax.data_ptr(), D.data_ptr(), mx.data_ptr(), _stream())
    _check(rc, "tdq_range_disparity")
    return D, med, mx


def f6_bytes(rows: int, K: int) -> int:
    return int(lib().tdq_f6_bytes(rows, K))


def tdq_quantize_act_f6(X: torch.Tensor, p: Params, gid: Optional[torch.Tensor], clip: torch.Tensor,
                        scale: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """tdq_quantize_act writing f6 fragments (uint8 [tdq_f6_bytes(B*T, C)])."""
    B, T, Cc, ld = _btc(X)
    if out is None:
        out = torch.empty((f6_bytes(B * T, Cc),), dtype=torch.uint8, device=X.device)
    rc = lib().tdq_quantize_act_f6(X.data_ptr(), _dt(X), B, T, Cc, ld, C.byref(p), _ptr(gid),
                                   clip.data_ptr(), scale.data_ptr(), out.data_ptr(), _stream())
    _check(rc, "tdq_quantize_act_f6")
    return out


def tdq_pack_codes_f6(Q: torch.Tensor, K: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Packed nibbles Q[rows, ld] -> f6 fragments (uint8 [tdq_f6_bytes(rows, K)])."""
    rows = Q.shape[0]
    if out is None:
        out = torch.empty((f6_bytes(rows, K),), dtype=torch.uint8, device=Q.device)
    rc = lib().tdq_pack_codes_f6(Q.data_ptr(), Q.stride(0), rows, K, out.data_ptr(), _stream())
    _check(rc, "tdq_pack_codes_f6")
    return out


def tdq_w4a4_linear_f6(Qx6: torch.Tensor, gid: Optional[torch.Tensor], scale: torch.Tensor, B: int,
                       T: int, K: int, Qw6: torch.Tensor, N: int, w_scale: torch.Tensor,
                       bias: Optional[torch.Tensor] = None, out_dtype=torch.float32,
                       out: Optional[torch.Tensor] = None, acc_dump: Optional[torch.Tensor] = None
                       ) -> torch.Tensor:
    """tdq_w4a4_linear on f6-fragment operands -> Y[B*T, N]."""
    G = scale.shape[1] if scale.dim() == 2 else scale.numel() // B
    if out is None:
        out = torch.empty((B * T, N), dtype=out_dtype, device=Qx6.device)
    rc = lib().tdq_w4a4_linear_f6(Qx6.data_ptr(), _ptr(gid), scale.data_ptr(), B, T, K, N, G,
                                  Qw6.data_ptr(), w_scale.data_ptr(), _ptr(bias), out.data_ptr(),
                                  _dt(out), out.stride(0), _ptr(acc_dump), _stream())
    _check(rc, "tdq_w4a4_linear_f6")
    return out


def tdq_w4a4_linear_blocks_f6(Qx6: torch.Tensor, block_scale: torch.Tensor, K: int,
                              Qw6: torch.Tensor, N: int, w_scale: torch.Tensor,
                              bias: Optional[torch.Tensor] = None, out_dtype=torch.float32,
                              out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """tdq_w4a4_linear_blocks on f6-fragment operands -> Y[M, N], M = block_scale.shape[0]."""
    M = block_scale.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=Qx6.device)
    rc = lib().tdq_w4a4_linear_blocks_f6(Qx6.data_ptr(), block_scale.data_ptr(), block_scale.stride(0),
                                         M, K, N, Qw6.data_ptr(), w_scale.data_ptr(), _ptr(bias),
                                         out.data_ptr(), _dt(out), out.stride(0), _stream())
    _check(rc, "tdq_w4a4_linear_blocks_f6")
    return out


PROBE_READ, PROBE_COPY, PROBE_MFMA_I8, PROBE_FMA_1WAVE, PROBE_FMA_2WAVES, PROBE_FMA_4WAVES = 0, 1, 2, 3, 4, 5


def tdq_probe(kind: int, buf: torch.Tensor, iters: int = 1, grid: int = 1) -> None:
    """One launch of a measurement probe on `buf` (uint8 device tensor); see tdq.h."""
    rc = lib().tdq_probe(kind, buf.data_ptr(), buf.numel() * buf.element_size(), iters, grid, _stream())
    _check(rc, "tdq_probe")


def tdq_quantize_weight(W: torch.Tensor) -> Tuple[torch.Tensor, torch.Tensor]:
    """W[N, K] fp32 (device) -> (Qw[N, ld_w] uint8 packed, w_scale[N] f32)."""
    if W.dtype != torch.float32 or W.dim() != 2 or W.stride(1) != 1:
        raise ValueError("W must be fp32 [N, K] with contiguous rows")
    N, K = W.shape
    Qw = torch.empty((N, packed_row_bytes(K)), dtype=torch.uint8, device=W.device)
    ws = torch.empty((N,), dtype=torch.float32, device=W.device)
    rc = lib().tdq_quantize_weight(W.data_ptr(), N, K, W.stride(0), Qw.data_ptr(), Qw.stride(0),
                                   ws.data_ptr(), _stream())
    _check(rc, "tdq_quantize_weight")
    return Qw, ws


def tdq_w4a4_linear(Qx: torch.Tensor, gid: Optional[torch.Tensor], scale: torch.Tensor, B: int,
                    T: int, K: int, Qw: torch.Tensor, w_scale: torch.Tensor,
                    bias: Optional[torch.Tensor] = None, out_dtype=torch.float32,
                    out: Optional[torch.Tensor] = None, acc_dump: Optional[torch.Tensor] = None
                    ) -> torch.Tensor:
    """-> Y[B*T, N].  scale is [B, G]; gid [B, T] (may be None when G == 1)."""
    N = Qw.shape[0]
    G = scale.shape[1] if scale.dim() == 2 else scale.numel() // B
    if out is None:
        out = torch.empty((B * T, N), dtype=out_dtype, device=Qx.device)
    rc = lib().tdq_w4a4_linear(Qx.data_ptr(), Qx.stride(0), _ptr(gid), scale.data_ptr(), B, T, K, N,
                               G, Qw.data_ptr(), Qw.stride(0), w_scale.data_ptr(), _ptr(bias),
                               out.data_ptr(), _dt(out), out.stride(0), _ptr(acc_dump), _stream())
    _check(rc, "tdq_w4a4_linear")
    return out


# the helper entry points under their C names as well
tdq_version = version
tdq_status_string = status_string
tdq_default_params = default_params
tdq_workspace_bytes = workspace_bytes
tdq_f6_bytes = f6_bytes
