"""Thin ctypes binding of ``liblc.so``: argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks shape,
dtype and contiguity, and passes raw device pointers plus the current HIP stream
to the C entry point of the same name (``include/lc.h``).  No arithmetic happens
here, and there is no fallback: if the library is missing the import of a symbol
fails loudly.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path
from typing import Optional, Tuple

import torch

_HERE = Path(__file__).resolve().parent
LIB_PATH = _HERE / "liblc.so"

LC_OK, LC_EINVAL, LC_ENULL, LC_EALIGN, LC_EWORKSPACE, LC_EUNSUPPORTED, LC_EHIP, LC_EINTERNAL = 0, -1, -2, -3, -4, -5, -6, -7
LC_F32, LC_BF16 = 0, 1
LC_OP_FORWARD, LC_OP_BACKWARD_DATA, LC_OP_BACKWARD_WEIGHTS, LC_OP_SAE_STEP = 0, 1, 2, 3
LC_SAE_PROJECT_ROWS, LC_SAE_LEARN_ALPHA = 1, 2
_STATUS = {0: "LC_OK", -1: "LC_EINVAL", -2: "LC_ENULL", -3: "LC_EALIGN", -4: "LC_EWORKSPACE",
           -5: "LC_EUNSUPPORTED", -6: "LC_EHIP", -7: "LC_EINTERNAL"}

EXPORTS = ("lc_geom_derive", "lc_workspace_bytes", "lc_forward", "lc_forward_dev_scale", "lc_backward_data", "lc_backward_weights",
           "l2pool_fwd", "l2pool_bwd", "lcn_fwd", "lcn_bwd", "l2pool_lcn_fwd", "lcn_l2pool_bwd", "lcn_variant_workspace_bytes", "lcn_variant_fwd",
           "lcn_variant_bwd", "lcn_variant_bwd_static", "sae_step", "lc_last_error", "lc_plan_query", "l2pool_lcn_plan_query")


class LcGeom(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "H", "W", "C", "R", "S", "F")]


class LcLaunch(C.Structure):
    """One planned kernel launch (``lc_launch_t`` of ``include/lc_plan.h``)."""
    _fields_ = [("kernel", C.c_char * 32), ("tparam", C.c_int32 * 12), ("arg", C.c_int32 * 12),
                ("grid", C.c_uint32 * 3), ("block", C.c_uint32), ("lds_bytes", C.c_uint64)]


class LcError(RuntimeError):
    def __init__(self, fn: str, code: int, detail: str = ""):
        self.code = code
        super().__init__(f"{fn} failed: {_STATUS.get(code, code)}{(' - ' + detail) if detail else ''}")


_lib = None


def lib() -> C.CDLL:
    """Load ``liblc.so`` (built by ``paper_1502_03409_amd.build``); raises if it is not there."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_1502_03409_amd.build` "
                                    "(there is no CPU fallback)")
        L = C.CDLL(str(LIB_PATH))
        vp, f32, i32, u32, sz = C.c_void_p, C.c_float, C.c_int32, C.c_uint32, C.c_size_t
        G = C.POINTER(LcGeom)
        L.lc_geom_derive.argtypes = [G, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        L.lc_workspace_bytes.argtypes = [G, C.c_int, C.c_int]
        L.lc_workspace_bytes.restype = sz
        L.lc_forward.argtypes = [G, vp, vp, vp, f32, vp, C.c_int, vp, sz, vp]
        L.lc_forward_dev_scale.argtypes = [G, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lc_backward_data.argtypes = [G, vp, vp, vp, C.c_int, vp, sz, vp]
        L.lc_backward_weights.argtypes = [G, vp, vp, f32, vp, C.c_int, vp, sz, vp]
        L.l2pool_fwd.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, f32, vp]
        L.l2pool_bwd.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp]
        L.lcn_fwd.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, vp]
        L.l2pool_lcn_fwd.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, f32, i32, f32, f32, vp]
        L.lcn_l2pool_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, f32, vp]
        L.lcn_bwd.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, vp]
        L.lcn_variant_workspace_bytes.argtypes = [i32, i32, i32, i32, C.c_uint32]
        L.lcn_variant_workspace_bytes.restype = C.c_size_t
        L.lcn_variant_fwd.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, f32, C.c_uint32, vp]
        L.lcn_variant_bwd.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, C.c_uint32, vp, C.c_size_t, vp]
        L.lcn_variant_bwd_static.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, f32, C.c_uint32, vp]
        L.sae_step.argtypes = [G, vp, vp, vp, vp, f32, f32, f32, u32, vp, vp, vp, sz, vp]
        L.lc_last_error.restype = C.c_char_p
        L.lc_plan_query.argtypes = [G, C.c_int, C.c_int, C.POINTER(LcLaunch), i32, C.POINTER(i32)]
        L.l2pool_lcn_plan_query.argtypes = [i32, i32, i32, i32, i32, i32, i32, f32, C.POINTER(LcLaunch), i32, C.POINTER(i32)]
        for name in EXPORTS:
            if name not in ("lc_workspace_bytes", "lc_last_error"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(fn: str, rc: int) -> None:
    if rc != LC_OK:
        with_text = rc in (LC_EHIP, LC_EINTERNAL) or (rc == LC_EWORKSPACE and fn == "lcn_variant_bwd_static")
        detail = lib().lc_last_error().decode() if with_text else ""
        raise LcError(fn, rc, detail)


def geom(B: int, H: int, W: int, Cc: int, R: int, S: int, F: int) -> LcGeom:
    return LcGeom(B, H, W, Cc, R, S, F)


def geom_derive(g: LcGeom) -> Tuple[int, int, int]:
    lh, lw, k = C.c_int32(), C.c_int32(), C.c_int32()
    _check("lc_geom_derive", lib().lc_geom_derive(C.byref(g), C.byref(lh), C.byref(lw), C.byref(k)))
    return lh.value, lw.value, k.value


def workspace_bytes(g: LcGeom, op: int, dtype: int = LC_F32) -> int:
    return int(lib().lc_workspace_bytes(C.byref(g), op, dtype))


def plan_query(g: LcGeom, op: int, dtype: int = LC_F32, max_out: int = 16):
    """The launches ``op`` would make for this geometry, as a list of dicts (host only; nothing is launched)."""
    out = (LcLaunch * max_out)()
    n = C.c_int32()
    _check("lc_plan_query", lib().lc_plan_query(C.byref(g), op, dtype, out, max_out, C.byref(n)))
    if n.value > max_out:
        return plan_query(g, op, dtype, n.value)
    return [{"kernel": out[i].kernel.decode(), "tparam": list(out[i].tparam), "arg": list(out[i].arg),
             "grid": tuple(out[i].grid), "block": int(out[i].block), "lds_bytes": int(out[i].lds_bytes)}
            for i in range(n.value)]


def l2pool_lcn_plan_query(shape, pool_ksize: int, pool_stride: int, lcn_ksize: int, gauss_sigma: float = 1.0):
    """The one-kernel launch of ``l2pool_lcn_fwd`` for a [B,H,W,C] map as a dict, or None where the call runs the
    two kernels one after the other (host only; nothing is launched)."""
    out = (LcLaunch * 1)()
    n = C.c_int32()
    B, H, W, Cc = shape
    _check("l2pool_lcn_plan_query", lib().l2pool_lcn_plan_query(B, H, W, Cc, pool_ksize, pool_stride, lcn_ksize,
                                                                gauss_sigma, out, 1, C.byref(n)))
    if n.value == 0:
        return None
    return {"kernel": out[0].kernel.decode(), "tparam": list(out[0].tparam), "arg": list(out[0].arg),
            "grid": tuple(out[0].grid), "block": int(out[0].block), "lds_bytes": int(out[0].lds_bytes)}


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: Optional[torch.Tensor], shape, dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def _op_dtype(dtype: int):
    return torch.float32 if dtype == LC_F32 else torch.bfloat16


def _ws(ws: Optional[torch.Tensor]):
    if ws is None:
        return None, 0
    return _dev(ws, None, ws.dtype, "ws"), ws.numel() * ws.element_size()


def lc_forward(g: LcGeom, x, w, bias, alpha: float, y, dtype: int = LC_F32, ws=None) -> None:
    LH, LW, K = geom_derive(g)
    dt = _op_dtype(dtype)
    wp, wb = _ws(ws)
    _check("lc_forward", lib().lc_forward(
        C.byref(g), _dev(x, (g.B, g.H, g.W, g.C), dt, "x"), _dev(w, (LH, LW, K, g.F), dt, "w"),
        _dev(bias, (LH, LW, g.F), torch.float32, "bias"), alpha, _dev(y, (g.B, LH, LW, g.F), torch.float32, "y"),
        dtype, wp, wb, _stream()))


def lc_forward_dev_scale(g: LcGeom, x, w, bias, alpha_dev, y, ws=None) -> None:
    LH, LW, K = geom_derive(g)
    wp, wb = _ws(ws)
    _check("lc_forward_dev_scale", lib().lc_forward_dev_scale(
        C.byref(g), _dev(x, (g.B, g.H, g.W, g.C), torch.float32, "x"), _dev(w, (LH, LW, K, g.F), torch.float32, "w"),
        _dev(bias, (LH, LW, g.F), torch.float32, "bias"), _dev(alpha_dev, None, torch.float32, "alpha_dev"),
        _dev(y, (g.B, LH, LW, g.F), torch.float32, "y"), wp, wb, _stream()))


def lc_backward_data(g: LcGeom, dy, w, dx, dtype: int = LC_F32, ws=None) -> None:
    LH, LW, K = geom_derive(g)
    dt = _op_dtype(dtype)
    wp, wb = _ws(ws)
    _check("lc_backward_data", lib().lc_backward_data(
        C.byref(g), _dev(dy, (g.B, LH, LW, g.F), dt, "dy"), _dev(w, (LH, LW, K, g.F), dt, "w"),
        _dev(dx, (g.B, g.H, g.W, g.C), torch.float32, "dx"), dtype, wp, wb, _stream()))


def lc_backward_weights(g: LcGeom, x, dy, beta: float, dw, dtype: int = LC_F32, ws=None) -> None:
    LH, LW, K = geom_derive(g)
    dt = _op_dtype(dtype)
    wp, wb = _ws(ws)
    _check("lc_backward_weights", lib().lc_backward_weights(
        C.byref(g), _dev(x, (g.B, g.H, g.W, g.C), dt, "x"), _dev(dy, (g.B, LH, LW, g.F), dt, "dy"), beta,
        _dev(dw, (LH, LW, K, g.F), torch.float32, "dw"), dtype, wp, wb, _stream()))


def _pool_out(H: int, ks: int, st: int) -> int:
    return (H - ks) // st + 1


def l2pool_fwd(x, y, ksize: int, stride: int, eps: float) -> None:
    B, H, W, Cc = x.shape
    _check("l2pool_fwd", lib().l2pool_fwd(
        _dev(x, None, torch.float32, "x"),
        _dev(y, (B, _pool_out(H, ksize, stride), _pool_out(W, ksize, stride), Cc), torch.float32, "y"),
        B, H, W, Cc, ksize, stride, eps, _stream()))


def l2pool_bwd(x, y, dy, dx, ksize: int, stride: int) -> None:
    B, H, W, Cc = x.shape
    oshape = (B, _pool_out(H, ksize, stride), _pool_out(W, ksize, stride), Cc)
    _check("l2pool_bwd", lib().l2pool_bwd(
        _dev(x, None, torch.float32, "x"), _dev(y, oshape, torch.float32, "y"), _dev(dy, oshape, torch.float32, "dy"),
        _dev(dx, x.shape, torch.float32, "dx"), B, H, W, Cc, ksize, stride, _stream()))


def lcn_fwd(x, y, mu, rstd, ksize: int, gauss_sigma: float, eps: float) -> None:
    B, H, W, Cc = x.shape
    _check("lcn_fwd", lib().lcn_fwd(
        _dev(x, None, torch.float32, "x"), _dev(y, x.shape, torch.float32, "y"),
        _dev(mu, (B, H, W), torch.float32, "mu"), _dev(rstd, (B, H, W), torch.float32, "rstd"),
        B, H, W, Cc, ksize, gauss_sigma, eps, _stream()))


def l2pool_lcn_fwd(x, p, y, mu, rstd, pool_ksize: int, pool_stride: int, pool_eps: float, lcn_ksize: int,
                   gauss_sigma: float, lcn_eps: float) -> None:
    B, H, W, Cc = x.shape
    Ho, Wo = _pool_out(H, pool_ksize, pool_stride), _pool_out(W, pool_ksize, pool_stride)
    _check("l2pool_lcn_fwd", lib().l2pool_lcn_fwd(
        _dev(x, None, torch.float32, "x"), _dev(p, (B, Ho, Wo, Cc), torch.float32, "p"),
        _dev(y, (B, Ho, Wo, Cc), torch.float32, "y"), _dev(mu, (B, Ho, Wo), torch.float32, "mu"),
        _dev(rstd, (B, Ho, Wo), torch.float32, "rstd"), B, H, W, Cc, pool_ksize, pool_stride, pool_eps, lcn_ksize,
        gauss_sigma, lcn_eps, _stream()))


def lcn_l2pool_bwd(x, p, mu, rstd, dy, scratch, dx, pool_ksize: int, pool_stride: int, lcn_ksize: int,
                   gauss_sigma: float) -> None:
    B, H, W, Cc = x.shape
    oshape = (B, _pool_out(H, pool_ksize, pool_stride), _pool_out(W, pool_ksize, pool_stride), Cc)
    _check("lcn_l2pool_bwd", lib().lcn_l2pool_bwd(
        _dev(x, None, torch.float32, "x"), _dev(p, oshape, torch.float32, "p"), _dev(mu, oshape[:3], torch.float32, "mu"),
        _dev(rstd, oshape[:3], torch.float32, "rstd"), _dev(dy, oshape, torch.float32, "dy"),
        _dev(scratch, oshape, torch.float32, "scratch"), _dev(dx, x.shape, torch.float32, "dx"),
        B, H, W, Cc, pool_ksize, pool_stride, lcn_ksize, gauss_sigma, _stream()))


def lcn_bwd(x, mu, rstd, dy, dx, ksize: int, gauss_sigma: float) -> None:
    B, H, W, Cc = x.shape
    _check("lcn_bwd", lib().lcn_bwd(
        _dev(x, None, torch.float32, "x"), _dev(mu, (B, H, W), torch.float32, "mu"),
        _dev(rstd, (B, H, W), torch.float32, "rstd"), _dev(dy, x.shape, torch.float32, "dy"),
        _dev(dx, x.shape, torch.float32, "dx"), B, H, W, Cc, ksize, gauss_sigma, _stream()))


LCN_PER_CHANNEL, LCN_ZERO_PAD, LCN_TWO_STAGE = 1, 2, 4


def lcn_variant_workspace_bytes(shape, flags: int) -> int:
    B, H, W, Cc = shape
    return int(lib().lcn_variant_workspace_bytes(B, H, W, Cc, flags))


def lcn_variant_fwd(x, y, mu, rstd, ksize: int, gauss_sigma: float, eps: float, flags: int) -> None:
    B, H, W, Cc = x.shape
    stat = (B, H, W, Cc) if flags & LCN_PER_CHANNEL else (B, H, W)
    _check("lcn_variant_fwd", lib().lcn_variant_fwd(
        _dev(x, None, torch.float32, "x"), _dev(y, x.shape, torch.float32, "y"),
        _dev(mu, stat, torch.float32, "mu"), _dev(rstd, stat, torch.float32, "rstd"),
        B, H, W, Cc, ksize, gauss_sigma, eps, flags, _stream()))


def lcn_variant_bwd(x, mu, rstd, dy, dx, ksize: int, gauss_sigma: float, flags: int, ws=None) -> None:
    B, H, W, Cc = x.shape
    stat = (B, H, W, Cc) if flags & LCN_PER_CHANNEL else (B, H, W)
    wp, wb = _ws(ws)
    _check("lcn_variant_bwd", lib().lcn_variant_bwd(
        _dev(x, None, torch.float32, "x"), _dev(mu, stat, torch.float32, "mu"),
        _dev(rstd, stat, torch.float32, "rstd"), _dev(dy, x.shape, torch.float32, "dy"),
        _dev(dx, x.shape, torch.float32, "dx"), B, H, W, Cc, ksize, gauss_sigma, flags, wp, wb, _stream()))


LCN_STATIC_SCRATCH_BYTES = 32 << 20


def lcn_variant_bwd_static(x, mu, rstd, dy, dx, ksize: int, gauss_sigma: float, flags: int) -> None:
    """`lcn_variant_bwd` with the library's own static scratch array (no workspace, no allocation)."""
    B, H, W, Cc = x.shape
    stat = (B, H, W, Cc) if flags & LCN_PER_CHANNEL else (B, H, W)
    _check("lcn_variant_bwd_static", lib().lcn_variant_bwd_static(
        _dev(x, None, torch.float32, "x"), _dev(mu, stat, torch.float32, "mu"),
        _dev(rstd, stat, torch.float32, "rstd"), _dev(dy, x.shape, torch.float32, "dy"),
        _dev(dx, x.shape, torch.float32, "dx"), B, H, W, Cc, ksize, gauss_sigma, flags, _stream()))


def sae_step(g: LcGeom, x, w, b, alpha, lam: float, eps_sparse: float, lr: float, flags: int, h_out, cost_out,
             ws) -> None:
    LH, LW, K = geom_derive(g)
    wp, wb = _ws(ws)
    _check("sae_step", lib().sae_step(
        C.byref(g), _dev(x, (g.B, g.H, g.W, g.C), torch.float32, "x"), _dev(w, (LH, LW, K, g.F), torch.float32, "w"),
        _dev(b, (g.H, g.W, g.C), torch.float32, "b"), _dev(alpha, None, torch.float32, "alpha"), lam, eps_sparse, lr,
        flags, _dev(h_out, (g.B, LH, LW, g.F), torch.float32, "h_out"),
        _dev(cost_out, None, torch.float32, "cost_out"), wp, wb, _stream()))
