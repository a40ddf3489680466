"""fp64 CPU oracle: Python face of ``lc_oracle.c``.

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product path never does.  The
arithmetic lives in ``lc_oracle.c`` (plain loops, double precision); this file
only compiles it with gcc and marshals numpy arrays.  Inputs may be fp32 or
fp64 arrays; they are up-cast to fp64 unchanged, and every result is fp64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "lc_oracle.c"
_LIB = _HERE / "liblc_oracle.so"
_lib = None

_D = C.POINTER(C.c_double)
_Fp = C.POINTER(C.c_float)


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (-O2, OpenMP)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               str(_SRC), "-o", str(_LIB), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(str(_LIB))
        _lib.orc_sae_cost.restype = C.c_double
        _lib.orc_sae_grad.restype = C.c_double
        _lib.orc_sae_step.restype = C.c_double
        _lib.orc_lc_forward_at.restype = C.c_double
        _lib.orc_lc_backward_data_at.restype = C.c_double
        _lib.orc_lc_backward_weights_at.restype = C.c_double
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(_D)


def _f(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32
    return a


def _fp(a: np.ndarray):
    return a.ctypes.data_as(_Fp)


def _geom(g):
    B, H, W, Cc, R, S, F = g
    return [C.c_int(int(v)) for v in (B, H, W, Cc, R, S, F)]


def n_loc(H: int, R: int, S: int) -> int:
    return (H - R) // S + 1


def lc_forward(g, x, w, bias=None, alpha=1.0):
    B, H, W, Cc, R, S, F = g
    LH, LW = n_loc(H, R, S), n_loc(W, R, S)
    x, w = _d(x), _d(w)
    assert x.size == B * H * W * Cc and w.size == LH * LW * R * R * Cc * F
    y = np.empty((B, LH, LW, F))
    bp = None
    if bias is not None:
        bias = _d(bias)
        assert bias.size == LH * LW * F
        bp = _p(bias)
    _load().orc_lc_forward(*_geom(g), _p(x), _p(w), bp, C.c_double(alpha), _p(y))
    return y


def lc_backward_data(g, dy, w):
    B, H, W, Cc, R, S, F = g
    LH, LW = n_loc(H, R, S), n_loc(W, R, S)
    dy, w = _d(dy), _d(w)
    assert dy.size == B * LH * LW * F and w.size == LH * LW * R * R * Cc * F
    dx = np.empty((B, H, W, Cc))
    _load().orc_lc_backward_data(*_geom(g), _p(dy), _p(w), _p(dx))
    return dx


def lc_backward_weights(g, x, dy, beta=0.0, dw=None):
    B, H, W, Cc, R, S, F = g
    LH, LW = n_loc(H, R, S), n_loc(W, R, S)
    x, dy = _d(x), _d(dy)
    assert x.size == B * H * W * Cc and dy.size == B * LH * LW * F
    out = np.zeros((LH, LW, R * R * Cc, F)) if dw is None else _d(dw).reshape(LH, LW, R * R * Cc, F).copy()
    _load().orc_lc_backward_weights(*_geom(g), _p(x), _p(dy), C.c_double(beta), _p(out))
    return out


def l2pool_fwd(x, ks=3, st=1, eps=1e-6):
    x = _d(x)
    B, H, W, Cc = x.shape
    y = np.empty((B, n_loc(H, ks, st), n_loc(W, ks, st), Cc))
    _load().orc_l2pool_fwd(C.c_int(B), C.c_int(H), C.c_int(W), C.c_int(Cc), C.c_int(ks), C.c_int(st),
                           C.c_double(eps), _p(x), _p(y))
    return y


def l2pool_bwd(x, y, dy, ks=3, st=1):
    x, y, dy = _d(x), _d(y), _d(dy)
    B, H, W, Cc = x.shape
    assert y.shape == dy.shape == (B, n_loc(H, ks, st), n_loc(W, ks, st), Cc)
    dx = np.empty_like(x)
    _load().orc_l2pool_bwd(C.c_int(B), C.c_int(H), C.c_int(W), C.c_int(Cc), C.c_int(ks), C.c_int(st),
                           _p(x), _p(y), _p(dy), _p(dx))
    return dx


def lcn_fwd(x, ks=5, sigma=1.0, eps=1e-4):
    x = _d(x)
    B, H, W, Cc = x.shape
    assert ks % 2 == 1 and ks <= 63
    y = np.empty_like(x)
    mu = np.empty((B, H, W))
    rstd = np.empty((B, H, W))
    _load().orc_lcn_fwd(C.c_int(B), C.c_int(H), C.c_int(W), C.c_int(Cc), C.c_int(ks), C.c_double(sigma),
                        C.c_double(eps), _p(x), _p(y), _p(mu), _p(rstd))
    return y, mu, rstd


def lcn_bwd(x, mu, rstd, dy, ks=5, sigma=1.0):
    x, mu, rstd, dy = _d(x), _d(mu), _d(rstd), _d(dy)
    B, H, W, Cc = x.shape
    assert mu.shape == rstd.shape == (B, H, W) and dy.shape == x.shape
    dx = np.empty_like(x)
    _load().orc_lcn_bwd(C.c_int(B), C.c_int(H), C.c_int(W), C.c_int(Cc), C.c_int(ks), C.c_double(sigma),
                        _p(x), _p(mu), _p(rstd), _p(dy), _p(dx))
    return dx


LCN_PER_CHANNEL, LCN_ZERO_PAD, LCN_TWO_STAGE = 1, 2, 4


def lcn_var_fwd(x, ks=5, sigma=1.0, eps=1e-4, flags=0):
    """LCN variants (flags: 1 per-channel statistics, 2 zero-padded borders, 4 two stages)."""
    x = _d(x)
    B, H, W, Cc = x.shape
    assert ks % 2 == 1 and ks <= 63 and 0 <= flags < 8
    stat = (B, H, W, Cc) if flags & LCN_PER_CHANNEL else (B, H, W)
    y, mu, rstd = np.empty_like(x), np.empty(stat), np.empty(stat)
    _load().orc_lcn_var_fwd(C.c_int(B), C.c_int(H), C.c_int(W), C.c_int(Cc), C.c_int(ks), C.c_double(sigma),
                            C.c_double(eps), C.c_uint(flags), _p(x), _p(y), _p(mu), _p(rstd))
    return y, mu, rstd


def lcn_var_bwd(x, mu, rstd, dy, ks=5, sigma=1.0, flags=0):
    x, mu, rstd, dy = _d(x), _d(mu), _d(rstd), _d(dy)
    B, H, W, Cc = x.shape
    stat = (B, H, W, Cc) if flags & LCN_PER_CHANNEL else (B, H, W)
    assert mu.shape == rstd.shape == stat and dy.shape == x.shape and 0 <= flags < 8
    dx = np.empty_like(x)
    _load().orc_lcn_var_bwd(C.c_int(B), C.c_int(H), C.c_int(W), C.c_int(Cc), C.c_int(ks), C.c_double(sigma),
                            C.c_uint(flags), _p(x), _p(mu), _p(rstd), _p(dy), _p(dx))
    return dx


def sae_cost(g, x, w, b, alpha=1.0, lam=0.1, eps_s=1e-6):
    B, H, W, Cc, R, S, F = g
    LH, LW = n_loc(H, R, S), n_loc(W, R, S)
    x, w, b = _d(x), _d(w), _d(b)
    assert b.size == H * W * Cc
    h = np.empty((B, LH, LW, F))
    r = np.empty((B, H, W, Cc))
    J = _load().orc_sae_cost(*_geom(g), _p(x), _p(w), _p(b), C.c_double(alpha), C.c_double(lam),
                             C.c_double(eps_s), _p(h), _p(r))
    return float(J), h, r


def sae_grad(g, x, w, b, alpha=1.0, lam=0.1, eps_s=1e-6):
    B, H, W, Cc, R, S, F = g
    LH, LW = n_loc(H, R, S), n_loc(W, R, S)
    x, w, b = _d(x), _d(w), _d(b)
    dw = np.empty((LH, LW, R * R * Cc, F))
    db = np.empty((H, W, Cc))
    da = C.c_double(0.0)
    h = np.empty((B, LH, LW, F))
    J = _load().orc_sae_grad(*_geom(g), _p(x), _p(w), _p(b), C.c_double(alpha), C.c_double(lam),
                             C.c_double(eps_s), _p(dw), _p(db), C.byref(da), _p(h))
    return float(J), dw, db, float(da.value), h


def sae_step(g, x, w, b, alpha=1.0, lam=0.1, eps_s=1e-6, lr=1e-3, flags=0):
    """Returns (J, w_new, b_new, alpha_new, h) and leaves its inputs untouched."""
    B, H, W, Cc, R, S, F = g
    LH, LW = n_loc(H, R, S), n_loc(W, R, S)
    x = _d(x)
    w = _d(w).copy().reshape(LH, LW, R * R * Cc, F)
    b = _d(b).copy().reshape(H, W, Cc)
    a = C.c_double(alpha)
    h = np.empty((B, LH, LW, F))
    J = _load().orc_sae_step(*_geom(g), _p(x), _p(w), _p(b), C.byref(a), C.c_double(lam), C.c_double(eps_s),
                             C.c_double(lr), C.c_uint(flags), _p(h))
    return float(J), w, b, float(a.value), h


def sae_step_one_field(g, x, w, b, alpha=1.0, lam=0.1, eps_s=1e-6, lr=1e-3, flags=0):
    """`sae_step` for a layer of ONE field that covers its whole input (R = H = W: the dense last layer of
    Sec. 3.1).  There `W x` of Eq. 1 is a plain matrix product, so the same steps, in the same order as the C
    oracle takes them, are written with numpy's fp64 matmul, which makes the paper-sized layer (92,256 x 4096
    weights) affordable.  Returns (J, w_new, b_new, alpha_new, h) like `sae_step`."""
    B, H, W, Cc, R, S, F = g
    if not (R == H == W):
        raise ValueError("one field covering the whole input is required")
    K = R * R * Cc
    X = _d(x).reshape(B, K)
    Wm = _d(w).reshape(K, F)
    a = X @ Wm                                    # W x
    h = alpha * a
    r = h @ Wm.T + _d(b).reshape(1, K) - X        # W^T h + b - x
    s = np.sqrt(h * h + eps_s)
    J = (np.sum(r * r) + lam * np.sum(s)) / B
    u = (2.0 / B) * r
    db = u.sum(axis=0)
    gh = u @ Wm + (lam / B) * h / s               # dJ/dh
    da = np.sum(a * gh)
    dW = u.T @ h + X.T @ (alpha * gh)             # decoder path + encoder path of the tied weights
    Wn = Wm - lr * dW
    bn = _d(b).reshape(K) - lr * db
    an = alpha - lr * da if flags & 2 else alpha
    if flags & 1:
        n2 = np.sum(Wn * Wn, axis=0)
        Wn = Wn * np.where(n2 > 0.0, 1.0 / np.sqrt(np.where(n2 > 0.0, n2, 1.0)), 0.0)[None, :]
    return float(J), Wn.reshape(1, 1, K, F), bn.reshape(H, W, Cc), float(an), h.reshape(B, 1, 1, F)


def lc_forward_at(g, x, w, bias, alpha, b, i, j, f):
    x, w = _f(x), _f(w)
    bp = None
    if bias is not None:
        bias = _f(bias)
        bp = _fp(bias)
    return float(_load().orc_lc_forward_at(*_geom(g), _fp(x), _fp(w), bp, C.c_double(alpha),
                                           C.c_int(b), C.c_int(i), C.c_int(j), C.c_int(f)))


def lc_backward_data_at(g, dy, w, b, row, col, c):
    dy, w = _f(dy), _f(w)
    return float(_load().orc_lc_backward_data_at(*_geom(g), _fp(dy), _fp(w), C.c_int(b), C.c_int(row),
                                                 C.c_int(col), C.c_int(c)))


def lc_backward_weights_at(g, x, dy, i, j, k, f):
    x, dy = _f(x), _f(dy)
    return float(_load().orc_lc_backward_weights_at(*_geom(g), _fp(x), _fp(dy), C.c_int(i), C.c_int(j),
                                                    C.c_int(k), C.c_int(f)))
