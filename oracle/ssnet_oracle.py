"""numpy-facing wrapper of the CPU oracle (oracle/ssnet_oracle.c).

TEST INFRASTRUCTURE: argument marshalling only; all arithmetic is in the C
file.  Arrays are numpy uint64, C-contiguous; share tensors are [n, ...].
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = C.CDLL(_build.build_sanitized() if os.environ.get("SSNET_ORACLE_SANITIZED") == "1" else _build.build())

u64 = C.c_uint64
i64 = C.c_int64
sz = C.c_size_t
P = C.c_void_p

DOM_SHARE, DOM_RESHARE, DOM_ZERO, DOM_MASK_E, DOM_MASK_ALPHA, DOM_MASK_ALPHAT, DOM_TRUNC_GEN = range(1, 8)
DOM_MASK_BETA, DOM_BETA_GEN, DOM_BETAINV_GEN = 8, 9, 10


def _sig(name, res, *args):
    fn = getattr(_lib, name)
    fn.restype = res
    fn.argtypes = list(args)
    return fn


_add = _sig("orc_add", u64, u64, u64, u64)
_sub = _sig("orc_sub", u64, u64, u64, u64)
_mul = _sig("orc_mul", u64, u64, u64, u64)
_pow = _sig("orc_pow", u64, u64, u64, u64)
_inv = _sig("orc_inv", u64, u64, u64)
_lift = _sig("orc_lift", None, P, sz, u64, P)
_from_signed = _sig("orc_from_signed", u64, i64, u64)
_encode = _sig("orc_encode", sz, P, sz, C.c_int, u64, P)
_decode = _sig("orc_decode", None, P, sz, C.c_int, u64, P)
_mix64 = _sig("orc_mix64", u64, u64)
_key = _sig("orc_key", u64, u64, u64, u64, u64, u64)
_draw = _sig("orc_draw", u64, u64, u64)
_draw_field = _sig("orc_draw_field", u64, u64, u64, u64)
_draw_coeffs = _sig("orc_draw_coeffs", None, u64, u64, u64, u64, C.c_int, sz, P, u64, P)
_share_explicit = _sig("orc_share_explicit", None, P, P, sz, C.c_int, C.c_int, u64, P)
_share = _sig("orc_share", None, P, sz, P, C.c_int, C.c_int, u64, u64, u64, P)
_lagrange = _sig("orc_lagrange", None, P, C.c_int, u64, P)
_reconstruct = _sig("orc_reconstruct", None, P, sz, P, C.c_int, u64, P)
_linear = _sig("orc_linear", None, P, P, C.c_int, C.c_int, C.c_int, C.c_int, u64, P)
_linear_strict = _sig("orc_linear_strict", None, P, P, C.c_int, C.c_int, C.c_int, C.c_int, u64, P)
_conv = _sig("orc_conv", None, P, P, *([C.c_int] * 10), u64, P)
_conv_points = _sig("orc_conv_points", None, P, P, *([C.c_int] * 10), u64, P, sz, P)
_red_matrix = _sig("orc_red_matrix", C.c_int, C.c_int, C.c_int, u64, P)
_dr_explicit = _sig("orc_degree_reduce_explicit", C.c_int, P, P, P, sz, C.c_int, C.c_int, u64, P, P, P, P)
_dr = _sig("orc_degree_reduce", C.c_int, P, sz, P, C.c_int, C.c_int, u64, u64, u64, P, P, P, P)
_tr_explicit = _sig("orc_truncate_explicit", None, P, P, P, P, P, sz, C.c_int, C.c_int, C.c_int, u64, P, P, P)
_tr = _sig("orc_truncate", None, P, sz, P, C.c_int, C.c_int, C.c_int, u64, u64, u64, P, P, P)


def _a(x, dtype=np.uint64):
    return np.ascontiguousarray(x, dtype=dtype)


def _p(x):
    return None if x is None else x.ctypes.data_as(P)


# ---- field ----
def add(a, b, p): return int(_add(a, b, p))
def sub(a, b, p): return int(_sub(a, b, p))
def mul(a, b, p): return int(_mul(a, b, p))
def power(a, e, p): return int(_pow(a, e, p))
def inv(a, p): return int(_inv(a, p))
def from_signed(v, p): return int(_from_signed(v, p))


def lift(u, p):
    u = _a(u)
    out = np.empty(u.shape, dtype=np.int64)
    _lift(_p(u), u.size, p, _p(out))
    return out


def encode(x, f, p):
    x = _a(x, np.float64)
    out = np.empty(x.shape, dtype=np.uint64)
    bad = _encode(_p(x), x.size, f, p, _p(out))
    if bad:
        raise ValueError(f"{bad} values exceed 2^40 after scaling")
    return out


def decode(u, s, p):
    u = _a(u)
    out = np.empty(u.shape, dtype=np.float64)
    _decode(_p(u), u.size, s, p, _p(out))
    return out


# ---- generator ----
def mix64(z): return int(_mix64(z))
def key(seed, domain, stream_id, party, j): return int(_key(seed, domain, stream_id, party, j))
def draw(k, e): return int(_draw(k, e))
def draw_field(k, e, p): return int(_draw_field(k, e, p))


def draw_coeffs(seed, domain, stream_id, party, degree, count, p, eidx=None):
    coef = np.empty((max(degree, 0), count), dtype=np.uint64)
    eidx = None if eidx is None else _a(eidx)
    _draw_coeffs(seed, domain, stream_id, party, degree, count, _p(eidx), p, _p(coef))
    return coef


# ---- GEN / REC ----
def share_explicit(secret, coef, n, degree, p):
    secret = _a(secret)
    coef = _a(coef).reshape(degree, secret.size) if degree else np.zeros((0, secret.size), np.uint64)
    out = np.empty((n,) + secret.shape, dtype=np.uint64)
    _share_explicit(_p(secret), _p(coef), secret.size, n, degree, p, _p(out))
    return out


def share(secret, n, degree, p, seed, stream_id, eidx=None):
    secret = _a(secret)
    eidx = None if eidx is None else _a(eidx)
    out = np.empty((n,) + secret.shape, dtype=np.uint64)
    _share(_p(secret), secret.size, _p(eidx), n, degree, p, seed, stream_id, _p(out))
    return out


def lagrange(ids, p):
    ids = _a(ids, np.int32)
    lam = np.empty(ids.size, dtype=np.uint64)
    _lagrange(_p(ids), ids.size, p, _p(lam))
    return lam


def reconstruct(shares, ids, p):
    shares = _a(shares)
    ids = _a(ids, np.int32)
    count = shares[0].size
    out = np.empty(shares.shape[1:], dtype=np.uint64)
    _reconstruct(_p(shares), count, _p(ids), ids.size, p, _p(out))
    return out


# ---- linear layers ----
def linear(x, w, p, strict=False):
    x, w = _a(x), _a(w)
    n, M, K = x.shape
    n2, K2, N = w.shape
    assert n == n2 and K == K2
    y = np.empty((n, M, N), dtype=np.uint64)
    (_linear_strict if strict else _linear)(_p(x), _p(w), n, M, K, N, p, _p(y))
    return y


def conv_out(H, k, stride, pad):
    return (H + 2 * pad - k) // stride + 1


def conv(x, w, stride, pad, p):
    x, w = _a(x), _a(w)
    n, B, Ci, H, W = x.shape
    n2, Co, Ci2, kh, kw = w.shape
    assert n == n2 and Ci == Ci2
    y = np.empty((n, B, Co, conv_out(H, kh, stride, pad), conv_out(W, kw, stride, pad)), dtype=np.uint64)
    _conv(_p(x), _p(w), n, B, Ci, H, W, Co, kh, kw, stride, pad, p, _p(y))
    return y


def conv_points(x, w, stride, pad, p, flat):
    x, w, flat = _a(x), _a(w), _a(flat)
    n, B, Ci, H, W = x.shape
    n2, Co, Ci2, kh, kw = w.shape
    assert n == n2 and Ci == Ci2
    out = np.empty(flat.size, dtype=np.uint64)
    _conv_points(_p(x), _p(w), n, B, Ci, H, W, Co, kh, kw, stride, pad, p, _p(flat), flat.size, _p(out))
    return out


# ---- RED / RERAND ----
def red_matrix(n, t, p):
    R = np.empty((2 * t + 1, n), dtype=np.uint64)
    rc = _red_matrix(n, t, p, _p(R))
    if rc:
        raise ValueError(f"orc_red_matrix failed: {rc}")
    return R


def degree_reduce_explicit(c, rcoef, zcoef, n, t, p, full=False):
    c, rcoef, zcoef = _a(c), _a(rcoef), _a(zcoef)
    count = c[0].size
    k, nr = t + 1, 2 * t + 1
    msg1 = np.empty((nr, k, count), np.uint64)
    msg2 = np.empty((k, n, count), np.uint64)
    red = np.empty((n, count), np.uint64)
    out = np.empty((n,) + c.shape[1:], np.uint64)
    rc = _dr_explicit(_p(c), _p(rcoef), _p(zcoef), count, n, t, p, _p(msg1), _p(msg2), _p(red), _p(out))
    if rc:
        raise ValueError(f"orc_degree_reduce_explicit failed: {rc}")
    return (out, msg1, msg2, red) if full else out


def degree_reduce(c, n, t, p, seed, stream_id, eidx=None, full=False):
    c = _a(c)
    eidx = None if eidx is None else _a(eidx)
    count = c[0].size
    k, nr = t + 1, 2 * t + 1
    msg1 = np.empty((nr, k, count), np.uint64) if full else None
    msg2 = np.empty((k, n, count), np.uint64) if full else None
    red = np.empty((n, count), np.uint64) if full else None
    out = np.empty((n,) + c.shape[1:], np.uint64)
    rc = _dr(_p(c), count, _p(eidx), n, t, p, seed, stream_id, _p(msg1), _p(msg2), _p(red), _p(out))
    if rc:
        raise ValueError(f"orc_degree_reduce failed: {rc}")
    return (out, msg1, msg2, red) if full else out


# ---- truncation ----
def truncate_explicit(x, evals, ca, cat, cw, n, t, f, p, full=False):
    x, evals, ca, cat, cw = _a(x), _a(evals), _a(ca), _a(cat), _a(cw)
    count = x[0].size
    u = np.empty((t + 1, count), np.uint64)
    wsh = np.empty((n, count), np.uint64)
    out = np.empty((n,) + x.shape[1:], np.uint64)
    _tr_explicit(_p(x), _p(evals), _p(ca), _p(cat), _p(cw), count, n, t, f, p, _p(u), _p(wsh), _p(out))
    return (out, u, wsh) if full else out


def truncate(x, n, t, f, p, seed, stream_id, eidx=None, full=False):
    x = _a(x)
    eidx = None if eidx is None else _a(eidx)
    count = x[0].size
    u = np.empty((t + 1, count), np.uint64) if full else None
    wsh = np.empty((n, count), np.uint64) if full else None
    out = np.empty((n,) + x.shape[1:], np.uint64)
    _tr(_p(x), count, _p(eidx), n, t, f, p, seed, stream_id, _p(u), _p(wsh), _p(out))
    return (out, u, wsh) if full else out


# ---- SSS-NonLinear (ReLU) ----
_nlm_explicit = _sig("orc_nonlinear_masks_explicit", None, P, P, P, sz, C.c_int, C.c_int, u64, P, P)
_nlm = _sig("orc_nonlinear_masks", None, sz, P, C.c_int, C.c_int, C.c_int, u64, u64, u64, P, P)
_relu = _sig("orc_relu", None, P, P, P, sz, C.c_int, C.c_int, u64, P, P, P)


def nonlinear_masks_explicit(beta, cb, cbi, n, t, p):
    """-> (shares of beta, shares of beta^-1), each [n, count]"""
    beta, cb, cbi = _a(beta), _a(cb), _a(cbi)
    count = beta.size
    sb, sbi = np.empty((n, count), np.uint64), np.empty((n, count), np.uint64)
    _nlm_explicit(_p(beta), _p(cb), _p(cbi), count, n, t, p, _p(sb), _p(sbi))
    return sb, sbi


def nonlinear_masks(count, n, t, bbits, p, seed, stream_id, eidx=None):
    eidx = None if eidx is None else _a(eidx)
    sb, sbi = np.empty((n, count), np.uint64), np.empty((n, count), np.uint64)
    _nlm(count, _p(eidx), n, t, bbits, p, seed, stream_id, _p(sb), _p(sbi))
    return sb, sbi


def relu(x, sh_b, sh_bi, n, t, p, full=False):
    """-> out [n, ...] (and with full: the 2t+1 masked products and the elite party's plain result)"""
    x, sh_b, sh_bi = _a(x), _a(sh_b), _a(sh_bi)
    count = x[0].size
    msg = np.empty((2 * t + 1, count), np.uint64) if full else None
    y = np.empty(count, np.uint64) if full else None
    out = np.empty(x.shape, np.uint64)
    _relu(_p(x), _p(sh_b), _p(sh_bi), count, n, t, p, _p(msg), _p(y), _p(out))
    return (out, msg, y) if full else out


# ---- truncation with the rounding division of an average pooling (Sec. VI-C, App. C) ----
_trd_explicit = _sig("orc_truncate_div_explicit", None, P, P, P, P, P, sz, C.c_int, C.c_int, C.c_int, C.c_int, u64,
                     P, P, P)
_trd = _sig("orc_truncate_div", None, P, sz, P, C.c_int, C.c_int, C.c_int, C.c_int, u64, u64, u64, P, P, P)


def truncate_div_explicit(x, evals, ca, cat, cw, n, t, f, kdiv, p, full=False):
    x, evals, ca, cat, cw = _a(x), _a(evals), _a(ca), _a(cat), _a(cw)
    count = x[0].size
    u = np.empty((t + 1, count), np.uint64)
    wsh = np.empty((n, count), np.uint64)
    out = np.empty((n,) + x.shape[1:], np.uint64)
    _trd_explicit(_p(x), _p(evals), _p(ca), _p(cat), _p(cw), count, n, t, f, kdiv, p, _p(u), _p(wsh), _p(out))
    return (out, u, wsh) if full else out


def truncate_div(x, n, t, f, kdiv, p, seed, stream_id, eidx=None, full=False):
    x = _a(x)
    eidx = None if eidx is None else _a(eidx)
    count = x[0].size
    u = np.empty((t + 1, count), np.uint64) if full else None
    wsh = np.empty((n, count), np.uint64) if full else None
    out = np.empty((n,) + x.shape[1:], np.uint64)
    _trd(_p(x), count, _p(eidx), n, t, f, kdiv, p, seed, stream_id, _p(u), _p(wsh), _p(out))
    return (out, u, wsh) if full else out


# ---- SSS-NonLinear with pooling ----
_pool_out = _sig("orc_pool_out_size", C.c_int, C.c_int, C.c_int, C.c_int, C.c_int)
_pool_masks = _sig("orc_pool_masks", None, sz, *([C.c_int] * 8), C.c_int, C.c_int, C.c_int, u64, u64, u64, P, P)
_relu_pool = _sig("orc_relu_pool", None, P, P, P, sz, *([C.c_int] * 8), C.c_int, C.c_int, C.c_int, u64, P, P, P)

POOL_MAX, POOL_SUM = 0, 1


def pool_out_size(H, k, s, pad):
    return _pool_out(H, k, s, pad)


def pool_masks(planes, H, W, kh, kw, sh, sw, ph, pw, n, t, bbits, p, seed, stream_id):
    """-> (shares of beta [n, planes*H*W], shares of beta^-1 [n, planes*Ho*Wo])"""
    Ho, Wo = _pool_out(H, kh, sh, ph), _pool_out(W, kw, sw, pw)
    sb, sbi = np.empty((n, planes * H * W), np.uint64), np.empty((n, planes * Ho * Wo), np.uint64)
    _pool_masks(planes, H, W, kh, kw, sh, sw, ph, pw, n, t, bbits, p, seed, stream_id, _p(sb), _p(sbi))
    return sb, sbi


def relu_pool(x, sh_b, sh_bi, planes, H, W, kh, kw, sh, sw, ph, pw, mode, n, t, p, full=False):
    """x [n, planes*H*W] -> out [n, planes*Ho*Wo] (with full: the masked products and the plain result)"""
    x, sh_b, sh_bi = _a(x), _a(sh_b), _a(sh_bi)
    Ho, Wo = _pool_out(H, kh, sh, ph), _pool_out(W, kw, sw, pw)
    cin, cout = planes * H * W, planes * Ho * Wo
    assert x.size == n * cin and sh_b.size == n * cin and sh_bi.size == n * cout
    msg = np.empty((2 * t + 1, cin), np.uint64) if full else None
    y = np.empty(cout, np.uint64) if full else None
    out = np.empty((n, cout), np.uint64)
    _relu_pool(_p(x), _p(sh_b), _p(sh_bi), planes, H, W, kh, kw, sh, sw, ph, pw, mode, n, t, p, _p(msg), _p(y), _p(out))
    return (out, msg, y) if full else out
