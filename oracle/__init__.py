"""ctypes binding of the CPU oracle (oracle/distr_attn_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package; the GPU library never does. Arrays are numpy, host memory: float32 in,
float64 out. Function names mirror the C entry points.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdistr_attn_oracle.so")
_lib = None


class OracleParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int), ("H", ctypes.c_int), ("Hkv", ctypes.c_int), ("N", ctypes.c_int),
        ("d", ctypes.c_int), ("Br", ctypes.c_int), ("n_groups", ctypes.c_int),
        ("causal", ctypes.c_int), ("n_planes", ctypes.c_int), ("gray_mode", ctypes.c_int),
        ("lsh_seed", ctypes.c_uint64), ("scale", ctypes.c_double),
        ("Nk", ctypes.c_int), ("side", ctypes.c_int), ("Bc", ctypes.c_int),
    ]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.oracle_gray_hash.restype = ctypes.c_uint32
        _lib.oracle_gray_hash.argtypes = [ctypes.c_uint32, ctypes.c_int, ctypes.c_int]
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _ptr(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype)) if a is not None else None


def params(B, H, Hkv, N, d, Br, n_groups, causal=False, n_planes=16, gray_mode=0, lsh_seed=0,
           scale=None, Nk=None, side=0, Bc=64):
    """Nk: keys per head (default N); side 1: the mirrored form (sample K, fuse Q, one grouping
    per K block of Bc rows)."""
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    return OracleParams(B, H, Hkv, N, d, Br, n_groups, int(bool(causal)), n_planes, gray_mode,
                        lsh_seed, float(scale), 0 if Nk is None else Nk, side, Bc)


def n_keys(p):
    return p.Nk if p.Nk > 0 else p.N


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name} returned {rc}")


def num_threads():
    return lib().oracle_num_threads()


def hyperplanes(seed, n_planes, Br):
    R = np.empty((n_planes, Br), dtype=np.float32)
    _check(lib().oracle_hyperplanes(ctypes.c_uint64(seed), n_planes, Br, _ptr(R, ctypes.c_float)),
           "oracle_hyperplanes")
    return R


def gray_hash(code, n_planes, gray_mode):
    return int(lib().oracle_gray_hash(code, n_planes, gray_mode))


def sort_channels(hashes):
    h = np.ascontiguousarray(hashes, dtype=np.uint32)
    perm = np.empty(h.shape[0], dtype=np.uint8)
    _check(lib().oracle_sort_channels(_ptr(h, ctypes.c_uint32), h.shape[0], _ptr(perm, ctypes.c_uint8)),
           "oracle_sort_channels")
    return perm


def lsh_group(q, p, R=None, want_proj=False):
    """-> (hash uint32 [B,H,Tq,d], perm uint8 [B,H,Tq,d], proj float32 [B,H,Tq,d,P] or None)."""
    q, qp = _f32(q)
    if R is None:
        R = hyperplanes(p.lsh_seed, p.n_planes, p.Br)
    R, Rp = _f32(R)
    Tq = (p.N + p.Br - 1) // p.Br
    hash_ = np.empty((p.B, p.H, Tq, p.d), dtype=np.uint32)
    perm = np.empty((p.B, p.H, Tq, p.d), dtype=np.uint8)
    proj = np.empty((p.B, p.H, Tq, p.d, p.n_planes), dtype=np.float32) if want_proj else None
    _check(lib().oracle_lsh_group(qp, ctypes.byref(p), Rp, _ptr(hash_, ctypes.c_uint32),
                                  _ptr(perm, ctypes.c_uint8), _ptr(proj, ctypes.c_float)),
           "oracle_lsh_group")
    return hash_, perm, proj


def exact_fwd(q, k, v, p):
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    o = np.zeros((p.B, p.H, p.N, p.d), dtype=np.float64)
    _check(lib().oracle_exact_fwd(qp, kp, vp, _ptr(o, ctypes.c_double), ctypes.byref(p)),
           "oracle_exact_fwd")
    return o


def distr_fwd(q, k, v, p, R=None, perm=None):
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    Rp = None
    if R is not None:
        R, Rp = _f32(R)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.uint8)
    o = np.zeros((p.B, p.H, p.N, p.d), dtype=np.float64)
    _check(lib().oracle_distr_fwd(qp, kp, vp, _ptr(o, ctypes.c_double), ctypes.byref(p), Rp,
                                  _ptr(perm, ctypes.c_uint8)), "oracle_distr_fwd")
    return o


def _tiles(tiles):
    t = np.ascontiguousarray(tiles, dtype=np.int32).reshape(-1, 3)
    return t, t.ctypes.data_as(ctypes.POINTER(ctypes.c_int))


def exact_fwd_tiles(q, k, v, p, tiles):
    """tiles: [(b, h, t), ...] -> float64 [n_tiles, Br, d] (rows past N stay NaN)."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    t, tp = _tiles(tiles)
    o = np.full((t.shape[0], p.Br, p.d), np.nan, dtype=np.float64)
    _check(lib().oracle_exact_fwd_tiles(qp, kp, vp, _ptr(o, ctypes.c_double), ctypes.byref(p), tp,
                                        t.shape[0]), "oracle_exact_fwd_tiles")
    return o


def distr_fwd_tiles(q, k, v, p, tiles, R=None, perm=None):
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    t, tp = _tiles(tiles)
    Rp = None
    if R is not None:
        R, Rp = _f32(R)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.uint8)
    o = np.full((t.shape[0], p.Br, p.d), np.nan, dtype=np.float64)
    _check(lib().oracle_distr_fwd_tiles(qp, kp, vp, _ptr(o, ctypes.c_double), ctypes.byref(p), Rp,
                                        _ptr(perm, ctypes.c_uint8), tp, t.shape[0]),
           "oracle_distr_fwd_tiles")
    return o


def scores(q, k, p, b=0, h=0, R=None, perm=None, want_exact=True, want_hat=True):
    """-> (s_hat [N,Nk] or None, s [N,Nk] or None): scaled, unmasked score matrices of one head."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    Rp = None
    if R is not None:
        R, Rp = _f32(R)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.uint8)
    s_hat = np.zeros((p.N, n_keys(p)), dtype=np.float64) if want_hat else None
    s = np.zeros((p.N, n_keys(p)), dtype=np.float64) if want_exact else None
    _check(lib().oracle_scores(qp, kp, _ptr(s_hat, ctypes.c_double), _ptr(s, ctypes.c_double),
                               ctypes.byref(p), Rp, _ptr(perm, ctypes.c_uint8), b, h),
           "oracle_scores")
    return s_hat, s


def lse(q, k, p, distr=True, R=None, perm=None):
    """-> float64 [B,H,N]: log-sum-exp of every row's visible scores (S^ if distr else S)."""
    q, qp = _f32(q)
    k, kp = _f32(k)
    Rp = None
    if R is not None:
        R, Rp = _f32(R)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.uint8)
    out = np.zeros((p.B, p.H, p.N), dtype=np.float64)
    _check(lib().oracle_lse(qp, kp, _ptr(out, ctypes.c_double), ctypes.byref(p), Rp,
                            _ptr(perm, ctypes.c_uint8), int(bool(distr))), "oracle_lse")
    return out


def _bwd(name, q, k, v, dout, p, extra):
    q, qp = _f32(q)
    k, kp = _f32(k)
    v, vp = _f32(v)
    dout, dop = _f32(dout)
    dq = np.zeros((p.B, p.H, p.N, p.d), dtype=np.float64)
    dk = np.zeros((p.B, p.Hkv, n_keys(p), p.d), dtype=np.float64)
    dv = np.zeros_like(dk)
    _check(getattr(lib(), name)(qp, kp, vp, dop, _ptr(dq, ctypes.c_double), _ptr(dk, ctypes.c_double),
                                _ptr(dv, ctypes.c_double), ctypes.byref(p), *extra), name)
    return dq, dk, dv


def exact_bwd(q, k, v, dout, p):
    """-> (dq, dk, dv) float64: gradient of sum(dout * exact_fwd) (Sec. 2.1)."""
    return _bwd("oracle_exact_bwd", q, k, v, dout, p, ())


def distr_bwd(q, k, v, dout, p, R=None, perm=None):
    """-> (dq, dk, dv) float64: gradient of sum(dout * distr_fwd) with the grouping held fixed."""
    Rp = None
    if R is not None:
        R, Rp = _f32(R)
    if perm is not None:
        perm = np.ascontiguousarray(perm, dtype=np.uint8)
    return _bwd("oracle_distr_bwd", q, k, v, dout, p, (Rp, _ptr(perm, ctypes.c_uint8)))
