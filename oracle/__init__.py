"""ctypes loader for the CPU oracle (oracle/signvote_oracle.c, oracle/qsgd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  Nothing under paper_1810_05291_amd/ imports this, and
this module imports nothing from there.  The functions below only marshal numpy
arrays into the C calls; all arithmetic is in the C file.

bf16 arrays are numpy uint16 arrays holding the bf16 bit patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

F32 = 0
BF16 = 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        _lib.ora_version.restype = ctypes.c_int
        _lib.ora_max_threads.restype = ctypes.c_int
        _lib.ora_qsgd_norm_f64.restype = ctypes.c_double
    return _lib


def max_threads() -> int:
    return int(lib().ora_max_threads())


def set_threads(n: int) -> None:
    lib().ora_set_threads(ctypes.c_int(int(n)))


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i64(x):
    return ctypes.c_int64(int(x))


def _f(x):
    return ctypes.c_float(float(x))


def _chk(a, dtype):
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a


def _dt_of(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(a.dtype)


def words_for(d: int) -> int:
    return (int(d) + 63) // 64


# ---- elementary steps -------------------------------------------------------------

def bf16_to_f32(h):
    h = _chk(np.ascontiguousarray(h), np.uint16)
    out = np.empty(h.shape, np.float32)
    lib().ora_bf16_to_f32(_p(h), _i64(h.size), _p(out))
    return out


def f32_to_bf16(x):
    x = _chk(np.ascontiguousarray(x), np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().ora_f32_to_bf16(_p(x), _i64(x.size), _p(out))
    return out


def sign_f32(x):
    x = _chk(np.ascontiguousarray(x), np.float32)
    s = np.empty(x.shape, np.int8)
    lib().ora_sign_f32(_p(x), _i64(x.size), _p(s))
    return s


def pack_signs(s):
    s = _chk(np.ascontiguousarray(s), np.int8)
    assert s.ndim == 1
    w = np.empty(words_for(s.size), np.uint64)
    lib().ora_pack_signs(_p(s), _i64(s.size), _p(w))
    return w


def unpack_signs(words, d):
    words = _chk(np.ascontiguousarray(words), np.uint64)
    assert words.size >= words_for(d)
    s = np.empty(int(d), np.int8)
    lib().ora_unpack_signs(_p(words), _i64(d), _p(s))
    return s


def momentum_f32(g, v, beta):
    """In place on v (fp32)."""
    _chk(g, np.float32), _chk(v, np.float32)
    assert g.size == v.size
    lib().ora_momentum_f32(_p(g), _p(v), _i64(g.size), _f(beta))
    return v


def momentum_f64(g, v, beta):
    _chk(g, np.float32), _chk(v, np.float32)
    out = np.empty(g.shape, np.float64)
    lib().ora_momentum_f64(_p(g), _p(v), _i64(g.size), _f(beta), _p(out))
    return out


def vote_sum(s):
    """s: int8 [M, d] of +-1 -> int32 [d]."""
    s = _chk(np.ascontiguousarray(s), np.int8)
    M, d = s.shape
    V = np.empty(d, np.int32)
    lib().ora_vote_sum(_p(s), ctypes.c_int(M), _i64(d), _i64(d), _p(V))
    return V


def sign_i32(V):
    V = _chk(np.ascontiguousarray(V), np.int32)
    s = np.empty(V.shape, np.int8)
    lib().ora_sign_i32(_p(V), _i64(V.size), _p(s))
    return s


def apply_f32(x, vote_pm1, lr, wd=0.0):
    """In place on x (fp32)."""
    _chk(x, np.float32), _chk(vote_pm1, np.int8)
    lib().ora_apply_f32(_p(x), _i64(x.size), _p(vote_pm1), _f(lr), _f(wd))
    return x


def apply_bf16(x, vote_pm1, lr, wd=0.0):
    _chk(x, np.uint16), _chk(vote_pm1, np.int8)
    lib().ora_apply_bf16(_p(x), _i64(x.size), _p(vote_pm1), _f(lr), _f(wd))
    return x


def apply_f64(x, vote_pm1, lr, wd=0.0):
    _chk(x, np.float32), _chk(vote_pm1, np.int8)
    out = np.empty(x.shape, np.float64)
    lib().ora_apply_f64(_p(x), _i64(x.size), _p(vote_pm1), _f(lr), _f(wd), _p(out))
    return out


# ---- composites with the C-ABI's argument lists, on host arrays --------------------

def _rows(a):
    assert a.ndim == 2 and a.strides[1] == a.itemsize and a.strides[0] % a.itemsize == 0
    return a.shape[0], a.shape[1], a.strides[0] // a.itemsize


def sign_pack(x2d, d=None, signs=None):
    M, dd, xs = _rows(x2d)
    d = dd if d is None else d
    if signs is None:
        signs = np.zeros((M, words_for(d)), np.uint64)
    _, _, ss = _rows(signs)
    rc = lib().ora_sign_pack(_p(x2d), ctypes.c_int(_dt_of(x2d)), ctypes.c_int(M), _i64(d), _i64(xs),
                             _p(signs), _i64(ss))
    assert rc == 0
    return signs


def signum_momentum_pack(g2d, v2d, beta, signs=None):
    M, d, gs = _rows(g2d)
    Mv, dv, vs = _rows(v2d)
    assert (M, d) == (Mv, dv) and v2d.dtype == np.float32
    if signs is None:
        signs = np.zeros((M, words_for(d)), np.uint64)
    _, _, ss = _rows(signs)
    rc = lib().ora_signum_momentum_pack(_p(g2d), ctypes.c_int(_dt_of(g2d)), _p(v2d), ctypes.c_int(M),
                                        _i64(d), _i64(gs), _i64(vs), _f(beta), _p(signs), _i64(ss))
    assert rc == 0
    return signs


def majority_vote(signs2d, d):
    M, W, ss = _rows(signs2d)
    assert signs2d.dtype == np.uint64 and W >= words_for(d)
    vote = np.zeros(words_for(d), np.uint64)
    rc = lib().ora_majority_vote(_p(signs2d), ctypes.c_int(M), _i64(d), _i64(ss), _p(vote))
    assert rc == 0
    return vote


def apply_sign_update(x, vote_words, lr, wd=0.0):
    assert x.ndim == 1 and x.flags["C_CONTIGUOUS"]
    _chk(vote_words, np.uint64)
    rc = lib().ora_apply_sign_update(_p(x), ctypes.c_int(_dt_of(x)), _i64(x.size), _p(vote_words),
                                     _f(lr), _f(wd))
    assert rc == 0
    return x


def vote_apply(signs2d, d, x, lr, wd=0.0):
    M, W, ss = _rows(signs2d)
    vote = np.zeros(words_for(d), np.uint64)
    rc = lib().ora_vote_apply(_p(signs2d), ctypes.c_int(M), _i64(d), _i64(ss), _p(x),
                              ctypes.c_int(_dt_of(x)), _f(lr), _f(wd), _p(vote))
    assert rc == 0
    return vote


def signum_step(g2d, v2d, beta, x, lr, wd=0.0, want_signs=False, worker_flip=None):
    """One iteration of Algorithm 1.  v2d may be None (signSGD, beta must be 0).
    Updates v2d and x in place; returns (vote_words, signs_words or None)."""
    M, d, gs = _rows(g2d)
    vs = 0
    if v2d is not None:
        Mv, dv, vs = _rows(v2d)
        assert (M, d) == (Mv, dv) and v2d.dtype == np.float32
    assert x.ndim == 1 and x.size == d and x.flags["C_CONTIGUOUS"]
    vote = np.zeros(words_for(d), np.uint64)
    signs = np.zeros((M, words_for(d)), np.uint64) if want_signs else None
    flip = None
    if worker_flip is not None:
        flip = np.ascontiguousarray(worker_flip, dtype=np.uint8)
        assert flip.size == M
    rc = lib().ora_signum_step(_p(g2d), ctypes.c_int(_dt_of(g2d)), _p(v2d), ctypes.c_int(M), _i64(d),
                               _i64(gs), _i64(vs), _f(beta), _p(x), ctypes.c_int(_dt_of(x)), _f(lr),
                               _f(wd), _p(vote), _p(signs), _i64(words_for(d)), _p(flip))
    assert rc == 0, rc
    return vote, signs


# ---- ternary QSGD (oracle/qsgd_oracle.c) -------------------------------------------------

QSGD_L2 = 0
QSGD_MAX = 1


def qsgd_norm_f64(g, kind):
    g = _chk(np.ascontiguousarray(g), np.float32)
    return float(lib().ora_qsgd_norm_f64(_p(g), _i64(g.size), ctypes.c_int(kind)))


def qsgd_quantize_row(g, u, norm):
    """codes in {-1, 0, +1} (int8) for one gradient row, uniforms u in [0, 1), and the row's norm (fp32)."""
    g, u = _chk(np.ascontiguousarray(g), np.float32), _chk(np.ascontiguousarray(u), np.float32)
    assert g.shape == u.shape and g.ndim == 1
    q = np.empty(g.size, np.int8)
    lib().ora_qsgd_quantize_row(_p(g), _p(u), _i64(g.size), _f(norm), _p(q))
    return q


def qsgd_pack(q):
    q = _chk(np.ascontiguousarray(q), np.int8)
    nz, sg = np.empty(words_for(q.size), np.uint64), np.empty(words_for(q.size), np.uint64)
    lib().ora_qsgd_pack(_p(q), _i64(q.size), _p(nz), _p(sg))
    return nz, sg


def qsgd_unpack(nz, sg, d):
    nz, sg = _chk(np.ascontiguousarray(nz), np.uint64), _chk(np.ascontiguousarray(sg), np.uint64)
    q = np.empty(int(d), np.int8)
    lib().ora_qsgd_unpack(_p(nz), _p(sg), _i64(d), _p(q))
    return q


def qsgd_average(q2d, norms):
    q2d, norms = _chk(np.ascontiguousarray(q2d), np.int8), _chk(np.ascontiguousarray(norms), np.float32)
    M, d = q2d.shape
    avg = np.empty(d, np.float32)
    lib().ora_qsgd_average(_p(q2d), _p(norms), ctypes.c_int(M), _i64(d), _p(avg))
    return avg


def qsgd_average_f64(q2d, norms):
    q2d, norms = _chk(np.ascontiguousarray(q2d), np.int8), _chk(np.ascontiguousarray(norms), np.float32)
    M, d = q2d.shape
    avg = np.empty(d, np.float64)
    lib().ora_qsgd_average_f64(_p(q2d), _p(norms), ctypes.c_int(M), _i64(d), _p(avg))
    return avg


def qsgd_update(x, avg, lr):
    """In place on x (fp32, or bf16 bit patterns as uint16)."""
    _chk(avg, np.float32)
    assert x.ndim == 1 and x.flags["C_CONTIGUOUS"] and x.size == avg.size
    if x.dtype == np.float32:
        lib().ora_qsgd_update_f32(_p(x), _p(avg), _i64(x.size), _f(lr))
    else:
        _chk(x, np.uint16)
        lib().ora_qsgd_update_bf16(_p(x), _p(avg), _i64(x.size), _f(lr))
    return x


def qsgd_norms(g2d, kind):
    M, d, gs = _rows(g2d)
    norms = np.empty(M, np.float32)
    rc = lib().ora_qsgd_norms(_p(g2d), ctypes.c_int(_dt_of(g2d)), ctypes.c_int(M), _i64(d), _i64(gs),
                              ctypes.c_int(kind), _p(norms))
    assert rc == 0
    return norms


def qsgd_quantize(g2d, u2d, norms):
    """Packed (nonzero, sign) planes, each uint64 [M, ceil(d/64)]."""
    M, d, gs = _rows(g2d)
    Mu, du, us = _rows(u2d)
    assert (M, d) == (Mu, du) and u2d.dtype == np.float32
    norms = _chk(np.ascontiguousarray(norms), np.float32)
    assert norms.size == M
    nz, sg = np.zeros((M, words_for(d)), np.uint64), np.zeros((M, words_for(d)), np.uint64)
    rc = lib().ora_qsgd_quantize(_p(g2d), ctypes.c_int(_dt_of(g2d)), _p(u2d), _p(norms), ctypes.c_int(M), _i64(d),
                                 _i64(gs), _i64(us), _p(nz), _p(sg), _i64(words_for(d)))
    assert rc == 0
    return nz, sg


def qsgd_aggregate_apply(nz2d, sg2d, norms, d, x=None, lr=0.0):
    """Average of the decoded vectors (returned, fp32); if x is given it is updated in place."""
    M, W, ss = _rows(nz2d)
    M2, W2, ss2 = _rows(sg2d)
    assert (M, W, ss) == (M2, W2, ss2) and W >= words_for(d)
    norms = _chk(np.ascontiguousarray(norms), np.float32)
    avg = np.empty(int(d), np.float32)
    rc = lib().ora_qsgd_aggregate_apply(_p(nz2d), _p(sg2d), _p(norms), ctypes.c_int(M), _i64(d), _i64(ss), _p(avg),
                                        _p(x), ctypes.c_int(_dt_of(x) if x is not None else F32), _f(lr))
    assert rc == 0
    return avg
