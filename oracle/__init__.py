"""CPU oracle -- TEST INFRASTRUCTURE, never part of the product path.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It defines what the GPU library must compute, written from the
paper's definitions (Sec. 2.1: sparse tensors, CSF, binary contractions, tensor
networks; Sec. 5.2 MTTKRP; Sec. 5.3 TTMc; Sec. 1 three-tensor product) and
shares no code with the GPU library.

  contractions   : COO loops with dense accumulation, in C (oracle.c), fp64
  abs-term sums  : the same routines on |inputs| (|a*b*c| = |a||b||c|), used as
                   the denominator of the error metric max|err|/sum|terms|
  csf_build      : reference CSF arrays from a lexicographic sort + linear scan
  unfused_*      : binary contraction sequences with full intermediates (Fig. 3a)

Parity pins (tests/test_oracle_*.py): dense nested-loop brute force on tiny
tensors, library einsum/matmul special cases, closed forms, linearity,
mode-permutation invariance, fused == unfused, CSF round trip.  The paper
prints no numeric worked example, so no pin uses printed values.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def lib():
    """Load (building if needed) liboracle.so."""
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        i64, i32p, f64p, i64p = (ctypes.c_int64, ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64))
        ci = ctypes.c_int
        L.oracle_num_threads.restype = ci
        L.oracle_ttmc3.restype = ci
        L.oracle_ttmc3.argtypes = [i64, i32p, i32p, i32p, f64p, i64p, ci, ci, ci, f64p, f64p, f64p]
        L.oracle_ttmc4.restype = ci
        L.oracle_ttmc4.argtypes = [i64, i32p, i32p, i32p, i32p, f64p, i64p, ci, ci, ci,
                                   f64p, f64p, f64p, f64p]
        L.oracle_mttkrp3.restype = ci
        L.oracle_mttkrp3.argtypes = [i64, i32p, i32p, i32p, f64p, i64p, ci, ci, f64p, f64p, f64p]
        L.oracle_sptn3.restype = ci
        L.oracle_sptn3.argtypes = [i64, i32p, i32p, i32p, f64p, i64, i64, i64, i64, f64p,
                                   i64, i32p, i32p, i32p, f64p, i64, f64p]
        _LIB = L
    return _LIB


def num_threads():
    return int(lib().oracle_num_threads())


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _dims(d):
    a = np.ascontiguousarray(d, dtype=np.int64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _check(rc, what):
    if rc != 0:
        raise ValueError("%s failed with code %d (bad argument or out-of-range coordinate)" % (what, rc))


def ttmc3(coords, vals, dims, Fa, Fb, mode=0):
    """Order-3 TTMc for output mode `mode` (Sec. 5.3).  Fa, Fb are the factors of the two
    other modes in increasing mode order.  Returns dims[mode] x Ra x Rb."""
    (k0, p0), (k1, p1), (k2, p2) = _i32(coords[0]), _i32(coords[1]), _i32(coords[2])
    v, pv = _f64(vals)
    fa, pa = _f64(Fa)
    fb, pb = _f64(Fb)
    d, pd = _dims(dims)
    other = [m for m in range(3) if m != mode]
    assert fa.shape[0] == dims[other[0]] and fb.shape[0] == dims[other[1]]
    Y = np.empty((int(dims[mode]), fa.shape[1], fb.shape[1]), dtype=np.float64)
    _check(lib().oracle_ttmc3(len(v), p0, p1, p2, pv, pd, mode, fa.shape[1], fb.shape[1], pa, pb,
                              Y.ctypes.data_as(ctypes.POINTER(ctypes.c_double))), "oracle_ttmc3")
    return Y


def ttmc4(coords, vals, dims, U1, U2, U3):
    """Order-4 TTMc, output mode 0.  Returns dims[0] x R1 x R2 x R3."""
    ks = [_i32(c) for c in coords]
    v, pv = _f64(vals)
    u1, p1 = _f64(U1)
    u2, p2 = _f64(U2)
    u3, p3 = _f64(U3)
    d, pd = _dims(dims)
    assert u1.shape[0] == dims[1] and u2.shape[0] == dims[2] and u3.shape[0] == dims[3]
    Y = np.empty((int(dims[0]), u1.shape[1], u2.shape[1], u3.shape[1]), dtype=np.float64)
    _check(lib().oracle_ttmc4(len(v), ks[0][1], ks[1][1], ks[2][1], ks[3][1], pv, pd,
                              u1.shape[1], u2.shape[1], u3.shape[1], p1, p2, p3,
                              Y.ctypes.data_as(ctypes.POINTER(ctypes.c_double))), "oracle_ttmc4")
    return Y


def mttkrp3(coords, vals, dims, Fa, Fb, mode=0):
    """Order-3 MTTKRP for output mode `mode` (Sec. 5.2).  Returns dims[mode] x R."""
    (k0, p0), (k1, p1), (k2, p2) = _i32(coords[0]), _i32(coords[1]), _i32(coords[2])
    v, pv = _f64(vals)
    fa, pa = _f64(Fa)
    fb, pb = _f64(Fb)
    d, pd = _dims(dims)
    other = [m for m in range(3) if m != mode]
    assert fa.shape[0] == dims[other[0]] and fb.shape[0] == dims[other[1]]
    assert fa.shape[1] == fb.shape[1]
    M = np.empty((int(dims[mode]), fa.shape[1]), dtype=np.float64)
    _check(lib().oracle_mttkrp3(len(v), p0, p1, p2, pv, pd, mode, fa.shape[1], pa, pb,
                                M.ctypes.data_as(ctypes.POINTER(ctypes.c_double))), "oracle_mttkrp3")
    return M


def sptn3(ucoords, uvals, udims, V, wcoords, wvals, wdims):
    """Z[i,m] = U[i,j,k] V[j,l] W[k,l,m] (Sec. 1).  Returns Ni x M."""
    ui, uj, uk = [_i32(c) for c in ucoords]
    wk, wl, wm = [_i32(c) for c in wcoords]
    uv, puv = _f64(uvals)
    wv, pwv = _f64(wvals)
    v, pv = _f64(V)
    Ni, Nj, Nk = [int(x) for x in udims]
    Nk2, L, Mm = [int(x) for x in wdims]
    assert Nk == Nk2 and v.shape == (Nj, L)
    Z = np.empty((Ni, Mm), dtype=np.float64)
    _check(lib().oracle_sptn3(len(uv), ui[1], uj[1], uk[1], puv, Ni, Nj, Nk, L, pv,
                              len(wv), wk[1], wl[1], wm[1], pwv, Mm,
                              Z.ctypes.data_as(ctypes.POINTER(ctypes.c_double))), "oracle_sptn3")
    return Z


# ---- sum of |terms|: the same contraction on absolute values --------------------------------

def ttmc3_abs(coords, vals, dims, Fa, Fb, mode=0):
    return ttmc3(coords, np.abs(vals), dims, np.abs(Fa), np.abs(Fb), mode)


def ttmc4_abs(coords, vals, dims, U1, U2, U3):
    return ttmc4(coords, np.abs(vals), dims, np.abs(U1), np.abs(U2), np.abs(U3))


def mttkrp3_abs(coords, vals, dims, Fa, Fb, mode=0):
    return mttkrp3(coords, np.abs(vals), dims, np.abs(Fa), np.abs(Fb), mode)


def sptn3_abs(ucoords, uvals, udims, V, wcoords, wvals, wdims):
    return sptn3(ucoords, np.abs(uvals), udims, np.abs(V), wcoords, np.abs(wvals), wdims)


def rel_err(got, want, abs_terms):
    """max over elements of |got-want| / sum|terms|; where sum|terms| == 0 both must be 0.0."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    S = np.asarray(abs_terms, dtype=np.float64)
    zero = S == 0.0
    if np.any(got[zero] != 0.0) or np.any(want[zero] != 0.0):
        return np.inf
    diff = np.abs(got - want)
    if not np.all(np.isfinite(got)):
        return np.inf
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.where(zero, 0.0, diff / np.where(zero, 1.0, S))
    return float(r.max()) if r.size else 0.0


from .csf_ref import csf_build, csf_expand                      # noqa: E402
from .unfused import (unfused_ttmc3, unfused_mttkrp3, unfused_ttmc4, unfused_sptn3)  # noqa: E402
