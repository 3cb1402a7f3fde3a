"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Loads ``oracle/liboracle.so`` (plain C, fp64, built with gcc by ``build()``)
and exposes one function per contraction.  Nothing here is used by the product
library; only tests, the smoke check and the benchmark's CPU-baseline leg may
import this module.  It imports nothing from the HIP package.

Every ``contract_*`` function up-converts its inputs to fp64 and evaluates the
linear loop nest that defines the contraction (see ``oracle.c``).  The
``abs_bound`` helper returns, per output element, the sum of the absolute
values of all partial products -- the quantity the error tolerances are scaled
by -- by running the same nest on element-wise absolute values (that sum
factorises exactly like the contraction itself).

``intermediate_*`` return the named intermediates of the fissioned schedules
(Section 4.2: the temporary's indices are those of the producer that also
occur in the consumer or the output), position-compressed along the sparse
prefix: row ``f`` belongs to the ``f``-th distinct coordinate prefix in
lexicographic order.  They are written with numpy scatter-adds.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

_i64 = ctypes.c_int64
_pi32 = ctypes.POINTER(ctypes.c_int32)
_pf64 = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile oracle.c into liboracle.so with gcc (OpenMP, no fast-math)."""
    src = os.path.join(_HERE, "oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-o", _LIB_PATH, src])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _p(a, typ):
    return a.ctypes.data_as(typ)


def _threads(nthreads):
    return int(nthreads) if nthreads else max_threads()


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"{name}: {'coordinate out of range' if rc == -2 else 'allocation failed'}")


def contract_ttmc3(coords, vals, dims, C, D, nthreads=None):
    """A(i,l,m) = sum_jk B(i,j,k) C(j,l) D(k,m)   (Table 2, kernel 6)."""
    ci, cj, ck = (_i32(c) for c in coords)
    v, C, D = _f64(vals), _f64(C), _f64(D)
    I, J, K = (int(d) for d in dims)
    L, M = C.shape[1], D.shape[1]
    assert C.shape[0] == J and D.shape[0] == K
    A = np.empty((I, L, M), dtype=np.float64)
    rc = _load().oracle_ttmc3(_i64(v.size), _p(ci, _pi32), _p(cj, _pi32), _p(ck, _pi32), _p(v, _pf64),
                              _i64(I), _i64(J), _i64(K), _p(C, _pf64), _i64(L), _p(D, _pf64), _i64(M),
                              _p(A, _pf64), ctypes.c_int(_threads(nthreads)))
    _check(rc, "oracle_ttmc3")
    return A


def contract_mttkrp3(coords, vals, dims, C, D, nthreads=None):
    """A(i,r) = sum_jk B(i,j,k) C(j,r) D(k,r)   (MTTKRP, Section 6 / Table 2 kernel 8 producer)."""
    ci, cj, ck = (_i32(c) for c in coords)
    v, C, D = _f64(vals), _f64(C), _f64(D)
    I, J, K = (int(d) for d in dims)
    R = C.shape[1]
    assert C.shape[0] == J and D.shape == (K, R)
    A = np.empty((I, R), dtype=np.float64)
    rc = _load().oracle_mttkrp3(_i64(v.size), _p(ci, _pi32), _p(cj, _pi32), _p(ck, _pi32), _p(v, _pf64),
                                _i64(I), _i64(J), _i64(K), _p(C, _pf64), _p(D, _pf64), _i64(R),
                                _p(A, _pf64), ctypes.c_int(_threads(nthreads)))
    _check(rc, "oracle_mttkrp3")
    return A


def contract_sddmm_spmm(coords, vals, dims, X, Y, Z, nthreads=None):
    """A(i,l) = sum_j S(i,j) (sum_k X(i,k) Y(j,k)) Z(j,l)   (Table 2, kernel 1)."""
    ci, cj = (_i32(c) for c in coords)
    v, X, Y, Z = _f64(vals), _f64(X), _f64(Y), _f64(Z)
    I, J = (int(d) for d in dims)
    K, L = X.shape[1], Z.shape[1]
    assert X.shape[0] == I and Y.shape == (J, K) and Z.shape[0] == J
    A = np.empty((I, L), dtype=np.float64)
    rc = _load().oracle_sddmm_spmm(_i64(v.size), _p(ci, _pi32), _p(cj, _pi32), _p(v, _pf64),
                                   _i64(I), _i64(J), _p(X, _pf64), _p(Y, _pf64), _i64(K),
                                   _p(Z, _pf64), _i64(L), _p(A, _pf64), ctypes.c_int(_threads(nthreads)))
    _check(rc, "oracle_sddmm_spmm")
    return A


def contract_ttmc4(coords, vals, dims, C, D, E, nthreads=None):
    """A(i,l,m,n) = sum_jkp B(i,j,k,p) C(j,l) D(k,m) E(p,n)   (order-4 TTM chain)."""
    ci, cj, ck, cp = (_i32(c) for c in coords)
    v, C, D, E = _f64(vals), _f64(C), _f64(D), _f64(E)
    I, J, K, P = (int(d) for d in dims)
    L, M, N = C.shape[1], D.shape[1], E.shape[1]
    assert C.shape[0] == J and D.shape[0] == K and E.shape[0] == P
    A = np.empty((I, L, M, N), dtype=np.float64)
    rc = _load().oracle_ttmc4(_i64(v.size), _p(ci, _pi32), _p(cj, _pi32), _p(ck, _pi32), _p(cp, _pi32),
                              _p(v, _pf64), _i64(I), _i64(J), _i64(K), _i64(P),
                              _p(C, _pf64), _i64(L), _p(D, _pf64), _i64(M), _p(E, _pf64), _i64(N),
                              _p(A, _pf64), ctypes.c_int(_threads(nthreads)))
    _check(rc, "oracle_ttmc4")
    return A


def contract_ttmc_all(coords, vals, dims, C, D, E, nthreads=None):
    """A(l,m,n) = sum_ijk B(i,j,k) C(i,l) D(j,m) E(k,n)   (Table 2, kernel 5; Figure 2a)."""
    ci, cj, ck = (_i32(c) for c in coords)
    v, C, D, E = _f64(vals), _f64(C), _f64(D), _f64(E)
    I, J, K = (int(d) for d in dims)
    L, M, N = C.shape[1], D.shape[1], E.shape[1]
    assert C.shape[0] == I and D.shape[0] == J and E.shape[0] == K
    A = np.empty((L, M, N), dtype=np.float64)
    rc = _load().oracle_ttmc_all(_i64(v.size), _p(ci, _pi32), _p(cj, _pi32), _p(ck, _pi32), _p(v, _pf64),
                                 _i64(I), _i64(J), _i64(K), _p(C, _pf64), _i64(L), _p(D, _pf64), _i64(M),
                                 _p(E, _pf64), _i64(N), _p(A, _pf64), ctypes.c_int(_threads(nthreads)))
    _check(rc, "oracle_ttmc_all")
    return A


def contract_mttkrp_gemm(coords, vals, dims, C, D, E, nthreads=None):
    """A(i,m) = sum_jkr B(i,j,k) C(j,r) D(k,r) E(r,m)   (Table 2, kernel 8)."""
    ci, cj, ck = (_i32(c) for c in coords)
    v, C, D, E = _f64(vals), _f64(C), _f64(D), _f64(E)
    I, J, K = (int(d) for d in dims)
    R, M = C.shape[1], E.shape[1]
    assert C.shape[0] == J and D.shape == (K, R) and E.shape[0] == R
    A = np.empty((I, M), dtype=np.float64)
    rc = _load().oracle_mttkrp_gemm(_i64(v.size), _p(ci, _pi32), _p(cj, _pi32), _p(ck, _pi32), _p(v, _pf64),
                                    _i64(I), _i64(J), _i64(K), _p(C, _pf64), _p(D, _pf64), _i64(R),
                                    _p(E, _pf64), _i64(M), _p(A, _pf64), ctypes.c_int(_threads(nthreads)))
    _check(rc, "oracle_mttkrp_gemm")
    return A


def contract_sddmm_spmm_gemm(coords, vals, dims, X, Y, Z, F, nthreads=None):
    """A(i,m) = sum_jkl S(i,j) X(i,k) Y(j,k) Z(j,l) F(l,m)   (Table 2, kernel 2)."""
    ci, cj = (_i32(c) for c in coords)
    v, X, Y, Z, F = _f64(vals), _f64(X), _f64(Y), _f64(Z), _f64(F)
    I, J = (int(d) for d in dims)
    K, L, M = X.shape[1], Z.shape[1], F.shape[1]
    assert X.shape[0] == I and Y.shape == (J, K) and Z.shape[0] == J and F.shape[0] == L
    A = np.empty((I, M), dtype=np.float64)
    rc = _load().oracle_sddmm_spmm_gemm(_i64(v.size), _p(ci, _pi32), _p(cj, _pi32), _p(v, _pf64),
                                        _i64(I), _i64(J), _p(X, _pf64), _p(Y, _pf64), _i64(K),
                                        _p(Z, _pf64), _i64(L), _p(F, _pf64), _i64(M), _p(A, _pf64),
                                        ctypes.c_int(_threads(nthreads)))
    _check(rc, "oracle_sddmm_spmm_gemm")
    return A


def contract_spmm(coords, vals, dims, C, nthreads=None):
    """A(i,k) = sum_j B(i,j) C(j,k)   (Figure 1b)."""
    ci, cj = (_i32(c) for c in coords)
    v, C = _f64(vals), _f64(C)
    I, J = (int(d) for d in dims)
    K = C.shape[1]
    assert C.shape[0] == J
    A = np.empty((I, K), dtype=np.float64)
    rc = _load().oracle_spmm(_i64(v.size), _p(ci, _pi32), _p(cj, _pi32), _p(v, _pf64),
                             _i64(I), _i64(J), _p(C, _pf64), _i64(K), _p(A, _pf64),
                             ctypes.c_int(_threads(nthreads)))
    _check(rc, "oracle_spmm")
    return A


_CONTRACT = {
    "ttmc3": contract_ttmc3,
    "mttkrp3": contract_mttkrp3,
    "sddmm_spmm": contract_sddmm_spmm,
    "ttmc4": contract_ttmc4,
    "ttmc_all": contract_ttmc_all,
    "mttkrp_gemm": contract_mttkrp_gemm,
    "sddmm_spmm_gemm": contract_sddmm_spmm_gemm,
}


def contract(kind, coords, vals, dims, factors, nthreads=None):
    """Dispatch on the contraction kind; returns the fp64 result."""
    return _CONTRACT[kind](coords, vals, dims, *factors, nthreads=nthreads)


def time_contract(kind, coords, vals, dims, factors, nthreads=None, warmup=1, runs=3):
    """Wall-clock seconds of `runs` evaluations of the C loop nest alone, after `warmup` untimed ones.
    The inputs are converted to the C types (fp64, int32, contiguous) once, before the clock starts:
    the conversions inside contract_* are then no-ops, and the clock covers the ctypes call and the
    allocation of the fp64 result only."""
    import time
    c = [_i32(x) for x in coords]
    v = _f64(vals)
    fs = [_f64(f) for f in factors]
    secs = []
    for r in range(warmup + runs):
        t0 = time.perf_counter()
        _CONTRACT[kind](c, v, dims, *fs, nthreads=nthreads)
        dt = time.perf_counter() - t0
        if r >= warmup:
            secs.append(dt)
    return secs


def abs_bound(kind, coords, vals, dims, factors, nthreads=None):
    """Per output element: sum over all partial products of their absolute values."""
    return _CONTRACT[kind](coords, np.abs(_f64(vals)), dims, *[np.abs(_f64(f)) for f in factors],
                           nthreads=nthreads)


# ---------------------------------------------------------------------------
# Index structure and named intermediates (numpy)
# ---------------------------------------------------------------------------

def prefixes(coords, dims, depth):
    """Distinct coordinate prefixes of length ``depth`` in lexicographic order.

    Returns (prefix_coords [depth, n_prefix] int64, inverse [nnz]) where
    ``inverse[n]`` is the prefix number of nonzero ``n``."""
    key = np.zeros(np.asarray(coords[0]).shape[0], dtype=np.int64)
    for m in range(depth):
        key = key * int(dims[m]) + np.asarray(coords[m], dtype=np.int64)
    uniq, inverse = np.unique(key, return_inverse=True)
    out = np.empty((depth, uniq.size), dtype=np.int64)
    rem = uniq
    for m in range(depth - 1, -1, -1):
        rem, out[m] = np.divmod(rem, int(dims[m]))
    return out, inverse


def intermediate_leaf(coords, vals, dims, last_factor):
    """T(f, x) = sum over the nonzeros z of leaf fiber f of  vals[z] * F(c_last[z], x),
    where f numbers the distinct prefixes of all but the last mode.  This is
    T(i,j,m) for kernel 6, T(i,j,r) for MTTKRP and T1(i,j,k,n) for the order-4 chain."""
    order = len(coords)
    pre, inv = prefixes(coords, dims, order - 1)
    Fm = _f64(last_factor)
    T = np.zeros((pre.shape[1], Fm.shape[1]), dtype=np.float64)
    np.add.at(T, inv, _f64(vals)[:, None] * Fm[np.asarray(coords[order - 1], dtype=np.int64)])
    return pre, T


def intermediate_t2_order4(coords, vals, dims, D, E):
    """T2(f2, m, n) = sum over nonzeros z with prefix (i,j) = f2 of vals[z] * D(k,m) * E(p,n)."""
    pre, inv = prefixes(coords, dims, 2)
    D, E = _f64(D), _f64(E)
    T2 = np.zeros((pre.shape[1], D.shape[1], E.shape[1]), dtype=np.float64)
    k = np.asarray(coords[2], dtype=np.int64)
    p = np.asarray(coords[3], dtype=np.int64)
    np.add.at(T2, inv, _f64(vals)[:, None, None] * D[k][:, :, None] * E[p][:, None, :])
    return pre, T2


def intermediate_slice_ttmc_all(coords, vals, dims, D, E):
    """Kernel 5, second and third schedule of Table 2: T(s, m, n) = sum over the nonzeros z of the
    s-th non-empty slice i of vals[z] * D(j,m) * E(k,n).  Returns (slice coordinates, T)."""
    pre, inv = prefixes(coords, dims, 1)
    D, E = _f64(D), _f64(E)
    T = np.zeros((pre.shape[1], D.shape[1], E.shape[1]), dtype=np.float64)
    j = np.asarray(coords[1], dtype=np.int64)
    k = np.asarray(coords[2], dtype=np.int64)
    np.add.at(T, inv, _f64(vals)[:, None, None] * D[j][:, :, None] * E[k][:, None, :])
    return pre, T


def intermediate_sampled(coords, vals, X, Y):
    """t(z) = S(i,j) * sum_k X(i,k) Y(j,k) for each stored (i,j), in the order given."""
    X, Y = _f64(X), _f64(Y)
    i = np.asarray(coords[0], dtype=np.int64)
    j = np.asarray(coords[1], dtype=np.int64)
    return _f64(vals) * np.einsum("zk,zk->z", X[i], Y[j])
