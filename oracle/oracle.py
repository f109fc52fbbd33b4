"""ctypes access to the CPU oracle (oracle/oz2_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's cpu_baseline
leg.  The product package never imports this module.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oz2_oracle.cpp")
_LIB = os.path.join(_HERE, "liboz2_oracle.so")

_lib = None


def build(force=False):
    """Compile the oracle with g++ (host only, OpenMP)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC]
    subprocess.check_call(cmd)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oz2o_sym_mod.restype = ctypes.c_int64
        _lib.oz2o_sym_mod.argtypes = [ctypes.c_int64, ctypes.c_int]
        _lib.oz2o_kappa.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_int64]
        _lib.oz2o_beta.argtypes = [ctypes.c_int, ctypes.c_void_p]
        _lib.oz2o_log2_budget.argtypes = [ctypes.c_int, ctypes.c_void_p]
        _lib.oz2o_native_gemm.argtypes = [ctypes.c_int, ctypes.c_int] + [ctypes.c_int64] * 3 + [
            ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
        _lib.oz2o_has_nonfinite.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64]
        _lib.oz2o_axpby.argtypes = [ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_double, ctypes.c_void_p]
        _lib.oz2o_kappa_sum.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_int64]
        _lib.oz2o_dgemm_sub.argtypes = ([ctypes.c_int64] * 3 + [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int64,
                                        ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p] + [ctypes.c_void_p] * 13)
        _lib.oz2o_exact_sub.argtypes = ([ctypes.c_int64] * 3 + [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                        ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p])
    return _lib


WORDS = 12


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _words_to_int(words):
    v = 0
    for i, w in enumerate(words):
        v |= int(w) << (32 * i)
    return v


def sym_mod(a, p):
    return int(lib().oz2o_sym_mod(int(a), int(p)))


def moduli(N):
    out = np.zeros(N, dtype=np.int32)
    rc = lib().oz2o_moduli(int(N), _ptr(out))
    if rc:
        raise ValueError("oz2o_moduli(%d) -> %d" % (N, rc))
    return [int(x) for x in out]


def kappa(N, k, mods=None):
    mods = np.asarray(moduli(N) if mods is None else mods, dtype=np.int32)
    return int(lib().oz2o_kappa(int(N), _ptr(mods), int(k)))


def kappa_sum(N, k, mods=None):
    """Largest S = k_A + k_B with k * 2^S <= M/2 - 1 (Section 3, first budget equation)."""
    mods = np.asarray(moduli(N) if mods is None else mods, dtype=np.int32)
    return lib().oz2o_kappa_sum(int(N), _ptr(mods), int(k))


def beta(N, mods=None):
    mods = np.asarray(moduli(N) if mods is None else mods, dtype=np.int32)
    return int(lib().oz2o_beta(int(N), _ptr(mods)))


def log2_budget(N, mods=None):
    """Largest b with 2^b <= M/2 - 1 (INT8-product shift selection)."""
    mods = np.asarray(moduli(N) if mods is None else mods, dtype=np.int32)
    return lib().oz2o_log2_budget(int(N), _ptr(mods))


def crt_constants(N, mods=None):
    """Return (M, [W_1..W_N]) as Python ints."""
    mods = np.asarray(moduli(N) if mods is None else mods, dtype=np.int32)
    Mw = np.zeros(WORDS, dtype=np.uint32)
    Ww = np.zeros((N, WORDS), dtype=np.uint32)
    rc = lib().oz2o_crt_constants(int(N), _ptr(mods), _ptr(Mw), _ptr(Ww))
    if rc:
        raise ValueError("oz2o_crt_constants -> %d" % rc)
    return _words_to_int(Mw), [_words_to_int(Ww[t]) for t in range(N)]


class Result(dict):
    __getattr__ = dict.__getitem__


def dgemm(A, B, N, mods=None, rows=None, cols=None, want=("C",), mode=0, delta=0):
    """Run Algorithm 1 on the CPU.  mode 0: shifts from the row/column maxima (Section 3); mode 1: shifts
    from the Cauchy-Schwarz bound (Section 4.1, "fast"); mode 2: shifts from the INT8 product of 6-bit upper
    bounds (Section 4.1, "accu"; the row and column maxima of that product always run over the whole of A and B,
    so A and B must be the full operands even when rows / cols select a subset).  A (m x k), B (k x n): numpy float64, any layout (copied to
    column-major).  delta: bits of budget moved from A to B (0: the equal split of the paper).
    rows / cols: optional index lists selecting the outputs to compute.
    want: any of "C", "shifts", "Ap", "Bp", "Ares", "Bres", "Cprod", "Cres", "X".
    Ap/Bp/X come back as nested Python-int lists (tiny inputs only)."""
    A = np.asfortranarray(A, dtype=np.float64)
    B = np.asfortranarray(B, dtype=np.float64)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    I = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    J = None if cols is None else np.ascontiguousarray(cols, dtype=np.int64)
    nI = m if I is None else len(I)
    nJ = n if J is None else len(J)
    mods_a = None if mods is None else np.asarray(mods, dtype=np.int32)
    w = set(want)
    C = np.zeros((nI, nJ), dtype=np.float64, order="F") if "C" in w else None
    sa = np.zeros(nI, dtype=np.int32) if "shifts" in w else None
    sb = np.zeros(nJ, dtype=np.int32) if "shifts" in w else None
    aps = np.zeros((nI, k), dtype=np.uint8) if "Ap" in w else None
    apm = np.zeros((nI, k, 4), dtype=np.uint32) if "Ap" in w else None
    bps = np.zeros((nJ, k), dtype=np.uint8) if "Bp" in w else None
    bpm = np.zeros((nJ, k, 4), dtype=np.uint32) if "Bp" in w else None
    ares = np.zeros((N, nI, k), dtype=np.int8) if "Ares" in w else None
    bres = np.zeros((N, nJ, k), dtype=np.int8) if "Bres" in w else None
    cprod = np.zeros((N, nJ, nI), dtype=np.int64) if "Cprod" in w else None
    cres = np.zeros((N, nJ, nI), dtype=np.uint8) if "Cres" in w else None
    xs = np.zeros((nJ, nI), dtype=np.uint8) if "X" in w else None
    xm = np.zeros((nJ, nI, WORDS), dtype=np.uint32) if "X" in w else None
    rc = lib().oz2o_dgemm_sub(m, n, k, _ptr(A), max(1, m), _ptr(B), max(1, k), int(N), int(mode), int(delta), _ptr(mods_a),
                              nI, _ptr(I), nJ, _ptr(J), _ptr(C), _ptr(sa), _ptr(sb), _ptr(aps), _ptr(apm),
                              _ptr(bps), _ptr(bpm), _ptr(ares), _ptr(bres), _ptr(cprod), _ptr(cres),
                              _ptr(xs), _ptr(xm))
    if rc:
        raise ValueError("oz2o_dgemm_sub -> %d" % rc)
    out = Result()
    if C is not None:
        out["C"] = C
    if sa is not None:
        out["sa"], out["sb"] = sa, sb
    if aps is not None:
        out["Ap"] = [[(-1 if aps[r, l] else 1) * _words_to_int(apm[r, l]) for l in range(k)] for r in range(nI)]
    if bps is not None:  # returned as k x nJ nested list: Bp[l][c]
        out["Bp"] = [[(-1 if bps[c, l] else 1) * _words_to_int(bpm[c, l]) for c in range(nJ)] for l in range(k)]
    if ares is not None:
        out["Ares"] = ares
    if bres is not None:
        out["Bres"] = bres
    if cprod is not None:  # [t][r][c]
        out["Cprod"] = np.ascontiguousarray(cprod.transpose(0, 2, 1))
    if cres is not None:
        out["Cres"] = np.ascontiguousarray(cres.transpose(0, 2, 1))
    if xs is not None:
        out["X"] = [[(-1 if xs[c, r] else 1) * _words_to_int(xm[c, r]) for c in range(nJ)] for r in range(nI)]
    return out


def native_gemm(opA, opB):
    """Textbook FP64 product (oz2o_native_gemm): the fallback for inputs with infinities or NaNs."""
    A = np.asfortranarray(opA, dtype=np.float64)
    B = np.asfortranarray(opB, dtype=np.float64)
    m, k = A.shape
    _, n = B.shape
    P = np.zeros((m, n), order="F")
    rc = lib().oz2o_native_gemm(0, 0, m, n, k, _ptr(A), max(1, m), _ptr(B), max(1, k), _ptr(P))
    if rc:
        raise ValueError("oz2o_native_gemm -> %d" % rc)
    return P


def has_nonfinite(X):
    X = np.asfortranarray(X, dtype=np.float64)
    return bool(lib().oz2o_has_nonfinite(X.shape[0], X.shape[1], _ptr(X), max(1, X.shape[0])))


def dgemm_ex(transa, transb, alpha, A, B, beta, C, N, mode=0, check_nonfinite=True):
    """C := alpha * op(A) op(B) + beta * C with the product formed by Algorithm 1 (see oz2o_axpby for the
    order of the floating-point operations of the update), or by the textbook FP64 loop when check_nonfinite
    is set and A or B holds an infinity or a NaN.  A, B as stored; returns the new C."""
    opA = A.T if transa in "TtCc" else A
    opB = B.T if transb in "TtCc" else B
    m, k = opA.shape
    if k == 0 or alpha == 0.0:
        P = np.zeros((m, opB.shape[1]), order="F")
    elif check_nonfinite and (has_nonfinite(opA) or has_nonfinite(opB)):
        P = native_gemm(opA, opB)
    else:
        P = dgemm(opA, opB, N, mode=mode).C
    out = np.array(C, dtype=np.float64, order="F", copy=True)
    Pf = np.asfortranarray(P)
    rc = lib().oz2o_axpby(out.size, float(alpha), _ptr(Pf), float(beta), _ptr(out))
    if rc:
        raise ValueError("oz2o_axpby -> %d" % rc)
    return out


def dsyrk(uplo, trans, alpha, A, beta, C, N, mode=0, check_nonfinite=True):
    """Symmetric rank-k update: the uplo triangle of C := alpha * op(A) op(A)^T + beta * C, every element of it as
    dgemm_ex forms it from (A, A^T); the other triangle of C comes back unchanged."""
    other = "T" if trans in "Nn" else "N"
    full = dgemm_ex(trans, other, alpha, A, A, beta, C, N, mode=mode, check_nonfinite=check_nonfinite)
    out = np.array(C, dtype=np.float64, order="F", copy=True)
    n = out.shape[0]
    ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    tri = (ii >= jj) if uplo in "Ll" else (ii <= jj)
    out[tri] = full[tri]
    return out


def triangular(A, uplo, diag):
    """The triangular matrix a BLAS routine sees in the array A: one triangle as stored, zeros elsewhere, ones
    on the diagonal when it is declared unit.  What is not referenced may hold anything, NaNs included."""
    A = np.asarray(A, dtype=np.float64)
    n = A.shape[0]
    ii, jj = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    keep = (ii >= jj) if uplo in "Ll" else (ii <= jj)
    T = np.where(keep, A, 0.0)
    if diag in "Uu":
        T[np.arange(n), np.arange(n)] = 1.0
    return np.asfortranarray(T)


def dtrmm(side, uplo, transa, diag, alpha, A, B, N, mode=0, check_nonfinite=True):
    """B := alpha * op(T) * B (side L) or alpha * B * op(T) (side R), T = triangular(A, uplo, diag), the product
    formed by Algorithm 1 (or by the FP64 fallback) on the explicit triangular matrix.  Returns the new B."""
    T = triangular(A, uplo, diag)
    B = np.asfortranarray(B, dtype=np.float64)
    zero = np.zeros(B.shape, order="F")
    if alpha == 0.0:
        return zero
    if side in "Ll":
        return dgemm_ex(transa, "N", alpha, T, B, 0.0, zero, N, mode=mode, check_nonfinite=check_nonfinite)
    return dgemm_ex("N", transa, alpha, B, T, 0.0, zero, N, mode=mode, check_nonfinite=check_nonfinite)


def exact(A, B, rows=None, cols=None):
    """binary128 reference: returns (C_ref, |A||B|) on the selected outputs, both rounded to double."""
    A = np.asfortranarray(A, dtype=np.float64)
    B = np.asfortranarray(B, dtype=np.float64)
    m, k = A.shape
    _, n = B.shape
    I = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    J = None if cols is None else np.ascontiguousarray(cols, dtype=np.int64)
    nI = m if I is None else len(I)
    nJ = n if J is None else len(J)
    C = np.zeros((nI, nJ), dtype=np.float64, order="F")
    S = np.zeros((nI, nJ), dtype=np.float64, order="F")
    rc = lib().oz2o_exact_sub(m, n, k, _ptr(A), max(1, m), _ptr(B), max(1, k), nI, _ptr(I), nJ, _ptr(J),
                              _ptr(C), _ptr(S))
    if rc:
        raise ValueError("oz2o_exact_sub -> %d" % rc)
    return C, S
