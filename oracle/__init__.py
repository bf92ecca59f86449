"""CPU oracle for Kron-Matmul (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It is independent of the HIP library: neither imports the other.

kron_matmul      -- Algorithm 1 of the paper (sliced multiply, last factor first),
                    wide accumulators, rounded once at the end.
sliced_multiply  -- one iteration of Algorithm 1.
kron_bruteforce  -- the definition: materialise F_1 (x) ... (x) F_N, dense matmul.
"""
import ctypes
import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        i64, ci, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        for name in ("kron_oracle_f32", "kron_oracle_f64",
                     "kron_bruteforce_f32", "kron_bruteforce_f64"):
            fn = getattr(lib, name)
            fn.restype = ci
            fn.argtypes = [i64, ci, vp, vp, vp, vp, vp]
        for name in ("kron_sliced_multiply_f32", "kron_sliced_multiply_f64"):
            fn = getattr(lib, name)
            fn.restype = ci
            fn.argtypes = [i64, i64, ci, ci, vp, vp, vp]
        lib.kron_oracle_threads.restype = ci
        lib.kron_oracle_threads.argtypes = []
        _lib = lib
    return _lib


def threads():
    """Number of OpenMP threads the oracle will use."""
    return int(_load().kron_oracle_threads())


def _prep(X, Fs):
    X = np.ascontiguousarray(X)
    if X.dtype not in (np.float32, np.float64):
        raise TypeError("X must be float32 or float64")
    if X.ndim != 2:
        raise ValueError("X must be 2-D")
    Fs = [np.ascontiguousarray(F, dtype=X.dtype) for F in Fs]
    if not Fs:
        raise ValueError("need at least one factor")
    for F in Fs:
        if F.ndim != 2:
            raise ValueError("factors must be 2-D")
    P = np.array([F.shape[0] for F in Fs], dtype=np.intc)
    Q = np.array([F.shape[1] for F in Fs], dtype=np.intc)
    if X.shape[1] != int(np.prod(P, dtype=np.int64)):
        raise ValueError("X has %d columns, factors need %d" % (X.shape[1], int(np.prod(P, dtype=np.int64))))
    return X, Fs, P, Q


def _call(stem, X, Fs):
    lib = _load()
    X, Fs, P, Q = _prep(X, Fs)
    M = X.shape[0]
    Y = np.empty((M, int(np.prod(Q, dtype=np.int64))), dtype=X.dtype)
    fptr = (ctypes.c_void_p * len(Fs))(*[F.ctypes.data for F in Fs])
    fn = getattr(lib, stem + ("_f32" if X.dtype == np.float32 else "_f64"))
    rc = fn(M, len(Fs), P.ctypes.data, Q.ctypes.data, X.ctypes.data,
            ctypes.cast(fptr, ctypes.c_void_p), Y.ctypes.data)
    if rc != 0:
        raise RuntimeError("%s failed with code %d" % (stem, rc))
    return Y


def kron_matmul(X, Fs):
    """Y = X (F_1 (x) ... (x) F_N) by Algorithm 1; Fs[0] is the leftmost factor."""
    return _call("kron_oracle", X, Fs)


def kron_bruteforce(X, Fs):
    """Same result from the definition (explicit Kronecker matrix); tiny sizes only."""
    return _call("kron_bruteforce", X, Fs)


def sliced_multiply(Yin, F):
    """One iteration of Algorithm 1: (M x K) with a (P x Q) factor -> M x (K/P)*Q."""
    lib = _load()
    Yin = np.ascontiguousarray(Yin)
    F = np.ascontiguousarray(F, dtype=Yin.dtype)
    M, K = Yin.shape
    P, Q = F.shape
    if K % P:
        raise ValueError("row width %d is not a multiple of P=%d" % (K, P))
    out = np.empty((M, K // P * Q), dtype=Yin.dtype)
    fn = lib.kron_sliced_multiply_f32 if Yin.dtype == np.float32 else lib.kron_sliced_multiply_f64
    rc = fn(M, K, P, Q, Yin.ctypes.data, F.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise RuntimeError("sliced_multiply failed with code %d" % rc)
    return out
