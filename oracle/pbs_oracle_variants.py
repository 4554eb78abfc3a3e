"""ctypes front end of pbs_oracle_variants.c: the fp64 CPU oracle of the variants the paper ablates (other proxies for
the importance score, key-aware query permutation).

TEST INFRASTRUCTURE ONLY, as oracle/pbs_oracle.py: imported by tests/, the smoke check and the benchmark's CPU leg; the
product package never imports it and it never imports the product package.  Wrappers only marshal arguments.
"""
import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pbs_oracle_variants.c")
_LIB = os.path.join(_HERE, "libpbs_oracle_variants.so")
_lib = None


def build(force=False):
    """Compile pbs_oracle_variants.c with gcc (plain -O2, OpenMP, strict IEEE, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _i32p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def key_scores_proxy(Q, K, rows=None, scale=0.0):
    """Importance score from the query rows `rows` (positions, the same for every head), or from the average query
    over all positions when rows is None.  Q [B,Hq,N,d], K [B,Hkv,N,d] -> s [B,Hkv,N] float64."""
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    Q, qp = _f32(Q)
    K, kp = _f32(K)
    s = np.empty((B, Hkv, N), dtype=np.float64)
    sc = float(scale) if scale else 1.0 / math.sqrt(d)
    if rows is None:
        rc = _load().pbsv_key_scores_proxy(B, Hq, Hkv, N, d, 1, 0, None, ctypes.c_double(sc), qp, kp,
                                           s.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        rc = _load().pbsv_key_scores_proxy(B, Hq, Hkv, N, d, 0, rows.size, _i32p(rows), ctypes.c_double(sc), qp, kp,
                                           s.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc:
        raise RuntimeError("pbsv_key_scores_proxy failed: %d" % rc)
    return s


def query_permutation(Q, K, block, segment, want_assigned=False):
    """Key-aware query permutation: qidx [B,Hq,N] int32 in gather form (and the centroid assigned to every query)."""
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    Q, qp = _f32(Q)
    K, kp = _f32(K)
    qidx = np.empty((B, Hq, N), dtype=np.int32)
    assigned = np.empty((B, Hq, N), dtype=np.int32) if want_assigned else None
    rc = _load().pbsv_query_permutation(B, Hq, Hkv, N, d, int(block), int(segment), qp, kp, _i32p(qidx),
                                        _i32p(assigned) if want_assigned else None)
    if rc:
        raise RuntimeError("pbsv_query_permutation failed: %d" % rc)
    return (qidx, assigned) if want_assigned else qidx


def query_permutation_segment(Q, K, block, segment, g):
    """The slice [g*segment, (g+1)*segment) of query_permutation's qidx, for one full segment g of every head, at the
    cost of that segment alone: [B,Hq,segment] int32."""
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    Q, qp = _f32(Q)
    K, kp = _f32(K)
    qseg = np.empty((B, Hq, int(segment)), dtype=np.int32)
    rc = _load().pbsv_query_permutation_segment(B, Hq, Hkv, N, d, int(block), int(segment), int(g), qp, kp, _i32p(qseg))
    if rc:
        raise RuntimeError("pbsv_query_permutation_segment failed: %d" % rc)
    return qseg
