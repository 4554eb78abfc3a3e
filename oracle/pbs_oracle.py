"""ctypes front end of the fp64 CPU oracle (pbs_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module
and this module never imports the product package.

All functions take numpy arrays.  Floating inputs are float32 arrays whose
values are already rounded to the storage type (bf16 values are exactly
representable in float32); the C code promotes them to double.  The wrappers
of the C functions only marshal arguments: that arithmetic is in pbs_oracle.c,
where every function cites the passage of the paper it follows.  Three functions
here are written in numpy instead and cite their passages themselves:
all_allowed_lists (the columns the extended causal mask admits), coverage (two
calls of the attention loop combined) and pipeline (the stages chained).
"""
import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pbs_oracle.c")
_LIB = os.path.join(_HERE, "libpbs_oracle.so")
_lib = None


def build(force=False):
    """Compile pbs_oracle.c with gcc (plain -O2, OpenMP, strict IEEE; no fast-math, no -march)."""
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


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _scale(scale, d):
    return float(scale) if scale else 1.0 / math.sqrt(d)


def num_threads():
    return int(_load().pbso_num_threads())


def key_scores(Q, K, block, scale=0.0):
    """Eq. 4 with group-averaged queries.  Q [B,Hq,N,d], K [B,Hkv,N,d] -> s [B,Hkv,N] float64."""
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    Q, qp = _f32(Q)
    K, kp = _f32(K)
    s = np.empty((B, Hkv, N), dtype=np.float64)
    rc = _load().pbso_key_scores(B, Hq, Hkv, N, d, int(block), ctypes.c_double(_scale(scale, d)), qp, kp, _f64p(s))
    if rc:
        raise RuntimeError("pbso_key_scores failed: %d" % rc)
    return s


def segment_argsort(s, segment):
    """Eq. 5 per segment, tail identity.  s [..., N] -> idx [..., N] int32 (gather form, absolute)."""
    s64 = np.ascontiguousarray(s, dtype=np.float64)
    N = s64.shape[-1]
    nbh = s64.size // N
    idx = np.empty(s64.shape, dtype=np.int32)
    rc = _load().pbso_segment_argsort(nbh, N, int(segment), _f64p(s64),
                                      idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc:
        raise RuntimeError("pbso_segment_argsort failed: %d" % rc)
    return idx


def gather_rows(X, idx):
    """X'[p] = X[idx[p]].  X [..., N, d] float32, idx [..., N]."""
    N, d = X.shape[-2:]
    X, xp = _f32(X)
    idx, ip = _i32(idx)
    out = np.empty_like(X)
    rc = _load().pbso_gather_rows(X.size // (N * d), N, d, xp, ip, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    if rc:
        raise RuntimeError("pbso_gather_rows failed: %d" % rc)
    return out


def scatter_rows(Op, idx):
    """O[idx[p]] = O'[p].  Op [..., N, d] float64, idx [..., N] or None (identity)."""
    N, d = Op.shape[-2:]
    Op = np.ascontiguousarray(Op, dtype=np.float64)
    out = np.empty_like(Op)
    ip = None
    if idx is not None:
        idx, ip = _i32(idx)
    rc = _load().pbso_scatter_rows(Op.size // (N * d), N, d, _f64p(Op), ip, _f64p(out))
    if rc:
        raise RuntimeError("pbso_scatter_rows failed: %d" % rc)
    return out


def block_mask(Qp, Kp, block, segment, tau, scale=0.0, flags=0, want_probs=False):
    """Algorithm 2 + forced blocks.  Returns (mask u8 [B,Hq,T,T], row_cnt, col_idx[, probs, k])."""
    B, Hq, N, d = Qp.shape
    Hkv = Kp.shape[1]
    T = -(-N // block)
    Qp, qp = _f32(Qp)
    Kp, kp = _f32(Kp)
    mask = np.empty((B, Hq, T, T), dtype=np.uint8)
    row_cnt = np.empty((B, Hq, T), dtype=np.int32)
    col_idx = np.empty((B, Hq, T, T), dtype=np.int32)
    probs = np.empty((B, Hq, T, T), dtype=np.float64) if want_probs else None
    kk = np.empty((B, Hq, T), dtype=np.int32) if want_probs else None
    rc = _load().pbso_block_mask(B, Hq, Hkv, N, d, int(block), int(segment), ctypes.c_double(float(tau)),
                                 ctypes.c_double(_scale(scale, d)), ctypes.c_uint(int(flags)), qp, kp,
                                 mask.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                 row_cnt.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                 col_idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                 _f64p(probs) if want_probs else None,
                                 kk.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) if want_probs else None)
    if rc:
        raise RuntimeError("pbso_block_mask failed: %d" % rc)
    return (mask, row_cnt, col_idx, probs, kk) if want_probs else (mask, row_cnt, col_idx)


def _attn_common(Qp, Kp, Vp, qidx, kidx, row_cnt, col_idx):
    Qp, qp = _f32(Qp)
    Kp, kp = _f32(Kp)
    Vp, vp = _f32(Vp)
    kidx, kip = _i32(kidx)
    qip = None
    if qidx is not None:
        qidx, qip = _i32(qidx)
    row_cnt, rcp = _i32(row_cnt)
    col_idx, cip = _i32(col_idx)
    keep = (Qp, Kp, Vp, qidx, kidx, row_cnt, col_idx)
    return keep, (qp, kp, vp, qip, kip, rcp, cip)


def attn_fwd(Qp, Kp, Vp, qidx, kidx, row_cnt, col_idx, block, scale=0.0, direct=False, want_lse=False):
    """Algorithm 1's masked online-softmax loop over the whole tensor -> O' [B,Hq,N,d] float64."""
    B, Hq, N, d = Qp.shape
    Hkv = Kp.shape[1]
    keep, ptrs = _attn_common(Qp, Kp, Vp, qidx, kidx, row_cnt, col_idx)
    out = np.zeros((B, Hq, N, d), dtype=np.float64)
    lse = np.zeros((B, Hq, N), dtype=np.float64) if want_lse else None
    rc = _load().pbso_attn_fwd(B, Hq, Hkv, N, d, int(block), ctypes.c_double(_scale(scale, d)), *ptrs,
                               int(bool(direct)), _f64p(out), _f64p(lse) if want_lse else None)
    if rc:
        raise RuntimeError("pbso_attn_fwd failed: %d" % rc)
    del keep
    return (out, lse) if want_lse else out


def attn_rows(Qp, Kp, Vp, qidx, kidx, row_cnt, col_idx, block, rows, scale=0.0, direct=False, want_lse=False):
    """Same, for sampled query blocks.  rows: int array [nrows, 3] of (b, hq, i) -> [nrows, block, d]."""
    B, Hq, N, d = Qp.shape
    Hkv = Kp.shape[1]
    keep, ptrs = _attn_common(Qp, Kp, Vp, qidx, kidx, row_cnt, col_idx)
    rows, rp = _i32(np.asarray(rows).reshape(-1, 3))
    out = np.zeros((rows.shape[0], block, d), dtype=np.float64)
    lse = np.zeros((rows.shape[0], block), dtype=np.float64) if want_lse else None
    rc = _load().pbso_attn_rows(B, Hq, Hkv, N, d, int(block), ctypes.c_double(_scale(scale, d)), *ptrs,
                                rows.shape[0], rp, int(bool(direct)), _f64p(out),
                                _f64p(lse) if want_lse else None)
    if rc:
        raise RuntimeError("pbso_attn_rows failed: %d" % rc)
    del keep
    return (out, lse) if want_lse else out


def all_allowed_lists(B, Hq, N, block, segment):
    """Block lists that name every key block the extended causal mask C admits (Section "Segmented Permutation
    for Causal Attention"): the whole own segment for query blocks of full segments, blocks 0..i in the tail."""
    T = -(-N // block)
    R, G = segment // block, N // segment
    i = np.arange(T)
    s = i // R
    allowed = np.where(s < G, np.minimum((s + 1) * R, T), i + 1).astype(np.int32)
    row_cnt = np.broadcast_to(allowed, (B, Hq, T)).copy()
    col_idx = np.broadcast_to(np.arange(T, dtype=np.int32), (B, Hq, T, T)).copy()
    return row_cnt, col_idx


def coverage(Qp, Kp, qidx, kidx, row_cnt, col_idx, block, segment, scale=0.0):
    """Attention mass captured by the listed blocks, per query slot [B,Hq,N]: the inner sums of the block-selection
    objective (Section "The Problem of Information Fragmentation"), with A the softmax over every visible key.
    Written as exp(lse over the listed blocks - lse over all admitted blocks)."""
    B, Hq, N, d = Qp.shape
    Vz = np.zeros_like(np.asarray(Kp, dtype=np.float32))
    _, lse_sel = attn_fwd(Qp, Kp, Vz, qidx, kidx, row_cnt, col_idx, block, scale, want_lse=True)
    rc_all, ci_all = all_allowed_lists(B, Hq, N, block, segment)
    _, lse_all = attn_fwd(Qp, Kp, Vz, qidx, kidx, rc_all, ci_all, block, scale, want_lse=True)
    with np.errstate(invalid="ignore"):
        cov = np.exp(lse_sel - lse_all)
    return np.where(np.isfinite(lse_sel), cov, 0.0)


def dense_causal(Q, K, V, scale=0.0):
    """Dense causal attention in the original token order -> O [B,Hq,N,d] float64."""
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    Q, qp = _f32(Q)
    K, kp = _f32(K)
    V, vp = _f32(V)
    out = np.empty((B, Hq, N, d), dtype=np.float64)
    rc = _load().pbso_dense_causal(B, Hq, Hkv, N, d, ctypes.c_double(_scale(scale, d)), qp, kp, vp, _f64p(out))
    if rc:
        raise RuntimeError("pbso_dense_causal failed: %d" % rc)
    return out


def pipeline(Q, K, V, block, segment, tau, scale=0.0, flags=0, qidx=None, score_dtype=np.float32):
    """Algorithm 1 end to end, each stage fed by the previous one.

    The score vector is rounded to `score_dtype` between Eq. 4 and Eq. 5 because
    that buffer is the hand-off between the two stages of the library under test.
    Returns a dict with every intermediate.
    """
    s = key_scores(Q, K, block, scale)
    s_h = s.astype(score_dtype)
    kidx = segment_argsort(s_h, segment)
    Kp = gather_rows(K, kidx)
    Vp = gather_rows(V, kidx)
    Qp = gather_rows(Q, qidx) if qidx is not None else np.ascontiguousarray(Q, dtype=np.float32)
    mask, row_cnt, col_idx = block_mask(Qp, Kp, block, segment, tau, scale, flags)
    Op, lse = attn_fwd(Qp, Kp, Vp, qidx, kidx, row_cnt, col_idx, block, scale, want_lse=True)
    O = scatter_rows(Op, qidx)
    return dict(s=s, s_handoff=s_h, kidx=kidx, Kp=Kp, Vp=Vp, Qp=Qp, mask=mask, row_cnt=row_cnt,
                col_idx=col_idx, Op=Op, lse=lse, O=O)
