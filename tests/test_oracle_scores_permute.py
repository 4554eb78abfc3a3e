"""Pins for the oracle's Eq. 4 (key scores) and Eq. 5 / segmented permutation.

The oracle is checked against things other than itself: closed forms worked by
hand, scipy/numpy library routines, invariants the paper states, and brute force
over all orders of a tiny segment.  CPU only.
"""
import itertools
import math

import numpy as np
import pytest
from scipy.special import softmax

from paper_2510_21270_amd import workloads as wl


# ---------------------------------------------------------------- Eq. 4
def test_scores_hand_case_two_keys(oracle):
    # one query q=1, d=1, keys 0 and ln3, scale 1: softmax([0, ln3]) = [1/4, 3/4]
    Q = np.array([[[[0.0], [1.0]]]], dtype=np.float32)            # [1,1,2,1]; the last block (B=1) is row 1
    K = np.array([[[[0.0], [np.float32(math.log(3.0))]]]], dtype=np.float32)
    s = oracle.key_scores(Q, K, block=1, scale=1.0)
    k1 = float(K[0, 0, 1, 0])
    want = np.array([1.0, math.exp(k1)]) / (1.0 + math.exp(k1))
    np.testing.assert_allclose(s[0, 0], want, rtol=1e-15)
    np.testing.assert_allclose(s[0, 0], [0.25, 0.75], rtol=1e-7)  # ln3 rounded to fp32


def test_scores_no_causal_mask_and_last_block_only(oracle):
    # A key placed AFTER every query of the last block's first row still gets mass (Eq. 4 has no mask),
    # and rows before the last block never matter.
    rng = np.random.default_rng(0)
    Q = rng.standard_normal((1, 1, 12, 4)).astype(np.float32)
    K = rng.standard_normal((1, 1, 12, 4)).astype(np.float32)
    s = oracle.key_scores(Q, K, block=4)
    assert (s > 0).all()
    Q2 = Q.copy()
    Q2[:, :, :8] = 99.0
    np.testing.assert_array_equal(oracle.key_scores(Q2, K, block=4), s)


@pytest.mark.parametrize("B,Hq,Hkv,N,d,block", [(1, 2, 2, 96, 16, 32), (2, 6, 2, 130, 8, 64), (1, 4, 1, 50, 32, 64)])
def test_scores_match_library_softmax(oracle, B, Hq, Hkv, N, d, block):
    rng = np.random.default_rng(7)
    Q = rng.standard_normal((B, Hq, N, d)).astype(np.float32)
    K = rng.standard_normal((B, Hkv, N, d)).astype(np.float32)
    s = oracle.key_scores(Q, K, block)
    r = Hq // Hkv
    bl = min(block, N)
    for b in range(B):
        for h in range(Hkv):
            qhat = Q[b, h * r:(h + 1) * r, N - bl:].astype(np.float64).mean(axis=0)       # group-averaged queries
            P = softmax(qhat @ K[b, h].astype(np.float64).T / math.sqrt(d), axis=1)
            np.testing.assert_allclose(s[b, h], P.mean(axis=0), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(s.sum(axis=-1), 1.0, rtol=1e-13)     # a mean of rows that each sum to one


def test_scores_gqa_is_query_averaging_not_score_averaging(oracle):
    # The two readings differ; pin which one the oracle implements with a case worked by hand:
    # two query heads q=+a and q=-a average to 0 -> uniform scores, whereas averaging per-head
    # score vectors would not be uniform.
    a = 3.0
    Q = np.tile(np.array([[[[a]], [[-a]]]], dtype=np.float32), (1, 1, 3, 1))     # [1,2,3,1]
    K = np.array([[[[1.0], [0.0], [-1.0]]]], dtype=np.float32)                   # [1,1,3,1]
    s = oracle.key_scores(Q, K, block=1, scale=1.0)
    np.testing.assert_allclose(s[0, 0], [1 / 3, 1 / 3, 1 / 3], rtol=1e-15)
    other = 0.5 * (softmax(a * K[0, 0, :, 0].astype(np.float64)) + softmax(-a * K[0, 0, :, 0].astype(np.float64)))
    assert abs(other[1] - 1 / 3) > 0.2                                           # the other reading is far away


# ---------------------------------------------------------------- Eq. 5 + segments
def test_argsort_matches_numpy_stable(oracle):
    rng = np.random.default_rng(3)
    N, S = 1000, 128
    s = rng.random((3, N))
    s[:, ::7] = s[:, 1::7][:, : s[:, ::7].shape[1]]                   # plant exact ties
    s32 = s.astype(np.float32)
    idx = oracle.segment_argsort(s32, S)
    G = N // S
    for bh in range(3):
        for g in range(G):
            want = g * S + np.argsort(-s32[bh, g * S:(g + 1) * S].astype(np.float64), kind="stable")
            np.testing.assert_array_equal(idx[bh, g * S:(g + 1) * S], want)
        np.testing.assert_array_equal(idx[bh, G * S:], np.arange(G * S, N))     # tail left unpermuted


def test_argsort_bijection_inside_each_segment(oracle):
    w = wl.c1_tiny(n=1500)
    s = oracle.key_scores(w.Q, w.K, w.block).astype(np.float32)
    idx = oracle.segment_argsort(s, w.segment)
    G = w.n // w.segment
    for bh in range(idx.shape[0] * idx.shape[1]):
        row = idx.reshape(-1, w.n)[bh]
        for g in range(G):
            seg = row[g * w.segment:(g + 1) * w.segment]
            np.testing.assert_array_equal(np.sort(seg), np.arange(g * w.segment, (g + 1) * w.segment))
        np.testing.assert_array_equal(row[G * w.segment:], np.arange(G * w.segment, w.n))


@pytest.mark.parametrize("S", [2, 3, 5, 6])
def test_argsort_brute_force_unique_order(oracle, S):
    # Enumerate all S! orders; exactly one is "descending score, equal scores by ascending index".
    rng = np.random.default_rng(S)
    for trial in range(6):
        s = rng.integers(0, 3, size=S).astype(np.float64)             # few distinct values -> many ties
        ok = [p for p in itertools.permutations(range(S))
              if all(s[p[t]] > s[p[t + 1]] or (s[p[t]] == s[p[t + 1]] and p[t] < p[t + 1]) for t in range(S - 1))]
        assert len(ok) == 1
        idx = oracle.segment_argsort(s[None, :], S)
        np.testing.assert_array_equal(idx[0], np.array(ok[0]))


def test_heavy_keys_lead_each_segment(oracle):
    # Gather form: slot 0 of a segment holds that segment's highest-scoring key
    # ("clusters heavy hitters into the leading blocks of each segment").
    s = np.array([[0.1, 0.9, 0.3, 0.2, 0.05, 0.6, 0.7, 0.01, 0.5]])
    idx = oracle.segment_argsort(s, 4)
    np.testing.assert_array_equal(idx[0], [1, 2, 3, 0, 6, 5, 4, 7, 8])


def test_gather_scatter_are_inverse(oracle):
    rng = np.random.default_rng(5)
    X = rng.standard_normal((2, 3, 40, 8)).astype(np.float32)
    idx = wl.random_segment_perm(11, 6, 40, 16).reshape(2, 3, 40)
    Xp = oracle.gather_rows(X, idx)
    for p in range(40):
        np.testing.assert_array_equal(Xp[1, 2, p], X[1, 2, idx[1, 2, p]])
    back = oracle.scatter_rows(Xp.astype(np.float64), idx)
    np.testing.assert_array_equal(back, X.astype(np.float64))
