"""Pins of the variant oracle (oracle/pbs_oracle_variants.c) against things other than itself: scipy's softmax, closed
forms and hand cases for the proxy scores; a numpy cosine-similarity brute force, planted clusters, invariants and
Theorem 1 for the key-aware query permutation."""
import numpy as np
import pytest
from scipy.special import softmax

from paper_2510_21270_amd import workloads as wl


def _rand(seed, *shape):
    return wl.round_to_bf16(np.random.default_rng(seed).standard_normal(shape).astype(np.float32))


# ------------------------------------------------------------------ proxies for the importance score
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (6, 2)])
def test_proxy_scores_from_given_rows_equal_scipy_softmax(oracle_variants, Hq, Hkv):
    # section "The Problem of Information Fragmentation", heuristic 4 / appendix "Task-wise Proxy Sensitivity":
    # mean over the chosen query rows of softmax(q K^T / sqrt(d)), group queries averaged first
    B, N, d = 2, 97, 16
    Q, K = _rand(1, B, Hq, N, d), _rand(2, B, Hkv, N, d)
    rows = np.array([3, 96, 40, 40, 0], dtype=np.int32)              # unsorted, one row twice
    got = oracle_variants.key_scores_proxy(Q, K, rows)
    r = Hq // Hkv
    Qg = Q.astype(np.float64).reshape(B, Hkv, r, N, d).mean(axis=2)  # [B,Hkv,N,d]
    L = np.einsum("bhtd,bhjd->bhtj", Qg[:, :, rows], K.astype(np.float64)) / np.sqrt(d)
    want = softmax(L, axis=-1).mean(axis=2)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(got.sum(-1), 1.0, rtol=1e-12)


def test_proxy_with_the_last_block_rows_is_eq4_and_row_order_does_not_matter(oracle, oracle_variants):
    B, Hq, Hkv, N, d, block = 1, 4, 2, 150, 32, 64
    Q, K = _rand(3, B, Hq, N, d), _rand(4, B, Hkv, N, d)
    last = np.arange(N - block, N, dtype=np.int32)
    want = oracle.key_scores(Q, K, block)                            # Eq. 4 (pinned on its own elsewhere)
    np.testing.assert_allclose(oracle_variants.key_scores_proxy(Q, K, last), want, rtol=1e-13)
    perm = np.random.default_rng(0).permutation(last)
    np.testing.assert_allclose(oracle_variants.key_scores_proxy(Q, K, perm), want, rtol=1e-12)
    # a row listed twice counts twice: [a, a, b] = (2 s_a + s_b) / 3
    sa = oracle_variants.key_scores_proxy(Q, K, np.array([7], dtype=np.int32))
    sb = oracle_variants.key_scores_proxy(Q, K, np.array([90], dtype=np.int32))
    saab = oracle_variants.key_scores_proxy(Q, K, np.array([7, 90, 7], dtype=np.int32))
    np.testing.assert_allclose(saab, (2 * sa + sb) / 3, rtol=1e-13)


def test_single_query_two_keys_is_the_logistic_function(oracle_variants):
    # one query, two keys: s = (sigmoid(x), 1 - sigmoid(x)) with x = (q.k0 - q.k1) * scale
    d = 4
    Q = np.zeros((1, 1, 2, d), dtype=np.float32)
    K = np.zeros((1, 1, 2, d), dtype=np.float32)
    Q[0, 0, 1] = [1.0, 2.0, 0.0, -1.0]
    K[0, 0, 0] = [0.5, 0.25, 3.0, 0.0]
    K[0, 0, 1] = [-1.0, 0.5, 1.0, 2.0]
    q64 = Q[0, 0, 1].astype(np.float64)
    x = (q64 @ K[0, 0, 0].astype(np.float64) - q64 @ K[0, 0, 1].astype(np.float64)) * 0.75
    got = oracle_variants.key_scores_proxy(Q, K, np.array([1], dtype=np.int32), scale=0.75)
    np.testing.assert_allclose(got[0, 0], [1 / (1 + np.exp(-x)), 1 / (1 + np.exp(x))], rtol=1e-14)


def test_average_query_proxy(oracle_variants):
    # reading of "Avg-Query-Attn": softmax of the mean query (over all positions and the group's heads) against all keys
    B, Hq, Hkv, N, d = 2, 4, 2, 61, 8
    Q, K = _rand(5, B, Hq, N, d), _rand(6, B, Hkv, N, d)
    got = oracle_variants.key_scores_proxy(Q, K, None)
    qbar = Q.astype(np.float64).reshape(B, Hkv, 2, N, d).mean(axis=(2, 3))         # [B,Hkv,d]
    want = softmax(np.einsum("bhd,bhjd->bhj", qbar, K.astype(np.float64)) / np.sqrt(d), axis=-1)
    np.testing.assert_allclose(got, want, rtol=1e-12)
    # queries that cancel: the average query is the zero vector and every key scores exactly 1/n
    Qz = np.concatenate([Q[:, :, :30], -Q[:, :, :30]], axis=2)
    Kz = K[:, :, :60]
    np.testing.assert_array_equal(oracle_variants.key_scores_proxy(Qz, Kz, None), np.full((B, Hkv, 60), 1.0 / 60))


# ------------------------------------------------------------------ key-aware query permutation
def _brute_assign(Q, K, block, segment):
    """numpy restatement with explicit cosines: normalise every vector, take the dot products, argmax over the
    centroids of the blocks the segment may see."""
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    r = Hq // Hkv
    T, R, G = -(-N // block), segment // block, N // segment
    out = np.full((B, Hq, N), -1, dtype=np.int32)
    for b in range(B):
        for hq in range(Hq):
            Kh = K[b, hq // r].astype(np.float64)
            cent = np.stack([Kh[j * block:min(N, (j + 1) * block)].mean(axis=0) for j in range(T)])
            cn = np.linalg.norm(cent, axis=1, keepdims=True)
            cent_unit = np.divide(cent, cn, out=np.zeros_like(cent), where=cn > 0)
            for t in range(G * segment):
                q = Q[b, hq, t].astype(np.float64)
                qn = np.linalg.norm(q)
                ncand = min((t // segment + 1) * R, T)
                cos = cent_unit[:ncand] @ (q / qn if qn > 0 else q)
                out[b, hq, t] = int(np.argmax(cos))
    return out


@pytest.mark.parametrize("N,block,segment,Hq,Hkv", [(96, 8, 32, 2, 1), (77, 4, 16, 4, 2), (40, 8, 8, 1, 1)])
def test_assignment_equals_cosine_brute_force_and_sigma_sorts_by_it(oracle_variants, N, block, segment, Hq, Hkv):
    d = 8
    Q, K = _rand(11, 1, Hq, N, d), _rand(12, 1, Hkv, N, d)
    qidx, assigned = oracle_variants.query_permutation(Q, K, block, segment, want_assigned=True)
    np.testing.assert_array_equal(assigned, _brute_assign(Q, K, block, segment))
    G = N // segment
    for h in range(Hq):
        for g in range(G):
            seg = np.arange(g * segment, (g + 1) * segment)
            # stable ascending order of the assigned centroid = numpy's stable argsort
            want = seg[np.argsort(assigned[0, h, seg], kind="stable")]
            np.testing.assert_array_equal(qidx[0, h, seg], want)
            assert sorted(qidx[0, h, seg].tolist()) == seg.tolist()              # a bijection of the segment
        np.testing.assert_array_equal(qidx[0, h, G * segment:], np.arange(G * segment, N))   # the tail stays


@pytest.mark.parametrize("N,block,segment,Hq,Hkv", [(96, 8, 32, 2, 1), (77, 4, 16, 4, 2)])
def test_one_segment_at_a_time_equals_the_brute_force_order(oracle_variants, N, block, segment, Hq, Hkv):
    # the per-segment entry (what the full-length GPU test can afford) against the numpy brute force, not against the
    # whole-sequence entry: assignment by cosine argmax, then numpy's stable argsort
    d = 8
    Q, K = _rand(21, 1, Hq, N, d), _rand(22, 1, Hkv, N, d)
    brute = _brute_assign(Q, K, block, segment)
    for g in range(N // segment):
        seg = np.arange(g * segment, (g + 1) * segment)
        got = oracle_variants.query_permutation_segment(Q, K, block, segment, g)
        for h in range(Hq):
            np.testing.assert_array_equal(got[0, h], seg[np.argsort(brute[0, h, seg], kind="stable")])
    with pytest.raises(RuntimeError):
        oracle_variants.query_permutation_segment(Q, K, block, segment, N // segment)     # not a full segment


def test_planted_clusters_are_recovered(oracle_variants):
    # keys: block j points along axis j (plus small noise); queries: positive multiples of a chosen axis.
    # Every query must be assigned to the block of its axis, unless that block lies in a later segment.
    block, segment, d, T = 4, 16, 16, 12
    N = T * block
    rng = np.random.default_rng(21)
    K = np.zeros((1, 1, N, d), dtype=np.float32)
    for j in range(T):
        K[0, 0, j * block:(j + 1) * block, j] = 1.0 + 0.25 * rng.random(block)
    K += 0.01 * rng.standard_normal(K.shape).astype(np.float32)
    Q = np.zeros((1, 1, N, d), dtype=np.float32)
    want = np.zeros(N, dtype=np.int32)
    for t in range(N):
        ncand = (t // segment + 1) * (segment // block)
        want[t] = rng.integers(0, ncand)
        Q[0, 0, t, want[t]] = 0.5 + rng.random()
    K, Q = wl.round_to_bf16(K), wl.round_to_bf16(Q)
    qidx, assigned = oracle_variants.query_permutation(Q, K, block, segment, want_assigned=True)
    np.testing.assert_array_equal(assigned[0, 0], want)
    # a negative multiple is the LEAST similar direction: never assigned to that block
    Qn = -Q
    _, assigned_n = oracle_variants.query_permutation(Qn, K, block, segment, want_assigned=True)
    assert not np.any(assigned_n[0, 0] == want)
    # a query of segment 0 that points at a block of segment 1 cannot be assigned to it (not visible to its segment)
    Q2 = Q.copy()
    Q2[0, 0, 3] = 0.0
    Q2[0, 0, 3, 6] = 1.0                                             # block 6 lies in segment 1
    _, a2 = oracle_variants.query_permutation(Q2, K, block, segment, want_assigned=True)
    assert a2[0, 0, 3] < segment // block


def test_identity_when_every_query_prefers_the_same_block_and_zero_centroids_score_zero(oracle_variants):
    block, segment, d = 4, 16, 8
    N = 3 * segment + 5
    rng = np.random.default_rng(31)
    K = -np.abs(_rand(32, 1, 1, N, d))                               # every other block points away from the queries
    K[0, 0, :block] = 5.0                                            # block 0 is the only centroid with a positive cosine
    Q = np.abs(_rand(33, 1, 2, N, d)) + 1.0
    qidx, assigned = oracle_variants.query_permutation(Q, wl.round_to_bf16(K), block, segment, want_assigned=True)
    assert np.all(assigned[:, :, :3 * segment] == 0) and np.all(assigned[:, :, 3 * segment:] == -1)
    np.testing.assert_array_equal(qidx, np.broadcast_to(np.arange(N, dtype=np.int32), qidx.shape))   # stable: identity
    # a block of zero keys has similarity 0: it wins against negative similarities and loses against positive ones
    Kz = np.zeros((1, 1, 8, 2), dtype=np.float32)
    Kz[0, 0, 4:] = [1.0, 0.0]                                        # block 0 = zero vector, block 1 = +x
    Qz = np.zeros((1, 1, 8, 2), dtype=np.float32)
    Qz[0, 0, :4] = [-1.0, 0.5]                                       # cos with block 1 negative -> block 0 (u = 0) wins
    Qz[0, 0, 4:] = [1.0, 0.5]                                        # cos with block 1 positive -> block 1
    _, az = oracle_variants.query_permutation(Qz, Kz, 4, 8, want_assigned=True)
    np.testing.assert_array_equal(az[0, 0], [0, 0, 0, 0, 1, 1, 1, 1])


def test_theorem_1_holds_with_the_key_aware_sigma(oracle, oracle_variants):
    # Theorem 1: permuting queries by sigma and keys by pi inside segments, attending over every admitted block and
    # undoing sigma gives dense causal attention, whatever sigma and pi are; here sigma is the key-aware one computed
    # on the permuted keys
    B, Hq, Hkv, N, d, block, segment = 1, 2, 1, 96, 8, 8, 32
    Q, K, V = _rand(41, B, Hq, N, d), _rand(42, B, Hkv, N, d), _rand(43, B, Hkv, N, d)
    kidx = oracle.segment_argsort(oracle.key_scores(Q, K, block).astype(np.float32), segment)
    Kp, Vp = oracle.gather_rows(K, kidx), oracle.gather_rows(V, kidx)
    qidx = oracle_variants.query_permutation(Q, Kp, block, segment)
    assert not np.array_equal(qidx[0, 0], np.arange(N))
    Qp = oracle.gather_rows(Q, qidx)
    rc, ci = oracle.all_allowed_lists(B, Hq, N, block, segment)
    Op = oracle.attn_fwd(Qp, Kp, Vp, qidx, kidx, rc, ci, block)
    O = oracle.scatter_rows(Op, qidx)
    np.testing.assert_allclose(O, oracle.dense_causal(Q, K, V), rtol=0, atol=1e-12)
