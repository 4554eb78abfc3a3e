"""GPU parity: every stage of the HIP path against the fp64 oracle, element by element, through the C ABI.

Stage k on the GPU receives the ORACLE's stage k-1 output, so each comparison isolates one stage:
  - permutation indices, permuted tensors, masks and block lists: bit-exact;
  - key scores: by value (rel 2e-3 for the bf16 matrix-core path: bf16 products are exact, the error is fp32
    accumulation over d=128 plus exp2 on logits of magnitude <~ 30; rel 1e-5 for fp32 inputs, which accumulate
    in fp64 and only round the result to float32);
  - attention output: max-abs 2e-2 and mean-abs 2e-3 against fp64 for bf16, 1e-4 for fp32.
Sizes span several tiles, a partial last block and an unpermuted tail, and finish in seconds in the oracle.
"""
import numpy as np
import pytest
import torch

from gpu_helpers import (check_close, coverage, i32_dev, make_problem, mask_from_bits, to_dev, to_host, vt_layout)
from paper_2510_21270_amd import binding as pbs
from paper_2510_21270_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _case(name):
    if name == "c1":
        return wl.c1_tiny()                                                     # config 1 exactly
    if name == "bf16_b128":                                                     # Llama-like, GQA 2:1, ragged
        return wl.planted("bf16_b128", 11, 4, 2, 4096 + 77, 128, 128, 1024, 0.9, "bf16", 16, rope_base=5e5)
    if name == "bf16_b64":
        return wl.planted("bf16_b64", 12, 6, 2, 1000, 128, 64, 256, 0.8, "bf16", 8, rope_base=1e6)
    if name == "f32_d128":
        return wl.planted("f32_d128", 13, 2, 1, 300, 128, 32, 64, 0.7, "f32", 4)
    if name == "bf16_d64":
        return wl.planted("bf16_d64", 14, 4, 4, 530, 64, 16, 128, 0.9, "bf16", 4)
    if name == "f32_b128":
        return wl.planted("f32_b128", 15, 2, 2, 700, 64, 128, 256, 0.9, "f32", 4)
    if name == "bf16_even":                                                     # whole blocks: 5 segments + 3 tail blocks
        return wl.planted("bf16_even", 17, 4, 2, 5 * 1024 + 384, 128, 128, 1024, 0.6, "bf16", 16, rope_base=5e5)
    if name == "bf16_r7":                                                       # Qwen-like GQA 7:1, bursts, ragged
        return wl.planted("bf16_r7", 16, 7, 1, 1536 + 19, 128, 128, 512, 0.95, "bf16", 8, rope_base=1e6, bursts=2,
                          burst_len=16)
    raise KeyError(name)


CASES = ["c1", "bf16_b128", "bf16_b64", "f32_d128", "bf16_d64", "f32_b128", "bf16_r7"]
_cache = {}


@pytest.fixture(scope="module")
def lib():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return pbs.load_library()


def _oracle_run(oracle, name, sigma):
    key = (name, sigma)
    if key not in _cache:
        w = _case(name)
        qidx = wl.random_segment_perm(77, w.batch * w.h_q, w.n, w.segment).reshape(w.batch, w.h_q, w.n) if sigma else None
        res = oracle.pipeline(w.Q, w.K, w.V, w.block, w.segment, w.tau, flags=w.flags, qidx=qidx)
        res["qidx"] = qidx
        _cache[key] = (w, res)
    return _cache[key]


@pytest.mark.parametrize("name", CASES)
def test_key_scores(lib, oracle, name):
    w, res = _oracle_run(oracle, name, False)
    p = make_problem(w)
    s = pbs.key_scores(p, to_dev(w.Q, w.dtype), to_dev(w.K, w.dtype))
    torch.cuda.synchronize()
    got = s.cpu().numpy().astype(np.float64)
    rtol = 2e-3 if (w.dtype == "bf16" and w.d == 128) else 1e-5
    np.testing.assert_allclose(got, res["s"], rtol=rtol, atol=1e-37)
    np.testing.assert_allclose(got.sum(-1), 1.0, rtol=1e-3)


@pytest.mark.parametrize("name", CASES)
def test_segment_permute_bit_exact(lib, oracle, name):
    w, res = _oracle_run(oracle, name, False)
    p = make_problem(w)
    scores = torch.from_numpy(res["s_handoff"]).cuda()
    kidx, Kp, Vt = pbs.segment_permute(p, scores, to_dev(w.K, w.dtype), to_dev(w.V, w.dtype))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(kidx.cpu().numpy(), res["kidx"])
    np.testing.assert_array_equal(to_host(Kp), res["Kp"].astype(np.float64))
    np.testing.assert_array_equal(to_host(Vt), vt_layout(res["Vp"], w.block).astype(np.float64))
    # indices only
    kidx2, _, _ = pbs.segment_permute(p, scores, None, None, indices_only=True)
    assert torch.equal(kidx2, kidx)


@pytest.mark.parametrize("name", ["c1", "bf16_b128"])
def test_permute_rows_and_unpermute_bit_exact(lib, oracle, name):
    w, res = _oracle_run(oracle, name, True)
    p = make_problem(w)
    qidx = i32_dev(res["qidx"])
    Q = to_dev(w.Q, w.dtype)
    Qp = pbs.permute_rows(p, Q, qidx)
    np.testing.assert_array_equal(to_host(Qp), res["Qp"].astype(np.float64))
    back = pbs.unpermute(p, Qp, qidx)                 # P^T P = I
    assert torch.equal(back, Q)
    same = pbs.unpermute(p, Qp, None)                 # identity sigma: nothing to do
    assert same.data_ptr() == Qp.data_ptr()
    copy = pbs.unpermute(p, Qp, None, torch.empty_like(Qp))
    assert torch.equal(copy, Qp)


@pytest.mark.parametrize("sigma", [False, True])
@pytest.mark.parametrize("name", CASES)
def test_block_mask_bit_exact(lib, oracle, name, sigma):
    w, res = _oracle_run(oracle, name, sigma)
    p = make_problem(w)
    bits, cnt, cols = pbs.block_mask(p, to_dev(res["Qp"], w.dtype), to_dev(res["Kp"], w.dtype))
    torch.cuda.synchronize()
    T = w.T
    np.testing.assert_array_equal(mask_from_bits(bits, T), res["mask"])
    cnt_h = cnt.cpu().numpy()
    np.testing.assert_array_equal(cnt_h, res["row_cnt"])
    cols_h = cols.cpu().numpy()
    valid = np.arange(T)[None, None, None, :] < cnt_h[..., None]
    np.testing.assert_array_equal(np.where(valid, cols_h, -1), res["col_idx"])


@pytest.mark.parametrize("sigma", [False, True])
@pytest.mark.parametrize("name", CASES)
def test_attn_fwd_and_unpermute(lib, oracle, name, sigma):
    w, res = _oracle_run(oracle, name, sigma)
    p = make_problem(w)
    qidx = i32_dev(res["qidx"]) if sigma else None
    Op, lse = pbs.attn_fwd(p, to_dev(res["Qp"], w.dtype), to_dev(res["Kp"], w.dtype),
                           to_dev(vt_layout(res["Vp"], w.block), w.dtype), qidx, i32_dev(res["kidx"]),
                           i32_dev(res["row_cnt"]), i32_dev(res["col_idx"]), want_lse=True)
    O = pbs.unpermute(p, Op, qidx)
    torch.cuda.synchronize()
    check_close(to_host(Op), res["Op"], w.dtype, name + " O'")
    check_close(to_host(O), res["O"], w.dtype, name + " O")
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], rtol=0, atol=2e-2 if w.dtype == "bf16" else 1e-4)


@pytest.mark.parametrize("sigma", [False, True])
@pytest.mark.parametrize("name", ["c1", "bf16_b128", "bf16_b64", "bf16_r7"])
def test_coverage_of_the_selected_blocks(lib, oracle, name, sigma):
    # attention mass captured by the mask (two pbs_attn_fwd calls: listed blocks, all admitted blocks)
    w, res = _oracle_run(oracle, name, sigma)
    p = make_problem(w)
    qidx = i32_dev(res["qidx"]) if sigma else None
    got, rc_all, ci_all = coverage(p, to_dev(res["Qp"], w.dtype), to_dev(res["Kp"], w.dtype),
                                   to_dev(vt_layout(res["Vp"], w.block), w.dtype), qidx, i32_dev(res["kidx"]),
                                   i32_dev(res["row_cnt"]), i32_dev(res["col_idx"]))
    torch.cuda.synchronize()
    # the admitted lists are pure geometry: bit-exact against the oracle's
    rc_want, ci_want = oracle.all_allowed_lists(w.batch, w.h_q, w.n, w.block, w.segment)
    assert np.array_equal(rc_all.cpu().numpy(), rc_want)
    listed = np.arange(w.T)[None, None, None, :] < rc_want[..., None]
    assert np.array_equal(np.where(listed, ci_all.cpu().numpy(), -1), np.where(listed, ci_want, -1))
    want = oracle.coverage(res["Qp"], res["Kp"], res["qidx"], res["kidx"], res["row_cnt"], res["col_idx"], w.block,
                           w.segment)
    got = got.cpu().numpy()
    assert got.min() >= 0.0 and got.max() <= 1.0 + 1e-3
    np.testing.assert_allclose(got, want, rtol=0, atol=5e-3 if w.dtype == "bf16" else 1e-4)
    assert want.mean() > 0.5                            # tau >= 0.7 on pooled scores keeps most of the true mass here


@pytest.mark.parametrize("sigma", [False, True])
@pytest.mark.parametrize("name", ["bf16_b128", "bf16_b64", "bf16_even", "bf16_r7"])
def test_index_remapped_attention_reads_the_original_keys(lib, oracle, name, sigma):
    # PBS_FLAG_INDEX_REMAP (appendix "Memory Overhead"): no K' is materialised; the permutation stage writes kidx, Vt
    # and the block means of the permuted keys, selection runs from those means, and the attention kernel gathers its
    # K tiles from the caller's K through kidx.  Everything must match the oracle as with a materialised K', and the
    # output must equal, bit for bit, the same kernel reading a materialised K' (PBS_FLAG_RUNNING_MAX_ONLY).
    w, res = _oracle_run(oracle, name, sigma)
    p = make_problem(w, flags=w.flags | pbs.FLAG_INDEX_REMAP)
    pk = make_problem(w, flags=w.flags | pbs.FLAG_INDEX_REMAP | pbs.FLAG_KBAR_IN_WS)
    K, V = to_dev(w.K, w.dtype), to_dev(w.V, w.dtype)
    ws = pbs.alloc_workspace(p, pbs.STAGE_BLOCK_MASK)
    ws.fill_(0xFF)
    kidx, Kp, Vt = pbs.segment_permute(p, torch.from_numpy(res["s_handoff"]).cuda(), K, V, ws=ws)
    assert Kp is None
    np.testing.assert_array_equal(kidx.cpu().numpy(), res["kidx"])
    np.testing.assert_array_equal(to_host(Vt), vt_layout(res["Vp"], w.block).astype(np.float64))
    Qp = to_dev(res["Qp"], w.dtype)
    bits, cnt, cols = pbs.block_mask(pk, Qp, K, ws=ws)           # K is not read: the means are in ws
    np.testing.assert_array_equal(mask_from_bits(bits, w.T), res["mask"])
    np.testing.assert_array_equal(cnt.cpu().numpy(), res["row_cnt"])
    qd = i32_dev(res["qidx"]) if sigma else None
    Op, lse = pbs.attn_fwd(p, Qp, K, Vt, qd, kidx, cnt, cols, want_lse=True)
    torch.cuda.synchronize()
    check_close(to_host(Op), res["Op"], w.dtype, name + " O' with index remapping")
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], rtol=0, atol=2e-2)
    p_mat = make_problem(w, flags=w.flags | pbs.FLAG_RUNNING_MAX_ONLY)
    Om, lsem = pbs.attn_fwd(p_mat, Qp, to_dev(res["Kp"], w.dtype), Vt, qd, kidx, cnt, cols, want_lse=True)
    assert torch.equal(Op, Om) and torch.equal(lse, lsem)
    # shapes the remapping kernels do not serve are refused
    if name == "bf16_b128":
        import ctypes
        bad = pbs.problem(1, 2, 2, 256, 64, 64, 128, "bf16", flags=pbs.FLAG_INDEX_REMAP)
        x = torch.zeros(64, device="cuda")
        assert pbs.load_library().pbs_attn_fwd(ctypes.byref(bad), *([x.data_ptr()] * 3), None, *([x.data_ptr()] * 4),
                                                None, None, 0, None) == 3


@pytest.mark.parametrize("on_permuted_keys", [False, True])
@pytest.mark.parametrize("name", CASES + ["bf16_even"])
def test_key_aware_query_permutation(lib, oracle, oracle_variants, name, on_permuted_keys):
    # the ablation of Section "Design Choice: Why Permute Keys but not Queries?": sigma is an argmax followed by a
    # stable sort, all in fp64 with the plain operation order on both sides, so the indices must agree bit for bit;
    # then the whole path with this sigma doing real work (Q' gathered, mask on Q', attention with qidx, O scattered)
    w, res = _oracle_run(oracle, name, False)
    p = make_problem(w)
    keys_h = res["Kp"] if on_permuted_keys else np.asarray(w.K, dtype=np.float32)
    want = oracle_variants.query_permutation(w.Q, keys_h, w.block, w.segment)
    Q = to_dev(w.Q, w.dtype)
    qidx = pbs.query_permutation(p, Q, to_dev(keys_h, w.dtype))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(qidx.cpu().numpy(), want)
    if not on_permuted_keys:
        return
    full = (w.n // w.segment) * w.segment
    if full:
        assert not np.array_equal(want[0, 0, :full], np.arange(full))          # it does reorder something
    ref = oracle.pipeline(w.Q, w.K, w.V, w.block, w.segment, w.tau, flags=w.flags, qidx=want)
    Qp = pbs.permute_rows(p, Q, qidx)
    np.testing.assert_array_equal(to_host(Qp), ref["Qp"].astype(np.float64))
    Kp, Vt = to_dev(ref["Kp"], w.dtype), to_dev(vt_layout(ref["Vp"], w.block), w.dtype)
    bits, cnt, cols = pbs.block_mask(p, Qp, Kp)
    np.testing.assert_array_equal(mask_from_bits(bits, w.T), ref["mask"])
    Op = pbs.attn_fwd(p, Qp, Kp, Vt, qidx, i32_dev(ref["kidx"]), cnt, cols)
    O = pbs.unpermute(p, Op, qidx)
    torch.cuda.synchronize()
    check_close(to_host(O), ref["O"], w.dtype, name + " O with the key-aware sigma")


@pytest.mark.parametrize("proxy", ["last", "rows", "rows_few", "avg"])
@pytest.mark.parametrize("name", ["c1", "bf16_b128", "bf16_b64", "bf16_d64", "bf16_r7"])
def test_key_scores_from_other_proxies(lib, oracle, oracle_variants, name, proxy):
    # the proxies the paper ablates: Eq. 4 evaluated on other query rows (random positions, the average query)
    w, res = _oracle_run(oracle, name, False)
    p = make_problem(w)
    Q, K = to_dev(w.Q, w.dtype), to_dev(w.K, w.dtype)
    if proxy == "last":
        got = pbs.key_scores_proxy(p, pbs.PROXY_LAST_BLOCK, None, Q, K)
        want = res["s"]
    elif proxy == "avg":
        got = pbs.key_scores_proxy(p, pbs.PROXY_AVG_QUERY, None, Q, K)
        want = oracle_variants.key_scores_proxy(w.Q, w.K, None)
    else:
        rows = wl.random_query_rows(5, w.n, 128 if proxy == "rows" else 3)
        if proxy == "rows_few":
            rows = np.array([rows[2], rows[0], rows[2]], dtype=np.int32)      # unsorted, one position twice
        got = pbs.key_scores_proxy(p, pbs.PROXY_QUERY_ROWS, i32_dev(rows), Q, K)
        want = oracle_variants.key_scores_proxy(w.Q, w.K, rows)
    torch.cuda.synchronize()
    got = got.cpu().numpy().astype(np.float64)
    rtol = 2e-3 if (w.dtype == "bf16" and w.d == 128) else 1e-5
    np.testing.assert_allclose(got, want, rtol=rtol, atol=1e-37)
    np.testing.assert_allclose(got.sum(-1), 1.0, rtol=1e-3)
    if proxy == "last":                                                        # the same kernels as pbs_key_scores
        assert torch.equal(pbs.key_scores_proxy(p, pbs.PROXY_LAST_BLOCK, None, Q, K), pbs.key_scores(p, Q, K))


@pytest.mark.parametrize("token_copy", [False, True])
@pytest.mark.parametrize("name", CASES + ["bf16_even"])
def test_block_means_left_by_the_permutation_stage(lib, oracle, name, token_copy):
    # pbs_segment_permute with a workspace also leaves the fp64 block means of K' there (by the gather kernel itself
    # for 2-byte storage and blocks of whole 1024-chunk batches, by the pooling kernel otherwise); pbs_block_mask with
    # PBS_FLAG_KBAR_IN_WS then must select exactly what the oracle selects, without reading K' (a poisoned K' is passed)
    w, res = _oracle_run(oracle, name, False)
    p = make_problem(w, flags=w.flags | (pbs.FLAG_TOKEN_ORDER_COPY if token_copy else 0))
    pk = make_problem(w, flags=p.flags | pbs.FLAG_KBAR_IN_WS)
    ws = pbs.alloc_workspace(p, pbs.STAGE_BLOCK_MASK)
    ws.fill_(0xFF)                                                      # NaN patterns wherever nothing is written
    kidx, Kp, Vt = pbs.segment_permute(p, torch.from_numpy(res["s_handoff"]).cuda(), to_dev(w.K, w.dtype),
                                       to_dev(w.V, w.dtype), ws=ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(kidx.cpu().numpy(), res["kidx"])
    np.testing.assert_array_equal(to_host(Kp), res["Kp"].astype(np.float64))
    poisoned = torch.full_like(Kp, float("nan"))
    bits, cnt, cols = pbs.block_mask(pk, to_dev(res["Qp"], w.dtype), poisoned, ws=ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mask_from_bits(bits, w.T), res["mask"])
    np.testing.assert_array_equal(cnt.cpu().numpy(), res["row_cnt"])
    valid = np.arange(w.T)[None, None, None, :] < res["row_cnt"][..., None]
    np.testing.assert_array_equal(np.where(valid, cols.cpu().numpy(), -1), res["col_idx"])
    # a workspace that is too small is refused before anything is launched
    lib_ = pbs.load_library()
    import ctypes
    st = lib_.pbs_segment_permute(ctypes.byref(p), None, Kp.data_ptr(), Kp.data_ptr(), kidx.data_ptr(), Kp.data_ptr(),
                                  Vt.data_ptr(), ws.data_ptr(), 16, None)
    assert st == 4


@pytest.mark.parametrize("name", CASES)
def test_pipeline_composed(lib, oracle, name):
    """All five stages chained on the GPU.  GPU scores are only close to the oracle's, so near-tied keys may swap
    places: index and mask agreement with the oracle chain is reported and every index disagreement must be a
    near-tie under the oracle's scores (config 1, fp32 inputs with fp64 accumulation, must agree exactly).
    The output is then checked against the oracle's attention evaluated on the GPU's own discrete decisions
    (its permutation and block lists), which is what the composed path promises."""
    w, res = _oracle_run(oracle, name, False)
    p = make_problem(w)
    pipe = pbs.Pipeline(p)
    O = pipe.run(to_dev(w.Q, w.dtype), to_dev(w.K, w.dtype), to_dev(w.V, w.dtype))
    torch.cuda.synchronize()
    kidx = pipe.kidx.cpu().numpy()
    agree = float((kidx == res["kidx"]).mean())
    mask = mask_from_bits(pipe.mask_bits, w.T)
    magree = float((mask == res["mask"]).mean())
    print("%s: index agreement %.6f, mask agreement %.6f" % (name, agree, magree))
    if w.dtype == "f32":
        assert agree == 1.0 and magree == 1.0
    else:
        s = res["s"]
        for b_, h_, pos in np.argwhere(kidx != res["kidx"])[:2000]:
            a, c = s[b_, h_, kidx[b_, h_, pos]], s[b_, h_, res["kidx"][b_, h_, pos]]
            assert abs(a - c) <= 4e-3 * max(abs(a), abs(c)) + 1e-37
    # the GPU's permutation is a valid segmented permutation
    G = w.n // w.segment
    srt = np.sort(kidx[..., :G * w.segment].reshape(w.batch, w.h_kv, G, w.segment), axis=-1)
    assert (srt == np.arange(G * w.segment).reshape(G, w.segment)).all()
    assert (kidx[..., G * w.segment:] == np.arange(G * w.segment, w.n)).all()
    cnt = pipe.row_cnt.cpu().numpy()
    cols = np.where(np.arange(w.T)[None, None, None, :] < cnt[..., None], pipe.col_idx.cpu().numpy(), -1)
    Kp, Vp = oracle.gather_rows(w.K, kidx), oracle.gather_rows(w.V, kidx)
    want = oracle.attn_fwd(w.Q, Kp, Vp, None, kidx, cnt, cols, w.block)
    check_close(to_host(O), want, w.dtype, name + " pipeline O")


def test_determinism(lib, oracle):
    w, res = _oracle_run(oracle, "bf16_b128", False)
    p = make_problem(w)
    Q, K, V = to_dev(w.Q, w.dtype), to_dev(w.K, w.dtype), to_dev(w.V, w.dtype)
    pipe = pbs.Pipeline(p)
    o1 = pipe.run(Q, K, V).clone()
    s1, k1, m1 = pipe.scores.clone(), pipe.kidx.clone(), pipe.mask_bits.clone()
    o2 = pipe.run(Q, K, V)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(s1, pipe.scores) and torch.equal(k1, pipe.kidx)
    assert torch.equal(m1, pipe.mask_bits)


def _random_shape(seed, wide):
    """A seeded random problem: the matrix-core path for block 128 (wide) or any supported combination."""
    rng = np.random.default_rng(1000 + seed)
    if wide:
        dtype, d, block = "bf16", 128, 128
        segment = int(rng.choice([128, 256, 512, 1024]))
        n = int(rng.integers(1, 2600))
    else:
        dtype = str(rng.choice(["bf16", "f32"]))
        d = int(rng.choice([64, 128]))
        block = int(rng.choice([16, 32, 64, 128]))
        segment = block * int(rng.choice([1, 2, 4, 8]))
        n = int(rng.integers(1, 900))
    h_kv = int(rng.choice([1, 2, 3]))
    h_q = h_kv * int(rng.choice([1, 2, 4]))
    tau = float(rng.choice([0.3, 0.6, 0.9, 0.99]))
    flags = int(rng.integers(0, 2))
    batch = int(rng.choice([1, 2, 3]))
    return wl.planted("rnd%d" % seed, 500 + seed, h_q, h_kv, n, d, block, segment, tau, dtype, 4,
                      rope_base=5e5 if seed % 2 else None, flags=flags, batch=batch)


@pytest.mark.parametrize("wide", [True, False])
@pytest.mark.parametrize("seed", range(30))
def test_random_shapes_stage_by_stage(lib, oracle, seed, wide):
    # every stage on the oracle's output of the stage before, for shapes no other test names
    w = _random_shape(seed, wide)
    sigma = seed % 3 == 0
    qidx = wl.random_segment_perm(seed, w.batch * w.h_q, w.n, w.segment).reshape(w.batch, w.h_q, w.n) if sigma else None
    scale = [0.0, float(np.float32(0.05)), float(np.float32(0.2))][seed % 3]   # 0 = the default 1 / sqrt(d); else a float
    res = oracle.pipeline(w.Q, w.K, w.V, w.block, w.segment, w.tau, scale=scale, flags=w.flags, qidx=qidx)
    p = make_problem(w, scale=scale)
    what = "%s batch=%d n=%d hq=%d hkv=%d d=%d block=%d segment=%d tau=%g flags=%d sigma=%s scale=%g" % (
        w.dtype, w.batch, w.n, w.h_q, w.h_kv, w.d, w.block, w.segment, w.tau, w.flags, sigma, scale)
    s = pbs.key_scores(p, to_dev(w.Q, w.dtype), to_dev(w.K, w.dtype)).cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(s, res["s"], rtol=2e-3 if (w.dtype == "bf16" and w.d == 128) else 1e-5, atol=1e-37,
                               err_msg=what)
    kidx, Kp, Vt = pbs.segment_permute(p, torch.from_numpy(res["s_handoff"]).cuda(), to_dev(w.K, w.dtype),
                                       to_dev(w.V, w.dtype))
    np.testing.assert_array_equal(kidx.cpu().numpy(), res["kidx"], err_msg=what)
    np.testing.assert_array_equal(to_host(Kp), res["Kp"].astype(np.float64), err_msg=what)
    np.testing.assert_array_equal(to_host(Vt), vt_layout(res["Vp"], w.block).astype(np.float64), err_msg=what)
    bits, cnt, cols = pbs.block_mask(p, to_dev(res["Qp"], w.dtype), Kp)
    np.testing.assert_array_equal(mask_from_bits(bits, w.T), res["mask"], err_msg=what)
    np.testing.assert_array_equal(cnt.cpu().numpy(), res["row_cnt"], err_msg=what)
    qd = i32_dev(qidx) if sigma else None
    Op, lse = pbs.attn_fwd(p, to_dev(res["Qp"], w.dtype), Kp, Vt, qd, kidx, cnt, cols, want_lse=True)
    O = pbs.unpermute(p, Op, qd)
    torch.cuda.synchronize()
    check_close(to_host(Op), res["Op"], w.dtype, what + " O'")
    check_close(to_host(O), res["O"], w.dtype, what + " O")
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], rtol=0, atol=2e-2 if w.dtype == "bf16" else 1e-4,
                               err_msg=what)


@pytest.mark.parametrize("name", ["bf16_even", "bf16_b128", "bf16_b64", "f32_d128"])
def test_token_order_copy_of_the_own_segment(lib, oracle, name):
    # PBS_FLAG_TOKEN_ORDER_COPY: the permutation stage writes K, V'^T and kidx a second time in token order, and the
    # 64-queries-per-wave attention kernel takes a query block's own segment from that copy (bf16_even: whole blocks;
    # bf16_b128: a ragged last block; the other cases write the copy and must ignore it).  Same visible keys, so the
    # oracle's O and lse must be met to the same tolerance; where the copy is ignored the output is bit-identical.
    w, res = _oracle_run(oracle, name, False)
    p0 = make_problem(w)
    p1 = make_problem(w, flags=w.flags | pbs.FLAG_TOKEN_ORDER_COPY)
    assert pbs.vt_bytes(p1) == 2 * pbs.vt_bytes(p0)
    K, V = to_dev(w.K, w.dtype), to_dev(w.V, w.dtype)
    scores = torch.from_numpy(res["s_handoff"]).cuda()
    kidx, Kp, Vt = pbs.segment_permute(p1, scores, K, V)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(kidx.cpu().numpy(), res["kidx"])
    np.testing.assert_array_equal(to_host(Kp), res["Kp"].astype(np.float64))
    np.testing.assert_array_equal(to_host(Vt), vt_layout(res["Vp"], w.block).astype(np.float64))
    iota = torch.arange(w.n, device="cuda", dtype=torch.int32).expand(w.batch, w.h_kv, w.n)
    assert torch.equal(pbs.token_copy(p1, kidx, 1), iota)
    assert torch.equal(pbs.token_copy(p1, Kp, w.d), K)
    np.testing.assert_array_equal(to_host(pbs.token_copy(p1, Vt, w.d)), vt_layout(w.V, w.block).astype(np.float64))
    kidx2 = pbs.alloc_kidx(p1)
    pbs.segment_permute(p1, scores, None, None, kidx=kidx2, indices_only=True)
    assert torch.equal(kidx2, kidx) and torch.equal(pbs.token_copy(p1, kidx2, 1), iota)
    # selection reads the permuted tensors only
    bits, cnt, cols = pbs.block_mask(p1, to_dev(res["Qp"], w.dtype), Kp)
    np.testing.assert_array_equal(cnt.cpu().numpy(), res["row_cnt"])
    # attention on the oracle's lists
    Q = to_dev(res["Qp"], w.dtype)
    rc, ci = i32_dev(res["row_cnt"]), i32_dev(res["col_idx"])
    O1, lse1 = pbs.attn_fwd(p1, Q, Kp, Vt, None, kidx, rc, ci, want_lse=True)
    O0, lse0 = pbs.attn_fwd(p0, Q, Kp, Vt, None, kidx, rc, ci, want_lse=True)
    torch.cuda.synchronize()
    check_close(to_host(O1), res["Op"], w.dtype, name + " O' with the token-order copy")
    np.testing.assert_allclose(lse1.cpu().numpy(), res["lse"], rtol=0, atol=2e-2 if w.dtype == "bf16" else 1e-4)
    if name in ("bf16_even", "bf16_b128"):
        assert not torch.equal(O1, O0)                       # a different order of the sums: the copy was used
        # lists in descending order do not end with the own segment: processed as listed, bit for bit
        T = w.T
        ar = torch.arange(T, device="cuda").view(1, 1, 1, T)
        src = torch.clamp(rc.unsqueeze(-1).long() - 1 - ar, min=0)
        rev = torch.where(ar < rc.unsqueeze(-1), torch.gather(ci, 3, src), ci)
        R1 = pbs.attn_fwd(p1, Q, Kp, Vt, None, kidx, rc, rev)
        R0 = pbs.attn_fwd(p0, Q, Kp, Vt, None, kidx, rc, rev)
        assert torch.equal(R1, R0)
        # a caller-supplied sigma switches the shortcut off as well
        sig = i32_dev(wl.random_segment_perm(5, w.batch * w.h_q, w.n, w.segment).reshape(w.batch, w.h_q, w.n))
        S1 = pbs.attn_fwd(p1, Q, Kp, Vt, sig, kidx, rc, ci)
        S0 = pbs.attn_fwd(p0, Q, Kp, Vt, sig, kidx, rc, ci)
        assert torch.equal(S1, S0)
    else:
        assert torch.equal(O1, O0) and torch.equal(lse1, lse0)
    # the composed pipeline with the flag
    pipe = pbs.Pipeline(p1)
    O = pipe.run(to_dev(w.Q, w.dtype), K, V)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all()


@pytest.mark.parametrize("seed", range(12))
def test_token_order_copy_on_random_shapes(lib, oracle, seed):
    # seeded shapes on which the copy is used: segments of 1 to 8 blocks, with and without an unpermuted tail, whole
    # blocks or a ragged last one, batches of one or two, GQA groups of 1, 2 or 4
    rng = np.random.default_rng(3000 + seed)
    segment = int(rng.choice([128, 256, 512, 1024]))
    n = 128 * int(rng.integers(1, 25)) + (int(rng.integers(1, 128)) if seed % 3 == 0 else 0)
    h_kv = int(rng.choice([1, 2, 3]))
    h_q = h_kv * int(rng.choice([1, 2, 4]))
    tau = float(rng.choice([0.3, 0.6, 0.9]))
    w = wl.planted("tok%d" % seed, 700 + seed, h_q, h_kv, n, 128, 128, segment, tau, "bf16", 4,
                   rope_base=5e5 if seed % 2 else None, flags=int(rng.integers(0, 2)), batch=int(rng.choice([1, 2])))
    res = oracle.pipeline(w.Q, w.K, w.V, w.block, w.segment, w.tau, flags=w.flags)
    p = make_problem(w, flags=w.flags | pbs.FLAG_TOKEN_ORDER_COPY)
    what = "batch=%d n=%d hq=%d hkv=%d segment=%d tau=%g flags=%d" % (w.batch, n, h_q, h_kv, segment, tau, w.flags)
    kidx, Kp, Vt = pbs.segment_permute(p, torch.from_numpy(res["s_handoff"]).cuda(), to_dev(w.K, "bf16"),
                                       to_dev(w.V, "bf16"))
    np.testing.assert_array_equal(kidx.cpu().numpy(), res["kidx"], err_msg=what)
    bits, cnt, cols = pbs.block_mask(p, to_dev(res["Qp"], "bf16"), Kp)
    np.testing.assert_array_equal(mask_from_bits(bits, w.T), res["mask"], err_msg=what)
    np.testing.assert_array_equal(cnt.cpu().numpy(), res["row_cnt"], err_msg=what)
    Op, lse = pbs.attn_fwd(p, to_dev(res["Qp"], "bf16"), Kp, Vt, None, kidx, cnt, cols, want_lse=True)
    torch.cuda.synchronize()
    check_close(to_host(Op), res["Op"], "bf16", what + " O'")
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], rtol=0, atol=2e-2, err_msg=what)
