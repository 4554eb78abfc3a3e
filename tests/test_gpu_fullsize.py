"""GPU parity at the FULL sizes of configs 2, 3 (Llama-3.1-8B-shaped layer, N = 32768 and N = 131072), 4 (Qwen2.5-7B-
shaped, N = 65536, GQA 7:1) and 5 (caller-supplied lists at N = 65536), in the launch configuration bench.py times (the same binding calls on the same preallocated Pipeline buffers).

Discrete outputs (permutation indices, permuted tensors, block masks, block lists) are compared in full and must be
bit-exact.  The attention output is compared on SAMPLED query blocks that the oracle computes one by one: first
block, last block, blocks at segment edges and random ones, spread over the query heads.  Every stage is fed the
oracle's previous stage, so each comparison isolates one stage.
"""
import numpy as np
import pytest
import torch

from gpu_helpers import (check_close, i32_dev, make_problem, mask_from_bits, to_dev, to_host, vt_layout,
                         with_token_copy)
from paper_2510_21270_amd import binding as pbs
from paper_2510_21270_amd import workloads as wl

pytestmark = pytest.mark.gpu
_state = {}


def _setup(name, oracle):
    """Generate the workload, run the oracle's stages 1-3 in full, upload, and keep everything for the tests."""
    if name in _state:
        return _state[name]
    _state.clear()                                   # one full-size workload in memory at a time
    torch.cuda.empty_cache()
    w = {"c2": wl.c2_llama, "c3": wl.c3_llama128k, "c4": wl.c4_qwen}[name]()
    s = oracle.key_scores(w.Q, w.K, w.block)
    s_h = s.astype(np.float32)
    kidx = oracle.segment_argsort(s_h, w.segment)
    Kp, Vp = oracle.gather_rows(w.K, kidx), oracle.gather_rows(w.V, kidx)
    mask, row_cnt, col_idx = oracle.block_mask(w.Q, Kp, w.block, w.segment, w.tau, flags=w.flags)
    p = make_problem(w)
    st = dict(w=w, p=p, s=s, s_h=s_h, kidx=kidx, Kp=Kp, Vp=Vp, mask=mask, row_cnt=row_cnt, col_idx=col_idx,
              Q=to_dev(w.Q, "bf16"), K=to_dev(w.K, "bf16"), V=to_dev(w.V, "bf16"), pipe=pbs.Pipeline(p))
    _state[name] = st
    return st


@pytest.mark.parametrize("name", ["c2", "c4", "c3"])
def test_full_size_scores_permutation_and_mask(oracle, name):
    st = _setup(name, oracle)
    w, p, pipe = st["w"], st["p"], st["pipe"]
    # stage 1: by value
    pbs.key_scores(p, st["Q"], st["K"], pipe.scores, pipe.ws1)
    torch.cuda.synchronize()
    got = pipe.scores.cpu().numpy().astype(np.float64)
    np.testing.assert_allclose(got, st["s"], rtol=2e-3, atol=1e-37)
    np.testing.assert_allclose(got.sum(-1), 1.0, rtol=1e-3)
    # stage 2 on the oracle's scores: bit-exact indices and permuted tensors
    pbs.segment_permute(p, torch.from_numpy(st["s_h"]).cuda(), st["K"], st["V"], pipe.kidx, pipe.Kp, pipe.Vt)
    torch.cuda.synchronize()
    assert np.array_equal(pipe.kidx.cpu().numpy(), st["kidx"])
    assert torch.equal(pipe.Kp, to_dev(st["Kp"], "bf16"))
    assert torch.equal(pipe.Vt, to_dev(vt_layout(st["Vp"], w.block), "bf16"))
    # stage 3 on the oracle's K': bit-exact mask and lists
    pbs.block_mask(p, st["Q"], pipe.Kp, pipe.mask_bits, pipe.row_cnt, pipe.col_idx, pipe.ws3)
    torch.cuda.synchronize()
    assert np.array_equal(mask_from_bits(pipe.mask_bits, w.T), st["mask"])
    cnt = pipe.row_cnt.cpu().numpy()
    assert np.array_equal(cnt, st["row_cnt"])
    cols = pipe.col_idx.cpu().numpy()
    valid = np.arange(w.T)[None, None, None, :] < cnt[..., None]
    assert np.array_equal(np.where(valid, cols, -1), st["col_idx"])
    # block accounting: every allowed block under segments is R^2 G(G+1)/2 (+ the plain causal tail)
    R, G = w.segment // w.block, w.n // w.segment
    assert int(st["row_cnt"].max()) <= w.T and int(st["row_cnt"].sum()) <= w.h_q * (R * R * G * (G + 1) // 2)


@pytest.mark.parametrize("name", ["c2", "c4", "c3"])
def test_full_size_attention_on_sampled_rows(oracle, name):
    st = _setup(name, oracle)
    w, p, pipe = st["w"], st["p"], st["pipe"]
    T, R = w.T, w.segment // w.block
    rng = np.random.default_rng(5)
    picks = [0, 1, R - 1, R, T // 2, T - R - 1, T - R, T - 2, T - 1] + rng.integers(0, T, size=7).tolist()
    rows = [[0, int(rng.integers(0, w.h_q)), int(i)] for i in picks]
    rows += [[0, h, T - 1] for h in (0, w.h_q - 1)]          # the longest rows of the first and last head
    # oracle's intermediates in, GPU attention out
    Kp_d, Vt_d = to_dev(st["Kp"], "bf16"), to_dev(vt_layout(st["Vp"], w.block), "bf16")
    Op, lse = pbs.attn_fwd(p, st["Q"], Kp_d, Vt_d, None, i32_dev(st["kidx"]), i32_dev(st["row_cnt"]),
                           i32_dev(st["col_idx"]), pipe.Op, want_lse=True)
    torch.cuda.synchronize()
    want, want_lse = oracle.attn_rows(w.Q, st["Kp"], st["Vp"], None, st["kidx"], st["row_cnt"], st["col_idx"],
                                      w.block, rows, want_lse=True)
    for u, (b, h, i) in enumerate(rows):
        sl = slice(i * w.block, (i + 1) * w.block)
        check_close(to_host(Op[b, h, sl]), want[u], "bf16", "%s row (%d,%d,%d)" % (name, b, h, i))
        np.testing.assert_allclose(lse[b, h, sl].cpu().numpy(), want_lse[u], rtol=0, atol=2e-2)
    # properties that hold at any size: finite everywhere, and every output row is a convex combination of V rows
    assert torch.isfinite(Op).all()
    vmax = st["V"].float().abs().amax(dim=2)                 # [1,Hkv,d]
    bound = vmax.repeat_interleave(w.h_q // w.h_kv, dim=1)[:, :, None, :] * 1.01 + 1e-3
    assert (Op.float().abs() <= bound).all()
    # the same rows with every own segment taken from a token-order copy of K, V'^T and kidx behind the permuted ones
    p2 = make_problem(w, flags=w.flags | pbs.FLAG_TOKEN_ORDER_COPY)
    Kp2 = with_token_copy(p2, "kp", Kp_d, st["K"])
    Vt2 = with_token_copy(p2, "vt", Vt_d, to_dev(vt_layout(w.V, w.block), "bf16"))
    del Kp_d, Vt_d
    kidx2 = with_token_copy(p2, "kidx", i32_dev(st["kidx"]),
                            torch.arange(w.n, device="cuda", dtype=torch.int32).expand(w.batch, w.h_kv, w.n))
    Op2, lse2 = pbs.attn_fwd(p2, st["Q"], Kp2, Vt2, None, kidx2, i32_dev(st["row_cnt"]), i32_dev(st["col_idx"]),
                             torch.empty_like(Op), want_lse=True)
    torch.cuda.synchronize()
    for u, (b, h, i) in enumerate(rows):
        sl = slice(i * w.block, (i + 1) * w.block)
        check_close(to_host(Op2[b, h, sl]), want[u], "bf16", "%s row (%d,%d,%d), token-order copy" % (name, b, h, i))
        np.testing.assert_allclose(lse2[b, h, sl].cpu().numpy(), want_lse[u], rtol=0, atol=2e-2)
    assert not torch.equal(Op2, Op)                          # the copy was used
    check_close(to_host(Op2[0, 0]), to_host(Op[0, 0]), "bf16", "%s head 0, copy against permuted order" % name)


def test_full_size_variants_proxies_query_permutation_and_index_remapping(oracle, oracle_variants):
    # the variants the paper ablates, at the headline layer's full size (N = 131072, 32 query heads, 8 kv heads), each
    # against what the oracle can afford there: the two other proxies in full (by value), the key-aware query
    # permutation on whole segments picked over the sequence (bit-exact), index-remapped attention on sampled rows
    st = _setup("c3", oracle)
    w, p, pipe = st["w"], st["p"], st["pipe"]
    T, R, G = w.T, w.segment // w.block, w.n // w.segment
    # proxies: 128 positions drawn from a seed; the average query
    rows = wl.random_query_rows(3, w.n, 128)
    got = pbs.key_scores_proxy(p, pbs.PROXY_QUERY_ROWS, torch.from_numpy(rows).cuda(), st["Q"], st["K"], pipe.scores,
                               pipe.ws1)
    torch.cuda.synchronize()
    np.testing.assert_allclose(got.cpu().numpy().astype(np.float64), oracle_variants.key_scores_proxy(w.Q, w.K, rows),
                               rtol=2e-3, atol=1e-37)
    got = pbs.key_scores_proxy(p, pbs.PROXY_AVG_QUERY, None, st["Q"], st["K"], pipe.scores, pipe.ws1)
    torch.cuda.synchronize()
    np.testing.assert_allclose(got.cpu().numpy().astype(np.float64), oracle_variants.key_scores_proxy(w.Q, w.K),
                               rtol=2e-3, atol=1e-37)
    # key-aware sigma on the permuted keys: first, second, a middle and the last segment of every head
    Kp_d = to_dev(st["Kp"], "bf16")
    qidx = pbs.query_permutation(p, st["Q"], Kp_d)
    torch.cuda.synchronize()
    qh = qidx.cpu().numpy()
    for g in (0, 1, G // 2, G - 1):
        want = oracle_variants.query_permutation_segment(w.Q, st["Kp"], w.block, w.segment, g)
        assert np.array_equal(qh[:, :, g * w.segment:(g + 1) * w.segment], want), "segment %d" % g
    # every segment is a bijection of itself (holds at any size)
    srt = np.sort(qh.reshape(w.batch, w.h_q, G, w.segment), axis=-1)
    assert np.array_equal(srt, np.broadcast_to(np.arange(G * w.segment, dtype=np.int32).reshape(G, w.segment), srt.shape))
    del qidx, qh, srt
    # index remapping: kidx, Vt and the block means from the permutation stage, no K'; attention gathers from K
    pr = make_problem(w, flags=w.flags | pbs.FLAG_INDEX_REMAP)
    prk = make_problem(w, flags=w.flags | pbs.FLAG_INDEX_REMAP | pbs.FLAG_KBAR_IN_WS)
    kidx, none, Vt = pbs.segment_permute(pr, torch.from_numpy(st["s_h"]).cuda(), st["K"], st["V"], ws=pipe.ws3)
    assert none is None and np.array_equal(kidx.cpu().numpy(), st["kidx"])
    pbs.block_mask(prk, st["Q"], st["K"], pipe.mask_bits, pipe.row_cnt, pipe.col_idx, pipe.ws3)
    torch.cuda.synchronize()
    assert np.array_equal(pipe.row_cnt.cpu().numpy(), st["row_cnt"])             # the means of K' came from the gather
    rng = np.random.default_rng(6)
    picks = [0, R - 1, R, T // 2, T - R, T - 1] + rng.integers(0, T, size=4).tolist()
    rws = [[0, int(rng.integers(0, w.h_q)), int(i)] for i in picks]
    Op, lse = pbs.attn_fwd(pr, st["Q"], st["K"], Vt, None, kidx, pipe.row_cnt, pipe.col_idx, pipe.Op, want_lse=True)
    torch.cuda.synchronize()
    want, want_lse = oracle.attn_rows(w.Q, st["Kp"], st["Vp"], None, st["kidx"], st["row_cnt"], st["col_idx"],
                                      w.block, rws, want_lse=True)
    for u, (b, h, i) in enumerate(rws):
        sl = slice(i * w.block, (i + 1) * w.block)
        check_close(to_host(Op[b, h, sl]), want[u], "bf16", "c3 row (%d,%d,%d), index remapping" % (b, h, i))
        np.testing.assert_allclose(lse[b, h, sl].cpu().numpy(), want_lse[u], rtol=0, atol=2e-2)
    assert torch.isfinite(Op).all()


@pytest.mark.parametrize("rho", [0.05, 0.10, 0.25, 0.50, 1.0])
def test_full_size_given_lists_on_sampled_rows(oracle, rho):
    """Config 5: identity key order, seeded block lists of density rho at N = 65536, attention only."""
    _state.clear()
    torch.cuda.empty_cache()
    w = wl.c5_density(rho)
    p = make_problem(w)
    T = w.T
    row_cnt, col_idx = w.extra["row_cnt"], w.extra["col_idx"]
    assert int(row_cnt.sum()) == w.h_q * (T * (T + 1) // 2 if rho >= 1.0 else int(round(rho * (T * (T + 1) // 2))))
    Q, K, V = to_dev(w.Q, "bf16"), to_dev(w.K, "bf16"), to_dev(w.V, "bf16")
    kidx, Kp, Vt = pbs.segment_permute(p, None, K, V)
    assert torch.equal(Kp, K) and torch.equal(kidx[0, 0].cpu(), torch.arange(w.n, dtype=torch.int32))
    Op, lse = pbs.attn_fwd(p, Q, Kp, Vt, None, kidx, i32_dev(row_cnt), i32_dev(col_idx), want_lse=True)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    rows = [[0, int(rng.integers(0, w.h_q)), int(i)] for i in [0, 1, T // 3, T - 2, T - 1] + rng.integers(0, T, size=5).tolist()]
    kid = np.tile(np.arange(w.n, dtype=np.int32), (1, w.h_kv, 1))
    want, want_lse = oracle.attn_rows(w.Q, w.K, w.V, None, kid, row_cnt, col_idx, w.block, rows, want_lse=True)
    for u, (b, h, i) in enumerate(rows):
        sl = slice(i * w.block, (i + 1) * w.block)
        check_close(to_host(Op[b, h, sl]), want[u], "bf16", "c5 rho=%g row (%d,%d,%d)" % (rho, b, h, i))
        np.testing.assert_allclose(lse[b, h, sl].cpu().numpy(), want_lse[u], rtol=0, atol=2e-2)
    assert torch.isfinite(Op).all()


def test_block_64_at_full_length_on_sampled_rows(oracle):
    """The block-64 matrix-core instantiation at N = 32768 (T = 512, segments of 8 blocks, GQA 4:1): every stage fed
    the oracle's previous stage; indices, mask and lists in full and bit-exact, attention on sampled query blocks."""
    _state.clear()
    torch.cuda.empty_cache()
    w = wl.planted("b64_full", 1064, 8, 2, 32768, 128, 64, 512, 0.9, "bf16", 64, rope_base=5e5)
    s_h = oracle.key_scores(w.Q, w.K, w.block).astype(np.float32)
    kidx = oracle.segment_argsort(s_h, w.segment)
    Kp, Vp = oracle.gather_rows(w.K, kidx), oracle.gather_rows(w.V, kidx)
    mask, row_cnt, col_idx = oracle.block_mask(w.Q, Kp, w.block, w.segment, w.tau, flags=w.flags)
    p = make_problem(w)
    Q, K, V = to_dev(w.Q, "bf16"), to_dev(w.K, "bf16"), to_dev(w.V, "bf16")
    kidx_g, Kp_g, Vt_g = pbs.segment_permute(p, torch.from_numpy(s_h).cuda(), K, V)
    assert np.array_equal(kidx_g.cpu().numpy(), kidx)
    assert torch.equal(Kp_g, to_dev(Kp, "bf16")) and torch.equal(Vt_g, to_dev(vt_layout(Vp, w.block), "bf16"))
    bits, cnt, cols = pbs.block_mask(p, Q, Kp_g)
    assert np.array_equal(mask_from_bits(bits, w.T), mask) and np.array_equal(cnt.cpu().numpy(), row_cnt)
    Op, lse = pbs.attn_fwd(p, Q, Kp_g, Vt_g, None, kidx_g, i32_dev(row_cnt), i32_dev(col_idx), want_lse=True)
    torch.cuda.synchronize()
    T, R = w.T, w.segment // w.block
    rng = np.random.default_rng(6)
    rows = [[0, int(rng.integers(0, w.h_q)), int(i)]
            for i in [0, 1, R - 1, R, T // 2, T - R, T - 2, T - 1] + rng.integers(0, T, size=6).tolist()]
    want, want_lse = oracle.attn_rows(w.Q, Kp, Vp, None, kidx, row_cnt, col_idx, w.block, rows, want_lse=True)
    for u, (b, h, i) in enumerate(rows):
        sl = slice(i * w.block, (i + 1) * w.block)
        check_close(to_host(Op[b, h, sl]), want[u], "bf16", "block 64 row (%d,%d,%d)" % (b, h, i))
        np.testing.assert_allclose(lse[b, h, sl].cpu().numpy(), want_lse[u], rtol=0, atol=2e-2)
    assert torch.isfinite(Op).all()


def test_maximum_length_dense_equals_causal_attention_on_sampled_blocks(oracle):
    # the largest supported length (T = 4096 blocks): tau > 1 keeps every admitted block, so whatever the scores made
    # of the key order, the pipeline must reproduce dense causal attention (Theorem 1).  Sampled query blocks are
    # compared with the oracle's attention loop fed the GPU's own permutation and lists, and with fp32 matrix
    # products of the very same bf16 inputs in token order.
    N, Hq, Hkv, d, B, S = 524288, 4, 1, 128, 128, 1024
    gen = torch.Generator(device="cuda").manual_seed(11)
    Q = torch.randn(1, Hq, N, d, device="cuda", generator=gen).to(torch.bfloat16)
    K = torch.randn(1, Hkv, N, d, device="cuda", generator=gen).to(torch.bfloat16)
    V = torch.randn(1, Hkv, N, d, device="cuda", generator=gen).to(torch.bfloat16)
    p = pbs.problem(1, Hq, Hkv, N, d, B, S, "bf16", tau=1.5)
    pipe = pbs.Pipeline(p)
    O = pipe.run(Q, K, V)
    torch.cuda.synchronize()
    T = N // B
    assert int(pipe.row_cnt.sum()) == Hq * (S // B) ** 2 * (N // S) * (N // S + 1) // 2     # R^2 G (G + 1) / 2 per head
    seg = torch.arange(N, device="cuda") // S
    assert torch.equal(pipe.kidx[0, 0].long() // S, seg)                  # every key stays in its segment
    picks = [(0, 0), (1, 1), (2, T // 2 + 3), (3, T - 1), (0, T - 8)]
    # oracle.attn_rows on these five query blocks: same inputs, the GPU's kidx and lists (only these rows are filled in)
    Qh, Kh, Vh = Q.float().cpu().numpy(), K.float().cpu().numpy(), V.float().cpu().numpy()
    kg = pipe.kidx.cpu().numpy()
    rc_h = np.zeros((1, Hq, T), dtype=np.int32)
    ci_h = np.zeros((1, Hq, T, T), dtype=np.int32)
    for (h, i) in picks:
        rc_h[0, h, i] = int(pipe.row_cnt[0, h, i])
        ci_h[0, h, i] = pipe.col_idx[0, h, i].cpu().numpy()
    want = oracle.attn_rows(Qh, oracle.gather_rows(Kh, kg), oracle.gather_rows(Vh, kg), None, kg, rc_h, ci_h, B,
                            [[0, h, i] for (h, i) in picks])
    for u, (h, i) in enumerate(picks):
        check_close(to_host(O[0, h, i * B:(i + 1) * B]), want[u], "bf16", "N = 524288 block (%d,%d)" % (h, i))
    del Qh, Kh, Vh, ci_h
    for (h, i) in picks:
        q = Q[0, h, i * B:(i + 1) * B].float()
        k = K[0, 0, :(i + 1) * B].float()
        v = V[0, 0, :(i + 1) * B].float()
        L = (q @ k.T) / d ** 0.5
        pos_q = torch.arange(i * B, (i + 1) * B, device="cuda")[:, None]
        pos_k = torch.arange((i + 1) * B, device="cuda")[None, :]
        ref = torch.softmax(L.masked_fill(pos_k > pos_q, float("-inf")), dim=1) @ v
        err = (O[0, h, i * B:(i + 1) * B].float() - ref).abs()
        assert float(err.max()) <= 2e-2 and float(err.mean()) <= 2e-3, (h, i, float(err.max()), float(err.mean()))


@pytest.mark.parametrize("dtype,d,Hq,Hkv,tau,flags", [("bf16", 128, 40, 10, 0.02, 0), ("f32", 64, 66, 33, 0.0, 0),
                                                      ("bf16", 128, 40, 10, 0.02, pbs.FLAG_TOKEN_ORDER_COPY)])
def test_element_offsets_beyond_32_bits_reproduce_the_last_group_run_on_its_own(dtype, d, Hq, Hkv, tau, flags):
    # 40 query heads x 524288 rows x 128 columns (66 x 524288 x 64 for the fp32 kernels) = 2.7e9 (2.2e9) elements per
    # tensor: the last GQA group lies wholly beyond element offset 2^31 in Q and O and beyond 2^32 in the block lists.
    # Every (batch, kv head) group is an independent pipeline with a fixed order of operations, so the big run must
    # reproduce, bit for bit, what the same group gives as a problem of its own (whose offsets are small).
    _state.clear()
    torch.cuda.empty_cache()
    N, B, S = 524288, 128, 1024
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cuda").manual_seed(23)
    Q = torch.empty(1, Hq, N, d, device="cuda", dtype=tdt)
    for h in range(Hq):
        Q[0, h] = torch.randn(N, d, device="cuda", generator=gen).to(tdt)
    K = torch.randn(1, Hkv, N, d, device="cuda", generator=gen).to(tdt)
    V = torch.randn(1, Hkv, N, d, device="cuda", generator=gen).to(tdt)
    assert Q.numel() > 2 ** 31
    big = pbs.Pipeline(pbs.problem(1, Hq, Hkv, N, d, B, S, dtype, tau=tau, flags=flags))
    O = big.run(Q, K, V)
    torch.cuda.synchronize()
    r = Hq // Hkv
    small = pbs.Pipeline(pbs.problem(1, r, 1, N, d, B, S, dtype, tau=tau, flags=flags))
    O1 = small.run(Q[:, Hq - r:].contiguous(), K[:, Hkv - 1:].contiguous(), V[:, Hkv - 1:].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(big.scores[:, Hkv - 1:], small.scores)
    # (with the token-order copy the attention kernel reaches up to 1.5e9 bytes beyond a head's base)
    assert torch.equal(big.kidx[:, Hkv - 1:], small.kidx)
    assert torch.equal(big.Kp[:, Hkv - 1:], small.Kp)
    assert torch.equal(big.Vt[:, Hkv - 1:], small.Vt)
    assert torch.equal(big.mask_bits[:, Hq - r:], small.mask_bits)
    assert torch.equal(big.row_cnt[:, Hq - r:], small.row_cnt)
    T = N // B
    listed = torch.arange(T, device="cuda").view(1, 1, 1, T) < small.row_cnt.unsqueeze(-1)
    assert torch.equal(torch.where(listed, big.col_idx[:, Hq - r:], -1), torch.where(listed, small.col_idx, -1))
    assert 0 < int(small.row_cnt.sum()) < r * T * (T + 1) // 8          # sparse, and not empty
    assert torch.equal(O[:, Hq - r:], O1)
    assert torch.isfinite(O[:, Hq - r:].float()).all()
    del big, small, Q, K, V, O, O1
    torch.cuda.empty_cache()
