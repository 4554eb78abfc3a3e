"""GPU parity on the degenerate and edge cases of the path (through the C ABI, against the oracle)."""
import numpy as np
import pytest
import torch

from gpu_helpers import (check_close, i32_dev, make_problem, mask_from_bits, to_dev, to_host, vt_layout,
                         with_token_copy)
from paper_2510_21270_amd import binding as pbs
from paper_2510_21270_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _full_pipeline_vs_oracle(oracle, w, tau=None, flags=None, exact_indices=True):
    p = make_problem(w, tau=tau, flags=flags)
    res = oracle.pipeline(w.Q, w.K, w.V, w.block, w.segment, p.tau, flags=p.flags)
    pipe = pbs.Pipeline(p)
    O = pipe.run(to_dev(w.Q, w.dtype), to_dev(w.K, w.dtype), to_dev(w.V, w.dtype))
    torch.cuda.synchronize()
    if exact_indices:
        np.testing.assert_array_equal(pipe.kidx.cpu().numpy(), res["kidx"])
        np.testing.assert_array_equal(mask_from_bits(pipe.mask_bits, w.T), res["mask"])
        check_close(to_host(O), res["O"], w.dtype, w.name)
    return pipe, res, O


@pytest.mark.parametrize("n", [1, 5, 63, 64, 65])
def test_tiny_lengths_f32(oracle, n):
    # shorter than one block / one segment: no permutation at all, partial blocks everywhere
    w = wl.planted("tiny%d" % n, 30 + n, 2, 1, n, 64, 64, 128, 0.9, "f32", 1)
    _full_pipeline_vs_oracle(oracle, w)


@pytest.mark.parametrize("n", [1, 100, 129])
def test_tiny_lengths_bf16_mfma(oracle, n):
    w = wl.planted("tinyb%d" % n, 40 + n, 2, 2, n, 128, 128, 128, 0.9, "bf16", 1)
    pipe, res, O = _full_pipeline_vs_oracle(oracle, w, exact_indices=False)
    # with at most two blocks everything allowed is forced, so the result is dense causal attention
    check_close(to_host(O), oracle.dense_causal(w.Q, w.K, w.V), "bf16", "tiny bf16")


@pytest.mark.parametrize("dtype,d,block,seg", [("f32", 64, 64, 256), ("bf16", 128, 128, 512), ("bf16", 128, 64, 256)])
def test_tau_above_one_is_dense_causal(oracle, dtype, d, block, seg):
    # every allowed block is kept, so the GPU pipeline must reproduce dense causal attention (Theorem 1),
    # whatever order its scores put the keys in.
    w = wl.planted("dense", 50, 4, 2, 1500, d, block, seg, 1.5, dtype, 8, rope_base=5e5)
    p = make_problem(w)
    pipe = pbs.Pipeline(p)
    O = pipe.run(to_dev(w.Q, dtype), to_dev(w.K, dtype), to_dev(w.V, dtype))
    torch.cuda.synchronize()
    check_close(to_host(O), oracle.dense_causal(w.Q, w.K, w.V), dtype, "dense")
    T, R, G = w.T, seg // block, 1500 // seg
    want_cnt = np.array([min((i // R + 1) * R, T) if i // R < G else i + 1 for i in range(T)])
    assert (pipe.row_cnt.cpu().numpy() == want_cnt).all()


def test_tau_zero_keeps_one_block_plus_forced(oracle):
    w = wl.planted("tau0", 51, 2, 1, 2048, 64, 64, 256, 0.0, "f32", 8)
    pipe, res, O = _full_pipeline_vs_oracle(oracle, w, tau=0.0, flags=0)
    R = 4
    cnt = pipe.row_cnt.cpu().numpy()
    assert cnt.max() <= R + 1


def test_identity_permutation_when_scores_are_null(oracle):
    # the unpermuted MeanPooling baseline: K' = K, V' = V
    w = wl.planted("ident", 52, 2, 2, 777, 128, 128, 256, 0.9, "bf16", 4)
    p = make_problem(w)
    kidx, Kp, Vt = pbs.segment_permute(p, None, to_dev(w.K, "bf16"), to_dev(w.V, "bf16"))
    torch.cuda.synchronize()
    assert (kidx.cpu().numpy() == np.arange(777)).all()
    np.testing.assert_array_equal(to_host(Kp), w.K.astype(np.float64))
    np.testing.assert_array_equal(to_host(Vt), vt_layout(w.V, 128).astype(np.float64))


def test_ties_and_signed_zero_scores(oracle):
    n, seg = 1024, 256
    p = pbs.problem(1, 1, 1, n, 64, 64, seg, "f32")
    rng = np.random.default_rng(3)
    s = rng.integers(0, 4, size=(1, 1, n)).astype(np.float32) * 0.25      # many exact ties
    s[0, 0, ::5] = -0.0                                                   # -0.0 ties with +0.0
    s[0, 0, 1::5] = 0.0
    want = oracle.segment_argsort(s, seg)
    kidx, _, _ = pbs.segment_permute(p, torch.from_numpy(s).cuda(), None, None, indices_only=True)
    np.testing.assert_array_equal(kidx.cpu().numpy(), want)
    s2 = np.zeros((1, 1, n), dtype=np.float32)                            # all equal -> identity
    kidx, _, _ = pbs.segment_permute(p, torch.from_numpy(s2).cuda(), None, None, indices_only=True)
    assert (kidx.cpu().numpy() == np.arange(n)).all()


def test_maximum_segment_and_non_power_of_two_segment(oracle):
    rng = np.random.default_rng(8)
    for n, seg, block in [(4096 * 2 + 100, 4096, 128), (384 * 3 + 7, 384, 128), (96 * 5, 96, 32)]:
        p = pbs.problem(1, 2, 2, n, 64, block, seg, "f32")
        s = rng.random((1, 2, n)).astype(np.float32)
        kidx, _, _ = pbs.segment_permute(p, torch.from_numpy(s).cuda(), None, None, indices_only=True)
        np.testing.assert_array_equal(kidx.cpu().numpy(), oracle.segment_argsort(s, seg))


@pytest.mark.parametrize("dtype,d,block", [("bf16", 128, 128), ("f32", 64, 32)])
def test_given_lists_any_order_empty_rows_and_out_of_range_entries(oracle, dtype, d, block):
    # config-5 style: identity key order, caller-supplied block lists
    T, Hq, Hkv = 12, 4, 2
    n = T * block - 9
    rng = np.random.default_rng(21)
    Q = rng.standard_normal((1, Hq, n, d)).astype(np.float32)
    K = rng.standard_normal((1, Hkv, n, d)).astype(np.float32)
    V = rng.standard_normal((1, Hkv, n, d)).astype(np.float32)
    if dtype == "bf16":
        Q, K, V = wl.round_to_bf16(Q), wl.round_to_bf16(K), wl.round_to_bf16(V)
    row_cnt, col_idx = wl.random_block_lists(5, 1, Hq, T, 0.4)
    kidx = np.tile(np.arange(n, dtype=np.int32), (1, Hkv, 1))
    p = pbs.problem(1, Hq, Hkv, n, d, block, block, dtype)              # segment = block: plain block causality
    want, want_lse = oracle.attn_fwd(Q, K, V, None, kidx, row_cnt, col_idx, block, want_lse=True)
    # the same lists reversed, plus junk entries that the kernel must ignore (beyond the causal region / negative)
    shuffled = col_idx.copy()
    cnt2 = row_cnt.copy()
    for h in range(Hq):
        for i in range(T):
            c = row_cnt[0, h, i]
            lst = col_idx[0, h, i, :c][::-1].tolist()
            if c + 2 <= T:
                lst = [-1] + lst + [T + 3 if i == T - 1 else min(T - 1, i + 1)]
                if lst[-1] <= i:
                    lst = lst[:-1]
            shuffled[0, h, i, :len(lst)] = lst
            cnt2[0, h, i] = len(lst)
    # one query block with an empty list: zero output rows and lse = -inf
    cnt2[0, 1, 3] = 0
    got, lse = pbs.attn_fwd(p, to_dev(Q, dtype), to_dev(K, dtype), to_dev(vt_layout(V, block), dtype), None,
                            i32_dev(kidx), i32_dev(cnt2), i32_dev(shuffled), want_lse=True)
    torch.cuda.synchronize()
    got, lse = to_host(got), lse.cpu().numpy()
    sl = slice(3 * block, 4 * block)
    assert (got[0, 1, sl] == 0).all() and np.isneginf(lse[0, 1, sl]).all()
    got[0, 1, sl] = want[0, 1, sl]
    check_close(got, want, dtype, "given lists")
    lse[0, 1, sl] = want_lse[0, 1, sl]
    np.testing.assert_allclose(lse, want_lse, atol=2e-2 if dtype == "bf16" else 1e-4, rtol=0)


def test_reversed_keys_rows_see_nothing_in_early_blocks(oracle):
    # keys reversed inside one segment: early visited blocks are fully masked for early queries (running max -inf)
    n, block, d = 512, 128, 128
    rng = np.random.default_rng(6)
    Q, K, V = (wl.round_to_bf16(rng.standard_normal((1, 1, n, d)).astype(np.float32)) for _ in range(3))
    kidx = np.arange(n - 1, -1, -1, dtype=np.int32).reshape(1, 1, n)
    Kp, Vp = oracle.gather_rows(K, kidx), oracle.gather_rows(V, kidx)
    row_cnt = np.full((1, 1, 4), 4, dtype=np.int32)
    col_idx = np.tile(np.arange(4, dtype=np.int32), (1, 1, 4, 1))
    p = pbs.problem(1, 1, 1, n, d, block, n, "bf16")
    got = pbs.attn_fwd(p, to_dev(Q, "bf16"), to_dev(Kp, "bf16"), to_dev(vt_layout(Vp, block), "bf16"), None,
                       i32_dev(kidx), i32_dev(row_cnt), i32_dev(col_idx))
    torch.cuda.synchronize()
    check_close(to_host(got), oracle.dense_causal(Q, K, V), "bf16", "reversed")


def test_scores_climbing_far_above_the_first_keys_take_the_second_pass(oracle):
    # The 64-queries-per-wave kernel fixes a query's softmax reference at its first visible keys and flags query
    # blocks whose probabilities outgrow it by more than 2^64; the library must then recompute those blocks with the
    # rescaling kernel.  Keys are built so that the logits rise by about 0.12 nats per key along the sequence:
    # every query block but the first meets keys many times 44 nats above their first sub-tile.
    n, block, d, Hq, Hkv = 1024, 128, 128, 2, 1
    rng = np.random.default_rng(17)
    u = np.zeros(d, dtype=np.float32)
    u[:4] = 1.0
    Q = np.tile(u * 4.0, (1, Hq, n, 1)).astype(np.float32)                       # q . u = 16 for every query
    ramp = (np.arange(n, dtype=np.float32) * 0.35)[None, None, :, None]        # logit = 16 * ramp * u.u/4 / sqrt(d)
    K = wl.round_to_bf16(ramp * (u / 4.0)[None, None, None, :] + 0.01 * rng.standard_normal((1, Hkv, n, d)).astype(np.float32))
    Q = wl.round_to_bf16(Q + 0.01 * rng.standard_normal(Q.shape).astype(np.float32))
    V = wl.round_to_bf16(rng.standard_normal((1, Hkv, n, d)).astype(np.float32))
    T = n // block
    kidx = np.tile(np.arange(n, dtype=np.int32), (1, Hkv, 1))
    row_cnt = np.tile(np.arange(1, T + 1, dtype=np.int32), (1, Hq, 1))
    col_idx = np.tile(np.arange(T, dtype=np.int32), (1, Hq, T, 1))
    p = pbs.problem(1, Hq, Hkv, n, d, block, block, "bf16")
    logit_span = float((Q[0, 0, -1] @ K[0, 0, -1] - Q[0, 0, -1] @ K[0, 0, 0]) / np.sqrt(d))
    assert logit_span > 100.0                                                    # far beyond 2^64 = e^44
    ws = pbs.alloc_workspace(p, pbs.STAGE_ATTN_FWD)
    got, lse = pbs.attn_fwd(p, to_dev(Q, "bf16"), to_dev(K, "bf16"), to_dev(vt_layout(V, block), "bf16"), None,
                            i32_dev(kidx), i32_dev(row_cnt), i32_dev(col_idx), want_lse=True, ws=ws)
    torch.cuda.synchronize()
    flags = ws[:Hq * T * 4].view(torch.int32).cpu().numpy()
    assert flags.sum() >= Hq * (T - 3), "the first pass was expected to flag the long query blocks"
    want, want_lse = oracle.attn_fwd(Q, K, V, None, kidx, row_cnt, col_idx, block, want_lse=True)
    check_close(to_host(got), want, "bf16", "second pass")
    np.testing.assert_allclose(lse.cpu().numpy(), want_lse, atol=2e-2, rtol=2e-4)
    # the same with segments of four blocks, every admitted block listed and the own segment taken from a token-order
    # copy: the first pass flags the blocks all the same, and the second pass recomputes them from the lists as given
    R = 4
    p4 = pbs.problem(1, Hq, Hkv, n, d, block, R * block, "bf16", flags=pbs.FLAG_TOKEN_ORDER_COPY)
    row_cnt4 = np.tile(((np.arange(T) // R + 1) * R).astype(np.int32), (1, Hq, 1))
    Kd, Vd, kd = to_dev(K, "bf16"), to_dev(vt_layout(V, block), "bf16"), i32_dev(kidx)
    ws.zero_()
    got4, lse4 = pbs.attn_fwd(p4, to_dev(Q, "bf16"), with_token_copy(p4, "kp", Kd, Kd),
                              with_token_copy(p4, "vt", Vd, Vd), None, with_token_copy(p4, "kidx", kd, kd),
                              i32_dev(row_cnt4), i32_dev(col_idx), want_lse=True, ws=ws)
    torch.cuda.synchronize()
    assert ws[:Hq * T * 4].view(torch.int32).sum().item() >= Hq * (T - 3)
    check_close(to_host(got4), want, "bf16", "second pass after a first pass on the token-order copy")
    np.testing.assert_allclose(lse4.cpu().numpy(), want_lse, atol=2e-2, rtol=2e-4)


def test_rescaling_kernel_alone_serves_block_128(oracle):
    # PBS_FLAG_RUNNING_MAX_ONLY sends block 128 through the 32-queries-per-wave kernel only (the recurrence of
    # Algorithm 1 as printed): same comparison with the oracle as the parity test
    w = wl.planted("narrow", 21, 4, 2, 2048 + 31, 128, 128, 512, 0.9, "bf16", 8, rope_base=5e5)
    res = oracle.pipeline(w.Q, w.K, w.V, w.block, w.segment, w.tau, flags=w.flags)
    p = make_problem(w, flags=w.flags | pbs.FLAG_RUNNING_MAX_ONLY)
    ws = torch.full((max(pbs.workspace_bytes(p, pbs.STAGE_ATTN_FWD), 256),), 0x55, dtype=torch.uint8, device="cuda")
    Op, lse = pbs.attn_fwd(p, to_dev(res["Qp"], "bf16"), to_dev(res["Kp"], "bf16"),
                           to_dev(vt_layout(res["Vp"], w.block), "bf16"), None, i32_dev(res["kidx"]),
                           i32_dev(res["row_cnt"]), i32_dev(res["col_idx"]), want_lse=True, ws=ws)
    torch.cuda.synchronize()
    assert bool((ws == 0x55).all())                    # the first pass, which writes its flags there, did not run
    check_close(to_host(Op), res["Op"], "bf16", "running maximum only")
    np.testing.assert_allclose(lse.cpu().numpy(), res["lse"], atol=2e-2, rtol=0)


def test_matrix_rate_probe_runs_and_counts_its_work():
    # measurement aid of bench.py: 1024 workgroups x 4 waves x iters x 32 instructions of 32 x 32 x 16 multiply-adds
    import ctypes
    lib = pbs.load_library()
    sink = torch.empty(262144, dtype=torch.float32, device="cuda")
    flop = ctypes.c_double(0.0)
    for random_operands in (0, 1):
        assert lib.pbs_mfma_rate_probe(random_operands, 100, sink.data_ptr(), sink.numel(), ctypes.byref(flop), None) == 0
        torch.cuda.synchronize()
        assert flop.value == 1024 * 4 * 100 * 32 * 2.0 * 32 * 32 * 16
        assert 500.0 < float(sink[0]) < 3000.0             # the shader clock one wave saw, MHz
        assert 31.0 < float(sink[1]) < 160.0               # 32 clocks per instruction, up to four waves on a SIMD
        assert torch.isfinite(sink).all()
    assert (sink != 0).any()                           # random operands leave non-zero accumulators
    rate, mhz = pbs.mfma_rate_probe(True, iters=2000, reps=1)
    assert rate > 100.0 and 500.0 < mhz < 3000.0
    # the clock meter beside a kernel that keeps the GPU busy for a while
    mhz2, watched = pbs.shader_clock_beside(lambda: lib.pbs_mfma_rate_probe(1, 40000, sink.data_ptr(), sink.numel(),
                                                                            ctypes.byref(flop), None), micros=5000)
    assert 500.0 < mhz2 < 3000.0 and watched >= 4900.0


@pytest.mark.parametrize("extra_flags", [0, pbs.FLAG_TOKEN_ORDER_COPY])
def test_pipeline_replayed_from_a_hip_graph_matches_eager_runs(extra_flags):
    # the five calls captured once; every replay, with new inputs copied into the captured tensors and eager work and
    # synchronisations in between, must reproduce the eager pipeline bit for bit (also in the configuration bench.py
    # times, with the token-order copy)
    w = wl.planted("graph", 21, 4, 2, 2048 + 45, 128, 128, 512, 0.9, "bf16", 8, rope_base=5e5)
    p = make_problem(w, flags=w.flags | extra_flags)
    eager, graphed = pbs.Pipeline(p), pbs.Pipeline(p)
    Q, K, V = to_dev(w.Q, "bf16"), to_dev(w.K, "bf16"), to_dev(w.V, "bf16")
    Qs, Ks, Vs = Q.clone(), K.clone(), V.clone()
    graphed.capture(Qs, Ks, Vs)
    gen = torch.Generator(device="cuda").manual_seed(3)
    for it in range(4):
        if it:
            Q = torch.randn(Q.shape, device="cuda", generator=gen).to(torch.bfloat16)
            K = (torch.randn(K.shape, device="cuda", generator=gen) * (1.0 + it)).to(torch.bfloat16)
            V = torch.randn(V.shape, device="cuda", generator=gen).to(torch.bfloat16)
        want = eager.run(Q, K, V).clone()
        torch.cuda.synchronize()
        Qs.copy_(Q), Ks.copy_(K), Vs.copy_(V)
        got = graphed.replay()
        torch.cuda.synchronize()
        assert torch.equal(graphed.kidx, eager.kidx), it
        assert torch.equal(graphed.mask_bits, eager.mask_bits), it
        assert torch.equal(got, want), it


def test_bench_prints_one_json_line_with_the_contract_fields():
    # bench.py on its small functional workload, as the child process the driver would start
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--workload", "small", "--steps", "2",
                          "--warmup", "1"], capture_output=True, text=True, timeout=600, cwd=root)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [ln for ln in res.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, res.stdout[-2000:]
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 2 and out["warmup"] == 1 and out["data"] == "synthetic"
    assert out["higher_is_better"] is True and out["vs_baseline"] is None and out["dtype"] == "bf16"
    assert "workload" in out["config"] and "model" not in out["config"]
    assert out["value"] > 0 and out["ms_per_step"] > 0
    rf = out["roofline"]
    assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and rf["peak"] == 2500.0 and "traffic" in rf
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-12 and 0 < rf["frac"] < 1
    cb = out["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["unit"] == out["unit"] and cb["cores"] >= 1 and cb["value"] > 0
    assert isinstance(cb["sample"], str) and cb["sample"]


@pytest.mark.parametrize("d,block", [(64, 64), (128, 32)])
def test_fp32_block_means_follow_the_row_order_of_the_definition(oracle, d, block):
    # fp32 storage, values spread over 24 binades inside every block: the fp64 block means then depend on the order
    # of the additions in their last bits, and so could a selection; the library adds the rows in ascending order, as
    # the plain definition does, so mask and lists must still match the oracle bit for bit (several tau, ragged length)
    rng = np.random.default_rng(41)
    n, Hq, Hkv, S = 1024 + 37, 4, 2, 4 * block
    def wide(shape):
        return (rng.standard_normal(shape) * np.exp2(rng.integers(-12, 13, size=shape))).astype(np.float32)
    Q, K = wide((1, Hq, n, d)), wide((1, Hkv, n, d))
    # keep the pooled logits of the order of one: the means are dominated by the largest binades
    Q *= np.float32(2.0 ** -9)
    K *= np.float32(2.0 ** -9)
    for tau in (0.5, float(np.float32(0.9)), float(np.float32(0.99))):   # as the float field of the problem holds them
        mask, row_cnt, col_idx = oracle.block_mask(Q, K, block, S, tau, flags=1)
        p = pbs.problem(1, Hq, Hkv, n, d, block, S, "f32", tau=tau, flags=1)
        bits, cnt, cols = pbs.block_mask(p, to_dev(Q, "f32"), to_dev(K, "f32"))
        torch.cuda.synchronize()
        T = -(-n // block)
        np.testing.assert_array_equal(mask_from_bits(bits, T), mask)
        np.testing.assert_array_equal(cnt.cpu().numpy(), row_cnt)
        valid = np.arange(T)[None, None, None, :] < row_cnt[..., None]
        np.testing.assert_array_equal(np.where(valid, cols.cpu().numpy(), -1), col_idx)
        assert 0.2 < mask.mean() / 0.5 < 1.9               # a real selection, neither empty nor everything


@pytest.mark.parametrize("h_q,n,segment", [(1, 65536, 64), (2, 65531, 128)])
def test_block_mask_at_the_largest_block_count(oracle, h_q, n, segment):
    # T = 4096 key blocks, the most the library accepts: a row of logits fills 32 KiB of LDS, so one query head takes
    # two query blocks per workgroup and two heads one; near-uniform rows of thousands of columns; ragged last block
    w = wl.planted("maxT", 11, h_q, 1, n, 64, 16, segment, 0.6, "bf16", 4)
    assert w.T == 4096
    mask, row_cnt, col_idx = oracle.block_mask(w.Q, w.K, w.block, w.segment, w.tau, flags=w.flags)
    bits, cnt, cols = pbs.block_mask(make_problem(w), to_dev(w.Q, "bf16"), to_dev(w.K, "bf16"))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mask_from_bits(bits, w.T), mask)
    np.testing.assert_array_equal(cnt.cpu().numpy(), row_cnt)
    valid = np.arange(w.T)[None, None, None, :] < row_cnt[..., None]
    np.testing.assert_array_equal(np.where(valid, cols.cpu().numpy(), -1), col_idx)

