#!/usr/bin/env python3
"""Benchmark of the PBS-Attn prefill hot path on one MI355X.

One "step" is one pass of the whole path (key scores -> segmented permutation -> block mask -> block-sparse
attention -> inverse permutation) over one synthetic layer input that is already resident in HBM.  The default
workload is the headline configuration: a Llama-3.1-8B-shaped layer (32 query heads, 8 kv heads, d=128, bf16) at
N=131072, block 128, segment 1024, tau 0.9.

Prints ONE JSON line.  `value` is the effective TFLOP/s of the whole step, counted over the blocks the attention
kernel actually visits (4 * block^2 * d FLOP per block per query head).  `roofline` covers the dominant kernel
(pbs_attn_fwd) from HIP-event timings taken inside the timed region; `cpu_baseline` is the fp64 oracle's attention
loop timed on the host cores on a bounded sample of query blocks.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0       # MI355X dense bf16 matrix peak
FP32_VECTOR_PEAK_TFLOPS = 157.3       # published fp32 vector rate (the shapes outside the matrix-core path)
HBM_PEAK_GBS = 8000.0                # MI355X HBM3E


def measured_attn_traffic(workload):
    """HBM bytes per pbs_attn_fwd launch as measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, scaled by what the
    same counters read for a plain copy of known size): read from the summary of that profiling run under profiles/,
    which carries a line `traffic_bytes_per_launch[<workload>] = <bytes>`.  None when no such run is on file: the
    timed run itself cannot read hardware counters."""
    import re
    path = os.path.join(ROOT, "profiles", "attn_fwd_hbm_traffic.md")
    try:
        text = open(path).read()
    except OSError:
        return None, None
    m = re.search(r"traffic_bytes_per_launch\[%s\]\s*=\s*([0-9.eE+]+)" % re.escape(workload), text)
    return (float(m.group(1)), "profiles/attn_fwd_hbm_traffic.md") if m else (None, None)


def make_workload(name):
    from paper_2510_21270_amd import workloads as wl
    if name == "c3":
        return wl.c3_llama128k()
    if name == "c2":
        return wl.c2_llama()
    if name == "c3s":                                    # extra: config 3 with keys that really are heavy
        return wl.c3_strong()
    if name == "c4":
        return wl.c4_qwen()
    if name == "c1":
        return wl.c1_tiny()
    if name.startswith("c5"):
        return wl.c5_density(float(name.split(":")[1]) if ":" in name else 0.25)
    if name == "small":                                  # quick functional check of the script itself
        return wl.c2_llama(n=8192, h_q=8, h_kv=2)
    raise SystemExit("unknown workload %r" % name)


def to_dev(x, dtype):
    import numpy as np
    import torch
    from paper_2510_21270_amd import workloads as wl
    if dtype == "bf16":
        return torch.from_numpy(wl.bf16_bits(x).view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def cpu_baseline(w, seconds_budget=20.0, visited=None):
    """The oracle's attention loop (Algorithm 1, fp64, plain C + OpenMP) on a sample of query blocks with every
    allowed block listed and the identity key order; reported in the metric's unit (TFLOP/s over visited blocks)."""
    import numpy as np
    from oracle import pbs_oracle as oracle
    threads = oracle.num_threads()
    T, R, G = w.T, w.segment // w.block, w.n // w.segment
    flop_per_block = 4.0 * w.block * w.block * w.d
    # calibrate on one short row, then pick rows until the budget is filled
    rng = np.random.default_rng(0)
    kidx = np.tile(np.arange(w.n, dtype=np.int32), (w.batch, w.h_kv, 1))

    # the oracle takes [B,Hq,T,T] lists; build them sparsely populated for the sampled rows only
    def run(rows):
        row_cnt = np.zeros((w.batch, w.h_q, T), dtype=np.int32)
        col_idx = np.zeros((w.batch, w.h_q, T, T), dtype=np.int32)
        blocks = 0
        for (b, h, i) in rows:
            g = i // R
            ni = min((g + 1) * R, T) if g < G else i + 1
            row_cnt[b, h, i] = ni
            col_idx[b, h, i, :ni] = np.arange(ni)
            blocks += ni
        t0 = time.perf_counter()
        oracle.attn_rows(w.Q, w.K, w.V, None, kidx, row_cnt, col_idx, w.block, rows)
        return time.perf_counter() - t0, blocks

    i_cal = min(T - 1, max(1, 2 * R - 1))
    t_cal, b_cal = run([[0, 0, i_cal]])
    per_block_core = t_cal / b_cal                               # seconds per block on one core
    budget_blocks = seconds_budget * threads / per_block_core
    rows, total = [], 0
    while total < budget_blocks and len(rows) < 4 * threads:
        i = int(rng.integers(T // 2, T))
        g = i // R
        ni = min((g + 1) * R, T) if g < G else i + 1
        rows.append([0, int(rng.integers(0, w.h_q)), i])
        total += ni
    secs, blocks = run(rows)
    out = {"value": blocks * flop_per_block / secs / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
           "sample": "%d query blocks (rows in the upper half, all allowed blocks listed, identity key order), "
                     "%d blocks of %dx%dx%d, fp64, %.1f s wall" % (len(rows), blocks, w.block, w.block, w.d, secs)}
    if visited is not None:
        # the other stages in full, and the attention loop scaled from the sample to the layer's visited blocks
        stages = {}
        t0 = time.perf_counter()
        s = oracle.key_scores(w.Q, w.K, w.block)
        stages["key_scores"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        kidx_o = oracle.segment_argsort(s.astype(np.float32), w.segment)
        Kp = oracle.gather_rows(w.K, kidx_o)
        oracle.gather_rows(w.V, kidx_o)
        stages["segment_permute"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.block_mask(w.Q, Kp, w.block, w.segment, w.tau, flags=w.flags)
        stages["block_mask"] = time.perf_counter() - t0
        stages["attn_fwd_extrapolated"] = secs * visited / blocks
        out["stages_s"] = stages
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-permute", action="store_true",
                    help="keep the keys in token order (identity permutation): what Algorithm 2 selects, and what "
                         "the attention costs, without the paper's permutation")
    ap.add_argument("--replicate-kv", action="store_true",
                    help="give every query head its own copy of its group's K and V (h_kv = h_q), i.e. one key "
                         "permutation per query head instead of one per kv head (appendix 'GQA Handling'); a "
                         "different configuration, named so in config.workload")
    ap.add_argument("--coverage", action="store_true",
                    help="after the timed region, also report the true attention mass inside the selected blocks "
                         "(two more attention passes, one of them over every admitted block)")
    ap.add_argument("--no-token-order-copy", action="store_true",
                    help="do not set PBS_FLAG_TOKEN_ORDER_COPY.  By default the permutation stage also writes K, V'^T "
                         "and kidx in token order (twice the bytes of that stage), and the attention evaluates every "
                         "query block's own segment from that copy: the blocks up to the diagonal, only the diagonal "
                         "one under the causal test (the same visible keys as the R permuted blocks of the segment, so "
                         "the same output)")
    ap.add_argument("--proxy", choices=["last", "random", "avg"], default="last",
                    help="which queries stand for all queries in the importance score: the last block (Eq. 4, the "
                         "paper's method), 128 positions drawn at random from a seed (Random-Query-Attn), or the average "
                         "query (Avg-Query-Attn); the other two are the paper's ablations, named so in config.workload")
    ap.add_argument("--key-aware-sigma", action="store_true",
                    help="also permute the queries, with the key-aware query permutation the paper ablates (sigma from "
                         "pbs_query_permutation on K', Q' gathered, output scattered back); adds the stage "
                         "'query_permute' and makes pbs_unpermute do real work; the own-segment shortcut is off then")
    ap.add_argument("--index-remap", action="store_true",
                    help="PBS_FLAG_INDEX_REMAP: no K' is materialised, the attention kernel gathers its K tiles from K "
                         "through kidx (the index remapping of the appendix 'Memory Overhead'); runs on the "
                         "running-maximum kernel")
    ap.add_argument("--dense-baseline", action="store_true",
                    help="after the timed region, also time plain causal attention in token order through the same "
                         "kernel (three more attention passes) and report the sparse layer's speed-up over it")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, run one plain device copy of known size through pbs_unpermute, so "
                         "that a rocprofv3 --pmc run of this command shows what FETCH_SIZE / WRITE_SIZE read for it")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the path shards by kv-head group with no exchange, and this "
                         "build runs on one MI355X only (--gpus 1)")
    import numpy as np
    import torch
    from paper_2510_21270_amd import binding as pbs

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    pbs.load_library()
    t_gen = time.perf_counter()
    w = make_workload(args.workload)
    t_gen = time.perf_counter() - t_gen
    if args.replicate_kv and w.h_kv != w.h_q:
        r = w.h_q // w.h_kv
        w.K, w.V = np.repeat(w.K, r, axis=1), np.repeat(w.V, r, axis=1)
        w.extra = {k: v for k, v in w.extra.items() if k != "planted"}      # keyed by kv head
        w.h_kv, w.name = w.h_q, w.name + "_replicated_kv"
    given = "row_cnt" in w.extra                      # config 5: caller-supplied block lists, identity key order
    variant = (args.proxy != "last") or args.key_aware_sigma or args.index_remap
    if args.key_aware_sigma and args.index_remap:
        raise SystemExit("--key-aware-sigma takes its centroids from K', which --index-remap does not materialise")
    if variant and given:
        raise SystemExit("--proxy / --key-aware-sigma / --index-remap need a workload that runs the whole path")
    token_copy = not (args.no_token_order_copy or given or args.key_aware_sigma or args.index_remap)
    flags = w.flags | (pbs.FLAG_TOKEN_ORDER_COPY if token_copy else 0) | (pbs.FLAG_INDEX_REMAP if args.index_remap else 0)
    if variant:
        w.name += "".join(["_proxy_" + args.proxy if args.proxy != "last" else "",
                           "_key_aware_sigma" if args.key_aware_sigma else "", "_index_remap" if args.index_remap else ""])
    p = pbs.problem(w.batch, w.h_q, w.h_kv, w.n, w.d, w.block, w.segment, w.dtype, tau=w.tau, flags=flags)
    Q, K, V = to_dev(w.Q, w.dtype), to_dev(w.K, w.dtype), to_dev(w.V, w.dtype)
    pipe = pbs.Pipeline(p, use_sigma=args.key_aware_sigma)
    if args.key_aware_sigma:
        qidx_buf = torch.empty((w.batch, w.h_q, w.n), dtype=torch.int32, device="cuda")
        ws6 = pbs.alloc_workspace(p, pbs.STAGE_QUERY_PERMUTE)
    qrows = None
    if args.proxy == "random":
        from paper_2510_21270_amd import workloads as wl_
        qrows = torch.from_numpy(wl_.random_query_rows(w.extra.get("seed", 0), w.n, 128)).cuda()
    proxy_code = {"last": pbs.PROXY_LAST_BLOCK, "random": pbs.PROXY_QUERY_ROWS, "avg": pbs.PROXY_AVG_QUERY}[args.proxy]
    if given:
        row_cnt = torch.from_numpy(w.extra["row_cnt"]).cuda()
        col_idx = torch.from_numpy(w.extra["col_idx"]).cuda()

    names = ["key_scores", "segment_permute", "query_permute", "block_mask", "attn_fwd", "unpermute"]

    def step(events=None):
        def mark(k):
            if events is not None:
                events[k].record()
        mark(0)
        qidx = None
        if given:
            mark(1)
            pbs.segment_permute(p, None, K, V, pipe.kidx, pipe.Kp, pipe.Vt)
            mark(2)
            mark(3)
            mark(4)
            pbs.attn_fwd(p, Q, pipe.Kp, pipe.Vt, None, pipe.kidx, row_cnt, col_idx, pipe.Op, ws=pipe.ws4)
        else:
            if args.proxy == "last":
                pbs.key_scores(p, Q, K, pipe.scores, pipe.ws1)
            else:
                pbs.key_scores_proxy(p, proxy_code, qrows, Q, K, pipe.scores, pipe.ws1)
            mark(1)
            pbs.segment_permute(p, None if args.no_permute else pipe.scores, K, V, pipe.kidx,
                                None if args.index_remap else pipe.Kp, pipe.Vt,
                                ws=pipe.ws3)          # the block means of K' come out of the gather
            keys = K if args.index_remap else pipe.Kp  # with index remapping the attention reads the caller's K
            mark(2)
            Qp = Q
            if args.key_aware_sigma:
                qidx = pbs.query_permutation(p, Q, pipe.Kp, qidx_buf, ws6)
                Qp = pbs.permute_rows(p, Q, qidx, pipe.Qp)
            mark(3)
            pbs.block_mask(pipe.p_kbar, Qp, keys, pipe.mask_bits, pipe.row_cnt, pipe.col_idx, pipe.ws3)
            mark(4)
            pbs.attn_fwd(p, Qp, keys, pipe.Vt, qidx, pipe.kidx, pipe.row_cnt, pipe.col_idx, pipe.Op, ws=pipe.ws4)
        mark(5)
        pbs.unpermute(p, pipe.Op, qidx, pipe.O)        # P_sigma = I in the paper's main setting: nothing to move
        mark(6)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = {nm: float(np.mean([evs[k][s].elapsed_time(evs[k][s + 1]) for k in range(args.steps)]))
                for s, nm in enumerate(names)}

    if args.copy_calibration:
        scratch = torch.empty_like(pipe.Op)
        pbs.unpermute(p, pipe.Op, None, scratch)           # identity sigma + distinct output = plain copy
        torch.cuda.synchronize()
        print("copy calibration: move_rows_kernel<true> read %d bytes and wrote %d bytes" %
              (scratch.numel() * scratch.element_size(), scratch.numel() * scratch.element_size()), file=sys.stderr)
        del scratch

    # ---- untimed extras: where the planted keys end up, the inverse permutation with a real sigma, a plain copy
    extras = {}
    if not given and "planted" in w.extra:
        kidx_h = pipe.kidx.cpu().numpy()
        seg = w.segment
        ranks = []
        for (b, h), pos in w.extra["planted"].items():
            slot_of = np.empty(w.n, dtype=np.int64)
            slot_of[kidx_h[b, h]] = np.arange(w.n)
            pos = pos[pos < (w.n // seg) * seg]
            ranks.append((slot_of[pos] % seg) / float(seg))
        ranks = np.concatenate(ranks) if ranks else np.zeros(0)
        if ranks.size:                                     # 0 = first slot of its segment, 0.5 = no better than chance
            extras["planted_keys_mean_rank_in_segment"] = float(ranks.mean())
            extras["planted_keys_in_first_block_of_segment"] = float((ranks < w.block / float(seg)).mean())
    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    if not args.copy_calibration:
        from paper_2510_21270_amd import workloads as wl
        scratch = torch.empty_like(pipe.Op)
        nbytes = 2.0 * scratch.numel() * scratch.element_size()
        ms_copy = timed(lambda: pbs.unpermute(p, pipe.Op, None, scratch))
        sigma = torch.from_numpy(wl.random_segment_perm(7, w.batch * w.h_q, w.n, w.segment)
                                 .reshape(w.batch, w.h_q, w.n)).cuda()
        ms_sigma = timed(lambda: pbs.unpermute(p, pipe.Op, sigma, scratch))
        extras["plain_copy"] = {"ms": ms_copy, "GBps": nbytes / ms_copy / 1e6, "bytes": nbytes}
        extras["unpermute_random_sigma"] = {"ms": ms_sigma, "GBps": (nbytes + sigma.numel() * 4) / ms_sigma / 1e6}
        del scratch, sigma
        if args.coverage and not given and not variant:
            # true attention mass inside the selected blocks (two more attention passes, untimed)
            _, lse_sel = pbs.attn_fwd(p, Q, pipe.Kp, pipe.Vt, None, pipe.kidx, pipe.row_cnt, pipe.col_idx, pipe.Op,
                                      want_lse=True, ws=pipe.ws4)
            rc_all, ci_all = pbs.admitted_lists(p)
            _, lse_all = pbs.attn_fwd(p, Q, pipe.Kp, pipe.Vt, None, pipe.kidx, rc_all, ci_all, pipe.Op, want_lse=True,
                                      ws=pipe.ws4)
            cov = pbs.mass_covered(p, lse_sel, lse_all)
            del rc_all, ci_all, lse_sel, lse_all
            extras["attention_mass_covered"] = {"mean": float(cov.mean()), "min_row": float(cov.min()),
                                                "rows_below_tau": float((cov < w.tau).float().mean())}
            del cov
        if args.dense_baseline and not given and not variant:
            # full causal attention in token order through the same kernel (every block up to the diagonal listed):
            # the dense pass that the paper's speed-ups are quoted against, on this GPU; overwrites K', V' and O'
            pbs.segment_permute(p, None, K, V, pipe.kidx, pipe.Kp, pipe.Vt)
            rc_dense = (torch.arange(w.T, device="cuda", dtype=torch.int32) + 1).view(1, 1, w.T) \
                .expand(w.batch, w.h_q, w.T).contiguous()
            ci_dense = torch.arange(w.T, device="cuda", dtype=torch.int32).view(1, 1, 1, w.T) \
                .expand(w.batch, w.h_q, w.T, w.T).contiguous()
            ms_dense = timed(lambda: pbs.attn_fwd(p, Q, pipe.Kp, pipe.Vt, None, pipe.kidx, rc_dense, ci_dense,
                                                  pipe.Op, ws=pipe.ws4), reps=2)
            dense_blocks = w.batch * w.h_q * w.T * (w.T + 1) // 2
            extras["dense_causal_same_kernel"] = {
                "ms": ms_dense, "tflops": dense_blocks * 4.0 * w.block * w.block * w.d / ms_dense / 1e9,
                "layer_speedup_of_the_sparse_path": ms_dense / ms_per_step}
            del rc_dense, ci_dense
        # what the matrix units sustain on their own, with operand bits that cost no / realistic switching power
        zero_rate, zero_mhz = pbs.mfma_rate_probe(False)
        rand_rate, rand_mhz = pbs.mfma_rate_probe(True)
        extras["mfma_alone_tflops"] = {"zero_operands": zero_rate, "random_operands": rand_rate}
        extras["shader_clock_mhz"] = {"mfma_alone_zero_operands": zero_mhz, "mfma_alone_random_operands": rand_mhz}
        if not given and not variant:
            # the clock pbs_attn_fwd runs at: one watching wave on a second stream beside two attention launches
            def two_attention_launches():
                for _ in range(2):
                    pbs.attn_fwd(p, Q, pipe.Kp, pipe.Vt, None, pipe.kidx, pipe.row_cnt, pipe.col_idx, pipe.Op,
                                 ws=pipe.ws4)
            mhz, watched_us = pbs.shader_clock_beside(two_attention_launches, micros=20000,
                                                      delay_s=min(0.02, stage_ms["attn_fwd"] * 0.3e-3))
            if watched_us < 1.2e3 * stage_ms["attn_fwd"]:      # the watch ended inside the launches
                extras["shader_clock_mhz"]["pbs_attn_fwd"] = mhz

    cnt = (row_cnt if given else pipe.row_cnt).cpu().numpy().astype(np.int64)
    visited = int(cnt.sum())                           # blocks the masks list
    T = w.T
    # blocks that are multiplied: with the token-order copy, a query block i of a full segment whose list ends with
    # its R own-segment blocks inside one staged chunk of 1024 entries takes i % R + 1 blocks for them instead of R
    computed = visited
    own_in_token_order = (token_copy and w.dtype == "bf16" and w.d == 128 and w.block == 128 and
                          (w.batch * w.h_kv + 1) * T * 128 * 256 < 2 ** 31 - 1)   # what pbs_attn_fwd requires for it
    if own_in_token_order:
        R, G = w.segment // w.block, w.n // w.segment
        i = np.arange(T, dtype=np.int64)[None, None, :]
        applies = (i // R < G) & (cnt >= R) & (((cnt - 1) % 1024) + 1 >= R)
        computed = int(visited - np.where(applies, R - (i % R + 1), 0).sum())
    causal_total = w.batch * w.h_q * T * (T + 1) // 2
    flop = computed * 4.0 * w.block * w.block * w.d     # effective TFLOP/s counts computed blocks only
    es = 2 if w.dtype == "bf16" else 4
    kv_bytes = 2 * w.batch * w.h_kv * w.n * w.d * es
    q_bytes = w.batch * w.h_q * w.n * w.d * es
    alg_bytes = {   # algorithmic HBM bytes of the bandwidth-bound stages (each tensor moved once)
        "key_scores": kv_bytes // 2 + w.batch * w.h_q * min(w.block, w.n) * w.d * es + w.batch * w.h_kv * w.n * 4,
        "segment_permute": 2 * kv_bytes + 2 * w.batch * w.h_kv * w.n * 4,
        "block_mask": q_bytes + kv_bytes // 2 + visited * 4 + w.batch * w.h_q * T * ((T + 63) // 64) * 8,
    }
    if given:
        alg_bytes = {"segment_permute": alg_bytes["segment_permute"] - w.batch * w.h_kv * w.n * 4}
    # bytes the permutation stage moves beyond the algorithmic ones: with the token-order copies K and V are read and
    # written a second time (the second read mostly from cache) and a second index vector is written
    moved_extra = {"segment_permute": 2 * kv_bytes + w.batch * w.h_kv * w.n * 4 if token_copy else 0}
    attn_tflops = flop / (stage_ms["attn_fwd"] * 1e-3) / 1e12
    visited_tflops = visited * 4.0 * w.block * w.block * w.d / (stage_ms["attn_fwd"] * 1e-3) / 1e12
    traffic, traffic_src = measured_attn_traffic(args.workload)
    roofline = {"kernel": "pbs_attn_fwd", "bound": "mfma", "achieved": attn_tflops,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS,
                "frac_from_visited_blocks": visited_tflops / MFMA_BF16_PEAK_TFLOPS,
                "traffic": traffic, "traffic_source": traffic_src or "not measured for this workload",
                "avg_launch_ms": stage_ms["attn_fwd"]}
    if not (w.dtype == "bf16" and w.d == 128 and w.block in (64, 128)):
        # every other shape runs on fp32 vector arithmetic (attn_vector_kernel): rated against the chip's fp32 vector
        # peak (256 compute units x 128 FMA lanes x 2 x 2.4 GHz = 157.3 TFLOP/s)
        roofline.update(bound="alu", peak=FP32_VECTOR_PEAK_TFLOPS, frac=attn_tflops / FP32_VECTOR_PEAK_TFLOPS,
                        frac_from_visited_blocks=visited_tflops / FP32_VECTOR_PEAK_TFLOPS)
    if given:
        # Caller-supplied lists drawn independently per query head: no two heads of a group share K'/V'^T tiles, so
        # every listed block fetches its 2 * block * d tile bytes (128 FLOP per byte), plus Q' and O' once.  Whichever
        # bound is nearer names the line.
        tile_bytes = visited * 2.0 * w.block * w.d * es + 2.0 * q_bytes
        hbm_gbs = tile_bytes / (stage_ms["attn_fwd"] * 1e-3) / 1e9
        roofline["frac_mfma"] = roofline["frac"]
        roofline["frac_hbm_unshared_tiles"] = hbm_gbs / HBM_PEAK_GBS
        # (above 1 the model is refuted: tiles are being shared in the caches, as they are at high densities, where
        # the heads of a cohort list many of the same blocks, and the line stays with the matrix bound)
        if roofline["frac_mfma"] < roofline["frac_hbm_unshared_tiles"] <= 1.0:
            roofline.update(bound="hbm", achieved=hbm_gbs, peak=HBM_PEAK_GBS, unit="GB/s",
                            frac=hbm_gbs / HBM_PEAK_GBS)
            roofline.pop("frac_from_visited_blocks")
    out = {
        "metric": "pbs_attn_prefill_effective_tflops", "value": flop / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_layer": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": dict(w.describe(), visited_blocks=visited, causal_blocks=causal_total,
                       token_order_copy=bool(token_copy), own_segment_in_token_order=bool(own_in_token_order),
                       computed_blocks=computed,
                       density_vs_causal=visited / causal_total, given_mask=bool(given),
                       permuted=not (given or args.no_permute)),
        "stages_ms": stage_ms,
        "stages_gbs": {k: alg_bytes[k] / (stage_ms[k] * 1e-3) / 1e9 for k in alg_bytes if stage_ms[k] > 0},
        "stages_frac_of_hbm_peak": {k: alg_bytes[k] / (stage_ms[k] * 1e-3) / 1e9 / HBM_PEAK_GBS
                                    for k in alg_bytes if stage_ms[k] > 0},
        "stages_algorithmic_bytes": alg_bytes, "stages_extra_bytes_moved": moved_extra,
        "roofline": roofline,
        "context": {"paper_h100_128k_ms": {"flashattention": 443.29, "pbs_total": 159.87, "speedup": 2.77},
                    "input_generation_s": t_gen, **extras},
    }
    if "mfma_alone_tflops" in extras and out["roofline"]["bound"] != "alu":
        out["roofline"]["frac_of_mfma_alone_random_operands"] = attn_tflops / extras["mfma_alone_tflops"]["random_operands"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, visited=None if given else visited)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
