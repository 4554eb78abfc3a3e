"""The entry point that allocates nothing (pbs_key_scores_static) against pbs_key_scores, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2510_21270_amd import binding as pbs

pytestmark = pytest.mark.gpu


def _scores_both_ways(n, h_q, h_kv, d, block, dtype, seed):
    lib = pbs.load_library()
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cuda").manual_seed(seed)
    Q = torch.randn(1, h_q, n, d, device="cuda", generator=gen).to(tdt)
    K = torch.randn(1, h_kv, n, d, device="cuda", generator=gen).to(tdt)
    p = pbs.problem(1, h_q, h_kv, n, d, block, 4 * block, dtype)
    # the existing entry point with a caller-supplied workspace
    ws = pbs.alloc_workspace(p, pbs.STAGE_KEY_SCORES)
    want = torch.full((1, h_kv, n), -1.0, dtype=torch.float32, device="cuda")
    st = lib.pbs_key_scores(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), want.data_ptr(), ws.data_ptr(), ws.numel(), None)
    assert st == 0
    # the one without: inputs and outputs only (allocated before the call)
    got = torch.full((1, h_kv, n), -2.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    st = lib.pbs_key_scores_static(ctypes.byref(p), Q.data_ptr(), K.data_ptr(), got.data_ptr(), None)
    assert st == 0
    torch.cuda.synchronize()
    return got, want


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    # a larger problem first, then a smaller one that finds the larger one's leftovers in the shared array; both
    # through the matrix-core sweeps (bf16, d = 128) with ragged lengths
    for (n, h_q, h_kv, seed) in [(24576 + 77, 8, 4, 1), (4096 + 5, 4, 2, 2)]:
        got, want = _scores_both_ways(n, h_q, h_kv, 128, 128, "bf16", seed)
        assert torch.equal(got, want), "n=%d" % n                 # same kernels, same order: bit-identical
        assert abs(float(got[0, 0].double().sum()) - 1.0) < 1e-3
    # and the fp64 vector path (fp32 inputs, d = 64), again larger then smaller
    for (n, seed) in [(3000, 3), (700, 4)]:
        got, want = _scores_both_ways(n, 2, 2, 64, 64, "f32", seed)
        assert torch.equal(got, want), "f32 n=%d" % n


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    lib = pbs.load_library()
    cap = lib.pbs_key_scores_static_scratch_bytes()
    assert cap == 4 << 20
    p = pbs.problem(1, 64, 64, 262144, 128, 128, 1024, "bf16")     # 64 kv heads: 18 MiB of scratch
    assert pbs.workspace_bytes(p, pbs.STAGE_KEY_SCORES) > cap
    x = torch.zeros(16, device="cuda")
    assert lib.pbs_key_scores_static(ctypes.byref(p), x.data_ptr(), x.data_ptr(), x.data_ptr(), None) == 4   # PBS_ERR_WORKSPACE
    torch.cuda.synchronize()
