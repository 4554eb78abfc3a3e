"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header declares,
validates arguments before launching anything, and sizes workspaces sensibly."""
import ctypes
import os
import re

import pytest

from paper_2510_21270_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(b.LIB_PATH):
        from paper_2510_21270_amd import build
        build.build()
    return b.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "pbs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pbs_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(b.EXPORTS) == names


def test_status_strings(lib):
    seen = {lib.pbs_status_string(code) for code in range(6)}
    assert len(seen) == 6 and all(seen)
    assert lib.pbs_status_string(99)


def _p(**kw):
    base = dict(batch=1, h_q=32, h_kv=8, n=131072, d=128, block=128, segment=1024, dtype="bf16", tau=0.9, scale=0.0,
                flags=1)
    base.update(kw)
    return b.problem(**base)


def test_validation_codes(lib):
    assert b.validate(_p()) == 0
    assert lib.pbs_validate(None) == 1
    assert b.validate(_p(h_q=30)) == 2                 # h_q % h_kv
    assert b.validate(_p(segment=1000)) == 2           # segment % block
    assert b.validate(_p(n=0)) == 2
    assert b.validate(_p(scale=-1.0)) == 2
    assert b.validate(_p(tau=float("nan"))) == 2
    assert b.validate(_p(d=96)) == 3
    assert b.validate(_p(block=48, segment=96)) == 3
    assert b.validate(_p(segment=8192)) == 3
    assert b.validate(_p(n=128 * 4097)) == 3           # T > 4096
    p = _p()
    p.dtype = 7
    assert b.validate(p) == 3
    assert b.validate(_p(n=5, block=16, segment=16, d=64, dtype="f32", h_q=2, h_kv=2)) == 0


def test_null_pointers_are_rejected_before_any_launch(lib):
    p = _p()
    ref = ctypes.byref(p)
    fake = ctypes.c_void_p(4096)                       # never dereferenced: a NULL elsewhere is found first
    assert lib.pbs_key_scores(ref, None, fake, fake, fake, 1 << 30, None) == 1
    assert lib.pbs_key_scores(ref, fake, fake, None, fake, 1 << 30, None) == 1
    assert lib.pbs_segment_permute(ref, fake, fake, fake, None, fake, fake, None, 0, None) == 1
    assert lib.pbs_segment_permute(ref, fake, fake, fake, fake, fake, None, None, 0, None) == 1   # Kp without Vt
    assert lib.pbs_segment_permute(ref, fake, None, fake, fake, fake, fake, None, 0, None) == 1   # Kp without K
    assert lib.pbs_permute_rows(ref, 32, fake, None, fake, None) == 1
    assert lib.pbs_block_mask(ref, fake, fake, None, fake, fake, fake, 1 << 30, None) == 1
    assert lib.pbs_attn_fwd(ref, fake, fake, fake, None, None, fake, fake, fake, None, None, 0, None) == 1
    assert lib.pbs_unpermute(ref, None, None, fake, None) == 1
    # workspace: missing, too small, misaligned
    assert lib.pbs_key_scores(ref, fake, fake, fake, None, 0, None) == 1
    assert lib.pbs_key_scores(ref, fake, fake, fake, fake, 16, None) == 4
    assert lib.pbs_key_scores(ref, fake, fake, fake, ctypes.c_void_p(4096 + 8), 1 << 30, None) == 4
    assert lib.pbs_block_mask(ref, fake, fake, fake, fake, fake, fake, 16, None) == 4
    assert lib.pbs_attn_fwd(ref, fake, fake, fake, None, fake, fake, fake, fake, None, None, 0, None) == 1
    assert lib.pbs_attn_fwd(ref, fake, fake, fake, None, fake, fake, fake, fake, None, fake, 16, None) == 4
    # misaligned tensors
    assert lib.pbs_unpermute(ref, ctypes.c_void_p(4096 + 4), None, fake, None) == 2
    # the measurement aid checks its arguments before launching as well
    flop = ctypes.c_double(0.0)
    assert lib.pbs_mfma_rate_probe(1, 10, None, 262144, ctypes.byref(flop), None) == 1
    assert lib.pbs_mfma_rate_probe(1, 10, fake, 262144, None, None) == 1
    assert lib.pbs_mfma_rate_probe(1, 0, fake, 262144, ctypes.byref(flop), None) == 2
    assert lib.pbs_mfma_rate_probe(1, 10, fake, 262143, ctypes.byref(flop), None) == 2
    assert lib.pbs_shader_clock_meter(None, 100, None) == 1
    assert lib.pbs_shader_clock_meter(fake, 0, None) == 2
    # invalid problem wins over everything
    bad = _p(h_q=30)
    assert lib.pbs_attn_fwd(ctypes.byref(bad), None, None, None, None, None, None, None, None, None, None, 0, None) == 2


def test_workspace_and_vt_sizes(lib):
    p = _p()
    T = 1024
    assert b.vt_bytes(p) == 8 * T * 128 * 128 * 2 == 8 * 131072 * 128 * 2
    # pooled means of K' in fp64 (those of Q' never leave the selection kernel)
    assert b.workspace_bytes(p, b.STAGE_BLOCK_MASK) == 8 * T * 128 * 8
    assert b.workspace_bytes(p, b.STAGE_KEY_SCORES) > 0
    # one redo flag per query block for the 64-queries-per-wave kernel (bf16, d = 128, block = 128), nothing otherwise
    assert b.workspace_bytes(p, b.STAGE_ATTN_FWD) == 32 * T * 4
    assert b.workspace_bytes(_p(block=64), b.STAGE_ATTN_FWD) == 0
    assert b.workspace_bytes(_p(h_q=30), b.STAGE_BLOCK_MASK) == 0
    # partial last block is padded in Vt
    q = _p(n=1000, block=64, segment=256, d=64, dtype="f32", h_q=2, h_kv=2)
    assert b.vt_bytes(q) == 2 * 16 * 64 * 64 * 4
    # a token-order copy behind the permuted tensor doubles it
    p.flags = b.FLAG_TOKEN_ORDER_COPY
    assert b.vt_bytes(p) == 2 * 8 * T * 128 * 128 * 2


def test_paper_memory_figures():
    # appendix "Memory Overhead": B x N bf16 scoring temp at B=128, N=128K, and one permuted K (or V) copy at
    # d=128, N=128K, are both about 32 MiB per head.
    assert 128 * 131072 * 2 == 32 * 2 ** 20
    assert 131072 * 128 * 2 == 32 * 2 ** 20


def test_bench_refuses_more_than_one_gpu():
    # every box of this build has one GPU; the bench must say so instead of starting ranks
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "one GPU" in (res.stderr + res.stdout)
