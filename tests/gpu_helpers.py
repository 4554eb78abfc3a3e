"""Helpers for the GPU parity tests: host<->device marshalling and layout conversions (data movement only)."""
import numpy as np
import torch

from paper_2510_21270_amd import binding as pbs
from paper_2510_21270_amd import workloads as wl

TOL = {"bf16": dict(max_abs=2e-2, mean_abs=2e-3), "f32": dict(max_abs=1e-4, mean_abs=1e-4)}


def to_dev(x_f32, dtype):
    """float32 numpy array with storage-exact values -> device tensor of the storage dtype."""
    x = np.ascontiguousarray(x_f32, dtype=np.float32)
    if dtype == "bf16":
        bits = torch.from_numpy(wl.bf16_bits(x).view(np.int16))
        return bits.view(torch.bfloat16).cuda()
    return torch.from_numpy(x).cuda()


def to_host(t):
    """device tensor -> float64 numpy (bf16 widened exactly)."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def i32_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def vt_layout(Vp, block):
    """[B,H,N,d] (numpy) -> the library's V' layout [B,H,T,block/G,d,G], G = min(block, 32), zero padded."""
    B, H, N, d = Vp.shape
    T = -(-N // block)
    G = min(block, 32)
    pad = np.zeros((B, H, T * block, d), dtype=Vp.dtype)
    pad[:, :, :N] = Vp
    return np.ascontiguousarray(pad.reshape(B, H, T, block // G, G, d).transpose(0, 1, 2, 3, 5, 4))


def mask_from_bits(bits, T):
    """int64 device tensor [B,Hq,T,W] -> uint8 numpy [B,Hq,T,T]."""
    words = bits.cpu().numpy().view(np.uint64)
    shifts = np.arange(64, dtype=np.uint64)
    m = ((words[..., None] >> shifts) & np.uint64(1)).astype(np.uint8)
    return m.reshape(words.shape[:-1] + (-1,))[..., :T]


def make_problem(w, tau=None, flags=None, segment=None, scale=0.0):
    return pbs.problem(w.batch, w.h_q, w.h_kv, w.n, w.d, w.block, segment or w.segment, w.dtype,
                       tau=w.tau if tau is None else tau, scale=scale, flags=w.flags if flags is None else flags)


def check_close(got, want, dtype, what=""):
    err = np.abs(got - want)
    tol = TOL[dtype]
    assert np.isfinite(got).all(), what
    assert err.max() <= tol["max_abs"], "%s max-abs %.3e > %.1e" % (what, err.max(), tol["max_abs"])
    assert err.mean() <= tol["mean_abs"], "%s mean-abs %.3e > %.1e" % (what, err.mean(), tol["mean_abs"])
    return float(err.max()), float(err.mean())


def with_token_copy(p, kind, first, second):
    """A K' ("kp"), Vt ("vt") or kidx ("kidx") tensor of problem p (PBS_FLAG_TOKEN_ORDER_COPY set) holding `first`,
    with `second` as the token-order copy behind it."""
    x = {"kp": pbs.alloc_kp, "vt": pbs.alloc_vt, "kidx": pbs.alloc_kidx}[kind](p)
    x.copy_(first)
    pbs.token_copy(p, x, 1 if kind == "kidx" else p.d).copy_(second)
    return x


def coverage(p, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx):
    """Attention mass inside the listed blocks [batch, h_q, n]: two pbs_attn_fwd calls (the listed blocks, every
    admitted block) and the two coverage entry points of the library."""
    Op = torch.empty_like(Qp)
    _, lse_sel = pbs.attn_fwd(p, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, want_lse=True)
    rc_all, ci_all = pbs.admitted_lists(p)
    _, lse_all = pbs.attn_fwd(p, Qp, Kp, Vt, qidx, kidx, rc_all, ci_all, Op, want_lse=True)
    return pbs.mass_covered(p, lse_sel, lse_all), rc_all, ci_all
