"""Seeded synthetic workloads for the PBS-Attn prefill path.

This module only MAKES INPUTS.  It holds none of the method's arithmetic (no
scoring, sorting, pooling, selection or attention) and is the one module that
both the CPU oracle's tests and the HIP path's tests/benchmark draw from.

The paper measures on LongBench / LongBench-v2 / RULER prompts run through
Llama-3.1-8B and Qwen2.5-7B weights (Section "Settings").  Neither is available
here, so the workloads below stand in for them: the models' head shapes, RoPE'd
Gaussian Q/K, and planted "heavy hitter" and "sink" keys that mimic the vertical
lines the paper describes (Section "Global-Importance-based Permutation").

Every array is generated in float32 from numpy's default_rng with a fixed seed
and a per-tensor sub-stream, then rounded once to the storage type.  Arrays are
returned as float32 holding storage-exact values (`f32`) plus, for bf16
workloads, the uint16 bit patterns (`bits`) ready to be viewed as bfloat16.
"""
from dataclasses import dataclass, field

import numpy as np

SEEDS = {"c1": 1001, "c2": 1002, "c3": 1003, "c4": 1004, "c5": 1005}


def round_to_bf16(x):
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    out = (u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return out.view(np.float32)


def bf16_bits(x_rounded):
    """uint16 bit patterns of float32 values that are already bf16-exact."""
    return (np.ascontiguousarray(x_rounded, dtype=np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


@dataclass
class Workload:
    name: str
    batch: int
    h_q: int
    h_kv: int
    n: int
    d: int
    block: int
    segment: int
    tau: float
    dtype: str              # "f32" or "bf16" (storage type of Q, K, V, O)
    flags: int
    Q: np.ndarray           # float32, storage-exact, [batch, h_q, n, d]
    K: np.ndarray           # float32, storage-exact, [batch, h_kv, n, d]
    V: np.ndarray
    extra: dict = field(default_factory=dict)

    @property
    def T(self):
        return -(-self.n // self.block)

    def describe(self):
        return dict(workload=self.name, batch=self.batch, h_q=self.h_q, h_kv=self.h_kv, n=self.n, d=self.d,
                    block=self.block, segment=self.segment, tau=float("%.6g" % self.tau), storage=self.dtype)


def _rng(seed, stream):
    return np.random.default_rng([int(seed), int(stream)])


def _normal(seed, stream, shape):
    return _rng(seed, stream).standard_normal(shape, dtype=np.float32)


def _rope_inplace(x, base):
    """Rotary embedding, rotate-half pairing (e, e + d/2), angle = pos * base**(-2e/d); x [..., n, d]."""
    n, d = x.shape[-2:]
    half = d // 2
    inv = np.power(float(base), -2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.arange(n, dtype=np.float64)[:, None] * inv[None, :]
    cos = np.cos(ang).astype(np.float32)
    sin = np.sin(ang).astype(np.float32)
    flat = x.reshape(-1, n, d)
    for h in range(flat.shape[0]):
        x1 = flat[h, :, :half].copy()
        x2 = flat[h, :, half:]
        flat[h, :, :half] = x1 * cos - x2 * sin
        flat[h, :, half:] = x2 * cos + x1 * sin
    return x


def _plant(Q, K, seed, n_scatter, n_sink=4, bursts=0, burst_len=0):
    """Overwrite chosen key rows by 4*u + noise, u = unit mean-query direction of the kv head's group."""
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    r = Hq // Hkv
    planted = {}
    for b in range(B):
        for h in range(Hkv):
            rng = _rng(seed, 100 + b * Hkv + h)
            u = Q[b, h * r:(h + 1) * r].reshape(-1, d).mean(axis=0, dtype=np.float64)
            u = (u / np.linalg.norm(u)).astype(np.float32)
            pos = []
            for _ in range(bursts):
                start = int(rng.integers(n_sink, max(n_sink + 1, N - burst_len)))
                pos.extend(range(start, min(N, start + burst_len)))
            k = min(n_scatter, max(0, N - n_sink))
            if k > 0:
                pos.extend((n_sink + rng.choice(N - n_sink, size=k, replace=False)).tolist())
            pos = np.unique(np.asarray(pos, dtype=np.int64))
            if pos.size:
                K[b, h, pos] = 4.0 * u[None, :] + 0.1 * rng.standard_normal((pos.size, d), dtype=np.float32)
            K[b, h, :min(n_sink, N)] = 4.0 * u[None, :]
            planted[(b, h)] = pos
    return planted


def _finish(name, Q, K, V, dtype, **kw):
    if dtype == "bf16":
        Q, K, V = round_to_bf16(Q), round_to_bf16(K), round_to_bf16(V)
    # like the tensors, the threshold is rounded once to the type it is handed over in (a float in the C ABI), so
    # that every consumer of the workload compares with the same number
    kw["tau"] = float(np.float32(kw["tau"]))
    return Workload(name=name, batch=Q.shape[0], h_q=Q.shape[1], h_kv=K.shape[1], n=Q.shape[2], d=Q.shape[3],
                    dtype=dtype, Q=Q, K=K, V=V, **kw)


def planted(name, seed, h_q, h_kv, n, d, block, segment, tau, dtype, n_scatter, rope_base=None, bursts=0,
            burst_len=0, batch=1, flags=1, shared_query=0.0):
    """The family behind configs 1-4: Gaussian Q/K/V, optional RoPE on Q/K, planted heavy hitters + 4 sinks.
    shared_query > 0 (not part of any numbered config) adds that multiple of one seeded unit vector per kv head to
    every query of its group, so that the mean-query direction the planted keys point along is one all queries share."""
    Q = _normal(seed, 1, (batch, h_q, n, d))
    K = _normal(seed, 2, (batch, h_kv, n, d))
    V = _normal(seed, 3, (batch, h_kv, n, d))
    if rope_base is not None:
        _rope_inplace(Q, rope_base)
        _rope_inplace(K, rope_base)
    if shared_query > 0.0:
        r = h_q // h_kv
        for b in range(batch):
            for h in range(h_kv):
                u0 = _rng(seed, 200 + b * h_kv + h).standard_normal(d).astype(np.float32)
                Q[b, h * r:(h + 1) * r] += np.float32(shared_query) * (u0 / np.linalg.norm(u0))
    pl = _plant(Q, K, seed, n_scatter, bursts=bursts, burst_len=burst_len)
    return _finish(name, Q, K, V, dtype, block=block, segment=segment, tau=tau, flags=flags,
                   extra={"planted": pl, "seed": seed})


def c1_tiny(n=2048, seed=SEEDS["c1"]):
    """Config 1: fp32, 2 heads, d=64, block 64, segment 512, tau 0.9, 16 heavy hitters per head."""
    return planted("c1_tiny_f32_n%d" % n, seed, 2, 2, n, 64, 64, 512, 0.9, "f32", 16)


def c2_llama(n=32768, h_q=32, h_kv=8, n_scatter=None, seed=SEEDS["c2"]):
    """Config 2: Llama-3.1-8B-shaped layer, bf16, d=128, block 128, segment 1024, RoPE base 5e5."""
    ns = n_scatter if n_scatter is not None else max(1, 64 * n // 32768)
    return planted("c2_llama_bf16_n%d" % n, seed, h_q, h_kv, n, 128, 128, 1024, 0.9, "bf16", ns, rope_base=5e5)


def c3_llama128k(n=131072, h_q=32, h_kv=8, seed=SEEDS["c3"]):
    """Config 3: the headline point, same layer at N=131072 with 256 heavy hitters per kv head."""
    ns = max(1, 256 * n // 131072)
    return planted("c3_llama_bf16_n%d" % n, seed, h_q, h_kv, n, 128, 128, 1024, 0.9, "bf16", ns, rope_base=5e5)


def c3_strong(n=131072, h_q=32, h_kv=8, seed=SEEDS["c3"]):
    """NOT one of the numbered configs: an extra, strengthened variant of config 3 in which the planted keys really
    are heavy hitters.  Every query carries a shared component of 24 along its kv head's direction (a planted key
    4u then has logit ~ 8.5 nats against every query, the Gaussian keys ~ N(0, 2.3^2)), and one key in eight is
    planted, so that after the segmented permutation the first block of each 1024-key segment is all heavy."""
    return planted("c3_strong_bf16_n%d" % n, seed, h_q, h_kv, n, 128, 128, 1024, 0.9, "bf16", n // 8, rope_base=5e5,
                   shared_query=24.0)


def c4_qwen(n=65536, h_q=28, h_kv=4, seed=SEEDS["c4"]):
    """Config 4: Qwen2.5-7B-shaped layer, GQA 7:1, segment 2048, tau 0.95, 8 bursts of 16 + 64 singletons."""
    return planted("c4_qwen_bf16_n%d" % n, seed, h_q, h_kv, n, 128, 128, 2048, 0.95, "bf16", 64, rope_base=1e6,
                   bursts=8, burst_len=16)


def random_block_lists(seed, batch, h_q, T, rho):
    """Config 5's masks: per query head the diagonal plus exactly round(rho*T(T+1)/2) - T strictly-lower
    blocks drawn without replacement (all of them when rho >= 1).  Returns (row_cnt, col_idx) with
    ascending columns and -1 fill."""
    total = T * (T + 1) // 2
    lower = total - T
    want = lower if rho >= 1.0 else max(0, min(lower, int(round(rho * total)) - T))
    ii, jj = np.tril_indices(T, k=-1)
    row_cnt = np.empty((batch, h_q, T), dtype=np.int32)
    col_idx = np.full((batch, h_q, T, T), -1, dtype=np.int32)
    for b in range(batch):
        for h in range(h_q):
            m = np.zeros((T, T), dtype=bool)
            m[np.arange(T), np.arange(T)] = True
            if want == lower:
                m[ii, jj] = True
            elif want > 0:
                pick = _rng(seed, 500 + b * h_q + h).choice(lower, size=want, replace=False)
                m[ii[pick], jj[pick]] = True
            cnt = m.sum(axis=1)
            row_cnt[b, h] = cnt
            order = np.argsort(~m, axis=1, kind="stable")      # True columns first, ascending
            cols = np.where(np.arange(T)[None, :] < cnt[:, None], order, -1)
            col_idx[b, h] = cols
    return row_cnt, col_idx


def c5_density(rho, n=65536, h_q=32, h_kv=8, seed=SEEDS["c5"]):
    """Config 5: i.i.d. Gaussian bf16 Q/K/V (no RoPE, no planting), identity key order, given block masks."""
    Q = _normal(seed, 1, (1, h_q, n, 128))
    K = _normal(seed, 2, (1, h_kv, n, 128))
    V = _normal(seed, 3, (1, h_kv, n, 128))
    w = _finish("c5_density%.2f_bf16_n%d" % (rho, n), Q, K, V, "bf16", block=128, segment=1024, tau=0.9, flags=0,
                extra={"seed": seed, "rho": rho})
    w.extra["row_cnt"], w.extra["col_idx"] = random_block_lists(seed, 1, h_q, w.T, rho)
    return w


def random_segment_perm(seed, nbh, n, segment):
    """A seeded segment-wise permutation (gather form, absolute positions; tail identity) used to exercise
    general sigma / pi in Theorem 1 and the inverse permutation."""
    rng = _rng(seed, 900)
    idx = np.tile(np.arange(n, dtype=np.int32), (nbh, 1))
    G = n // segment
    for bh in range(nbh):
        for g in range(G):
            idx[bh, g * segment:(g + 1) * segment] = g * segment + rng.permutation(segment).astype(np.int32)
    return idx


def random_query_rows(seed, n, m):
    """m distinct query positions drawn uniformly from [0, n), ascending (the Random-Query proxy draws its queries at
    random; the draw is an input of the scoring call, not something the library does)."""
    rng = _rng(seed, 300)
    return np.sort(rng.choice(n, size=min(m, n), replace=False)).astype(np.int32)
