"""Thin ctypes binding of libpbs.so (include/pbs.h).  Argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the library's HIP kernels.
The functions carry the names of the C entry points.  There is no CPU fallback: if the library is missing
or a call fails, an exception is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpbs.so")
_lib = None

PBS_F32, PBS_BF16 = 0, 1
STAGE_KEY_SCORES, STAGE_SEGMENT_PERMUTE, STAGE_BLOCK_MASK, STAGE_ATTN_FWD, STAGE_UNPERMUTE = 1, 2, 3, 4, 5
STAGE_QUERY_PERMUTE = 6
FLAG_FORCE_FIRST_BLOCK, FLAG_TOKEN_ORDER_COPY, FLAG_RUNNING_MAX_ONLY, FLAG_KBAR_IN_WS, FLAG_INDEX_REMAP = 1, 2, 4, 8, 16

EXPORTS = ["pbs_status_string", "pbs_validate", "pbs_workspace_bytes", "pbs_vt_bytes", "pbs_key_scores",
           "pbs_segment_permute", "pbs_permute_rows", "pbs_block_mask", "pbs_attn_fwd", "pbs_unpermute",
           "pbs_mfma_rate_probe", "pbs_key_scores_static", "pbs_key_scores_static_scratch_bytes", "pbs_admitted_lists",
           "pbs_mass_covered", "pbs_key_scores_proxy", "pbs_query_permutation", "pbs_shader_clock_meter"]


class PbsError(RuntimeError):
    pass


class pbs_problem(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("h_q", ctypes.c_int32), ("h_kv", ctypes.c_int32), ("n", ctypes.c_int32),
                ("d", ctypes.c_int32), ("block", ctypes.c_int32), ("segment", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("tau", ctypes.c_float), ("scale", ctypes.c_float),
                ("flags", ctypes.c_uint32)]


def load_library():
    """Load libpbs.so built in-tree (python -m paper_2510_21270_amd.build).  Fails loudly when it is missing."""
    global _lib
    if _lib is None:
        path = LIB_PATH
        if not os.path.exists(path):
            raise PbsError("libpbs.so not found at %s: build it with `python -m paper_2510_21270_amd.build`" % path)
        lib = ctypes.CDLL(path)
        P, V, Z = ctypes.POINTER(pbs_problem), ctypes.c_void_p, ctypes.c_size_t
        lib.pbs_status_string.restype = ctypes.c_char_p
        lib.pbs_status_string.argtypes = [ctypes.c_int]
        lib.pbs_validate.argtypes = [P]
        lib.pbs_workspace_bytes.restype = Z
        lib.pbs_workspace_bytes.argtypes = [P, ctypes.c_int]
        lib.pbs_vt_bytes.restype = Z
        lib.pbs_vt_bytes.argtypes = [P]
        lib.pbs_key_scores.argtypes = [P, V, V, V, V, Z, V]
        lib.pbs_key_scores_proxy.argtypes = [P, ctypes.c_int, V, ctypes.c_int32, V, V, V, V, Z, V]
        lib.pbs_key_scores_static.argtypes = [P, V, V, V, V]
        lib.pbs_key_scores_static_scratch_bytes.restype = Z
        lib.pbs_key_scores_static_scratch_bytes.argtypes = []
        lib.pbs_segment_permute.argtypes = [P, V, V, V, V, V, V, V, Z, V]
        lib.pbs_permute_rows.argtypes = [P, ctypes.c_int32, V, V, V, V]
        lib.pbs_block_mask.argtypes = [P, V, V, V, V, V, V, Z, V]
        lib.pbs_attn_fwd.argtypes = [P, V, V, V, V, V, V, V, V, V, V, Z, V]
        lib.pbs_unpermute.argtypes = [P, V, V, V, V]
        lib.pbs_query_permutation.argtypes = [P, V, V, V, V, Z, V]
        lib.pbs_admitted_lists.argtypes = [P, V, V, V]
        lib.pbs_mass_covered.argtypes = [P, V, V, V, V]
        lib.pbs_mfma_rate_probe.argtypes = [ctypes.c_int, ctypes.c_int, V, Z, ctypes.POINTER(ctypes.c_double), V]
        lib.pbs_shader_clock_meter.argtypes = [V, ctypes.c_int, V]
        _lib = lib
    return _lib


def problem(batch, h_q, h_kv, n, d, block, segment, dtype, tau=0.9, scale=0.0, flags=0):
    code = {"bf16": PBS_BF16, "f32": PBS_F32, torch.bfloat16: PBS_BF16, torch.float32: PBS_F32}[dtype]
    return pbs_problem(batch, h_q, h_kv, n, d, block, segment, code, tau, scale, flags)


def torch_dtype(p):
    return torch.bfloat16 if p.dtype == PBS_BF16 else torch.float32


def _check(st, what):
    if st != 0:
        raise PbsError("%s: %s (status %d)" % (what, load_library().pbs_status_string(st).decode(), st))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def validate(p):
    return load_library().pbs_validate(ctypes.byref(p))


def workspace_bytes(p, stage):
    return int(load_library().pbs_workspace_bytes(ctypes.byref(p), stage))


def vt_bytes(p):
    return int(load_library().pbs_vt_bytes(ctypes.byref(p)))


def T_of(p):
    return -(-p.n // p.block)


def alloc_workspace(p, stage, device="cuda"):
    nbytes = workspace_bytes(p, stage)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)   # torch allocations are 512-B aligned


def has_token_copy(p):
    return bool(p.flags & FLAG_TOKEN_ORDER_COPY)


def _tok_rows(p):
    """Rows between the start of a permuted tensor and the start of its token-order copy (PBS_FLAG_TOKEN_ORDER_COPY)."""
    return p.batch * p.h_kv * T_of(p) * p.block


def _alloc_with_copy(p, shape, row_elems, dtype, device):
    """A [batch, h_kv, ...] tensor; with PBS_FLAG_TOKEN_ORDER_COPY it is the head of a larger allocation whose tail
    holds the token-order copy (token_copy() returns that view; the storage lives as long as either view does)."""
    numel = 1
    for v in shape:
        numel *= v
    if not has_token_copy(p):
        return torch.empty(shape, dtype=dtype, device=device)
    flat = torch.empty(_tok_rows(p) * row_elems + numel, dtype=dtype, device=device)
    return flat[:numel].view(shape)


def token_copy(p, x, row_elems):
    """The token-order copy that lies behind a K' (row_elems = d), Vt (d) or kidx (1) tensor from the allocators here."""
    off = x.storage_offset() + _tok_rows(p) * row_elems
    return torch.as_strided(x, x.shape, x.stride(), off)


def alloc_vt(p, device="cuda"):
    G = min(p.block, 32)                                   # keys per transposed group
    return _alloc_with_copy(p, (p.batch, p.h_kv, T_of(p), p.block // G, p.d, G), p.d, torch_dtype(p), device)


def alloc_kp(p, device="cuda"):
    return _alloc_with_copy(p, (p.batch, p.h_kv, p.n, p.d), p.d, torch_dtype(p), device)


def alloc_kidx(p, device="cuda"):
    return _alloc_with_copy(p, (p.batch, p.h_kv, p.n), 1, torch.int32, device)


def _ws_args(p, stage, ws):
    if ws is None:
        ws = alloc_workspace(p, stage)
    return ws, _ptr(ws), ws.numel()


def key_scores(p, Q, K, scores=None, ws=None):
    if scores is None:
        scores = torch.empty((p.batch, p.h_kv, p.n), dtype=torch.float32, device=K.device)
    ws, wp, wn = _ws_args(p, STAGE_KEY_SCORES, ws)
    _check(load_library().pbs_key_scores(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(scores), wp, wn, _stream()),
           "pbs_key_scores")
    return scores


PROXY_LAST_BLOCK, PROXY_QUERY_ROWS, PROXY_AVG_QUERY = 0, 1, 2


def key_scores_proxy(p, proxy, qrows, Q, K, scores=None, ws=None):
    if scores is None:
        scores = torch.empty((p.batch, p.h_kv, p.n), dtype=torch.float32, device=K.device)
    ws, wp, wn = _ws_args(p, STAGE_KEY_SCORES, ws)
    m = 0 if qrows is None else qrows.numel()
    _check(load_library().pbs_key_scores_proxy(ctypes.byref(p), proxy, _ptr(qrows), m, _ptr(Q), _ptr(K), _ptr(scores),
                                               wp, wn, _stream()), "pbs_key_scores_proxy")
    return scores


def key_scores_static(p, Q, K, scores=None):
    if scores is None:
        scores = torch.empty((p.batch, p.h_kv, p.n), dtype=torch.float32, device=K.device)
    _check(load_library().pbs_key_scores_static(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(scores), _stream()),
           "pbs_key_scores_static")
    return scores


def segment_permute(p, scores, K, V, kidx=None, Kp=None, Vt=None, indices_only=False, ws=None):
    dev = (K if K is not None else scores).device
    if kidx is None:
        kidx = alloc_kidx(p, dev)
    if not indices_only:
        if Kp is None and not (p.flags & FLAG_INDEX_REMAP):
            Kp = alloc_kp(p, dev)
        if Vt is None:
            Vt = alloc_vt(p, dev)
    _check(load_library().pbs_segment_permute(ctypes.byref(p), _ptr(scores), _ptr(K), _ptr(V), _ptr(kidx), _ptr(Kp),
                                              _ptr(Vt), _ptr(ws), 0 if ws is None else ws.numel(), _stream()),
           "pbs_segment_permute")
    return kidx, Kp, Vt


def permute_rows(p, X, idx, Xp=None):
    if Xp is None:
        Xp = torch.empty_like(X)
    _check(load_library().pbs_permute_rows(ctypes.byref(p), X.shape[1], _ptr(X), _ptr(idx), _ptr(Xp), _stream()),
           "pbs_permute_rows")
    return Xp


def query_permutation(p, Q, Kc, qidx=None, ws=None):
    if qidx is None:
        qidx = torch.empty((p.batch, p.h_q, p.n), dtype=torch.int32, device=Q.device)
    ws, wp, wn = _ws_args(p, STAGE_QUERY_PERMUTE, ws)
    _check(load_library().pbs_query_permutation(ctypes.byref(p), _ptr(Q), _ptr(Kc), _ptr(qidx), wp, wn, _stream()),
           "pbs_query_permutation")
    return qidx


def block_mask(p, Qp, Kp, mask_bits=None, row_cnt=None, col_idx=None, ws=None):
    T = T_of(p)
    dev = Qp.device
    if mask_bits is None:
        mask_bits = torch.empty((p.batch, p.h_q, T, (T + 63) // 64), dtype=torch.int64, device=dev)
    if row_cnt is None:
        row_cnt = torch.empty((p.batch, p.h_q, T), dtype=torch.int32, device=dev)
    if col_idx is None:
        col_idx = torch.empty((p.batch, p.h_q, T, T), dtype=torch.int32, device=dev)
    ws, wp, wn = _ws_args(p, STAGE_BLOCK_MASK, ws)
    _check(load_library().pbs_block_mask(ctypes.byref(p), _ptr(Qp), _ptr(Kp), _ptr(mask_bits), _ptr(row_cnt),
                                         _ptr(col_idx), wp, wn, _stream()), "pbs_block_mask")
    return mask_bits, row_cnt, col_idx


def attn_fwd(p, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op=None, lse=None, want_lse=False, ws=None):
    if Op is None:
        Op = torch.empty_like(Qp)
    if lse is None and want_lse:
        lse = torch.empty((p.batch, p.h_q, p.n), dtype=torch.float32, device=Qp.device)
    ws, wp, wn = _ws_args(p, STAGE_ATTN_FWD, ws)
    _check(load_library().pbs_attn_fwd(ctypes.byref(p), _ptr(Qp), _ptr(Kp), _ptr(Vt), _ptr(qidx), _ptr(kidx),
                                       _ptr(row_cnt), _ptr(col_idx), _ptr(Op), _ptr(lse), wp, wn, _stream()),
           "pbs_attn_fwd")
    return (Op, lse) if want_lse else Op


def unpermute(p, Op, qidx, O=None):
    if O is None:
        O = Op if qidx is None else torch.empty_like(Op)
    _check(load_library().pbs_unpermute(ctypes.byref(p), _ptr(Op), _ptr(qidx), _ptr(O), _stream()), "pbs_unpermute")
    return O


def admitted_lists(p, row_cnt=None, col_idx=None, device="cuda"):
    T = T_of(p)
    if row_cnt is None:
        row_cnt = torch.empty((p.batch, p.h_q, T), dtype=torch.int32, device=device)
    if col_idx is None:
        col_idx = torch.empty((p.batch, p.h_q, T, T), dtype=torch.int32, device=device)
    _check(load_library().pbs_admitted_lists(ctypes.byref(p), _ptr(row_cnt), _ptr(col_idx), _stream()),
           "pbs_admitted_lists")
    return row_cnt, col_idx


def mass_covered(p, lse_listed, lse_admitted, covered=None):
    if covered is None:
        covered = torch.empty_like(lse_listed)
    _check(load_library().pbs_mass_covered(ctypes.byref(p), _ptr(lse_listed), _ptr(lse_admitted), _ptr(covered),
                                           _stream()), "pbs_mass_covered")
    return covered


def mfma_rate_probe(random_operands, iters=20000, reps=3):
    """(TFLOP/s, shader clock in MHz) of the matrix units alone: best of `reps` launches timed with events on the
    current stream, and the clock one wave of that launch saw."""
    sink = torch.empty(262144, dtype=torch.float32, device="cuda")
    flop = ctypes.c_double(0.0)
    best, mhz = 0.0, 0.0
    for _ in range(reps + 1):                              # the first launch warms up
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        _check(load_library().pbs_mfma_rate_probe(int(bool(random_operands)), iters, _ptr(sink), sink.numel(),
                                                  ctypes.byref(flop), _stream()), "pbs_mfma_rate_probe")
        e1.record()
        e1.synchronize()
        rate = flop.value / (e0.elapsed_time(e1) * 1e-3) / 1e12
        if rate > best:
            best, mhz = rate, float(sink[0])
    return best, mhz


def shader_clock_beside(fn, micros=20000, delay_s=0.02):
    """Shader clock in MHz while fn()'s kernels run on the current stream: fn() is enqueued, then, after delay_s, one
    watching wave on a second stream (default priority) for `micros` microseconds.  fn's work must outlast both."""
    import time
    out = torch.zeros(2, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    fn()
    time.sleep(delay_s)
    with torch.cuda.stream(side):
        _check(load_library().pbs_shader_clock_meter(_ptr(out), int(micros), ctypes.c_void_p(side.cuda_stream)),
               "pbs_shader_clock_meter")
    torch.cuda.synchronize()
    return float(out[0]), float(out[1])


class Pipeline:
    """Algorithm 1 end to end on preallocated buffers: the five library calls, nothing else."""

    def __init__(self, p, device="cuda", use_sigma=False):
        self.p = p
        self.p_kbar = pbs_problem.from_buffer_copy(p)
        self.p_kbar.flags |= FLAG_KBAR_IN_WS
        T, dt = T_of(p), torch_dtype(p)
        self.scores = torch.empty((p.batch, p.h_kv, p.n), dtype=torch.float32, device=device)
        self.kidx = alloc_kidx(p, device)
        self.Kp = alloc_kp(p, device)
        self.Vt = alloc_vt(p, device)
        self.mask_bits = torch.empty((p.batch, p.h_q, T, (T + 63) // 64), dtype=torch.int64, device=device)
        self.row_cnt = torch.empty((p.batch, p.h_q, T), dtype=torch.int32, device=device)
        self.col_idx = torch.empty((p.batch, p.h_q, T, T), dtype=torch.int32, device=device)
        self.Op = torch.empty((p.batch, p.h_q, p.n, p.d), dtype=dt, device=device)
        self.O = torch.empty_like(self.Op) if use_sigma else self.Op
        self.Qp = torch.empty_like(self.Op) if use_sigma else None
        self.ws1 = alloc_workspace(p, STAGE_KEY_SCORES, device)
        self.ws3 = alloc_workspace(p, STAGE_BLOCK_MASK, device)
        self.ws4 = alloc_workspace(p, STAGE_ATTN_FWD, device)

    def run(self, Q, K, V, qidx=None):
        p = self.p
        key_scores(p, Q, K, self.scores, self.ws1)
        # the block means of K' that Algorithm 2 starts from come out of the gather (PBS_FLAG_KBAR_IN_WS)
        segment_permute(p, self.scores, K, V, self.kidx, self.Kp, self.Vt, ws=self.ws3)
        Qp = Q if qidx is None else permute_rows(p, Q, qidx, self.Qp)
        block_mask(self.p_kbar, Qp, self.Kp, self.mask_bits, self.row_cnt, self.col_idx, self.ws3)
        attn_fwd(p, Qp, self.Kp, self.Vt, qidx, self.kidx, self.row_cnt, self.col_idx, self.Op, ws=self.ws4)
        return unpermute(p, self.Op, qidx, self.O)

    def capture(self, Q, K, V, qidx=None):
        """Record the pipeline into a HIP graph that reads these very tensors (refill them in place, then replay()).
        The library allocates nothing, never synchronises and records no memset nodes, so the calls can be captured
        as they are; short sequences, where the dozen launches cost more than the kernels, gain from it."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.run(Q, K, V, qidx)                        # everything lazily initialised happens outside the capture
        torch.cuda.current_stream().wait_stream(side)
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self._graph_out = self.run(Q, K, V, qidx)
        return self._graph_out

    def replay(self):
        self.graph.replay()
        return self._graph_out
