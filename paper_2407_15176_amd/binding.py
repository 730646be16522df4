"""Thin ctypes front of libreattn.so: the same names as include/reattn.h.

Argument marshalling only: tensors are torch device tensors whose data pointers
are handed to the C ABI; every step of the path runs in the library's HIP
kernels on the current torch stream.  There is no CPU fallback: if the library
has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch  # loads the HIP runtime the library binds to; used for memory and streams only

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libreattn.so")

F32, BF16, F16 = 0, 1, 2
_DTYPE_CODE = {"f32": F32, "bf16": BF16, "f16": F16}
AGG_SUM, AGG_MAX = 0, 1
ROUTE_AUTO, ROUTE_FILTER, ROUTE_SCORES = 0, 1, 2

OK = 0
ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_RANGE, ERR_WINDOW, ERR_WORKSPACE, ERR_ALIGN, ERR_HIP, ERR_STATIC_LIMIT = (
    -1, -2, -3, -4, -5, -6, -7, -8, -9)

EXPORTS = [
    "reattn_version", "reattn_status_string", "reattn_validate", "reattn_scope",
    "reattn_workspace_bytes", "reattn_score", "reattn_topk", "reattn_gather_rope",
    "reattn_attend", "reattn_decode_step", "reattn_prefill_chunk", "reattn_decode_step_timed",
    "reattn_probe_read_bandwidth", "reattn_prefill_chunk_timed",
    "reattn_vote_workspace_bytes", "reattn_vote_topk", "reattn_vote_merge", "reattn_vote_layer",
    "reattn_vote_layer_timed", "reattn_cache_append", "reattn_prefill_sequence_chunks",
    "reattn_prefill_sequence_workspace_bytes", "reattn_prefill_sequence", "reattn_decode_token",
    "reattn_static_scratch_bytes", "reattn_decode_step_static", "reattn_redo_list_offset",
    "reattn_prefill_sequence_chunk_bounds", "reattn_params_bytes", "reattn_vote_bytes",
]
PREFILL_STAGES = ("sample_threshold", "score_gemm_filter", "candidate_topk", "attend")
STAGES = ("prep", "scan", "topk", "attend")
VOTE_STAGES = ("head_topk_scan", "vote_merge", "attend")


class CParams(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("dtype", C.c_int32), ("n_ctx", C.c_int64), ("n_query", C.c_int32),
        ("n_sink", C.c_int32), ("n_local", C.c_int32), ("top_k", C.c_int32),
        ("rope_theta", C.c_float), ("max_position", C.c_int32), ("agg", C.c_int32),
        ("softmax_scale", C.c_float),
        ("k_stride_head", C.c_int64), ("k_stride_tok", C.c_int64),
        ("v_stride_head", C.c_int64), ("v_stride_tok", C.c_int64),
        ("page_table", C.c_void_p), ("page_size", C.c_int32), ("route", C.c_int32),
        ("ws_warm", C.c_int32),
    ]


class CVote(C.Structure):
    _fields_ = [("vote_k", C.c_int32), ("n_centres", C.c_int32), ("span", C.c_int32), ("n_seq", C.c_int32)]


class ReattnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    """Loads libreattn.so (built by paper_2407_15176_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2407_15176_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        P, PP = C.c_void_p, C.POINTER(CParams)
        L.reattn_version.restype = C.c_int
        L.reattn_params_bytes.restype = C.c_size_t
        L.reattn_vote_bytes.restype = C.c_size_t
        if L.reattn_params_bytes() != C.sizeof(CParams) or L.reattn_vote_bytes() != C.sizeof(CVote):
            raise RuntimeError(
                f"{LIB_PATH}: reattn_params / reattn_vote are {L.reattn_params_bytes()} / {L.reattn_vote_bytes()} bytes "
                f"in the library, {C.sizeof(CParams)} / {C.sizeof(CVote)} in this binding; rebuild the library")
        L.reattn_status_string.argtypes = [C.c_int]
        L.reattn_status_string.restype = C.c_char_p
        L.reattn_validate.argtypes = [PP]
        L.reattn_scope.argtypes = [PP] + [C.POINTER(C.c_int64)] * 5
        L.reattn_workspace_bytes.argtypes = [PP]
        L.reattn_workspace_bytes.restype = C.c_size_t
        L.reattn_score.argtypes = [PP, P, P, P, P, C.c_size_t, P]
        L.reattn_topk.argtypes = [PP, P, P, P, C.c_size_t, P]
        L.reattn_gather_rope.argtypes = [PP, P, P, P, P, P, P]
        L.reattn_attend.argtypes = [PP, P, P, P, P, P, C.c_size_t, P]
        L.reattn_decode_step.argtypes = [PP, P, P, P, P, P, P, C.c_size_t, P]
        L.reattn_prefill_chunk.argtypes = [PP, P, P, P, P, P, P, C.c_size_t, P]
        L.reattn_decode_step_static.argtypes = [PP, P, P, P, P, P, P]
        L.reattn_static_scratch_bytes.restype = C.c_size_t
        L.reattn_redo_list_offset.argtypes = [PP, C.POINTER(C.c_size_t)]
        L.reattn_decode_step_timed.argtypes = [PP, P, P, P, P, P, P, C.c_size_t, P,
                                               C.POINTER(C.c_float)]
        L.reattn_prefill_chunk_timed.argtypes = L.reattn_decode_step_timed.argtypes
        L.reattn_probe_read_bandwidth.argtypes = [P, C.c_size_t, C.c_int, P, C.POINTER(C.c_float)]
        PV = C.POINTER(CVote)
        L.reattn_vote_workspace_bytes.argtypes = [PP, PV]
        L.reattn_vote_workspace_bytes.restype = C.c_size_t
        L.reattn_vote_topk.argtypes = [PP, PV, P, P, P, P, C.c_size_t, P]
        L.reattn_vote_merge.argtypes = [PP, PV, P, P, P, P, C.c_size_t, P]
        L.reattn_vote_layer.argtypes = [PP, PV, P, P, P, P, P, P, P, C.c_size_t, P]
        L.reattn_vote_layer_timed.argtypes = L.reattn_vote_layer.argtypes + [C.POINTER(C.c_float)]
        L.reattn_cache_append.argtypes = [PP, C.c_int64, C.c_int32, P, P, P, P, P]
        L.reattn_prefill_sequence_chunk_bounds.argtypes = [PP, C.c_int32, C.c_int64, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.reattn_prefill_sequence_chunks.argtypes = [PP, C.c_int32]
        L.reattn_prefill_sequence_chunks.restype = C.c_int64
        L.reattn_prefill_sequence_workspace_bytes.argtypes = [PP, PV, C.c_int32]
        L.reattn_prefill_sequence_workspace_bytes.restype = C.c_size_t
        L.reattn_decode_token.argtypes = [PP, PV, C.c_int32] + [C.POINTER(C.c_void_p)] * 6 + [P, C.c_size_t, P]
        L.reattn_prefill_sequence.argtypes = [PP, PV, C.c_int32, P, P, P, P, P, P, P, P, P, P, C.c_size_t, P]
        _lib = L
    return _lib


@dataclass
class Params:
    """reattn_params in Python clothing (paper Eq. 1-3 notation; see include/reattn.h)."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: int
    n_ctx: int
    n_query: int = 1
    n_sink: int = 4
    n_local: int = 4096
    top_k: int = 4096
    rope_theta: float = 500000.0
    max_position: int = 0
    agg: int = AGG_SUM
    softmax_scale: float = 0.0
    k_stride_head: int = 0
    k_stride_tok: int = 0
    v_stride_head: int = 0
    v_stride_tok: int = 0
    page_table: "torch.Tensor | None" = None     # int32 device tensor [ceil(n_ctx / page_size)], or None
    page_size: int = 0
    route: int = 0                               # ROUTE_AUTO / ROUTE_FILTER / ROUTE_SCORES (long decode steps)
    ws_warm: int = 0                             # decode steps: the workspace was last written by a step of the same shape

    def c(self) -> CParams:
        pt = None
        if self.page_table is not None:
            t = self.page_table
            if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
                raise ValueError("page_table must be a contiguous int32 device tensor")
            if t.numel() * max(self.page_size, 1) < self.n_ctx:
                raise ValueError("page_table does not cover n_ctx tokens")
            pt = t.data_ptr()
        return CParams(self.n_q_heads, self.n_kv_heads, self.head_dim, self.dtype, self.n_ctx,
                       self.n_query, self.n_sink, self.n_local, self.top_k, self.rope_theta,
                       self.max_position, self.agg, self.softmax_scale,
                       self.k_stride_head, self.k_stride_tok, self.v_stride_head, self.v_stride_tok,
                       pt, self.page_size, self.route, self.ws_warm)

    @classmethod
    def from_workload(cls, w) -> "Params":
        return cls(w.n_q_heads, w.n_kv_heads, w.head_dim, _DTYPE_CODE[w.dtype],
                   w.n_ctx, w.n_query, w.n_sink, w.n_local, w.top_k, w.rope_theta, w.max_position)

    def torch_dtype(self):
        return {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16}[self.dtype]


def version() -> int:
    return lib().reattn_version()


def status_string(status: int) -> str:
    return lib().reattn_status_string(status).decode()


def validate(p: Params) -> int:
    cp = p.c()
    return lib().reattn_validate(C.byref(cp))


def scope(p: Params):
    """(s_eff, l_eff, n_mid, k_eff, S) of Eq. 1 with the clamping rules."""
    cp = p.c()
    v = [C.c_int64() for _ in range(5)]
    rc = lib().reattn_scope(C.byref(cp), *[C.byref(x) for x in v])
    if rc:
        raise ReattnError(rc, "reattn_scope")
    return tuple(x.value for x in v)


def workspace_bytes(p: Params) -> int:
    cp = p.c()
    return lib().reattn_workspace_bytes(C.byref(cp))


def alloc_workspace(p: Params, device="cuda") -> torch.Tensor:
    n = workspace_bytes(p)
    if n == 0:
        raise ReattnError(validate(p), "reattn_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _dev(t: torch.Tensor | None, name: str, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, where: str):
    if rc != OK:
        raise ReattnError(rc, where)


def score(p: Params, q, k_cache, scores=None, ws=None):
    s_eff, l_eff, n_mid, k_eff, S = scope(p)
    if scores is None:
        scores = torch.empty(p.n_query, p.n_kv_heads, n_mid, dtype=torch.float32, device=q.device)
    cp = p.c()
    _check(lib().reattn_score(C.byref(cp), _dev(q, "q", p.torch_dtype()),
                              _dev(k_cache, "k_cache", p.torch_dtype()),
                              _dev(scores, "scores", torch.float32), _dev(ws, "ws"),
                              ws.numel() if ws is not None else 0, _stream()), "reattn_score")
    return scores


def topk(p: Params, scores, ws, idx=None):
    s_eff, l_eff, n_mid, k_eff, S = scope(p)
    if idx is None:
        idx = torch.empty(p.n_query, p.n_kv_heads, k_eff, dtype=torch.int32, device=scores.device)
    cp = p.c()
    _check(lib().reattn_topk(C.byref(cp), _dev(scores, "scores", torch.float32),
                             _dev(idx, "idx", torch.int32), _dev(ws, "ws"), ws.numel(), _stream()),
           "reattn_topk")
    return idx


def gather_rope(p: Params, k_cache, v_cache, idx, k_sel=None, v_sel=None):
    s_eff, l_eff, n_mid, k_eff, S = scope(p)
    shape = (p.n_query, p.n_kv_heads, S, p.head_dim)
    if k_sel is None:
        k_sel = torch.empty(shape, dtype=torch.float32, device=k_cache.device)
    if v_sel is None:
        v_sel = torch.empty(shape, dtype=p.torch_dtype(), device=k_cache.device)
    cp = p.c()
    _check(lib().reattn_gather_rope(C.byref(cp), _dev(k_cache, "k_cache", p.torch_dtype()),
                                    _dev(v_cache, "v_cache", p.torch_dtype()),
                                    _dev(idx, "idx", torch.int32),
                                    _dev(k_sel, "k_sel", torch.float32),
                                    _dev(v_sel, "v_sel", p.torch_dtype()), _stream()),
           "reattn_gather_rope")
    return k_sel, v_sel


def attend(p: Params, q, k_sel, v_sel, ws, out=None):
    if out is None:
        out = torch.empty(p.n_query, p.n_q_heads, p.head_dim, dtype=torch.float32, device=q.device)
    cp = p.c()
    _check(lib().reattn_attend(C.byref(cp), _dev(q, "q", p.torch_dtype()),
                               _dev(k_sel, "k_sel", torch.float32),
                               _dev(v_sel, "v_sel", p.torch_dtype()),
                               _dev(out, "out", torch.float32), _dev(ws, "ws"), ws.numel(), _stream()),
           "reattn_attend")
    return out


def _layer(fn_name: str, p: Params, q, k_cache, v_cache, ws, idx_out, out, want_idx: bool):
    s_eff, l_eff, n_mid, k_eff, S = scope(p)
    if out is None:
        out = torch.empty(p.n_query, p.n_q_heads, p.head_dim, dtype=torch.float32, device=q.device)
    if idx_out is None and want_idx:
        idx_out = torch.empty(p.n_query, p.n_kv_heads, k_eff, dtype=torch.int32, device=q.device)
    cp = p.c()
    fn = getattr(lib(), fn_name)
    _check(fn(C.byref(cp), _dev(q, "q", p.torch_dtype()), _dev(k_cache, "k_cache", p.torch_dtype()),
              _dev(v_cache, "v_cache", p.torch_dtype()), _dev(idx_out, "idx_out", torch.int32),
              _dev(out, "out", torch.float32), _dev(ws, "ws"), ws.numel(), _stream()), fn_name)
    return out, idx_out


def decode_step(p: Params, q, k_cache, v_cache, ws, idx_out=None, out=None, want_idx=True):
    return _layer("reattn_decode_step", p, q, k_cache, v_cache, ws, idx_out, out, want_idx)


def redo_list(p: Params, ws: torch.Tensor):
    """(count, row ids) the last decode step / prefill chunk over `ws` left in its redo list (synchronises).
    Row ids are listed for chunks only.  Returns None when the params take a route without such a list."""
    cp, off = p.c(), C.c_size_t(0)
    rc = lib().reattn_redo_list_offset(C.byref(cp), C.byref(off))
    if rc == ERR_SHAPE:
        return None
    _check(rc, "reattn_redo_list_offset")
    words = ws[off.value:].view(torch.int32)
    n = int(words[0].item())
    rows = words[1:1 + n].cpu().tolist() if p.n_query > 1 else []
    return n, rows


def static_scratch_bytes() -> int:
    return lib().reattn_static_scratch_bytes()


def decode_step_static(p: Params, q, k_cache, v_cache, idx_out, out):
    """reattn_decode_step over the library's own scratch array: the caller passes every buffer, nothing is allocated."""
    cp = p.c()
    _check(lib().reattn_decode_step_static(
        C.byref(cp), _dev(q, "q", p.torch_dtype()), _dev(k_cache, "k_cache", p.torch_dtype()),
        _dev(v_cache, "v_cache", p.torch_dtype()), _dev(idx_out, "idx_out", torch.int32),
        _dev(out, "out", torch.float32), _stream()), "reattn_decode_step_static")
    return out, idx_out


def prefill_chunk(p: Params, q, k_cache, v_cache, ws, idx_out=None, out=None, want_idx=True):
    return _layer("reattn_prefill_chunk", p, q, k_cache, v_cache, ws, idx_out, out, want_idx)


def prefill_chunk_timed(p: Params, q, k_cache, v_cache, ws, idx_out=None, out=None):
    """prefill_chunk (MFMA path) with per-stage HIP-event timing; synchronises."""
    return _timed("reattn_prefill_chunk_timed", PREFILL_STAGES, p, q, k_cache, v_cache, ws, idx_out, out)


def decode_step_timed(p: Params, q, k_cache, v_cache, ws, idx_out=None, out=None):
    """decode_step with per-stage HIP-event timing; synchronises.  Returns (out, idx, {stage: ms})."""
    return _timed("reattn_decode_step_timed", STAGES, p, q, k_cache, v_cache, ws, idx_out, out)


def _timed(fn_name, names, p: Params, q, k_cache, v_cache, ws, idx_out=None, out=None):
    s_eff, l_eff, n_mid, k_eff, S = scope(p)
    if out is None:
        out = torch.empty(p.n_query, p.n_q_heads, p.head_dim, dtype=torch.float32, device=q.device)
    if idx_out is None:
        idx_out = torch.empty(p.n_query, p.n_kv_heads, k_eff, dtype=torch.int32, device=q.device)
    ms = (C.c_float * len(names))()
    cp = p.c()
    _check(getattr(lib(), fn_name)(
        C.byref(cp), _dev(q, "q", p.torch_dtype()), _dev(k_cache, "k_cache", p.torch_dtype()),
        _dev(v_cache, "v_cache", p.torch_dtype()), _dev(idx_out, "idx_out", torch.int32),
        _dev(out, "out", torch.float32), _dev(ws, "ws"), ws.numel(), _stream(), ms), fn_name)
    return out, idx_out, dict(zip(names, [float(x) for x in ms]))


def probe_read_bandwidth(buf: torch.Tensor, iters: int = 10) -> float:
    """GB/s of a plain streaming read of `buf` with the scan's load shape (measurement aid)."""
    out = C.c_float(0.0)
    _check(lib().reattn_probe_read_bandwidth(_dev(buf, "buf"), buf.numel() * buf.element_size(),
                                             iters, _stream(), C.byref(out)),
           "reattn_probe_read_bandwidth")
    return float(out.value)


# ---- vote selection (heads and query rows vote; top-k' centres; spans) ------------------------
@dataclass
class Vote:
    """reattn_vote: the paper's k (votes per list), k' (centres) and span m."""
    vote_k: int = 4
    n_centres: int = 127
    span: int = 32
    n_seq: int = 1          # equal-length sequences folded into the head axis (decode only)

    def c(self) -> CVote:
        return CVote(self.vote_k, self.n_centres, self.span, self.n_seq)


def vote_workspace_bytes(p: Params, v: Vote) -> int:
    cp, cv = p.c(), v.c()
    return lib().reattn_vote_workspace_bytes(C.byref(cp), C.byref(cv))


def alloc_vote_workspace(p: Params, v: Vote, device="cuda") -> torch.Tensor:
    n = vote_workspace_bytes(p, v)
    if n == 0:
        raise ReattnError(validate(p) or ERR_RANGE, "reattn_vote_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def vote_cap(p: Params, v: Vote) -> int:
    """Largest selection length min(n_centres * span, N_mid)."""
    _, _, n_mid, _, _ = scope(p)
    return min(v.n_centres * v.span, n_mid)


def vote_topk(p: Params, v: Vote, q, k_cache, ws, head_topk=None):
    _, _, n_mid, _, _ = scope(p)
    kk = min(v.vote_k, n_mid)
    if head_topk is None:
        head_topk = torch.empty(p.n_query, p.n_q_heads, kk, dtype=torch.int32, device=q.device)
    cp, cv = p.c(), v.c()
    _check(lib().reattn_vote_topk(C.byref(cp), C.byref(cv), _dev(q, "q", p.torch_dtype()),
                                  _dev(k_cache, "k_cache", p.torch_dtype()),
                                  _dev(head_topk, "head_topk", torch.int32), _dev(ws, "ws"), ws.numel(),
                                  _stream()), "reattn_vote_topk")
    return head_topk


def vote_merge(p: Params, v: Vote, head_topk, ws, sel=None, n_sel=None):
    if sel is None:
        sel = torch.empty(max(v.n_seq, 1) * max(vote_cap(p, v), 1), dtype=torch.int32, device=head_topk.device)
    if n_sel is None:
        n_sel = torch.zeros(max(v.n_seq, 1), dtype=torch.int32, device=head_topk.device)
    cp, cv = p.c(), v.c()
    _check(lib().reattn_vote_merge(C.byref(cp), C.byref(cv), _dev(head_topk, "head_topk", torch.int32),
                                   _dev(sel, "sel", torch.int32), _dev(n_sel, "n_sel", torch.int32),
                                   _dev(ws, "ws"), ws.numel(), _stream()), "reattn_vote_merge")
    return sel, n_sel


def vote_layer(p: Params, v: Vote, q, k_cache, v_cache, ws, sel=None, n_sel=None, out=None, want_sel=True):
    if out is None:
        out = torch.empty(p.n_query, p.n_q_heads, p.head_dim, dtype=torch.float32, device=q.device)
    if want_sel and sel is None:
        sel = torch.empty(max(v.n_seq, 1) * max(vote_cap(p, v), 1), dtype=torch.int32, device=q.device)
    if want_sel and n_sel is None:
        n_sel = torch.zeros(max(v.n_seq, 1), dtype=torch.int32, device=q.device)
    cp, cv = p.c(), v.c()
    _check(lib().reattn_vote_layer(C.byref(cp), C.byref(cv), _dev(q, "q", p.torch_dtype()),
                                   _dev(k_cache, "k_cache", p.torch_dtype()),
                                   _dev(v_cache, "v_cache", p.torch_dtype()),
                                   _dev(sel, "sel", torch.int32), _dev(n_sel, "n_sel", torch.int32),
                                   _dev(out, "out", torch.float32), _dev(ws, "ws"), ws.numel(), _stream()),
           "reattn_vote_layer")
    return out, sel, n_sel


def vote_layer_timed(p: Params, v: Vote, q, k_cache, v_cache, ws, sel=None, n_sel=None, out=None):
    """vote_layer with per-stage HIP-event timing; synchronises.  Returns (out, sel, n_sel, {stage: ms})."""
    if out is None:
        out = torch.empty(p.n_query, p.n_q_heads, p.head_dim, dtype=torch.float32, device=q.device)
    if sel is None:
        sel = torch.empty(max(vote_cap(p, v), 1), dtype=torch.int32, device=q.device)
    if n_sel is None:
        n_sel = torch.zeros(1, dtype=torch.int32, device=q.device)
    ms = (C.c_float * len(VOTE_STAGES))()
    cp, cv = p.c(), v.c()
    _check(lib().reattn_vote_layer_timed(C.byref(cp), C.byref(cv), _dev(q, "q", p.torch_dtype()),
                                         _dev(k_cache, "k_cache", p.torch_dtype()),
                                         _dev(v_cache, "v_cache", p.torch_dtype()),
                                         _dev(sel, "sel", torch.int32), _dev(n_sel, "n_sel", torch.int32),
                                         _dev(out, "out", torch.float32), _dev(ws, "ws"), ws.numel(),
                                         _stream(), ms), "reattn_vote_layer_timed")
    return out, sel, n_sel, dict(zip(VOTE_STAGES, [float(x) for x in ms]))


# ---- streaming prefill of one layer (chunk loop with cache append) ---------------------------
def cache_append(p: Params, first_tok: int, k_new, v_new, k_cache, v_cache):
    """cache[h][first_tok + t] = new[t][h]; k_new, v_new token-major [n_tok, Hkv, D]."""
    cp = p.c()
    _check(lib().reattn_cache_append(C.byref(cp), first_tok, k_new.shape[0], _dev(k_new, "k_new", p.torch_dtype()),
                                     _dev(v_new, "v_new", p.torch_dtype()), _dev(k_cache, "k_cache", p.torch_dtype()),
                                     _dev(v_cache, "v_cache", p.torch_dtype()), _stream()), "reattn_cache_append")


def sequence_chunks(p: Params, chunk: int):
    """[(first, end)] of the chunk loop, as the library cuts it (reattn_prefill_sequence_chunk_bounds)."""
    cp = p.c()
    n = lib().reattn_prefill_sequence_chunks(C.byref(cp), chunk)
    out = []
    for c in range(n):
        s, e = C.c_int64(), C.c_int64()
        _check(lib().reattn_prefill_sequence_chunk_bounds(C.byref(cp), chunk, c, C.byref(s), C.byref(e)),
               "reattn_prefill_sequence_chunk_bounds")
        out.append((s.value, e.value))
    return out


def prefill_sequence(p: Params, chunk: int, q, k_new, v_new, k_cache=None, v_cache=None, vote: Vote | None = None,
                     ws=None, want_sets: bool = True):
    """Chunk loop of one layer.  Returns dict(out [L,Hq,D], k_cache, v_cache, and per mode
    idx = [per chunk [M,Hkv,k_eff]] or sel = [per chunk 1-D tensor])."""
    L, dev = p.n_ctx, q.device
    cp = p.c()
    cv = vote.c() if vote is not None else None
    pv = C.byref(cv) if cv is not None else None
    if k_cache is None:
        k_cache = torch.empty(p.n_kv_heads, L, p.head_dim, dtype=p.torch_dtype(), device=dev)
        v_cache = torch.empty_like(k_cache)
    need = lib().reattn_prefill_sequence_workspace_bytes(C.byref(cp), pv, chunk)
    if ws is None:
        if need == 0:
            raise ReattnError(validate(p) or ERR_RANGE, "reattn_prefill_sequence_workspace_bytes")
        ws = torch.empty(need, dtype=torch.uint8, device=dev)
    out = torch.empty(L, p.n_q_heads, p.head_dim, dtype=torch.float32, device=dev)
    chunks = sequence_chunks(p, chunk)
    idx_flat = sel_all = n_sel_all = None
    shapes = []
    if want_sets and vote is None:
        for s, e in chunks:                                    # every chunk's k_eff from the library's own Eq. 1
            k_eff = scope(Params(**{**p.__dict__, "n_ctx": e, "n_query": e - s, "max_position": 0}))[3]
            shapes.append((e - s, p.n_kv_heads, k_eff))
        idx_flat = torch.empty(max(1, sum(a * b * c for a, b, c in shapes)), dtype=torch.int32, device=dev)
    if want_sets and vote is not None:
        cap = max(1, vote_cap(Params(**{**p.__dict__, "n_query": 1, "max_position": 0}), vote))
        sel_all = torch.empty(len(chunks), cap, dtype=torch.int32, device=dev)
        n_sel_all = torch.zeros(len(chunks), dtype=torch.int32, device=dev)
    _check(lib().reattn_prefill_sequence(
        C.byref(cp), pv, chunk, _dev(q, "q", p.torch_dtype()), _dev(k_new, "k_new", p.torch_dtype()),
        _dev(v_new, "v_new", p.torch_dtype()), _dev(k_cache, "k_cache", p.torch_dtype()),
        _dev(v_cache, "v_cache", p.torch_dtype()), _dev(out, "out", torch.float32),
        _dev(idx_flat, "idx_out", torch.int32), _dev(sel_all, "sel_out", torch.int32),
        _dev(n_sel_all, "n_sel_out", torch.int32), _dev(ws, "ws"), ws.numel(), _stream()), "reattn_prefill_sequence")
    res = {"out": out, "k_cache": k_cache, "v_cache": v_cache, "chunks": chunks}
    if idx_flat is not None:
        res["idx"], at = [], 0
        for a, b, c in shapes:
            res["idx"].append(idx_flat[at:at + a * b * c].view(a, b, c))
            at += a * b * c
    if sel_all is not None:
        res["sel"], res["n_sel"] = sel_all, n_sel_all
    return res


# ---- one decode token through all layers -------------------------------------------------------
def decode_token(p: Params, qs, k_news, v_news, k_caches, v_caches, ws, outs=None, vote: Vote | None = None):
    """qs[l] [1,Hq,D]; k_news[l], v_news[l] [1,Hkv,D] (or [Hkv,D]); caches [Hkv,cap,D] with p's strides.
    p.n_ctx counts the new token.  Returns outs (list of [1,Hq,D] fp32)."""
    n = len(qs)
    if outs is None:
        outs = [torch.empty(1, p.n_q_heads, p.head_dim, dtype=torch.float32, device=qs[0].device) for _ in range(n)]
    dt = p.torch_dtype()

    def arr(ts, name, dtype):
        return (C.c_void_p * n)(*[_dev(t, name, dtype).value for t in ts])
    cp = p.c()
    cv = vote.c() if vote is not None else None
    _check(lib().reattn_decode_token(C.byref(cp), C.byref(cv) if cv is not None else None, n,
                                     arr(qs, "q", dt), arr(k_news, "k_new", dt), arr(v_news, "v_new", dt),
                                     arr(k_caches, "k_cache", dt), arr(v_caches, "v_cache", dt),
                                     arr(outs, "out", torch.float32), _dev(ws, "ws"), ws.numel(), _stream()),
           "reattn_decode_token")
    return outs
