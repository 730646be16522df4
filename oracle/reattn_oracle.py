"""ctypes/numpy front for the fp64 CPU oracle (oracle/reattn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module and
this module never imports the product package.

Arrays are numpy; q / K / V are passed as their exact stored bytes: float32
arrays, or bfloat16 / IEEE half as uint16 bit patterns (dtype="bf16" / "f16").
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "reattn_oracle.c")
_LIB = os.path.join(_HERE, "libreattn_oracle.so")

F32, BF16, F16 = 0, 1, 2
_DTYPE_CODE = {"f32": F32, "bf16": BF16, "f16": F16}
AGG_SUM, AGG_MAX = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Shape(C.Structure):
    _fields_ = [
        ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("dtype", C.c_int32), ("n_ctx", C.c_int64), ("n_sink", C.c_int32),
        ("n_local", C.c_int32), ("top_k", C.c_int32), ("agg", C.c_int32),
        ("rope_theta", C.c_double), ("softmax_scale", C.c_double),
        ("k_stride_head", C.c_int64), ("k_stride_tok", C.c_int64),
        ("v_stride_head", C.c_int64), ("v_stride_tok", C.c_int64),
    ]


@dataclass
class Shape:
    """Problem description in the paper's terms (Eq. 1-3)."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # "f32" | "bf16" | "f16"
    n_ctx: int
    n_sink: int
    n_local: int
    top_k: int
    rope_theta: float
    agg: int = AGG_SUM
    softmax_scale: float = 0.0

    def c(self) -> _Shape:
        D, N = self.head_dim, self.n_ctx
        return _Shape(self.n_q_heads, self.n_kv_heads, D, _DTYPE_CODE[self.dtype],
                      N, self.n_sink, self.n_local, self.top_k, self.agg,
                      float(self.rope_theta), float(self.softmax_scale),
                      N * D, D, N * D, D)

    def partition(self):
        """(s_eff, l_eff, n_mid, k_eff) of Eq. 1 with the clamping rules."""
        lib = _lib()
        s, l, m, k = (C.c_int64() for _ in range(4))
        lib.ro_partition(self.n_ctx, self.n_sink, self.n_local, self.top_k,
                         C.byref(s), C.byref(l), C.byref(m), C.byref(k))
        return s.value, l.value, m.value, k.value


_cached = None


def _lib():
    global _cached
    if _cached is None:
        lib = C.CDLL(build())
        P = C.c_void_p
        lib.ro_partition.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_int32, P, P, P, P]
        lib.ro_partition.restype = None
        lib.ro_widen_bf16.argtypes = [C.c_uint16]
        lib.ro_widen_bf16.restype = C.c_double
        lib.ro_widen_f16.argtypes = [C.c_uint16]
        lib.ro_widen_f16.restype = C.c_double
        lib.ro_score.argtypes = [P, C.c_int32, P, P, P]
        lib.ro_topk_row.argtypes = [P, C.c_int64, C.c_int64, C.c_int64, P, P]
        lib.ro_topk.argtypes = [P, C.c_int64, C.c_int64, C.c_int64, C.c_int64, P, P]
        lib.ro_gather_rope.argtypes = [P, P, P, P, C.c_int64, C.c_double, P, P]
        lib.ro_gather_rope.restype = C.c_int64
        lib.ro_attend.argtypes = [P, C.c_int32, P, P, P, P, P, C.c_double, P]
        lib.ro_forward.argtypes = [P, C.c_int32, P, P, P, P, P, P, P, P]
        lib.ro_head_scores.argtypes = [P, C.c_int32, P, P, P]
        lib.ro_vote_merge.argtypes = [P, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                      P, P, P, P]
        _cached = lib
    return _cached


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check_store(a: np.ndarray, sh: Shape, name: str) -> np.ndarray:
    want = np.float32 if sh.dtype == "f32" else np.uint16        # bf16 / f16 travel as bit patterns
    if a.dtype != want:
        raise TypeError(f"{name}: expected {want} storage for dtype {sh.dtype}, got {a.dtype}")
    if not a.flags.c_contiguous:
        raise ValueError(f"{name}: must be C-contiguous")
    return a


def _check_rc(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def widen_bf16(bits: int) -> float:
    return _lib().ro_widen_bf16(int(bits) & 0xFFFF)


def widen_f16(bits: int) -> float:
    return _lib().ro_widen_f16(int(bits) & 0xFFFF)


def score(sh: Shape, q: np.ndarray, k_cache: np.ndarray) -> np.ndarray:
    """Eq. 2 scores: q [M,Hq,D], K [Hkv,N,D] -> float64 [M,Hkv,N_mid]."""
    _check_store(q, sh, "q"); _check_store(k_cache, sh, "k_cache")
    M = q.shape[0]
    _, _, n_mid, _ = sh.partition()
    out = np.empty((M, sh.n_kv_heads, n_mid), dtype=np.float64)
    cs = sh.c()
    _check_rc(_lib().ro_score(C.byref(cs), M, _ptr(q), _ptr(k_cache), _ptr(out)), "score")
    return out


def topk_rows(scores: np.ndarray, k: int, index_base: int = 0):
    """scores float64 [R, n] -> (idx int32 [R, min(k,n)] ascending absolute, kth float64 [R])."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    R, n = scores.shape
    k_eff = max(0, min(k, n))
    idx = np.empty((R, k_eff), dtype=np.int32)
    kth = np.zeros((R,), dtype=np.float64)
    _check_rc(_lib().ro_topk(_ptr(scores), R, n, k_eff, index_base, _ptr(idx), _ptr(kth)), "topk")
    return idx, kth


def gather_rope(sh: Shape, k_cache, v_cache, idx: np.ndarray, q_tok: int | None = None,
                pos_offset: float = 0.0):
    """Concatenation of Eq. 3 for one query: (K rotated [Hkv,S,D], V [Hkv,S,D], kept length)."""
    _check_store(k_cache, sh, "k_cache"); _check_store(v_cache, sh, "v_cache")
    s, l, _, k = sh.partition()
    S = s + k + l
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(sh.n_kv_heads, k)
    ks = np.zeros((sh.n_kv_heads, S, sh.head_dim), dtype=np.float64)
    vs = np.zeros_like(ks)
    cs = sh.c()
    n = _lib().ro_gather_rope(C.byref(cs), _ptr(k_cache), _ptr(v_cache), _ptr(idx),
                              sh.n_ctx - 1 if q_tok is None else q_tok, float(pos_offset),
                              _ptr(ks), _ptr(vs))
    return ks, vs, int(n)


def attend(sh: Shape, q, k_cache, v_cache, idx: np.ndarray, q_tok=None,
           pos_offset: float = 0.0) -> np.ndarray:
    """Eq. 3 attention on given index sets: idx [M,Hkv,k_eff] -> float64 [M,Hq,D]."""
    _check_store(q, sh, "q"); _check_store(k_cache, sh, "k_cache"); _check_store(v_cache, sh, "v_cache")
    M = q.shape[0]
    _, _, _, k = sh.partition()
    idx = np.ascontiguousarray(idx, dtype=np.int32).reshape(M, sh.n_kv_heads, k)
    qt = _q_tok(sh, M, q_tok)
    out = np.empty((M, sh.n_q_heads, sh.head_dim), dtype=np.float64)
    cs = sh.c()
    _check_rc(_lib().ro_attend(C.byref(cs), M, _ptr(q), _ptr(qt), _ptr(k_cache), _ptr(v_cache),
                               _ptr(idx), float(pos_offset), _ptr(out)), "attend")
    return out


def _q_tok(sh: Shape, M: int, q_tok) -> np.ndarray:
    if q_tok is None:  # queries are the last M cached tokens (appendix: append, then select)
        q_tok = np.arange(sh.n_ctx - M, sh.n_ctx)
    qt = np.ascontiguousarray(q_tok, dtype=np.int64)
    assert qt.shape == (M,)
    return qt


def forward(sh: Shape, q, k_cache, v_cache, q_tok=None, want_scores: bool = False):
    """Whole step.  Returns dict(idx [M,Hkv,k_eff], kth [M,Hkv], out [M,Hq,D], scores?)."""
    _check_store(q, sh, "q"); _check_store(k_cache, sh, "k_cache"); _check_store(v_cache, sh, "v_cache")
    M = q.shape[0]
    _, _, n_mid, k = sh.partition()
    qt = _q_tok(sh, M, q_tok)
    idx = np.empty((M, sh.n_kv_heads, k), dtype=np.int32)
    kth = np.zeros((M, sh.n_kv_heads), dtype=np.float64)
    sc = np.empty((M, sh.n_kv_heads, n_mid), dtype=np.float64) if want_scores else None
    out = np.empty((M, sh.n_q_heads, sh.head_dim), dtype=np.float64)
    cs = sh.c()
    _check_rc(_lib().ro_forward(C.byref(cs), M, _ptr(q), _ptr(qt), _ptr(k_cache), _ptr(v_cache),
                                _ptr(idx), _ptr(kth), _ptr(sc), _ptr(out)), "forward")
    return {"idx": idx, "kth": kth, "out": out, "scores": sc}


# ---- vote selection (paper: votes over heads and query rows, top-k' centres, spans) ----------
def head_scores(sh: Shape, q: np.ndarray, k_cache: np.ndarray) -> np.ndarray:
    """Per-head raw scores: q [M,Hq,D], K [Hkv,N,D] -> float64 [M,Hq,N_mid]."""
    _check_store(q, sh, "q"); _check_store(k_cache, sh, "k_cache")
    M = q.shape[0]
    _, _, n_mid, _ = sh.partition()
    out = np.empty((M, sh.n_q_heads, n_mid), dtype=np.float64)
    cs = sh.c()
    _check_rc(_lib().ro_head_scores(C.byref(cs), M, _ptr(q), _ptr(k_cache), _ptr(out)), "head_scores")
    return out


def vote_merge(head_topk: np.ndarray, n_mid: int, index_base: int, n_centres: int, span: int):
    """head_topk int32 [R, vote_k] absolute -> dict(votes [n_mid], centres [<=n_centres], sel [n_sel])."""
    head_topk = np.ascontiguousarray(head_topk, dtype=np.int32)
    R, vote_k = head_topk.shape
    votes = np.zeros((max(n_mid, 0),), dtype=np.int32)
    centres = np.full((max(n_centres, 0),), -1, dtype=np.int32)
    sel = np.empty((max(n_centres * span, 1),), dtype=np.int32)
    n_sel = C.c_int64(0)
    _check_rc(_lib().ro_vote_merge(_ptr(head_topk), R, vote_k, n_mid, index_base, n_centres, span,
                                   _ptr(votes), _ptr(centres), _ptr(sel), C.byref(n_sel)), "vote_merge")
    return {"votes": votes, "centres": centres[centres >= 0], "sel": sel[:n_sel.value].copy()}


def vote_forward(sh: Shape, q, k_cache, v_cache, vote_k: int, n_centres: int, span: int, q_tok=None,
                 head_topk=None):
    """Whole step with the vote selection: per-head top-k -> votes -> centres -> spans ->
    attention of every query row over [global, shared selection, local].  `head_topk`
    (int32 [M,Hq,vote_k]) replaces the oracle's own per-head lists when given.
    Returns dict(head_topk, head_kth [M,Hq], votes, centres, sel, out [M,Hq,D], head_scores)."""
    M = q.shape[0]
    s_eff, l_eff, n_mid, _ = sh.partition()
    hs = head_scores(sh, q, k_cache)
    kk = max(0, min(vote_k, n_mid))
    own, kth = topk_rows(hs.reshape(M * sh.n_q_heads, n_mid), kk, index_base=s_eff)
    lists = own if head_topk is None else np.ascontiguousarray(head_topk, dtype=np.int32).reshape(own.shape)
    m = vote_merge(lists, n_mid, s_eff, n_centres, span)
    sel = m["sel"]
    from dataclasses import replace as _replace
    sh2 = _replace(sh, top_k=int(sel.size))
    idx = np.broadcast_to(sel, (M, sh.n_kv_heads, sel.size)).copy()
    out = attend(sh2, q, k_cache, v_cache, idx, q_tok=q_tok)
    return {"head_topk": own.reshape(M, sh.n_q_heads, kk), "head_kth": kth.reshape(M, sh.n_q_heads),
            "votes": m["votes"], "centres": m["centres"], "sel": sel, "out": out, "head_scores": hs}


# ---- streaming prefill of one layer (appendix, prefilling phase) -------------------------------
def prefill_sequence(sh: Shape, q, k_new, v_new, chunk: int, vote=None):
    """The chunk loop of the prefilling phase for ONE layer: the first chunk holds
    n_sink + n_local tokens, every later one `chunk` tokens; a chunk's keys and values are
    appended to the cache, then its query rows select from the middle and attend (Eq. 1-3).
    sh.n_ctx = L is the sequence length.  q [L,Hq,D]; k_new, v_new [L,Hkv,D] token-major, as
    the projections deliver them.  vote = (vote_k, n_centres, span) switches to the vote
    selection.  Returns dict(out [L,Hq,D], chunks = [(start, end, per-chunk result dict)])."""
    from dataclasses import replace as _replace
    L = sh.n_ctx
    assert q.shape[0] == L and k_new.shape[0] == L and v_new.shape[0] == L
    k_cache = np.ascontiguousarray(np.transpose(k_new, (1, 0, 2)))      # [Hkv, L, D]: row t is token t
    v_cache = np.ascontiguousarray(np.transpose(v_new, (1, 0, 2)))
    out = np.empty((L, sh.n_q_heads, sh.head_dim), dtype=np.float64)
    chunks = []
    s, e = 0, min(L, sh.n_sink + sh.n_local)
    while s < L:
        she = _replace(sh, n_ctx=e)
        kc = np.ascontiguousarray(k_cache[:, :e])                        # the cache as it stands after the append
        vc = np.ascontiguousarray(v_cache[:, :e])
        qc = np.ascontiguousarray(q[s:e])
        if vote is None:
            r = forward(she, qc, kc, vc, want_scores=True)
        else:
            r = vote_forward(she, qc, kc, vc, *vote)
        out[s:e] = r["out"]
        chunks.append((s, e, r))
        s, e = e, min(L, e + chunk)
    return {"out": out, "chunks": chunks}
