"""Shared comparison rules for the GPU parity tests (HIP path vs fp64 CPU oracle).

Bars (from the benchmark spec):
  * top-k index sets bit-exact, except that entries whose ORACLE score lies within
    1e-3 relative of the oracle's k-th score may be swapped for one another;
  * attention outputs within max-abs 2e-2 (bf16 storage) / 1e-4 (fp32 storage) of the
    oracle: on the oracle's own set for every row whose GPU set equals it, and on the
    GPU's set for all rows when some GPU set differs inside the tie band (a swapped entry
    is as good by the position-agnostic score but not by the rotary-encoded logit).
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import reattn_oracle as ro
from paper_2407_15176_amd import binding as B
from paper_2407_15176_amd import workloads as wl

TIE_BAND = 1e-3
# f16 storage: not named by the benchmark spec; the arithmetic is the bf16 path's (fp32 on exactly
# widened inputs, hi + lo halves on the matrix cores), measured at 1e-5..5e-4, so it is held to 1e-3
OUT_TOL = {"bf16": 2e-2, "f32": 1e-4, "f16": 1e-3}


def oracle_shape(w: wl.Workload, agg: int = ro.AGG_SUM) -> ro.Shape:
    return ro.Shape(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, w.n_ctx, w.n_sink, w.n_local,
                    w.top_k, w.rope_theta, agg=agg)


def host_inputs(t: dict):
    return wl.to_numpy_store(t["q"]), wl.to_numpy_store(t["k"]), wl.to_numpy_store(t["v"])


def check_index_sets(gpu_idx: np.ndarray, ora_idx: np.ndarray, ora_scores: np.ndarray,
                     kth: np.ndarray, s_eff: int, n_mid: int):
    """gpu_idx/ora_idx [R,k]; ora_scores [R,n_mid] fp64; kth [R].  Returns #rows that differ."""
    R, k = ora_idx.shape
    assert gpu_idx.shape == (R, k), (gpu_idx.shape, ora_idx.shape)
    differ = 0
    for r in range(R):
        g, o = gpu_idx[r].astype(np.int64), ora_idx[r].astype(np.int64)
        if k:
            assert np.all(np.diff(g) > 0), f"row {r}: indices not strictly ascending"
            assert g[0] >= s_eff and g[-1] < s_eff + n_mid, f"row {r}: index outside the middle"
        if np.array_equal(g, o):
            continue
        differ += 1
        only_g = np.setdiff1d(g, o, assume_unique=True)
        only_o = np.setdiff1d(o, g, assume_unique=True)
        assert only_g.size == only_o.size
        band = TIE_BAND * abs(kth[r])
        sg = ora_scores[r, only_g - s_eff]
        so = ora_scores[r, only_o - s_eff]
        assert np.all(np.abs(sg - kth[r]) <= band), (
            f"row {r}: GPU picked {only_g.size} entries outside the tie band "
            f"(worst {np.abs(sg - kth[r]).max():.3e} vs band {band:.3e})")
        assert np.all(np.abs(so - kth[r]) <= band), (
            f"row {r}: GPU missed entries outside the tie band "
            f"(worst {np.abs(so - kth[r]).max():.3e} vs band {band:.3e})")
    return differ


def check_layer(w: wl.Workload, t: dict, gpu_out: torch.Tensor, gpu_idx: torch.Tensor,
                q_rows=None, agg: int = ro.AGG_SUM):
    """Full comparison of one decode step / prefill chunk.  q_rows: subset of query rows the
    oracle evaluates (None = all)."""
    sh = oracle_shape(w, agg)
    q, k, v = host_inputs(t)
    M = w.n_query
    rows = np.arange(M) if q_rows is None else np.asarray(q_rows)
    q_tok = (w.n_ctx - M + rows).astype(np.int64)
    res = ro.forward(sh, np.ascontiguousarray(q[rows]), k, v, q_tok=q_tok, want_scores=True)
    s_eff, l_eff, n_mid, k_eff = sh.partition()
    g_idx = gpu_idx.cpu().numpy()[rows]
    g_out = gpu_out.cpu().numpy().astype(np.float64)[rows]
    nr = rows.size * w.n_kv_heads
    differ = check_index_sets(g_idx.reshape(nr, k_eff), res["idx"].reshape(nr, k_eff),
                              res["scores"].reshape(nr, n_mid), res["kth"].reshape(nr), s_eff, n_mid)
    tol = OUT_TOL[w.dtype]
    assert np.isfinite(g_out).all()
    # Where the GPU's set equals the oracle's, the outputs must agree.  Where it differs inside the
    # tie band, the swapped entries were equally good by the position-agnostic score of Eq. 2 but
    # can carry very different attention weights once rotary-encoded (Eq. 3), so the two outputs may
    # legitimately differ: there the GPU is held to the oracle evaluated on the GPU's own set.
    same = np.ones(rows.size * w.n_kv_heads, dtype=bool)
    for r_ in range(same.size):
        same[r_] = np.array_equal(g_idx.reshape(nr, k_eff)[r_], res["idx"].reshape(nr, k_eff)[r_])
    same_q = np.repeat(same.reshape(rows.size, w.n_kv_heads), w.n_q_heads // w.n_kv_heads, axis=1)   # [rows, Hq]
    diff_all = np.abs(g_out - res["out"]).max(axis=2)
    err = float(diff_all[same_q].max()) if same_q.any() else 0.0
    assert err <= tol, f"output max-abs error {err:.3e} > {tol}"
    err2 = 0.0
    if differ:
        out2 = ro.attend(sh, np.ascontiguousarray(q[rows]), k, v, g_idx, q_tok=q_tok)
        err2 = np.abs(g_out - out2).max()
        assert err2 <= tol, f"output vs oracle-on-GPU-set max-abs error {err2:.3e} > {tol}"
    return {"rows_differ": differ, "max_abs_err": float(err), "max_abs_err_own_set": float(err2)}


def run_layer(w: wl.Workload, t: dict, agg: int = B.AGG_SUM, route: int = 0):
    p = B.Params.from_workload(w)
    p.agg = agg
    p.route = route
    ws = B.alloc_workspace(p)
    fn = B.decode_step if w.n_query == 1 else B.prefill_chunk
    out, idx = fn(p, t["q"], t["k"], t["v"], ws)
    torch.cuda.synchronize()
    return out, idx
