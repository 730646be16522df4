"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times.  The oracle evaluates the whole decode step (its cost is
seconds on the host cores); config 4 (prefill) samples query rows."""
import numpy as np
import pytest
import torch

from paper_2407_15176_amd import binding as B
from paper_2407_15176_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _decode_full(cfg):
    w = wl.CONFIGS[cfg]
    t = wl.generate(w, "cuda")
    out, idx = P.run_layer(w, t)
    r = P.check_layer(w, t, out, idx)
    print(f"\n{w.name}: {r}", flush=True)
    idx_h = idx.cpu().numpy()[0]
    needles = set(t["needles"].tolist())
    assert len(needles) == w.n_needles
    for h in range(w.n_kv_heads):
        assert needles <= set(idx_h[h].tolist())          # every planted needle is retrieved
    return r


def test_config2_decode_128k():
    _decode_full(2)


def test_config3_decode_1m():
    _decode_full(3)


@pytest.mark.timeout(600)
def test_config5_decode_4m_three_query_heads_per_group():
    r = _decode_full(5)
    assert r["max_abs_err"] <= 2e-2


@pytest.mark.timeout(900)
def test_config4_prefill_chunk_4096_queries_sampled_rows():
    """Config 4: every query row is computed on the GPU; the oracle checks a seeded sample of rows
    (first, last and 22 others), index sets and outputs."""
    w = wl.CONFIGS[4]
    t = wl.generate(w, "cuda")
    out, idx = P.run_layer(w, t)
    rows = np.unique(np.concatenate([[0, 1, w.n_query - 2, w.n_query - 1],
                                     np.random.default_rng(4).integers(0, w.n_query, 20)]))
    r = P.check_layer(w, t, out, idx, q_rows=rows)
    print(f"\n{w.name}: rows {rows.tolist()} -> {r}", flush=True)
    # structural checks on ALL rows: ascending, in range, finite outputs
    idx_h = idx.cpu().numpy()
    assert np.all(np.diff(idx_h, axis=-1) > 0)
    assert idx_h.min() >= w.n_sink and idx_h.max() < w.n_ctx - w.n_local
    assert torch.isfinite(out).all()


# ---------------------------------------------------------------- vote selection at full size
def _vote_decode_full(cfg):
    from oracle import reattn_oracle as ro
    w = wl.CONFIGS[cfg].scaled(top_k=0, max_position=0)
    v = B.Vote(4, 127, 32)
    t = wl.generate(w, "cuda")
    p = B.Params.from_workload(w)
    ws = B.alloc_vote_workspace(p, v)
    lists = B.vote_topk(p, v, t["q"], t["k"], ws)
    out, sel, n_sel = B.vote_layer(p, v, t["q"], t["k"], t["v"], ws)
    torch.cuda.synchronize()
    sh = P.oracle_shape(w)
    q, k, vv = P.host_inputs(t)
    res = ro.vote_forward(sh, q, k, vv, v.vote_k, v.n_centres, v.span, head_topk=lists.cpu().numpy())
    s_eff, l_eff, n_mid, _ = sh.partition()
    P.check_index_sets(lists.cpu().numpy().reshape(w.n_q_heads, 4), res["head_topk"].reshape(w.n_q_heads, 4),
                       res["head_scores"].reshape(w.n_q_heads, n_mid), res["head_kth"].reshape(w.n_q_heads),
                       s_eff, n_mid)
    n = int(n_sel.item())
    assert sel.cpu().numpy()[:n].tolist() == res["sel"].tolist()
    err = np.abs(out.cpu().numpy().astype(np.float64) - res["out"]).max()
    print(f"\n{w.name} vote: n_sel {n}, max_abs_err {err:.3e}", flush=True)
    assert err <= P.OUT_TOL[w.dtype]


@pytest.mark.timeout(600)
def test_config3_vote_decode_1m():
    _vote_decode_full(3)


@pytest.mark.timeout(900)
def test_config5_vote_decode_4m():
    _vote_decode_full(5)


@pytest.mark.timeout(900)
def test_config4_vote_chunk_4096_queries():
    """Config 4's cache, all 4,096 query rows on the GPU with the vote selection.  The oracle checks
    (1) the per-head lists of a seeded sample of rows, (2) the integer pipeline votes -> centres ->
    spans exactly, on ALL of the GPU's 524,288 votes, (3) the attention of the sampled rows over the
    shared selection."""
    from dataclasses import replace
    from oracle import reattn_oracle as ro
    w = wl.CONFIGS[4].scaled(top_k=0, max_position=0)
    v = B.Vote(4, 127, 32)
    t = wl.generate(w, "cuda")
    p = B.Params.from_workload(w)
    ws = B.alloc_vote_workspace(p, v)
    lists = B.vote_topk(p, v, t["q"], t["k"], ws)
    out, sel, n_sel = B.vote_layer(p, v, t["q"], t["k"], t["v"], ws)
    torch.cuda.synchronize()
    sh = P.oracle_shape(w)
    q, k, vv = P.host_inputs(t)
    s_eff, l_eff, n_mid, _ = sh.partition()
    rows = np.unique(np.concatenate([[0, 1, w.n_query - 1], np.random.default_rng(9).integers(0, w.n_query, 5)]))
    lists_h = lists.cpu().numpy()
    # (1) lists of the sampled rows
    hs = ro.head_scores(sh, np.ascontiguousarray(q[rows]), k)                       # [R, Hq, n_mid]
    R = rows.size * w.n_q_heads
    own, kth = ro.topk_rows(hs.reshape(R, n_mid), 4, index_base=s_eff)
    P.check_index_sets(lists_h[rows].reshape(R, 4), own, hs.reshape(R, n_mid), kth, s_eff, n_mid)
    # (2) the merge, exactly, on everything the GPU voted
    want = ro.vote_merge(lists_h.reshape(-1, 4), n_mid, s_eff, v.n_centres, v.span)
    n = int(n_sel.item())
    sel_h = sel.cpu().numpy()[:n]
    assert sel_h.tolist() == want["sel"].tolist()
    # (3) attention of the sampled rows over the shared selection
    idx = np.broadcast_to(sel_h, (rows.size, w.n_kv_heads, n)).copy()
    ref = ro.attend(replace(sh, top_k=n), np.ascontiguousarray(q[rows]), k, vv, idx,
                    q_tok=(w.n_ctx - w.n_query + rows).astype(np.int64))
    err = np.abs(out.cpu().numpy().astype(np.float64)[rows] - ref).max()
    print(f"\n{w.name} vote chunk: n_sel {n}, rows {rows.tolist()}, max_abs_err {err:.3e}", flush=True)
    assert err <= P.OUT_TOL[w.dtype]
    assert torch.isfinite(out).all()
