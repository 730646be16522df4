"""Seeded random shapes: decode steps, chunks and vote layers at sizes the oracle finishes in
milliseconds, drawn to hit the corners the fixed cases miss (tiny middles, k around N_mid, spans
larger than the middle, query counts around tile boundaries, every supported group size)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import reattn_oracle as ro
from paper_2407_15176_amd import binding as B
from paper_2407_15176_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _draw(seed: int):
    r = np.random.default_rng(1000 + seed)
    dtype = ["bf16", "f16", "f32"][seed % 3]
    D = 128 if dtype != "f32" else int(r.choice([64, 128]))
    G = int(r.choice([1, 2, 3, 4, 8]))
    Hkv = int(r.choice([1, 2, 3]))
    n_sink = int(r.choice([0, 1, 4, 33]))
    n_local = int(r.choice([1, 7, 64, 200, 513]))
    n_mid = int(r.choice([0, 1, 5, 63, 64, 65, 1000, 4097, 8193, 20000]))
    M = int(r.choice([1, 1, 1, 2, 5, 33])) if n_mid > 0 else int(r.choice([1, 3, 40]))
    M = min(M, n_local) if n_mid > 0 else M
    n_ctx = n_sink + n_local + n_mid if n_mid > 0 else int(r.integers(1, n_sink + n_local + 1))
    M = min(M, n_ctx)                                   # an empty middle takes any M <= N (the first chunk of the prefilling phase)
    top_k = int(r.choice([0, 1, 3, 64, 500, 5000]))
    base = wl.CONFIGS[2] if dtype != "f32" else wl.CONFIGS[1]
    w = base.scaled(dtype=dtype, head_dim=D, n_q_heads=G * Hkv, n_kv_heads=Hkv, n_ctx=n_ctx, n_query=M, n_sink=n_sink,
                    n_local=n_local, top_k=top_k, max_position=0, n_needles=int(r.choice([0, 3])), cfg=int(r.integers(1, 90)),
                    scale_q=bool(r.integers(0, 2)))
    vote = B.Vote(int(r.choice([1, 2, 4, 8])), int(r.choice([1, 5, 127, 1024])), int(r.choice([1, 2, 32, 100000])))
    return w, vote


@pytest.mark.parametrize("seed", range(72))
def test_layer_random_shape(seed):
    w, _ = _draw(seed)
    p = B.Params.from_workload(w)
    if B.validate(p) != B.OK:
        pytest.skip("shape outside the library's domain")
    t = wl.generate(w, "cuda")
    out, idx = P.run_layer(w, t)
    P.check_layer(w, t, out, idx)


@pytest.mark.parametrize("seed", range(0, 72, 3))
def test_layer_random_shape_max_aggregation(seed):
    """The same draws with the largest per-head score of a group instead of the sum (REATTN_AGG_MAX)."""
    w, _ = _draw(seed)
    t = wl.generate(w, "cuda")
    out, idx = P.run_layer(w, t, agg=B.AGG_MAX)
    P.check_layer(w, t, out, idx, agg=B.AGG_MAX)


@pytest.mark.parametrize("seed", range(72))
def test_vote_layer_random_shape(seed):
    w, v = _draw(seed)
    w = w.scaled(top_k=0)
    p = B.Params.from_workload(w)
    if B.vote_workspace_bytes(p, v) == 0:
        pytest.skip("shape outside the vote path's domain")
    t = wl.generate(w, "cuda")
    ws = B.alloc_vote_workspace(p, v)
    lists = B.vote_topk(p, v, t["q"], t["k"], ws)
    out, sel, n_sel = B.vote_layer(p, v, t["q"], t["k"], t["v"], ws)
    torch.cuda.synchronize()
    sh = P.oracle_shape(w)
    q, k, vv = P.host_inputs(t)
    res = ro.vote_forward(sh, q, k, vv, v.vote_k, v.n_centres, v.span, head_topk=lists.cpu().numpy())
    s_eff, l_eff, n_mid, _ = sh.partition()
    kk = res["head_topk"].shape[-1]
    R = w.n_query * w.n_q_heads
    P.check_index_sets(lists.cpu().numpy().reshape(R, kk), res["head_topk"].reshape(R, kk),
                       res["head_scores"].reshape(R, n_mid), res["head_kth"].reshape(R), s_eff, n_mid)
    n = int(n_sel.item())
    assert sel.cpu().numpy()[:n].tolist() == res["sel"].tolist()
    err = np.abs(out.cpu().numpy().astype(np.float64) - res["out"]).max()
    assert err <= P.OUT_TOL[w.dtype], err


def _draw_large(seed: int):
    """Longer middles (the chip-wide top-k past 65,536 scores), chunks of several query tiles and odd query
    counts, more heads: what the draws above do not reach."""
    r = np.random.default_rng(5000 + seed)
    dtype = ["bf16", "f16", "bf16", "f32"][seed % 4]
    D = 128 if dtype != "f32" else int(r.choice([64, 128]))
    G = int(r.choice([1, 3, 4, 7, 8]))
    Hkv = int(r.choice([1, 2, 4]))
    n_sink = int(r.choice([0, 4, 32]))
    n_local = int(r.choice([64, 300, 1024]))
    n_mid = int(r.choice([3000, 30000, 66000, 70001, 140000]))
    M = min(int(r.choice([1, 1, 2, 5, 64, 129, 300, 511])), n_local)
    top_k = int(r.choice([1, 100, 1024, 4096]))
    base = wl.CONFIGS[2] if dtype != "f32" else wl.CONFIGS[1]
    w = base.scaled(dtype=dtype, head_dim=D, n_q_heads=G * Hkv, n_kv_heads=Hkv, n_ctx=n_sink + n_local + n_mid, n_query=M,
                    n_sink=n_sink, n_local=n_local, top_k=top_k, max_position=0, n_needles=int(r.choice([0, 3])),
                    cfg=int(r.integers(1, 90)), scale_q=bool(r.integers(0, 2)))
    rows = None if M <= 8 else sorted(set([0, 1, M // 2, M - 2, M - 1] + [int(x) for x in r.integers(0, M, 3)]))
    return w, rows


@pytest.mark.parametrize("seed", range(48))
def test_layer_random_large_shape(seed):
    w, rows = _draw_large(seed)
    p = B.Params.from_workload(w)
    if B.validate(p) != B.OK:
        pytest.skip("shape outside the library's domain")
    t = wl.generate(w, "cuda")
    out, idx = P.run_layer(w, t)
    P.check_layer(w, t, out, idx, q_rows=rows)
