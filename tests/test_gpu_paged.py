"""Paged caches: pools [Hkv][P * page_size][D] behind a device page table.

A paged call reads exactly the rows a contiguous call reads, through one more indirection, and runs the
same arithmetic in the same order: every result must equal the contiguous call's bit for bit (and the
contiguous call is what the oracle tests pin).  Pages are scattered over a pool with spare pages that hold
garbage, so a wrong translation shows."""
from dataclasses import replace

import pytest
import torch

from paper_2407_15176_amd import binding as B
from paper_2407_15176_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _paged(w: wl.Workload, t: dict, page_size: int, seed: int, spare: int = 7):
    """Scatters the contiguous caches of t over pools; returns (params, k_pool, v_pool, rows) with
    rows[tok] = the pool row of token tok."""
    N, Hkv, D = w.n_ctx, w.n_kv_heads, w.head_dim
    n_pages = -(-N // page_size)
    P = n_pages + spare
    g = torch.Generator().manual_seed(seed)
    table = torch.randperm(P, generator=g)[:n_pages].to(torch.int32)
    tok = torch.arange(N)
    rows = table[tok // page_size].long() * page_size + tok % page_size
    dt = t["k"].dtype
    gd = torch.Generator(device="cuda").manual_seed(seed)
    k_pool = torch.randn(Hkv, P * page_size, D, generator=gd, device="cuda").to(dt)   # garbage in the unused rows
    v_pool = torch.randn(Hkv, P * page_size, D, generator=gd, device="cuda").to(dt)
    k_pool[:, rows.cuda()] = t["k"]
    v_pool[:, rows.cuda()] = t["v"]
    p = replace(B.Params.from_workload(w), k_stride_head=P * page_size * D, k_stride_tok=D,
                v_stride_head=P * page_size * D, v_stride_tok=D, page_table=table.cuda(), page_size=page_size)
    return p, k_pool, v_pool, rows.cuda()


CASES = {
    "bf16_d128_g4": (wl.CONFIGS[2].scaled(n_ctx=20_011, n_local=300, top_k=333), 64),
    "bf16_d128_long": (wl.CONFIGS[2].scaled(n_ctx=150_001, n_local=1_000, top_k=2_000), 256),   # several workgroups per head
    "f32_d64_g4": (wl.CONFIGS[1].scaled(n_ctx=9_973, n_local=200, top_k=100), 128),
    "f16_d128_g3": (wl.CONFIGS[5].scaled(dtype="f16", n_ctx=17_000, n_local=257, top_k=128, max_position=0), 1024),
    "bf16_one_page": (wl.CONFIGS[2].scaled(n_ctx=700, n_local=64, top_k=50), 1024),
}


@pytest.mark.parametrize("name", list(CASES))
def test_paged_decode_step_equals_contiguous(name):
    w, ps = CASES[name]
    t = wl.generate(w, "cuda")
    p0 = B.Params.from_workload(w)
    out0, idx0 = B.decode_step(p0, t["q"], t["k"], t["v"], B.alloc_workspace(p0), want_idx=True)
    p, kp, vp, _ = _paged(w, t, ps, seed=11)
    out1, idx1 = B.decode_step(p, t["q"], kp, vp, B.alloc_workspace(p), want_idx=True)
    torch.cuda.synchronize()
    assert torch.equal(idx0, idx1)
    assert torch.equal(out0, out1)


@pytest.mark.parametrize("name", ["bf16_d128_g4", "f32_d64_g4"])
def test_paged_separate_calls_equal_contiguous(name):
    w, ps = CASES[name]
    t = wl.generate(w, "cuda")
    p0 = B.Params.from_workload(w)
    p, kp, vp, _ = _paged(w, t, ps, seed=12)
    ws0, ws1 = B.alloc_workspace(p0), B.alloc_workspace(p)
    s0 = B.score(p0, t["q"], t["k"], ws=ws0)
    s1 = B.score(p, t["q"], kp, ws=ws1)
    torch.cuda.synchronize()
    assert torch.equal(s0, s1)
    idx = B.topk(p0, s0, ws0)
    k0, v0 = B.gather_rope(p0, t["k"], t["v"], idx)
    k1, v1 = B.gather_rope(p, kp, vp, idx)
    torch.cuda.synchronize()
    assert torch.equal(k0, k1) and torch.equal(v0, v1)


def test_paged_append_and_decode_token():
    """Three layers over paged pools that share one page table: the token's rows land in the right pool rows
    and every layer's output equals the contiguous call's."""
    n_layers, ps = 3, 128
    w = wl.CONFIGS[2].scaled(n_ctx=9_000, n_local=200, top_k=150, max_position=0, n_needles=0)
    dt = w.torch_dtype()
    Hq, Hkv, D, N = w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_ctx
    g = torch.Generator(device="cuda").manual_seed(240715000 + 91)
    ts = [wl.generate(w, "cuda") for _ in range(n_layers)]
    for l in range(1, n_layers):                                 # distinct caches per layer
        ts[l]["k"] = torch.randn(Hkv, N, D, generator=g, device="cuda").to(dt)
        ts[l]["v"] = torch.randn(Hkv, N, D, generator=g, device="cuda").to(dt)
    qs = [torch.randn(1, Hq, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    kn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    vn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    p0 = replace(B.Params.from_workload(w), n_query=1)
    k0 = [t["k"].clone() for t in ts]; v0 = [t["v"].clone() for t in ts]
    want = B.decode_token(p0, qs, kn, vn, k0, v0, B.alloc_workspace(p0))
    pools = [_paged(w, t, ps, seed=13) for t in ts]              # the same seed: one page table for all layers
    p = pools[0][0]
    kps = [x[1] for x in pools]; vps = [x[2] for x in pools]
    rows = pools[0][3]
    got = B.decode_token(p, qs, kn, vn, kps, vps, B.alloc_workspace(p))
    torch.cuda.synchronize()
    for l in range(n_layers):
        assert torch.equal(kps[l][:, rows[N - 1]], kn[l][0]) and torch.equal(vps[l][:, rows[N - 1]], vn[l][0])
        assert torch.equal(kps[l][:, rows], k0[l]) and torch.equal(vps[l][:, rows], v0[l])
        assert torch.equal(got[l], want[l]), l
    # a block of tokens through reattn_cache_append
    k_new = torch.randn(300, Hkv, D, generator=g, device="cuda").to(dt)
    v_new = torch.randn(300, Hkv, D, generator=g, device="cuda").to(dt)
    B.cache_append(p, 4_000, k_new, v_new, kps[0], vps[0])
    torch.cuda.synchronize()
    assert torch.equal(kps[0][:, rows[4_000:4_300]], k_new.transpose(0, 1))
    assert torch.equal(vps[0][:, rows[4_000:4_300]], v_new.transpose(0, 1))


VOTES = {
    "bf16_d128_g4": B.Vote(4, 12, 16),
    "bf16_d128_long": B.Vote(8, 127, 32),          # lists of 8 from many workgroups
    "f32_d64_g4": B.Vote(2, 20, 8),                # the vector-ALU scan
    "f16_d128_g3": B.Vote(1, 64, 4),
    "bf16_one_page": B.Vote(4, 5, 7),
}


@pytest.mark.parametrize("name", list(CASES))
def test_paged_vote_layer_equals_contiguous(name):
    w, ps = CASES[name]
    v = VOTES[name]
    t = wl.generate(w, "cuda")
    p0 = B.Params.from_workload(w)
    out0, sel0, n0 = B.vote_layer(p0, v, t["q"], t["k"], t["v"], B.alloc_vote_workspace(p0, v))
    p, kp, vp, _ = _paged(w, t, ps, seed=15)
    ws = B.alloc_vote_workspace(p, v)
    lists1 = B.vote_topk(p, v, t["q"], kp, ws)
    lists0 = B.vote_topk(p0, v, t["q"], t["k"], B.alloc_vote_workspace(p0, v))
    out1, sel1, n1 = B.vote_layer(p, v, t["q"], kp, vp, ws)
    torch.cuda.synchronize()
    assert torch.equal(lists0, lists1)
    assert int(n0) == int(n1) and torch.equal(sel0[: int(n0)], sel1[: int(n1)])
    assert torch.equal(out0, out1)


def test_paged_vote_decode_token():
    n_layers, ps = 2, 64
    w = wl.CONFIGS[2].scaled(n_ctx=12_345, n_local=200, top_k=0, max_position=0, n_needles=0)
    v = B.Vote(4, 12, 16)
    dt = w.torch_dtype()
    Hq, Hkv, D, N = w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_ctx
    g = torch.Generator(device="cuda").manual_seed(240715000 + 92)
    ts = [wl.generate(w, "cuda") for _ in range(n_layers)]
    ts[1]["k"] = torch.randn(Hkv, N, D, generator=g, device="cuda").to(dt)
    ts[1]["v"] = torch.randn(Hkv, N, D, generator=g, device="cuda").to(dt)
    qs = [torch.randn(1, Hq, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    kn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    vn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    p0 = replace(B.Params.from_workload(w), n_query=1)
    k0 = [t["k"].clone() for t in ts]; v0 = [t["v"].clone() for t in ts]
    want = B.decode_token(p0, qs, kn, vn, k0, v0, B.alloc_vote_workspace(p0, v), vote=v)
    pools = [_paged(w, t, ps, seed=16) for t in ts]
    p = pools[0][0]
    kps = [x[1] for x in pools]; vps = [x[2] for x in pools]
    rows = pools[0][3]
    got = B.decode_token(p, qs, kn, vn, kps, vps, B.alloc_vote_workspace(p, v), vote=v)
    torch.cuda.synchronize()
    for l in range(n_layers):
        assert torch.equal(kps[l][:, rows], k0[l]) and torch.equal(vps[l][:, rows], v0[l])
        assert torch.equal(got[l], want[l]), l


CHUNKS = {
    # matrix-core selection and attention, several query tiles, key splits of the filter
    "bf16_mfma": (wl.CONFIGS[4].scaled(n_ctx=40_003, n_query=300, n_local=512, top_k=700, max_position=0), 128),
    "f16_mfma": (wl.CONFIGS[4].scaled(dtype="f16", n_ctx=20_000, n_query=65, n_local=300, top_k=256, max_position=0), 64),
    # the streaming scan once per query row and the flash-decoding kernel
    "f32_scan": (wl.CONFIGS[1].scaled(n_ctx=6_001, n_query=5, n_local=64, top_k=100, max_position=0), 256),
    # a zero query row: every score ties, the exact redo reads the pages
    "bf16_redo": (wl.CONFIGS[4].scaled(n_ctx=15_000, n_query=9, n_local=300, top_k=200, max_position=0), 1024),
}


@pytest.mark.parametrize("name", list(CHUNKS))
def test_paged_prefill_chunk_equals_contiguous(name):
    w, ps = CHUNKS[name]
    t = wl.generate(w, "cuda")
    if name == "bf16_redo":
        t["q"][4].zero_()
    p0 = B.Params.from_workload(w)
    out0, idx0 = B.prefill_chunk(p0, t["q"], t["k"], t["v"], B.alloc_workspace(p0), want_idx=True)
    p, kp, vp, _ = _paged(w, t, ps, seed=21)
    out1, idx1 = B.prefill_chunk(p, t["q"], kp, vp, B.alloc_workspace(p), want_idx=True)
    torch.cuda.synchronize()
    assert torch.equal(idx0, idx1)
    assert torch.equal(out0, out1)


@pytest.mark.parametrize("M,dtype,ps", [(6, "bf16", 128), (40, "bf16", 128), (300, "f16", 128), (3, "f32", 128),
                                        (600, "bf16", 64), (600, "f16", 256)])
def test_paged_vote_chunk_equals_contiguous(M, dtype, ps):
    """6 query rows take the streaming scan with two column blocks, 40 and 300 the tiled contraction (256-column
    workgroups) and the shared-set attention, 600 the 512-column workgroups (a key tile of 128 tokens then lies in up
    to three 64-token pages), fp32 the vector-ALU scan."""
    base = wl.CONFIGS[4] if dtype != "f32" else wl.CONFIGS[1]
    w = base.scaled(dtype=dtype, n_ctx=18_000, n_query=M, n_local=max(400, M + 37), top_k=0, max_position=0)
    v = B.Vote(4, 30, 16)
    t = wl.generate(w, "cuda")
    p0 = B.Params.from_workload(w)
    ws0 = B.alloc_vote_workspace(p0, v)
    lists0 = B.vote_topk(p0, v, t["q"], t["k"], ws0)
    out0, sel0, n0 = B.vote_layer(p0, v, t["q"], t["k"], t["v"], ws0)
    p, kp, vp, _ = _paged(w, t, ps, seed=22)
    ws = B.alloc_vote_workspace(p, v)
    lists1 = B.vote_topk(p, v, t["q"], kp, ws)
    out1, sel1, n1 = B.vote_layer(p, v, t["q"], kp, vp, ws)
    torch.cuda.synchronize()
    assert torch.equal(lists0, lists1)
    assert int(n0) == int(n1) and torch.equal(sel0[: int(n0)], sel1[: int(n1)])
    assert torch.equal(out0, out1)


@pytest.mark.parametrize("mode", ["topk", "vote"])
def test_paged_prefill_sequence_equals_contiguous(mode):
    """The chunk loop of one layer writes the rows of every chunk through the page table and reads them back
    through it: outputs and the pools' contents equal the contiguous run."""
    L, chunk, ps = 3_000, 256, 64
    w = wl.CONFIGS[2].scaled(n_ctx=L, n_local=300, top_k=0 if mode == "vote" else 128, max_position=0, n_needles=0)
    vote = B.Vote(4, 12, 16) if mode == "vote" else None
    dt = w.torch_dtype()
    Hq, Hkv, D = w.n_q_heads, w.n_kv_heads, w.head_dim
    g = torch.Generator(device="cuda").manual_seed(240715000 + 93)
    q = torch.randn(L, Hq, D, generator=g, device="cuda").to(dt)
    k_new = torch.randn(L, Hkv, D, generator=g, device="cuda").to(dt)
    v_new = torch.randn(L, Hkv, D, generator=g, device="cuda").to(dt)
    p0 = replace(B.Params.from_workload(w), n_query=1)
    want = B.prefill_sequence(p0, chunk, q, k_new, v_new, vote=vote)
    # empty pools behind a scattered page table
    n_pages = -(-L // ps); P = n_pages + 5
    table = torch.randperm(P, generator=torch.Generator().manual_seed(23))[:n_pages].to(torch.int32)
    kp = torch.zeros(Hkv, P * ps, D, dtype=dt, device="cuda"); vp = torch.zeros_like(kp)
    p = replace(p0, k_stride_head=P * ps * D, k_stride_tok=D, v_stride_head=P * ps * D, v_stride_tok=D,
                page_table=table.cuda(), page_size=ps)
    got = B.prefill_sequence(p, chunk, q, k_new, v_new, kp, vp, vote=vote)
    torch.cuda.synchronize()
    tok = torch.arange(L)
    rows = (table[tok // ps].long() * ps + tok % ps).cuda()
    assert torch.equal(kp[:, rows], k_new.transpose(0, 1)) and torch.equal(vp[:, rows], v_new.transpose(0, 1))
    assert torch.equal(got["out"], want["out"])


def test_paged_batch_folded_into_heads():
    """Two equal-length sequences folded into the head axis share one page table (the pools hold 2 * Hkv
    head slices): the top-k step and the vote step with votes pooled per sequence equal the contiguous calls."""
    batch = 2
    base = wl.CONFIGS[2]
    w = base.scaled(n_ctx=11_003, n_local=256, top_k=200, n_q_heads=base.n_q_heads * batch,
                    n_kv_heads=base.n_kv_heads * batch, max_position=0)
    t = wl.generate(w, "cuda")
    p0 = B.Params.from_workload(w)
    p, kp, vp, _ = _paged(w, t, 128, seed=17)
    out0, idx0 = B.decode_step(p0, t["q"], t["k"], t["v"], B.alloc_workspace(p0), want_idx=True)
    out1, idx1 = B.decode_step(p, t["q"], kp, vp, B.alloc_workspace(p), want_idx=True)
    torch.cuda.synchronize()
    assert torch.equal(idx0, idx1) and torch.equal(out0, out1)
    v = B.Vote(4, 12, 16, n_seq=batch)
    pv0, pv = replace(p0, top_k=0), replace(p, top_k=0)
    o0, s0, n0 = B.vote_layer(pv0, v, t["q"], t["k"], t["v"], B.alloc_vote_workspace(pv0, v))
    o1, s1, n1 = B.vote_layer(pv, v, t["q"], kp, vp, B.alloc_vote_workspace(pv, v))
    torch.cuda.synchronize()
    assert torch.equal(n0, n1)
    cap = B.vote_cap(pv0, v)
    for b in range(batch):                                       # the lists' tails past n_sel are not written
        assert torch.equal(s0[b * cap: b * cap + int(n0[b])], s1[b * cap: b * cap + int(n1[b])]), b
    assert torch.equal(o0, o1)


@pytest.mark.parametrize("seed", range(40))
def test_paged_random_shape_equals_contiguous(seed):
    """The seeded random shapes of test_gpu_random_shapes (small and large draws alternating), decode steps and
    chunks alike, over pages of a random size: indices and outputs equal the contiguous call's bit for bit."""
    from tests import test_gpu_random_shapes as R
    w = R._draw(seed)[0] if seed % 2 else R._draw_large(seed)[0]
    p0 = B.Params.from_workload(w)
    if B.validate(p0) != B.OK:
        pytest.skip("shape outside the library's domain")
    ps = [64, 128, 1024][seed % 3]
    t = wl.generate(w, "cuda")
    fn = B.decode_step if w.n_query == 1 else B.prefill_chunk
    out0, idx0 = fn(p0, t["q"], t["k"], t["v"], B.alloc_workspace(p0), want_idx=True)
    p, kp, vp, _ = _paged(w, t, ps, seed=100 + seed, spare=3)
    out1, idx1 = fn(p, t["q"], kp, vp, B.alloc_workspace(p), want_idx=True)
    torch.cuda.synchronize()
    assert torch.equal(idx0, idx1)
    assert torch.equal(out0, out1)


# ------------------------------------------------------ the filter route of long decode steps over pools
@pytest.mark.parametrize("name,ps", [("bf16_d128_long", 256), ("bf16_d128_long", 64)])
def test_paged_filter_route_equals_contiguous_and_oracle(name, ps):
    """The sampling launch, the filtering scan and (through a planted miss of the bound) the exact redo all
    find their rows through the page table; checked bit for bit against the contiguous call and, directly,
    against the oracle on the gathered cache."""
    from tests import parity as P
    w, _ = CASES[name]
    t = wl.generate(w, "cuda")
    p0 = replace(B.Params.from_workload(w), route=B.ROUTE_FILTER)
    ws0 = B.alloc_workspace(p0)
    out0, idx0 = B.decode_step(p0, t["q"], t["k"], t["v"], ws0)
    assert B.redo_list(p0, ws0) == (0, [])
    p, kp, vp, rows = _paged(w, t, ps, seed=21)
    p = replace(p, route=B.ROUTE_FILTER)
    ws = B.alloc_workspace(p)
    out1, idx1 = B.decode_step(p, t["q"], kp, vp, ws)
    torch.cuda.synchronize()
    assert B.redo_list(p, ws) == (0, [])
    assert torch.equal(idx0, idx1) and torch.equal(out0, out1)
    P.check_layer(w, t, out1, idx1)
    # keys that score high exactly where the sample looks: fewer than k pairs pass, every row is redone
    step = w.n_mid // 8192
    qbar = t["q"][0].float().reshape(w.n_kv_heads, w.group, w.head_dim).sum(dim=1)
    pos = torch.arange(w.n_sink, w.n_sink + w.n_mid, step, device="cuda")[:1500]
    needle = (qbar / qbar.norm(dim=1, keepdim=True) * 60.0).to(t["k"].dtype).unsqueeze(1)
    t["k"][:, pos, :] = needle
    kp[:, rows[pos], :] = needle
    out2, idx2 = B.decode_step(p, t["q"], kp, vp, ws)
    torch.cuda.synchronize()
    assert B.redo_list(p, ws)[0] == w.n_kv_heads
    P.check_layer(w, t, out2, idx2)


# ------------------------------------------------------------ paged calls against the oracle itself
# (the oracle reads the contiguous cache the pools were scattered from: t["k"], t["v"])
@pytest.mark.parametrize("agg", [B.AGG_SUM, B.AGG_MAX])
@pytest.mark.parametrize("name", ["bf16_d128_g4", "f32_d64_g4", "f16_d128_g3"])
def test_paged_decode_step_against_oracle(name, agg):
    from tests import parity as P
    w, ps = CASES[name]
    t = wl.generate(w, "cuda")
    p, kp, vp, _ = _paged(w, t, ps, seed=31)
    p = replace(p, agg=agg)
    out, idx = B.decode_step(p, t["q"], kp, vp, B.alloc_workspace(p), want_idx=True)
    torch.cuda.synchronize()
    P.check_layer(w, t, out, idx, agg=agg)


@pytest.mark.parametrize("name", list(CASES)[:2])
def test_paged_decode_step_on_a_warm_workspace(name):
    """reattn_params.ws_warm over a paged cache: the second step on the same workspace skips the clearing / table
    launch and returns what the cold step returned."""
    from tests import parity as P
    w, ps = CASES[name]
    t = wl.generate(w, "cuda")
    p, kp, vp, _ = _paged(w, t, ps, seed=34)
    ws = B.alloc_workspace(p)
    out0, idx0 = B.decode_step(p, t["q"], kp, vp, ws, want_idx=True)
    out1, idx1 = B.decode_step(replace(p, ws_warm=1), t["q"], kp, vp, ws, want_idx=True)
    torch.cuda.synchronize()
    assert torch.equal(idx0, idx1) and torch.equal(out0, out1)
    P.check_layer(w, t, out1, idx1)


@pytest.mark.parametrize("name", ["bf16_mfma", "f32_scan"])
def test_paged_prefill_chunk_against_oracle(name):
    from tests import parity as P
    w, ps = CHUNKS[name]
    w = w.scaled(n_needles=0, scale_q=True)
    t = wl.generate(w, "cuda")
    p, kp, vp, _ = _paged(w, t, ps, seed=32)
    out, idx = B.prefill_chunk(p, t["q"], kp, vp, B.alloc_workspace(p), want_idx=True)
    torch.cuda.synchronize()
    P.check_layer(w, t, out, idx)


@pytest.mark.parametrize("M", [1, 40])
def test_paged_vote_layer_against_oracle(M):
    import numpy as np
    from oracle import reattn_oracle as ro
    from tests import parity as P
    w = wl.CONFIGS[4].scaled(n_ctx=30_011, n_query=M, n_local=300, top_k=0, max_position=0)
    v = B.Vote(4, 40, 16)
    t = wl.generate(w, "cuda")
    p, kp, vp, _ = _paged(w, t, 128, seed=33)
    ws = B.alloc_vote_workspace(p, v)
    lists = B.vote_topk(p, v, t["q"], kp, ws)
    out, sel, n_sel = B.vote_layer(p, v, t["q"], kp, vp, ws)
    torch.cuda.synchronize()
    sh = P.oracle_shape(w)
    q, k, vv = P.host_inputs(t)
    res = ro.vote_forward(sh, q, k, vv, v.vote_k, v.n_centres, v.span, head_topk=lists.cpu().numpy())
    s_eff, _, n_mid, _ = sh.partition()
    R = M * w.n_q_heads
    P.check_index_sets(lists.cpu().numpy().reshape(R, 4), res["head_topk"].reshape(R, 4),
                       res["head_scores"].reshape(R, n_mid), res["head_kth"].reshape(R), s_eff, n_mid)
    n = int(n_sel.item())
    assert sel.cpu().numpy()[:n].tolist() == res["sel"].tolist()
    err = np.abs(out.cpu().numpy().astype(np.float64) - res["out"]).max()
    assert err <= P.OUT_TOL[w.dtype], err
