"""GPU parity of the streaming prefill of one layer (chunk loop with cache append) against the
fp64 CPU oracle's loop, through the C ABI: reattn_cache_append, reattn_prefill_sequence.

Per chunk the rules of the single-chunk tests apply: index sets bit-exact outside the 1e-3 tie
band of the k-th score, outputs within 2e-2 (bf16) / 1e-4 (fp32) of the oracle on its own sets
or, where a GPU set differs inside the band, of the oracle evaluated on the GPU's sets."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import reattn_oracle as ro
from paper_2407_15176_amd import binding as B
from paper_2407_15176_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _sequence_inputs(w: wl.Workload, seed: int):
    """q [L,Hq,D], k_new, v_new [L,Hkv,D] in the storage dtype, with the recipe's channel scales."""
    g = torch.Generator(device="cuda").manual_seed(240715000 + seed)
    L, dt = w.n_ctx, w.torch_dtype()
    sig = wl.channel_sigma(w).to("cuda") if w.channel_scales else None        # [Hkv, D]
    q = torch.randn(L, w.n_q_heads, w.head_dim, generator=g, device="cuda")
    k = torch.randn(L, w.n_kv_heads, w.head_dim, generator=g, device="cuda")
    v = torch.randn(L, w.n_kv_heads, w.head_dim, generator=g, device="cuda")
    if sig is not None:
        k, v = k * sig[None], v * sig[None]
    return q.to(dt).contiguous(), k.to(dt).contiguous(), v.to(dt).contiguous()


CASES = {
    "f32_d64": (wl.CONFIGS[1].scaled(n_ctx=1_500, n_local=200, top_k=50, max_position=0, n_needles=0), 64),
    "bf16_d128": (wl.CONFIGS[2].scaled(n_ctx=3_011, n_local=256, top_k=100, n_needles=0), 128),
    "bf16_g3_ragged": (wl.CONFIGS[5].scaled(n_ctx=2_000, n_local=300, top_k=77, max_position=0, n_needles=0), 300),
    "bf16_short": (wl.CONFIGS[2].scaled(n_ctx=150, n_local=256, top_k=100, n_needles=0), 64),   # one chunk, no middle
}


@pytest.mark.parametrize("name,agg", [(n, B.AGG_SUM) for n in CASES] + [(n, B.AGG_MAX) for n in list(CASES)[:2]])
def test_sequence_topk_matches_oracle_loop(name, agg):
    w, chunk = CASES[name]
    q, k_new, v_new = _sequence_inputs(w, 1)
    p = replace(B.Params.from_workload(replace(w, n_query=1)), agg=agg)
    res = B.prefill_sequence(p, chunk, q, k_new, v_new)
    torch.cuda.synchronize()
    assert torch.equal(res["k_cache"], k_new.transpose(0, 1).contiguous())       # the append is a plain copy
    assert torch.equal(res["v_cache"], v_new.transpose(0, 1).contiguous())
    sh = P.oracle_shape(w, agg)
    qh, kh, vh = wl.to_numpy_store(q), wl.to_numpy_store(k_new), wl.to_numpy_store(v_new)
    want = ro.prefill_sequence(sh, qh, kh, vh, chunk)
    assert [(a, b) for a, b, _ in want["chunks"]] == res["chunks"]
    got = res["out"].cpu().numpy().astype(np.float64)
    tol = P.OUT_TOL[w.dtype]
    kc = np.ascontiguousarray(np.transpose(kh, (1, 0, 2))); vc = np.ascontiguousarray(np.transpose(vh, (1, 0, 2)))
    for c, (a, b, r) in enumerate(want["chunks"]):
        she = replace(sh, n_ctx=b)
        s_eff, l_eff, n_mid, k_eff = she.partition()
        g_idx = res["idx"][c].cpu().numpy()
        M = b - a
        differ = P.check_index_sets(g_idx.reshape(M * w.n_kv_heads, k_eff), r["idx"].reshape(M * w.n_kv_heads, k_eff),
                                    r["scores"].reshape(M * w.n_kv_heads, n_mid), r["kth"].reshape(M * w.n_kv_heads),
                                    s_eff, n_mid)
        ref = r["out"]
        if differ:      # swapped tie-band entries can weigh differently after the rotary encoding: judge on the GPU's set
            ref = ro.attend(she, np.ascontiguousarray(qh[a:b]), np.ascontiguousarray(kc[:, :b]),
                            np.ascontiguousarray(vc[:, :b]), g_idx)
        err = np.abs(got[a:b] - ref).max()
        assert err <= tol, (c, err)


@pytest.mark.parametrize("name", ["bf16_d128", "bf16_g3_ragged", "f32_d64", "bf16_short"])
def test_sequence_vote_matches_oracle_loop(name):
    w, chunk = CASES[name]
    q, k_new, v_new = _sequence_inputs(w, 2)
    v = B.Vote(4, 9, 16)
    p = B.Params.from_workload(replace(w, n_query=1, top_k=0, max_position=0))
    res = B.prefill_sequence(p, chunk, q, k_new, v_new, vote=v)
    torch.cuda.synchronize()
    sh = P.oracle_shape(replace(w, top_k=0))
    qh, kh, vh = wl.to_numpy_store(q), wl.to_numpy_store(k_new), wl.to_numpy_store(v_new)
    want = ro.prefill_sequence(sh, qh, kh, vh, chunk, vote=(v.vote_k, v.n_centres, v.span))
    got = res["out"].cpu().numpy().astype(np.float64)
    sel, n_sel = res["sel"].cpu().numpy(), res["n_sel"].cpu().numpy()
    tol = P.OUT_TOL[w.dtype]
    kc = np.ascontiguousarray(np.transpose(kh, (1, 0, 2))); vc = np.ascontiguousarray(np.transpose(vh, (1, 0, 2)))
    for c, (a, b, r) in enumerate(want["chunks"]):
        g_sel = sel[c, : n_sel[c]]
        if g_sel.tolist() != r["sel"].tolist():
            # a per-head list may differ inside its tie band; then the shared set may: evaluate the
            # oracle's attention on the GPU's set (valid: ascending, inside the middle, right length bound)
            she = replace(sh, n_ctx=b)
            s_eff, l_eff, n_mid, _ = she.partition()
            assert np.all(np.diff(g_sel) > 0) and g_sel[0] >= s_eff and g_sel[-1] < s_eff + n_mid
            assert g_sel.size <= v.n_centres * v.span
            M = b - a
            idx = np.broadcast_to(g_sel, (M, w.n_kv_heads, g_sel.size)).copy()
            ref = ro.attend(replace(she, top_k=int(g_sel.size)), np.ascontiguousarray(qh[a:b]),
                            np.ascontiguousarray(kc[:, :b]), np.ascontiguousarray(vc[:, :b]), idx)
        else:
            ref = r["out"]
        assert np.abs(got[a:b] - ref).max() <= tol, c


def test_cache_append_strided_cache():
    """A cache with room to grow (token capacity above L) takes the rows where the strides say."""
    w = wl.CONFIGS[2].scaled(n_ctx=1000, n_local=64, top_k=16)
    cap = 1536
    p = B.Params.from_workload(w)
    p = replace(p, k_stride_head=cap * w.head_dim, k_stride_tok=w.head_dim,
                v_stride_head=cap * w.head_dim, v_stride_tok=w.head_dim)
    kc = torch.zeros(w.n_kv_heads, cap, w.head_dim, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    k_new = torch.randn(300, w.n_kv_heads, w.head_dim, device="cuda").bfloat16()
    v_new = torch.randn(300, w.n_kv_heads, w.head_dim, device="cuda").bfloat16()
    B.cache_append(p, 700, k_new, v_new, kc, vc)
    torch.cuda.synchronize()
    assert torch.equal(kc[:, 700:1000], k_new.transpose(0, 1))
    assert torch.equal(vc[:, 700:1000], v_new.transpose(0, 1))
    assert not kc[:, :700].any() and not kc[:, 1000:].any()
    with pytest.raises(B.ReattnError):
        B.cache_append(p, 701, k_new, v_new, kc, vc)          # would run past n_ctx


# --------------------------------------------------------- decode tokens through several layers
@pytest.mark.parametrize("mode", ["topk", "vote"])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_decode_tokens_through_layers(mode, dtype):
    """Three layers, each with its own cache (room to grow), four decode tokens in a row: every layer's
    step is the oracle's decode step on that layer's cache as it stands after the append."""
    n_layers, n0, n_tok, cap = 3, 5_000, 4, 5_008
    base = wl.CONFIGS[2].scaled(dtype=dtype, n_ctx=n0, n_local=200, top_k=0 if mode == "vote" else 120, max_position=0)
    vote = B.Vote(4, 12, 16) if mode == "vote" else None
    dt = base.torch_dtype()
    g = torch.Generator(device="cuda").manual_seed(240715000 + 55)
    Hq, Hkv, D = base.n_q_heads, base.n_kv_heads, base.head_dim
    kcs = [torch.zeros(Hkv, cap, D, dtype=dt, device="cuda") for _ in range(n_layers)]
    vcs = [torch.zeros(Hkv, cap, D, dtype=dt, device="cuda") for _ in range(n_layers)]
    for l in range(n_layers):                                   # the prompt's cache
        kcs[l][:, :n0] = torch.randn(Hkv, n0, D, generator=g, device="cuda").to(dt)
        vcs[l][:, :n0] = torch.randn(Hkv, n0, D, generator=g, device="cuda").to(dt)
    for step in range(n_tok):
        n = n0 + step + 1
        w = base.scaled(n_ctx=n)
        p = replace(B.Params.from_workload(w), k_stride_head=cap * D, k_stride_tok=D, v_stride_head=cap * D, v_stride_tok=D)
        ws = B.alloc_vote_workspace(p, vote) if vote else B.alloc_workspace(p)
        qs = [torch.randn(1, Hq, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
        kn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
        vn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
        outs = B.decode_token(p, qs, kn, vn, kcs, vcs, ws, vote=vote)
        torch.cuda.synchronize()
        sh = P.oracle_shape(w)
        for l in range(n_layers):
            assert torch.equal(kcs[l][:, n - 1], kn[l][0]) and torch.equal(vcs[l][:, n - 1], vn[l][0])
            k = wl.to_numpy_store(kcs[l][:, :n].contiguous()); v = wl.to_numpy_store(vcs[l][:, :n].contiguous())
            q = wl.to_numpy_store(qs[l])
            if vote:
                ref = ro.vote_forward(sh, q, k, v, vote.vote_k, vote.n_centres, vote.span)["out"]
            else:
                ref = ro.forward(sh, q, k, v)["out"]
            err = np.abs(outs[l].cpu().numpy().astype(np.float64) - ref).max()
            # random keys leave a margin of ~1e-3 relative at the k-th score: a set flip would show as a large error
            assert err <= P.OUT_TOL[dtype], (step, l, err)


@pytest.mark.parametrize("n_ctx,route", [(9_001, 0), (80_001, 0), (80_001, 1)])
def test_decode_token_layers_equal_separate_steps(n_ctx, route):
    """Layers after the first skip the clearing launch (the previous layer's top-k leaves the histograms
    zeroed) and copy the token's rows inside the scan: every layer must equal cache_append + decode_step
    on its own workspace, bit for bit.  80,001 tokens take the chip-wide select / refine / emit kernels,
    9,001 the one-workgroup-per-row kernel; route 1 asks for the filter route (sampled bound, filtering scan,
    pick), whose sampling launch skips the rotary table after the first layer."""
    n_layers = 4
    w = wl.CONFIGS[2].scaled(n_ctx=n_ctx, n_local=300, top_k=500, max_position=0, n_needles=0)
    dt = w.torch_dtype()
    Hq, Hkv, D, N = w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_ctx
    g = torch.Generator(device="cuda").manual_seed(240715000 + 56)
    kcs = [torch.randn(Hkv, N, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    vcs = [torch.randn(Hkv, N, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    qs = [torch.randn(1, Hq, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    kn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    vn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    p = replace(B.Params.from_workload(w), n_query=1, route=route)
    k2 = [x.clone() for x in kcs]; v2 = [x.clone() for x in vcs]
    ws = B.alloc_workspace(p)
    assert (B.redo_list(p, ws) is not None) == (route == 1)
    for rep in range(2):                                        # the second call starts on the workspace the first left
        outs = B.decode_token(p, qs, kn, vn, kcs, vcs, ws)
        torch.cuda.synchronize()
        for l in range(n_layers):
            B.cache_append(p, N - 1, kn[l], vn[l], k2[l], v2[l])
            want, _ = B.decode_step(p, qs[l], k2[l], v2[l], B.alloc_workspace(p), want_idx=True)
            torch.cuda.synchronize()
            assert torch.equal(kcs[l], k2[l]) and torch.equal(vcs[l], v2[l]), (rep, l)
            assert torch.equal(outs[l], want), (rep, l)


@pytest.mark.parametrize("seed", range(30))
def test_decode_token_random_shapes_equal_separate_steps(seed):
    """Seeded random shapes (small and large draws alternating), three layers, both selections: every layer of
    decode_token equals cache_append followed by the layer's own step on a fresh workspace, bit for bit."""
    from tests import test_gpu_random_shapes as R
    w, vote = R._draw(seed) if seed % 2 else (R._draw_large(seed)[0], B.Vote(4, 20, 8))
    use_vote = seed % 4 >= 2
    w = w.scaled(n_query=1, top_k=0 if use_vote else w.top_k, n_needles=0)
    p = replace(B.Params.from_workload(w), n_query=1)
    if B.validate(p) != B.OK or (use_vote and B.vote_workspace_bytes(p, vote) == 0):
        pytest.skip("shape outside the library's domain")
    n_layers = 3
    dt = w.torch_dtype()
    Hq, Hkv, D, N = w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_ctx
    g = torch.Generator(device="cuda").manual_seed(240715000 + 300 + seed)
    kcs = [torch.randn(Hkv, N, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    vcs = [torch.randn(Hkv, N, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    qs = [torch.randn(1, Hq, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    kn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    vn = [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)]
    k2 = [x.clone() for x in kcs]; v2 = [x.clone() for x in vcs]
    alloc = (lambda: B.alloc_vote_workspace(p, vote)) if use_vote else (lambda: B.alloc_workspace(p))
    outs = B.decode_token(p, qs, kn, vn, kcs, vcs, alloc(), vote=vote if use_vote else None)
    torch.cuda.synchronize()
    for l in range(n_layers):
        B.cache_append(p, N - 1, kn[l], vn[l], k2[l], v2[l])
        if use_vote:
            want = B.vote_layer(p, vote, qs[l], k2[l], v2[l], alloc())[0]
        else:
            want = B.decode_step(p, qs[l], k2[l], v2[l], alloc(), want_idx=False)[0]
        torch.cuda.synchronize()
        assert torch.equal(kcs[l], k2[l]) and torch.equal(vcs[l], v2[l]), l
        assert torch.equal(outs[l], want), l
