"""A decode token through several layers, captured once into a HIP graph and replayed.

The library allocates nothing, keeps no state and only enqueues kernels on the caller's stream, so a
caller may capture its calls (the way a serving loop hides the launch cost of the ~8 small kernels of a
layer).  The replays are checked against the same call made eagerly: several replays, with new inputs
copied into the captured buffers and eager work and synchronisations between them."""
from dataclasses import replace

import pytest
import torch

from paper_2407_15176_amd import binding as B
from paper_2407_15176_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode", ["topk", "vote"])
def test_decode_token_replays_from_a_graph(mode):
    n_layers, n0, cap = 4, 6_001, 6_016
    base = wl.CONFIGS[2].scaled(n_ctx=n0 + 1, n_local=200, top_k=0 if mode == "vote" else 150, max_position=0)
    vote = B.Vote(4, 12, 16) if mode == "vote" else None
    dt = base.torch_dtype()
    g = torch.Generator(device="cuda").manual_seed(240715000 + 77)
    Hq, Hkv, D = base.n_q_heads, base.n_kv_heads, base.head_dim
    p = replace(B.Params.from_workload(base), k_stride_head=cap * D, k_stride_tok=D, v_stride_head=cap * D,
                v_stride_tok=D)

    def caches():
        gg = torch.Generator(device="cuda").manual_seed(240715000 + 78)
        ks = [torch.zeros(Hkv, cap, D, dtype=dt, device="cuda") for _ in range(n_layers)]
        vs = [torch.zeros(Hkv, cap, D, dtype=dt, device="cuda") for _ in range(n_layers)]
        for l in range(n_layers):
            ks[l][:, :n0] = torch.randn(Hkv, n0, D, generator=gg, device="cuda").to(dt)
            vs[l][:, :n0] = torch.randn(Hkv, n0, D, generator=gg, device="cuda").to(dt)
        return ks, vs

    def token():
        return ([torch.randn(1, Hq, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)],
                [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)],
                [torch.randn(1, Hkv, D, generator=g, device="cuda").to(dt) for _ in range(n_layers)])

    def workspace():
        return B.alloc_vote_workspace(p, vote) if vote else B.alloc_workspace(p)

    # captured buffers
    kcs, vcs = caches()
    qs, kn, vn = token()
    ws = workspace()
    outs = [torch.zeros(1, Hq, D, dtype=torch.float32, device="cuda") for _ in range(n_layers)]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.decode_token(p, qs, kn, vn, kcs, vcs, ws, outs=outs, vote=vote)

    # the eager twin works on its own caches and workspace
    e_kcs, e_vcs = caches()
    e_ws = workspace()
    for replay in range(4):
        nq, nk, nv = token()                                   # a new token for the same position
        for l in range(n_layers):
            qs[l].copy_(nq[l]); kn[l].copy_(nk[l]); vn[l].copy_(nv[l])
        for o in outs:
            o.fill_(float("nan"))                              # eager work on the captured outputs between replays
        graph.replay()
        want = B.decode_token(p, nq, nk, nv, e_kcs, e_vcs, e_ws, vote=vote)
        torch.cuda.synchronize()
        for l in range(n_layers):
            assert torch.equal(outs[l], want[l]), (replay, l)
            assert torch.equal(kcs[l], e_kcs[l]) and torch.equal(vcs[l], e_vcs[l]), (replay, l)
