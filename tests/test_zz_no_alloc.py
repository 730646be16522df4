"""The decode step that allocates nothing (reattn_decode_step_static: its scratch is a fixed array inside the
library's device image) against reattn_decode_step on a caller's workspace: same kernels, so the index sets
are identical and the outputs agree bit for bit; two calls in a row share the array, the second on a smaller
problem, so anything the first left behind would show."""
from dataclasses import replace

import pytest
import torch

from paper_2407_15176_amd import binding as B
from paper_2407_15176_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _both(w):
    t = wl.generate(w, "cuda")
    p = B.Params.from_workload(w)
    assert 0 < B.workspace_bytes(p) <= B.static_scratch_bytes()
    ws = B.alloc_workspace(p)
    out_ref, idx_ref = B.decode_step(p, t["q"], t["k"], t["v"], ws)
    out = torch.full((1, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
    idx = torch.full((1, w.n_kv_heads, w.k_eff), -1, dtype=torch.int32, device="cuda")
    B.decode_step_static(p, t["q"], t["k"], t["v"], idx, out)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx_ref)
    assert torch.equal(out, out_ref)
    return t, out, idx


def test_static_decode_step_matches_workspace_call_twice_in_a_row():
    big = wl.CONFIGS[2].scaled(n_ctx=150_001, top_k=4096)        # several scan slices, the chip-wide top-k
    small = wl.CONFIGS[2].scaled(n_ctx=20_011, n_local=300, top_k=333, n_needles=8)   # one-workgroup top-k, ragged sizes
    _both(big)
    t, out, idx = _both(small)
    r = P.check_layer(small, t, out, idx)                        # and the second call against the oracle itself
    assert r["max_abs_err"] <= P.OUT_TOL[small.dtype]


def test_static_decode_step_fp32_after_bf16():
    _both(wl.CONFIGS[1])
    _both(wl.CONFIGS[1].scaled(n_ctx=3_001, n_local=64, top_k=17))


def test_static_decode_step_on_its_warm_array():
    """reattn_params.ws_warm through the entry point that allocates nothing: the second and third step of one shape
    (the context one token longer each time) skip the clearing / table launch and still equal the workspace call."""
    base = wl.CONFIGS[2].scaled(n_ctx=30_011, n_local=300, top_k=333, n_needles=8)
    for i in range(3):
        w = base.scaled(n_ctx=base.n_ctx + i)
        t = wl.generate(w, "cuda")
        p = B.Params.from_workload(w)
        out_ref, idx_ref = B.decode_step(p, t["q"], t["k"], t["v"], B.alloc_workspace(p))
        out = torch.full((1, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        idx = torch.full((1, w.n_kv_heads, w.k_eff), -1, dtype=torch.int32, device="cuda")
        B.decode_step_static(replace(p, ws_warm=int(i > 0)), t["q"], t["k"], t["v"], idx, out)
        torch.cuda.synchronize()
        assert torch.equal(idx, idx_ref) and torch.equal(out, out_ref), i
