"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2407_15176_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "reattn.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(reattn_[a-z_]+)\s*\(", text)))


def good(**kw):
    base = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=B.BF16, n_ctx=131072, n_query=1,
                n_sink=4, n_local=4096, top_k=4096, rope_theta=500000.0, max_position=131072)
    base.update(kw)
    return B.Params(**base)


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings():
    assert B.version() >= 100
    seen = set()
    for s in range(0, -10, -1):
        msg = B.status_string(s)
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 10
    assert B.status_string(-99) == "unknown status"


def test_scope_matches_eq1_on_the_five_configs():
    from paper_2407_15176_amd import workloads as wl
    want = {1: (15868, 256, 772), 2: (126972, 4096, 8196), 3: (1044476, 8192, 12292),
            4: (258044, 4096, 8196), 5: (4190204, 8192, 12292)}
    for cfg, w in wl.CONFIGS.items():
        p = B.Params.from_workload(w)
        assert B.validate(p) == B.OK
        s, l, mid, k, S = B.scope(p)
        assert (mid, k, S) == want[cfg]
        assert (s, l) == (4, w.n_local)
        assert (mid, k, S) == (w.n_mid, w.k_eff, w.scope)
        assert B.workspace_bytes(p) > 0


def test_scope_clamping():
    assert B.scope(good(n_ctx=100, n_local=16, top_k=10, max_position=0)) == (4, 16, 80, 10, 30)
    assert B.scope(good(n_ctx=100, n_local=16, top_k=500, max_position=0)) == (4, 16, 80, 80, 100)
    assert B.scope(good(n_ctx=10, n_local=16, top_k=10, max_position=0)) == (4, 6, 0, 0, 10)


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=30), B.ERR_SHAPE),
    (dict(n_kv_heads=0), B.ERR_SHAPE),
    (dict(head_dim=96), B.ERR_SHAPE),
    (dict(n_q_heads=34, n_kv_heads=2), B.ERR_SHAPE),          # G = 17
    (dict(dtype=7), B.ERR_DTYPE),
    (dict(agg=3), B.ERR_DTYPE),
    (dict(n_ctx=0), B.ERR_RANGE),
    (dict(n_ctx=2 ** 31), B.ERR_RANGE),
    (dict(n_query=0), B.ERR_RANGE),
    (dict(n_query=5000), B.ERR_RANGE),                        # M > n_local
    (dict(n_sink=-1), B.ERR_RANGE),
    (dict(n_local=0), B.ERR_RANGE),
    (dict(top_k=-1), B.ERR_RANGE),
    (dict(route=3), B.ERR_RANGE),
    (dict(rope_theta=1.0), B.ERR_RANGE),
    (dict(rope_theta=float("nan")), B.ERR_RANGE),
    (dict(softmax_scale=-0.5), B.ERR_RANGE),
    (dict(max_position=8192), B.ERR_WINDOW),                  # S = 8196
    (dict(k_stride_tok=64, k_stride_head=64 * 131072), B.ERR_SHAPE),   # row shorter than D
    (dict(k_stride_tok=132, k_stride_head=132 * 131072), B.ERR_ALIGN), # 264-byte rows
    (dict(v_stride_tok=128, v_stride_head=0), B.ERR_SHAPE),
])
def test_validate_rejects(kw, status):
    p = good(**kw)
    assert B.validate(p) == status
    assert B.workspace_bytes(p) == 0


def test_paged_cache_parameters_are_checked_on_the_host():
    """Paged caches: pools [Hkv][P * page_size][D] behind a device page table (never read on the host)."""
    L = B.lib()

    def status(page_size=256, table=0x1000, **kw):
        base = dict(n_ctx=10_000, n_local=256, top_k=64, max_position=0, k_stride_tok=128,
                    k_stride_head=128 * 16_384, v_stride_tok=128, v_stride_head=128 * 16_384)
        base.update(kw)
        cp = good(**base).c()
        cp.page_table, cp.page_size = table, page_size
        return L.reattn_validate(C.byref(cp)), L.reattn_workspace_bytes(C.byref(cp)), cp

    rc, ws, cp = status()
    assert rc == B.OK and ws > 0
    assert status(page_size=100)[0] == B.ERR_RANGE                 # not a power of two
    assert status(page_size=32)[0] == B.ERR_RANGE                  # below the smallest page
    assert status(table=None)[0] == B.ERR_NULL                     # a page size without a table
    assert status(k_stride_tok=0, k_stride_head=0)[0] == B.ERR_SHAPE      # the pool's extent must be given
    assert status(n_query=8)[0] == B.OK                            # chunks read pages too
    assert status(k_stride_head=128 * 2 ** 31, v_stride_head=128 * 2 ** 31)[0] == B.ERR_RANGE   # pool rows are int32
    cv = B.Vote(4, 20, 8).c()
    assert L.reattn_vote_workspace_bytes(C.byref(cp), C.byref(cv)) > 0     # the vote selection reads pages too
    cp8 = status(n_query=8)[2]
    assert L.reattn_vote_workspace_bytes(C.byref(cp8), C.byref(cv)) > 0


def test_empty_middle_takes_any_query_count():
    # N = 3 < sink: no middle, the kept entries are simply the 3 tokens in order: plain attention
    assert B.validate(good(n_ctx=3, n_local=16, top_k=10, max_position=0)) == B.OK
    assert B.validate(good(n_ctx=3, n_sink=2, n_local=16, top_k=10, max_position=0)) == B.OK
    # the first prefill chunk: sink + local tokens at once, all of them queries
    assert B.validate(good(n_ctx=4 + 256, n_sink=4, n_local=256, n_query=4 + 256, top_k=10)) == B.OK
    # with a middle a chunk must lie inside the local window
    assert B.validate(good(n_ctx=4 + 256 + 1, n_sink=4, n_local=256, n_query=257, top_k=10)) == B.ERR_RANGE
    assert B.validate(good(n_ctx=4 + 256 + 1, n_sink=4, n_local=256, n_query=256, top_k=10)) == B.OK


def test_sequence_loop_is_planned_on_the_host():
    p = good(n_ctx=10_000, n_sink=4, n_local=256, top_k=64, max_position=0)
    cp = p.c()
    L = B.lib()
    assert L.reattn_prefill_sequence_chunks(C.byref(cp), 128) == 1 + -(-(10_000 - 260) // 128)
    assert L.reattn_prefill_sequence_chunks(C.byref(cp), 0) == 0
    # the chunks as the appendix's prefilling loop cuts them: sink + local tokens first, then 128 at a time
    chunks = B.sequence_chunks(p, 128)
    assert chunks[0] == (0, 260) and chunks[1] == (260, 388) and chunks[-1] == (9_988, 10_000)
    assert all(a[1] == b[0] for a, b in zip(chunks, chunks[1:]))
    s, e = C.c_int64(), C.c_int64()
    assert L.reattn_prefill_sequence_chunk_bounds(C.byref(cp), 128, len(chunks), C.byref(s), C.byref(e)) == B.ERR_RANGE
    assert L.reattn_prefill_sequence_chunk_bounds(C.byref(cp), 128, -1, None, None) == B.ERR_RANGE
    assert L.reattn_prefill_sequence_chunk_bounds(C.byref(cp), 0, 0, None, None) == B.ERR_RANGE
    assert B.sequence_chunks(good(n_ctx=100, n_sink=4, n_local=256, max_position=0), 64) == [(0, 100)]
    assert L.reattn_prefill_sequence_workspace_bytes(C.byref(cp), None, 128) > 0
    assert L.reattn_prefill_sequence_workspace_bytes(C.byref(cp), None, 257) == 0     # chunk above the local window
    cv = B.Vote(4, 20, 8).c()
    assert L.reattn_prefill_sequence_workspace_bytes(C.byref(cp), C.byref(cv), 128) > 0
    fake = C.c_void_p(0x1000)
    assert L.reattn_prefill_sequence(C.byref(cp), None, 128, fake, fake, None, fake, fake, fake, None, None, None,
                                     fake, 1 << 40, None) == B.ERR_NULL
    assert L.reattn_prefill_sequence(C.byref(cp), None, 257, fake, fake, fake, fake, fake, fake, None, None, None,
                                     fake, 1 << 40, None) == B.ERR_RANGE
    assert L.reattn_prefill_sequence(C.byref(cp), None, 128, fake, fake, fake, fake, fake, fake, None, None, None,
                                     fake, 16, None) == B.ERR_WORKSPACE
    ptrs = (C.c_void_p * 2)(0x1000, 0x2000)
    holes = (C.c_void_p * 2)(0x1000, None)
    need1 = B.workspace_bytes(p)
    assert L.reattn_decode_token(C.byref(cp), None, 2, ptrs, ptrs, ptrs, ptrs, ptrs, holes, fake, need1, None) == B.ERR_NULL
    assert L.reattn_decode_token(C.byref(cp), None, 0, ptrs, ptrs, ptrs, ptrs, ptrs, ptrs, fake, need1, None) == B.ERR_RANGE
    assert L.reattn_decode_token(C.byref(cp), None, 2, ptrs, ptrs, ptrs, ptrs, ptrs, ptrs, fake, 16, None) == B.ERR_WORKSPACE
    assert L.reattn_cache_append(C.byref(cp), 9_990, 11, fake, fake, fake, fake, None) == B.ERR_RANGE
    assert L.reattn_cache_append(C.byref(cp), 9_990, 10, fake, None, fake, fake, None) == B.ERR_NULL


def test_null_and_workspace_errors_before_any_launch():
    lib = B.lib()
    p = good(n_ctx=8192, n_local=256, top_k=64)
    cp = p.c()
    fake = C.c_void_p(0x1000)       # never dereferenced: the checks below fire first
    need = B.workspace_bytes(p)
    assert lib.reattn_validate(None) == B.ERR_NULL
    assert lib.reattn_score(C.byref(cp), None, fake, fake, None, 0, None) == B.ERR_NULL
    assert lib.reattn_topk(C.byref(cp), None, fake, fake, need, None) == B.ERR_NULL
    assert lib.reattn_topk(C.byref(cp), fake, fake, None, need, None) == B.ERR_WORKSPACE
    assert lib.reattn_topk(C.byref(cp), fake, fake, fake, need - 1, None) == B.ERR_WORKSPACE
    assert lib.reattn_topk(C.byref(cp), fake, fake, C.c_void_p(0x1010), need, None) == B.ERR_ALIGN
    assert lib.reattn_gather_rope(C.byref(cp), fake, fake, None, fake, fake, None) == B.ERR_NULL
    assert lib.reattn_attend(C.byref(cp), fake, None, fake, fake, fake, need, None) == B.ERR_NULL
    assert lib.reattn_decode_step(C.byref(cp), fake, fake, None, None, fake, fake, need, None) == B.ERR_NULL
    assert lib.reattn_decode_step(C.byref(cp), fake, fake, fake, None, fake, fake, 16, None) == B.ERR_WORKSPACE
    assert lib.reattn_decode_step(C.byref(cp), C.c_void_p(0x1004), fake, fake, None, fake, fake, need,
                                  None) == B.ERR_ALIGN
    pm = good(n_ctx=8192, n_local=256, top_k=64, n_query=4).c()
    assert lib.reattn_decode_step(C.byref(pm), fake, fake, fake, None, fake, fake, 1 << 40, None) == B.ERR_RANGE
    assert lib.reattn_prefill_chunk(C.byref(pm), fake, fake, fake, None, None, fake, 1 << 40, None) == B.ERR_NULL


def test_workspace_is_modest_for_decode():
    from paper_2407_15176_amd import workloads as wl
    for cfg in (1, 2, 3, 5):
        w = wl.CONFIGS[cfg]
        need = B.workspace_bytes(B.Params.from_workload(w))
        # scores + candidate list + bitmap: about 8.2 bytes per middle token per KV head
        assert need < 10 * w.n_mid * w.n_kv_heads + (8 << 20)


def test_vote_parameters_are_checked_on_the_host():
    p = good(top_k=0)
    need = B.vote_workspace_bytes(p, B.Vote(4, 127, 32))
    assert 0 < need < (4 << 20)            # a decode step: partial lists, rotary table, split-S partials
    for bad in (B.Vote(0, 127, 32), B.Vote(9, 127, 32), B.Vote(4, 0, 32), B.Vote(4, 1025, 32), B.Vote(4, 127, 0)):
        assert B.vote_workspace_bytes(p, bad) == 0
    # the paper's own setting fills an 8K window exactly: 32 + 4096 + 127 * 32 = 8192
    p8k = good(n_sink=32, top_k=0, max_position=8192)
    assert B.vote_workspace_bytes(p8k, B.Vote(4, 127, 32)) > 0
    assert B.vote_workspace_bytes(p8k, B.Vote(4, 128, 32)) == 0          # one more span overflows the window
    # every shape the library takes has a vote path: 16-bit storage with D = 64, fp32 with D = 128, groups of up to 16
    assert B.vote_workspace_bytes(good(head_dim=64, top_k=0), B.Vote()) > 0
    assert B.vote_workspace_bytes(good(dtype=B.F32, top_k=0), B.Vote()) > 0
    assert B.vote_workspace_bytes(good(n_q_heads=72, top_k=0), B.Vote()) > 0          # G = 9
    assert B.vote_workspace_bytes(good(n_q_heads=128, top_k=0), B.Vote()) > 0         # G = 16
    assert B.vote_workspace_bytes(good(n_q_heads=136, top_k=0), B.Vote()) == 0        # G = 17: no shape of the library's
    # NULL pointers are reported before anything is launched
    L = B.lib()
    cp, cv = p.c(), B.Vote().c()
    assert L.reattn_vote_layer(C.byref(cp), C.byref(cv), None, None, None, None, None, None, None, 0, None) == B.ERR_NULL
    assert L.reattn_vote_merge(C.byref(cp), C.byref(cv), None, None, None, None, 0, None) == B.ERR_NULL


def test_static_entry_point_rejects_steps_past_its_scratch_on_the_host():
    """The no-allocation decode step refuses, before any HIP call, a step whose workspace exceeds its fixed array."""
    lib = B.lib()
    assert B.static_scratch_bytes() == 32 << 20
    big = good(n_ctx=1 << 20, max_position=0)
    assert B.workspace_bytes(big) > B.static_scratch_bytes()
    cp = big.c()
    one = C.c_void_p(256)       # never dereferenced: the size check comes first
    assert lib.reattn_decode_step_static(C.byref(cp), one, one, one, None, one, None) == B.ERR_STATIC_LIMIT
    cp = good(n_query=2).c()
    assert lib.reattn_decode_step_static(C.byref(cp), one, one, one, None, one, None) == B.ERR_RANGE
    assert "scratch" in B.status_string(B.ERR_STATIC_LIMIT)


def test_both_aggregations_validate():
    """REATTN_AGG_SUM and REATTN_AGG_MAX are the reattn_agg values; workspace sizes do not depend on the choice
    except where max aggregation leaves the matrix-core chunk path (it then needs no split-query buffers)."""
    from dataclasses import replace
    from paper_2407_15176_amd import workloads as wl
    p = B.Params.from_workload(wl.CONFIGS[2])
    for agg in (B.AGG_SUM, B.AGG_MAX):
        q = replace(p, agg=agg)
        assert B.validate(q) == B.OK
        assert B.workspace_bytes(q) > 0
    assert B.workspace_bytes(replace(p, agg=B.AGG_MAX)) == B.workspace_bytes(p)      # a decode step: the same plan but the route


def test_struct_sizes_match_the_binding():
    """The ctypes structs are declared by hand: the library reports its own sizeof for both."""
    import ctypes as C
    from paper_2407_15176_amd import binding as B
    L = B.lib()                                              # raises on a mismatch
    assert L.reattn_params_bytes() == C.sizeof(B.CParams)
    assert L.reattn_vote_bytes() == C.sizeof(B.CVote)
