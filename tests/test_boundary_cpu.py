"""Host-side checks of the C-ABI library that need no GPU: symbols, validation, workspace queries."""
import ctypes as C
import os
import re

import pytest

from paper_2511_12201_amd import binding as ob


@pytest.fixture(scope="module")
def lib():
    return ob.load_library()


def _desc(**kw):
    d = ob.LayerDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim, d.n_tokens = 1, 4, 2, 64, 300
    d.vis_begin, d.vis_end, d.sink_index, d.causal, d.dtype = 0, 256, 0, 1, ob.OMNI_BF16
    d.softmax_scale = 0.125
    d.q_stride = (C.c_int64 * 3)(4 * 300 * 64, 300 * 64, 64)
    d.kv_stride = (C.c_int64 * 3)(2 * 300 * 64, 300 * 64, 64)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_library_exports_every_declared_symbol(lib, repo_root):
    header = open(os.path.join(repo_root, "include/omnisparse.h")).read()
    declared = set(re.findall(r"\b(omni_[a-z_]+)\s*\(", header))
    declared -= {"omni_workspace_bytes"} - set(re.findall(r"size_t\s+(omni_workspace_bytes)\(", header))
    assert {"omni_score_queries", "omni_select_queries", "omni_kv_budget", "omni_select_kv", "omni_sparse_attn_fwd",
            "omni_sparse_attn_bwd", "omni_slim_decode"} <= declared
    for name in declared:
        assert hasattr(lib, name), name
    assert set(ob.EXPORTED) == declared
    assert lib.omni_version() >= 100


def test_workspace_queries(lib):
    d = _desc()
    for call in (ob.CALL_SCORE_QUERIES, ob.CALL_SELECT_QUERIES, ob.CALL_SELECT_KV, ob.CALL_DENSE_ATTN_FWD):
        assert ob.workspace_bytes(call, d) > 0
    small = ob.workspace_bytes(ob.CALL_SPARSE_ATTN_FWD, d, 64)
    big = ob.workspace_bytes(ob.CALL_SPARSE_ATTN_FWD, d, 300)
    assert 0 < small < big
    # packed K and V for every query head, padded to whole 64-key tiles, plus the index list
    assert big >= 4 * 320 * 64 * 2 * 2 + 4 * 320 * 4
    assert ob.workspace_bytes(ob.CALL_KV_BUDGET, d, 256) > 0
    with pytest.raises(ob.OmniError):
        ob.workspace_bytes(ob.CALL_KV_BUDGET, d, 0)
    with pytest.raises(ob.OmniError):
        ob.workspace_bytes(ob.CALL_SCORE_QUERIES, _desc(head_dim=96))
    with pytest.raises(ob.OmniError):
        ob.workspace_bytes(99, d)
    dd = ob.DecodeDesc()
    dd.batch, dd.n_q_heads, dd.n_kv_heads, dd.head_dim, dd.cache_capacity = 2, 4, 2, 128, 1000
    dd.vis_begin, dd.vis_end, dd.dtype, dd.softmax_scale, dd.tau = 0, 900, ob.OMNI_BF16, 0.088, 0.08
    dd.kv_stride = (C.c_int64 * 3)(2 * 1000 * 128, 1000 * 128, 128)
    assert ob.workspace_bytes(ob.CALL_SLIM_DECODE, dd) > 0


FAKE = C.c_void_p(0x10000)       # non-null, 256-byte aligned; never dereferenced: validation fails first


@pytest.mark.parametrize("kw,code,needle", [
    (dict(head_dim=96), -2, "head_dim"),
    (dict(n_kv_heads=3), -1, "multiple"),
    (dict(vis_begin=10, vis_end=10), -1, "vis_begin"),
    (dict(vis_end=301), -1, "vis_begin"),
    (dict(sink_index=300), -1, "sink_index"),
    (dict(dtype=7), -2, "dtype"),
    (dict(softmax_scale=0.0), -1, "softmax_scale"),
    (dict(causal=2), -1, "causal"),
    (dict(n_tokens=0), -1, "positive"),
])
def test_invalid_descriptors_are_rejected_before_any_launch(lib, kw, code, needle):
    d = _desc(**kw)
    rc = lib.omni_score_queries(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None)
    assert rc == code
    assert needle in ob.last_error()


def test_argument_errors(lib):
    d = _desc()
    assert lib.omni_score_queries(C.byref(d), None, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert "null" in ob.last_error()
    assert lib.omni_score_queries(None, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    # workspace too small / misaligned / null
    assert lib.omni_score_queries(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, 8, None) == -3
    assert "too small" in ob.last_error()
    assert lib.omni_score_queries(C.byref(d), FAKE, FAKE, FAKE, FAKE, C.c_void_p(0x10010), 1 << 30, None) == -3
    assert lib.omni_score_queries(C.byref(d), FAKE, FAKE, FAKE, FAKE, None, 1 << 30, None) == -1
    # misaligned tensor pointer
    assert lib.omni_score_queries(C.byref(d), C.c_void_p(0x10004), FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert "aligned" in ob.last_error()
    # stride not a multiple of 8 elements
    bad = _desc()
    bad.q_stride = (C.c_int64 * 3)(4 * 300 * 64, 300 * 64, 68)
    assert lib.omni_score_queries(C.byref(bad), FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    # per-call parameter checks
    assert lib.omni_select_queries(C.byref(d), FAKE, 2, 0.1, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.omni_select_queries(C.byref(d), FAKE, 1, 1.5, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.omni_kv_budget(C.byref(d), FAKE, FAKE, 1.5, 256, 0, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 1 << 30, None) == -1
    assert lib.omni_kv_budget(C.byref(d), FAKE, FAKE, 0.9, 0, 0, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 1 << 30, None) == -1
    assert lib.omni_kv_budget(C.byref(d), FAKE, FAKE, 0.9, 256, 3, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, 1 << 30, None) == -1
    assert lib.omni_select_kv(C.byref(d), FAKE, FAKE, 0, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.omni_sparse_attn_fwd(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.omni_sparse_attn_fwd(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 300, FAKE, FAKE, FAKE, 16, None) == -3
    # the fused selection call, the per-head variants and the compacted decode store validate like their base calls
    ps = lambda **kw: lib.omni_prefill_select(
        C.byref(d), FAKE, FAKE, kw.get("q_mode", 0), kw.get("q_param", 0.08), kw.get("p", 0.95), kw.get("pb", 256),
        kw.get("mode", 0), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, kw.get("kv", FAKE), kw.get("cap", 300),
        FAKE, kw.get("ws", 1 << 30), None)
    assert ps(mode=3) == -1 and "budget_mode" in ob.last_error()
    assert ps(q_mode=2) == -1 and ps(q_mode=1, q_param=0.0) == -1 and ps(p=0.0) == -1 and ps(pb=0) == -1 and ps(cap=0) == -1
    assert ps(kv=None) == -1 and "null" in ob.last_error()
    assert ps(ws=64) == -3
    assert ob.workspace_bytes(ob.CALL_PREFILL_SELECT, d, 256) >= ob.workspace_bytes(ob.CALL_KV_BUDGET, d, 256)
    with pytest.raises(ob.OmniError):
        ob.workspace_bytes(ob.CALL_PREFILL_SELECT, d, 0)
    assert lib.omni_select_kv_per_head(C.byref(d), FAKE, FAKE, 0, FAKE, FAKE, 1 << 30, None) == -1
    assert lib.omni_sparse_attn_fwd_per_head(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 300, FAKE, FAKE, FAKE,
                                             1 << 30, None) == -1
    assert lib.omni_group_subset_per_head(C.byref(d), FAKE, FAKE, 300, FAKE, FAKE, FAKE, 0, FAKE, 1 << 30, None) == -1
    dd = ob.DecodeDesc()
    dd.batch, dd.n_q_heads, dd.n_kv_heads, dd.head_dim, dd.cache_capacity = 2, 4, 2, 128, 1000
    dd.vis_begin, dd.vis_end, dd.dtype, dd.softmax_scale, dd.tau = 0, 900, ob.OMNI_BF16, 0.088, 0.08
    dd.kv_stride = (C.c_int64 * 3)(2 * 1000 * 128, 1000 * 128, 128)
    assert lib.omni_compact_cache(C.byref(dd), FAKE, FAKE, FAKE, FAKE, 0, FAKE, FAKE, None) == -1
    assert lib.omni_compact_cache(C.byref(dd), FAKE, FAKE, FAKE, FAKE, 64, None, FAKE, None) == -1
    assert lib.omni_slim_decode_compact(C.byref(dd), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, FAKE,
                                        FAKE, FAKE, 16, None) == -3
    # block lists walked in place: bf16, block a multiple of the key tile, bounded list length
    ba = lambda dd_=d, **kw: lib.omni_block_attn_fwd(
        C.byref(dd_), FAKE, FAKE, FAKE, FAKE, FAKE, kw.get("blk", FAKE), FAKE, kw.get("cap", 4), kw.get("block", 64), FAKE,
        FAKE, FAKE, kw.get("ws", 1 << 30), None)
    assert ba(block=100) == -2 and "multiple of 64" in ob.last_error()
    assert ba(cap=0) == -1 and ba(blk=None) == -1 and ba(ws=16) == -3
    assert ba(cap=4096, block=64) == -2
    assert ba(_desc(dtype=ob.OMNI_F32)) == -2 and "bf16" in ob.last_error()
    assert ba(_desc(causal=0), block=128) == -2
    assert lib.omni_expand_blocks(C.byref(_desc(causal=0)), FAKE, FAKE, 3, 128, FAKE, FAKE, 384, None) == -2
    assert lib.omni_expand_blocks(C.byref(d), FAKE, FAKE, 3, 128, FAKE, FAKE, 383, None) == -1
    assert ob.workspace_bytes(ob.CALL_BLOCK_ATTN_FWD, d, 5 * 64) > 0
    with pytest.raises(ob.OmniError):
        ob.workspace_bytes(ob.CALL_BLOCK_ATTN_FWD, d, 100)
    # paged store: the pool descriptor is validated before any launch
    def pool(**kw):
        pp = ob.PagePool()
        pp.K, pp.V, pp.page_table = kw.get("K", 0x10000), 0x10000, kw.get("table", 0x10000)
        pp.n_pages, pp.page_rows, pp.pages_cap = kw.get("n_pages", 8), kw.get("page_rows", 16), kw.get("pages_cap", 4)
        return pp
    cp = lambda pp, u_cap=64: lib.omni_compact_cache_paged(C.byref(dd), FAKE, FAKE, FAKE, FAKE, u_cap,
                                                           C.byref(pp) if pp else None, None)
    assert cp(None) == -1 and "pool" in ob.last_error()
    assert cp(pool(K=None)) == -1 and cp(pool(table=None)) == -1 and cp(pool(K=0x10008)) == -1
    assert cp(pool(page_rows=24)) == -2 and "power of two" in ob.last_error()
    assert cp(pool(n_pages=0)) == -1 and cp(pool(n_pages=1 << 28, page_rows=16)) == -2
    assert cp(pool(), u_cap=65) == -1 and "pages_cap" in ob.last_error()
    assert cp(pool(), u_cap=0) == -1
    pp = pool()
    assert lib.omni_slim_decode_paged(C.byref(dd), FAKE, FAKE, FAKE, FAKE, FAKE, C.byref(pp), FAKE, FAKE, FAKE, 64, FAKE,
                                      FAKE, FAKE, 16, None) == -3
    assert lib.omni_slim_decode_paged(C.byref(dd), FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 64, FAKE,
                                      FAKE, FAKE, 1 << 30, None) == -1
    assert lib.omni_debug_key_split_len(0) == 0
    # a successful validation path clears the message
    assert ob.workspace_bytes(ob.CALL_SELECT_KV, d) > 0
    assert ob.last_error() == ""


def test_argument_errors_of_the_fused_and_batched_calls(lib):
    """omni_sparse_prefill, omni_prefill_select_varlen, omni_block_attn_bwd, omni_slim_decode_prepare and the decode
    call without workspace refuse bad arguments before any launch."""
    d = _desc()
    sp = lambda **kw: lib.omni_sparse_prefill(
        C.byref(d), FAKE, FAKE, kw.get("V", FAKE), kw.get("q_mode", 0), kw.get("q_param", 0.08), kw.get("p", 0.95),
        kw.get("pb", 256), kw.get("mode", 0), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, kw.get("cap", 300),
        kw.get("O", FAKE), FAKE, FAKE, kw.get("ws", 1 << 32), None)
    assert sp(mode=3) == -1 and sp(q_mode=2) == -1 and sp(p=1.5) == -1 and sp(pb=0) == -1 and sp(cap=0) == -1
    assert sp(V=None) == -1 and "null" in ob.last_error()
    assert sp(O=None) == -1
    assert sp(ws=1024) == -3 and "too small" in ob.last_error()
    need = lib.omni_sparse_prefill_workspace_bytes(C.byref(d), 256, 300)
    assert need > ob.workspace_bytes(ob.CALL_PREFILL_SELECT, d, 256) + ob.workspace_bytes(ob.CALL_SPARSE_ATTN_FWD, d, 300) - 256
    assert lib.omni_sparse_prefill_workspace_bytes(C.byref(d), 0, 300) == 0 and "probe_block" in ob.last_error()
    assert lib.omni_sparse_prefill_workspace_bytes(C.byref(d), 256, 0) == 0
    assert lib.omni_sparse_prefill_workspace_bytes(C.byref(_desc(head_dim=96)), 256, 300) == 0
    # per-sequence lengths: host arrays, checked against the padded length, the visual range and the sink
    arr = lambda *v: (C.c_int32 * len(v))(*v)
    d2 = _desc(batch=2)
    vl = lambda n, v0, v1, **kw: lib.omni_prefill_select_varlen(
        C.byref(d2), FAKE, FAKE, n, v0, v1, 0, 0.08, 0.95, 256, kw.get("mode", 0), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
        FAKE, FAKE, FAKE, 300, FAKE, kw.get("ws", 1 << 32), None)
    assert vl(arr(300, 301), arr(1, 1), arr(200, 200)) == -1 and "seq_tokens" in ob.last_error()
    assert vl(arr(300, 0), arr(1, 1), arr(200, 200)) == -1
    assert vl(arr(300, 100), arr(1, 1), arr(200, 101)) == -1 and "vis_begin" in ob.last_error()
    assert vl(arr(300, 100), arr(1, 50), arr(200, 50)) == -1
    assert vl(None, arr(1, 1), arr(200, 50)) == -1
    assert vl(arr(300, 100), arr(1, 1), arr(200, 50), mode=5) == -1
    assert vl(arr(300, 100), arr(1, 1), arr(200, 50), ws=64) == -3
    d3 = _desc(batch=2, sink_index=120)
    assert lib.omni_prefill_select_varlen(C.byref(d3), FAKE, FAKE, arr(300, 100), arr(1, 1), arr(200, 50), 0, 0.08, 0.95, 256, 0,
                                          FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 300, FAKE, 1 << 32,
                                          None) == -1 and "sink_index" in ob.last_error()
    # backward on block lists: as the forward
    bb = lambda dd_=d, **kw: lib.omni_block_attn_bwd(
        C.byref(dd_), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, kw.get("blk", FAKE), FAKE, kw.get("cap", 4),
        kw.get("block", 64), FAKE, FAKE, kw.get("dV", FAKE), FAKE, kw.get("ws", 1 << 32), None)
    assert bb(block=100) == -2 and bb(cap=0) == -1 and bb(blk=None) == -1 and bb(dV=None) == -1 and bb(ws=16) == -3
    assert bb(_desc(dtype=ob.OMNI_F32)) == -2 and bb(_desc(causal=0), block=128) == -2
    assert ob.workspace_bytes(ob.CALL_BLOCK_ATTN_BWD, d, 5 * 64) > 0
    # decode: the prepare call wants a descriptor with static_lists, whose workspace holds the merged lists too
    dd = ob.DecodeDesc()
    dd.batch, dd.n_q_heads, dd.n_kv_heads, dd.head_dim, dd.cache_capacity = 2, 4, 2, 128, 1000
    dd.vis_begin, dd.vis_end, dd.dtype, dd.softmax_scale, dd.tau = 0, 900, ob.OMNI_BF16, 0.088, 0.08
    dd.kv_stride = (C.c_int64 * 3)(2 * 1000 * 128, 1000 * 128, 128)
    plain = ob.workspace_bytes(ob.CALL_SLIM_DECODE, dd)
    assert lib.omni_slim_decode_prepare(C.byref(dd), FAKE, FAKE, 64, FAKE, 1 << 30, None) == -1
    assert "static_lists" in ob.last_error()
    dd.static_lists = 1
    with_lists = ob.workspace_bytes(ob.CALL_SLIM_DECODE, dd)
    assert with_lists >= plain + 2 * 2 * 900 * 8
    assert lib.omni_slim_decode_prepare(C.byref(dd), None, FAKE, 64, FAKE, 1 << 30, None) == -1
    assert lib.omni_slim_decode_prepare(C.byref(dd), FAKE, FAKE, 0, FAKE, 1 << 30, None) == -1
    assert lib.omni_slim_decode_prepare(C.byref(dd), FAKE, FAKE, 64, FAKE, plain, None) == -3
    assert lib.omni_slim_decode(C.byref(dd), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 64, FAKE, FAKE, FAKE, plain, None) == -3
    dd.static_lists = 2
    assert lib.omni_slim_decode_prepare(C.byref(dd), FAKE, FAKE, 64, FAKE, 1 << 30, None) == -1
    dd.static_lists = 0
    assert lib.omni_static_scratch_bytes() == 16 << 20
    assert lib.omni_slim_decode_grouped_static(C.byref(dd), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 64, FAKE,
                                               FAKE, None) == -1
    assert lib.omni_slim_decode_grouped_static(C.byref(dd), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE,
                                               FAKE, None) == -1


@pytest.mark.parametrize("q_cnt,budget,n_heads,n_tokens,causal", [
    ([1859, 500, 300, 0, 20, 129, 128, 1], [700], 8, 1859, 1),
    (None, None, 8, 1859, 1),
    ([65536] + [17000 + 13 * i for i in range(27)], [35000], 28, 65536, 1),
    ([0, 0, 5, 0], [3], 4, 537, 0),
    ([0, 0, 0, 0], [3], 4, 537, 1),
])
@pytest.mark.parametrize("tile_rows", [128, 256])
def test_device_work_list_covers_every_query_tile_exactly_once(lib, q_cnt, budget, n_heads, n_tokens, causal, tile_rows):
    import numpy as np
    d = _desc(n_q_heads=n_heads, n_kv_heads=n_heads, n_tokens=n_tokens, vis_end=min(256, n_tokens), causal=causal)
    head, tile, cost = ob.debug_work_list(d, q_cnt, budget, n_tokens, tile_rows)
    counts = q_cnt if q_cnt is not None else [n_tokens] * n_heads
    want = {(h, t) for h in range(n_heads) for t in range((counts[h] + tile_rows - 1) // tile_rows)}
    got = list(zip(head.tolist(), tile.tolist()))
    assert len(got) == len(want) and set(got) == want
    # handed out longest first; among equals in head-major, tile-ascending order
    assert np.all(np.diff(cost) <= 0)
    for (a, ca), (b, cb) in zip(zip(got, cost), zip(got[1:], cost[1:])):
        if ca == cb:
            assert b > a
    # the cost is the number of 64-key tiles the item streams: under the causal mask it grows with the tile index
    nk = n_tokens if budget is None else min(budget[0], n_tokens)
    for (h, t), cst in zip(got, cost.tolist()):
        nt = (counts[h] + tile_rows - 1) // tile_rows
        keys = nk if not causal else -(-nk * (t + 1) // nt)
        assert cst == -(-keys // 64)


@pytest.mark.parametrize("q_cnt,budget,n_heads,n_tokens", [
    ([65536] + [17000 + 13 * i for i in range(27)], [35000], 28, 65536),
    ([1859, 500, 300, 0, 20, 129, 128, 1], [700], 8, 1859),
    ([0, 0, 5, 0], [3], 4, 537),
    ([400] * 3, [300], 3, 537),
    ([900 + 37 * i for i in range(24)], [1500], 24, 1859),
])
def test_queued_work_list_places_whole_heads_and_balances_the_queues(lib, q_cnt, budget, n_heads, n_tokens):
    """One list per XCD: every tile once, a head in one queue only and in one stretch of it, longest item first
    inside a head, heads placed largest first onto the least loaded queue (checked by replaying that rule)."""
    import numpy as np
    tile_rows = 256
    d = _desc(n_q_heads=n_heads, n_kv_heads=n_heads, n_tokens=n_tokens, vis_end=min(256, n_tokens), causal=1)
    head, tile, cost, qend = ob.debug_work_list(d, q_cnt, budget, n_tokens, tile_rows, queues=8)
    want = {(h, t) for h in range(n_heads) for t in range((q_cnt[h] + tile_rows - 1) // tile_rows)}
    got = list(zip(head.tolist(), tile.tolist()))
    assert len(got) == len(want) and set(got) == want
    assert np.all(np.diff(qend) >= 0) and qend[-1] == len(got)
    total = {h: int(cost[head == h].sum()) for h in range(n_heads)}
    if 2 * max(total.values()) * 8 > 3 * sum(total.values()):
        # one head outweighs 1.5 fair shares of a queue: one longest-first list after all
        assert np.all(qend == len(got)) and np.all(np.diff(cost) <= 0)
        return
    starts = np.concatenate([[0], qend[:-1]])
    queue_of, loads, order_in_queue = {}, [], []
    for q in range(8):
        seg_h, seg_c = head[starts[q]:qend[q]], cost[starts[q]:qend[q]]
        loads.append(int(seg_c.sum()))
        heads_here = []
        for h in seg_h.tolist():
            if not heads_here or heads_here[-1] != h:
                heads_here.append(h)
        assert len(heads_here) == len(set(heads_here))            # a head is one contiguous stretch
        for h in heads_here:
            assert h not in queue_of
            queue_of[h] = q
            assert np.all(np.diff(seg_c[seg_h == h]) <= 0)       # longest item first inside the head
        order_in_queue.append(heads_here)
    # replay: heads by total cost (descending, lower index first among equals) onto the least loaded queue
    sim_load, sim_order = [0] * 8, [[] for _ in range(8)]
    for h in sorted(range(n_heads), key=lambda x: (-total[x], x)):
        q = min(range(8), key=lambda r: (sim_load[r], r))
        sim_load[q] += total[h]
        if q_cnt[h] > 0:
            sim_order[q].append(h)
    assert sim_order == order_in_queue
    assert loads == sim_load
