"""GPU parity at the full sizes of the measured workloads, in the launch configuration bench.py times.

The oracle cannot run whole attention at these sizes in test time, so it does what it can do exactly:
the whole selection (cheap), and attention / gradients for sampled queries and keys, one by one; sums over
all keys that the definition fixes at any size cover the rest.
"""
import numpy as np
import pytest
import torch

from oracle import omni_oracle as oc
from paper_2511_12201_amd import binding as ob
from paper_2511_12201_amd import synth
from tests.helpers import (check_selection_on_gpu_scores, grad_bar, lists_to_padded, padded_to_lists, stored, to_device,
                           to_host)

pytestmark = pytest.mark.gpu

TAU, RECALL_P, PROBE_BLOCK = 0.08, 0.95, 256          # the hyper-parameters of the bench
TOL = 2e-2                                            # bf16 bar for outputs and gradients


class FullCase:
    """Seeded layer of a measured configuration with the oracle's own selection (cached per session)."""
    _cache = {}

    def __init__(self, cfg):
        self.cfg = cfg
        L = synth.make_layer(cfg)
        self.Q, self.K, self.V = L["Q"], L["K"], L["V"]
        self.dQ, self.dK, self.dV = (to_device(x, cfg.dtype) for x in (self.Q, self.K, self.V))
        self.desc = ob.make_layer_desc(self.dQ, self.dK, cfg.vis_begin, cfg.vis_end, cfg.sink_index, cfg.causal)
        probe = oc.probe_keys(self.K, cfg.vis_begin, cfg.vis_end, cfg.sink_index)
        self.scores32 = oc.score_queries(self.Q, probe, cfg.scale).astype(np.float32)
        self.q_lists = oc.select_queries(self.scores32, 0, TAU, cfg.vis_begin, cfg.vis_end)
        self.a32 = oc.pooled_key_scores(self.Q, self.K, PROBE_BLOCK, cfg.causal, cfg.scale).astype(np.float32)
        self.bud = oc.kv_budget(self.a32, RECALL_P, 0)
        self.kv_lists = [list(x) for x in oc.select_kv(self.a32, self.bud["budget"])]

    @classmethod
    def get(cls, cfg):
        if cfg.name not in cls._cache:
            cls._cache.clear()                        # one full-size layer in memory at a time
            cls._cache[cfg.name] = cls(cfg)
        return cls._cache[cfg.name]


def _sample_queries(rng, q_list, n, lo=0):
    """A few kept queries of one head: the first, the last, some around 256-row tile edges, the rest random."""
    q = q_list[q_list >= lo]
    if q.size == 0:
        return np.zeros(0, dtype=np.int64)
    picks = {0, q.size - 1}
    for edge in (255, 256, 257, q.size - 256, q.size // 2):
        if 0 <= edge < q.size:
            picks.add(int(edge))
    picks.update(int(x) for x in rng.integers(0, q.size, n))
    return np.sort(q[sorted(picks)]).astype(np.int64)


def test_c3_64k_selection_and_forward_on_sampled_rows():
    cfg = synth.C3_64K
    c = FullCase.get(cfg)
    N, H = cfg.n_tokens, cfg.n_q_heads
    # free-running selection, exactly as bench.py calls it, against the oracle's
    sel = ob.omni_prefill_select(c.desc, c.dQ, c.dK, 0, TAU, RECALL_P, PROBE_BLOCK, 0, N)
    torch.cuda.synchronize()
    got_q = padded_to_lists(sel.q_idx, sel.q_cnt)
    s_gpu, a_gpu = to_host(sel.scores), to_host(sel.budget.key_scores)
    # the score arrays numerically against the oracle's ...
    assert np.max(np.abs(s_gpu.astype(np.float64) - c.scores32)) <= 2e-5
    assert np.max(np.abs(a_gpu.astype(np.float64) - c.a32)) <= 1e-4 * c.a32.max()
    np.testing.assert_allclose(a_gpu.astype(np.float64).sum(-1), N, rtol=1e-5)
    # ... and the selection kernels on the arrays they saw: the oracle's selection on the GPU's scores gives the GPU's sets
    gpu_kv_lists = check_selection_on_gpu_scores(oc, s_gpu, a_gpu, got_q, to_host(sel.budget.flattest),
                                                 to_host(sel.budget.budget), to_host(sel.kv_idx), 0, TAU, RECALL_P, 0,
                                                 cfg.vis_begin, cfg.vis_end)
    assert int(to_host(sel.budget.flattest)[0]) == int(c.bud["flattest"][0])
    bg, bo = len(gpu_kv_lists[0][0]), int(c.bud["budget"][0])
    assert abs(bg - bo) <= max(2, int(2e-3 * bo))          # informational: distance to the oracle's own pipeline
    # attention of the free-running step on its own sets, sampled rows of every head against the oracle
    Of, lsef = ob.omni_sparse_attn_fwd(c.desc, c.dQ, c.dK, c.dV, sel.q_idx, sel.q_cnt, sel.kv_idx, sel.budget.budget, N)
    torch.cuda.synchronize()
    rng = np.random.default_rng(43)
    samples = [[_sample_queries(rng, got_q[0][h], 4) for h in range(H)]]
    Oo, Lo = oc.sparse_attn_fwd(c.Q, c.K, c.V, samples, gpu_kv_lists, cfg.causal, cfg.scale)
    Og, Lg = to_host(Of), to_host(lsef)
    for h in range(H):
        rows = samples[0][h]
        assert np.max(np.abs(Og[0, h, rows] - Oo[0, h, rows])) <= TOL, f"free-running attention, head {h}"
        assert np.max(np.abs(Lg[0, h, rows] - Lo[0, h, rows])) <= 2e-3
    # the same step as one call (key lists formed inside the attention's gather): every output bit for bit
    one, O1, lse1 = ob.omni_sparse_prefill(c.desc, c.dQ, c.dK, c.dV, 0, TAU, RECALL_P, PROBE_BLOCK, 0, N)
    torch.cuda.synchronize()
    assert torch.equal(O1, Of) and torch.equal(lse1, lsef)
    assert torch.equal(one.scores, sel.scores) and torch.equal(one.budget.key_scores, sel.budget.key_scores)
    assert torch.equal(one.budget.budget, sel.budget.budget) and torch.equal(one.q_cnt, sel.q_cnt)
    assert torch.equal(one.kv_idx[0, :, :bg], sel.kv_idx[0, :, :bg])
    del Of, lsef, one, O1, lse1

    # attention on the oracle's sets (b_cap = N as in the bench), sampled rows against the oracle
    q_idx, q_cnt = lists_to_padded(c.q_lists, H, N)
    kv_idx, _ = lists_to_padded([c.kv_lists[0]], H, N)
    budget = torch.tensor([bo], dtype=torch.int32, device="cuda")
    O, lse = ob.omni_sparse_attn_fwd(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, kv_idx, budget, N)
    torch.cuda.synchronize()
    rng = np.random.default_rng(41)
    samples = [[_sample_queries(rng, c.q_lists[0][h], 6) for h in range(H)]]
    Oo, Lo = oc.sparse_attn_fwd(c.Q, c.K, c.V, samples, c.kv_lists, cfg.causal, cfg.scale)
    Og, Lg = to_host(O), to_host(lse)
    worst = 0.0
    for h in range(H):
        rows = samples[0][h]
        fin = np.isfinite(Lo[0, h, rows])
        np.testing.assert_array_equal(np.isfinite(Lg[0, h, rows]), fin)
        worst = max(worst, float(np.max(np.abs(Og[0, h, rows] - Oo[0, h, rows]))))
        assert np.max(np.abs(Lg[0, h, rows][fin] - Lo[0, h, rows][fin])) <= 2e-3
    assert worst <= TOL
    # rows that are not kept: zero output, lse = -inf -- every one of them
    for h in range(H):
        kept = np.zeros(N, dtype=bool)
        kept[c.q_lists[0][h]] = True
        assert np.all(Lg[0, h, ~kept] == -np.inf)
        assert not Og[0, h, ~kept].any()
        assert np.all(np.isfinite(Lg[0, h, kept]))       # the sink key is selected, so every kept query sees a key


def test_c3_64k_block_lists_in_place_equal_the_gathered_path():
    """Block lists at the bench's granularity (256) on the 64k layer: the in-place kernel against expand + gather,
    bit for bit, and sampled rows of it against the oracle."""
    cfg = synth.C3_64K
    c = FullCase.get(cfg)
    N, H = cfg.n_tokens, cfg.n_q_heads
    block = 256
    nb = N // block
    rng = np.random.default_rng(59)
    nsel = int(0.6 * nb)
    lists = [[np.sort(np.concatenate([[0], 1 + rng.choice(nb - 1, nsel - 1, replace=False)])).astype(np.int32)
              for _ in range(H)]]
    blk_idx, _ = lists_to_padded(lists, H, nb)
    blk_budget = torch.tensor([nsel], dtype=torch.int32, device="cuda")
    q_idx, q_cnt = lists_to_padded(c.q_lists, H, N)
    O1, lse1 = ob.omni_block_attn_fwd(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, blk_idx, blk_budget, block)
    kv_idx, budget = ob.omni_expand_blocks(c.desc, blk_idx, blk_budget, block)
    O2, lse2 = ob.omni_sparse_attn_fwd(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, kv_idx, budget, kv_idx.shape[-1])
    torch.cuda.synchronize()
    assert torch.equal(O1.view(torch.int16), O2.view(torch.int16))
    assert torch.equal(lse1.view(torch.int32), lse2.view(torch.int32))
    tok = oc.expand_blocks(lists, block, N)
    samples = [[_sample_queries(rng, c.q_lists[0][h], 3) for h in range(H)]]
    Oo, Lo = oc.sparse_attn_fwd(c.Q, c.K, c.V, samples, tok, cfg.causal, cfg.scale)
    Og, Lg = to_host(O1), to_host(lse1)
    for h in range(H):
        rows = samples[0][h]
        assert np.max(np.abs(Og[0, h, rows] - Oo[0, h, rows])) <= TOL
        assert np.max(np.abs(Lg[0, h, rows] - Lo[0, h, rows])) <= 2e-3


def test_c4_32k_backward_on_sampled_rows_and_sums_over_all_keys():
    cfg = synth.C4_TRAIN_32K
    c = FullCase.get(cfg)
    N, H, Hkv = cfg.n_tokens, cfg.n_q_heads, cfg.n_kv_heads
    G = H // Hkv
    dO_np = synth.make_grad_output(cfg)
    dO = to_device(dO_np, cfg.dtype)
    bo = int(c.bud["budget"][0])
    q_idx, q_cnt = lists_to_padded(c.q_lists, H, N)
    kv_idx, _ = lists_to_padded([c.kv_lists[0]], H, N)
    budget = torch.tensor([bo], dtype=torch.int32, device="cuda")
    assert len(c.q_lists[0][0]) == N                       # head 0 keeps every query: its first key tiles are split
    O, lse = ob.omni_sparse_attn_fwd(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, kv_idx, budget, N)
    torch.cuda.synchronize()
    # The backward is handed the forward's output as the layer stores it, and both sides must read the same one
    # (its row sums with dO enter every gradient): for the rows the oracle works on, the oracle's own forward,
    # rounded to bf16, replaces the GPU's in what the GPU backward gets -- after it has been checked against it.
    tail = N - 1536
    rng = np.random.default_rng(43)
    late = [[ql[ql >= tail] for ql in c.q_lists[0]]]
    early = [[_sample_queries(rng, c.q_lists[0][h][c.q_lists[0][h] < tail], 4) for h in range(H)]]
    rows_o = [[np.concatenate([early[0][h], late[0][h]]) for h in range(H)]]
    Oo, Lo = oc.sparse_attn_fwd(c.Q, c.K, c.V, rows_o, c.kv_lists, cfg.causal, cfg.scale)
    O_h, lse_h = to_host(O).copy(), to_host(lse).copy()
    for h in range(H):
        r = rows_o[0][h]
        assert np.max(np.abs(O_h[0, h, r] - Oo[0, h, r])) <= TOL, f"forward, head {h}"
        assert np.max(np.abs(lse_h[0, h, r] - Lo[0, h, r])) <= 2e-3
        O_h[0, h, r] = stored(Oo[0, h, r], cfg.dtype)
        lse_h[0, h, r] = Lo[0, h, r].astype(np.float32)
    gQ, gK, gV = ob.omni_sparse_attn_bwd(c.desc, c.dQ, c.dK, c.dV, to_device(O_h, cfg.dtype), dO,
                                         torch.from_numpy(lse_h).cuda(), q_idx, q_cnt, kv_idx, budget, N)
    torch.cuda.synchronize()
    gQ, gK, gV = to_host(gQ), to_host(gK), to_host(gV)

    # (1) exact rows: every kept query from `tail` on goes to the oracle, which then holds the whole gradient
    # of every key >= tail (only later queries see a key) and of those queries
    dQo, dKo, dVo = oc.sparse_attn_bwd(c.Q, c.K, c.V, dO_np, late, c.kv_lists, cfg.causal, cfg.scale, O=O_h)
    rQ, rK, rV = oc.sparse_attn_bwd_term_rss(c.Q, c.K, c.V, dO_np, late, c.kv_lists, cfg.causal, cfg.scale, O=O_h)
    for h in range(H):
        rows = late[0][h]
        assert np.all(np.abs(gQ[0, h, rows] - dQo[0, h, rows]) <= grad_bar(dQo[0, h, rows], cfg.dtype, rQ[0, h, rows])), \
            f"dQ, head {h}"
    assert np.all(np.abs(gK[0, :, tail:] - dKo[0, :, tail:]) <= grad_bar(dKo[0, :, tail:], cfg.dtype, rK[0, :, tail:]))
    assert np.all(np.abs(gV[0, :, tail:] - dVo[0, :, tail:]) <= grad_bar(dVo[0, :, tail:], cfg.dtype, rV[0, :, tail:]))
    # (2) sampled early queries (dQ needs only the query's own softmax row)
    dQe, _, _ = oc.sparse_attn_bwd(c.Q, c.K, c.V, dO_np, early, c.kv_lists, cfg.causal, cfg.scale, O=O_h)
    rQe, _, _ = oc.sparse_attn_bwd_term_rss(c.Q, c.K, c.V, dO_np, early, c.kv_lists, cfg.causal, cfg.scale, O=O_h)
    for h in range(H):
        rows = early[0][h]
        assert np.all(np.abs(gQ[0, h, rows] - dQe[0, h, rows]) <= grad_bar(dQe[0, h, rows], cfg.dtype, rQe[0, h, rows])), \
            f"dQ early, head {h}"
    # (3) sums over all keys, fixed by the definition: rows of P sum to 1, rows of dS to 0, so
    #     sum_k dV[g, k] = sum over the group's heads and kept queries of dO,   sum_k dK[g, k] = 0.
    # bf16 outputs: every summed element carries an independent rounding error of at most half an ulp
    # (2^-8 relative), so the sum is off by about 2^-8 / sqrt(3) * sqrt(sum v^2); the bar is six of those
    for g in range(Hkv):
        want = np.zeros(cfg.head_dim)
        for h in range(g * G, (g + 1) * G):
            want += dO_np[0, h, c.q_lists[0][h]].astype(np.float64).sum(0)
        got_v = gV[0, g].astype(np.float64).sum(0)
        got_k = gK[0, g].astype(np.float64).sum(0)
        bar_v = 6 * 2.0 ** -8 / np.sqrt(3) * np.sqrt((gV[0, g].astype(np.float64) ** 2).sum(0)) + 2e-3
        # dK also inherits the rounding of the forward's bf16 O through delta = rowsum(dO * O): the rows of dS then
        # sum to the (small, random) error of delta instead of 0, which adds over all queries -- four times the bar
        bar_k = 24 * 2.0 ** -8 / np.sqrt(3) * np.sqrt((gK[0, g].astype(np.float64) ** 2).sum(0)) + 2e-3
        assert np.all(np.abs(got_v - want) <= bar_v), f"sum of dV, group {g}: {np.max(np.abs(got_v - want) / bar_v)}"
        assert np.all(np.abs(got_k) <= bar_k), f"sum of dK, group {g}: {np.max(np.abs(got_k) / bar_k)}"
    # (4) tokens no head of the group selected have zero gradient, queries not kept too
    for g in range(Hkv):
        used = np.zeros(N, dtype=bool)
        for h in range(g * G, (g + 1) * G):
            used[c.kv_lists[0][h]] = True
        assert not gK[0, g, ~used].any() and not gV[0, g, ~used].any()
    for h in range(H):
        kept = np.zeros(N, dtype=bool)
        kept[c.q_lists[0][h]] = True
        assert not gQ[0, h, ~kept].any()


def test_c4_32k_block_lists_backward_in_place_equals_the_gathered_path():
    """Block lists at the bench's granularity (256) on the 32k training layer: the backward that walks them in place
    against expand + gather, bit for bit (the gathered path is checked against the oracle above)."""
    cfg = synth.C4_TRAIN_32K
    c = FullCase.get(cfg)
    N, H = cfg.n_tokens, cfg.n_q_heads
    block = 256
    nb = N // block
    rng = np.random.default_rng(61)
    nsel = int(0.6 * nb)
    lists = [[np.sort(np.concatenate([[0], 1 + rng.choice(nb - 1, nsel - 1, replace=False)])).astype(np.int32)
              for _ in range(H)]]
    blk_idx, _ = lists_to_padded(lists, H, nb)
    blk_budget = torch.tensor([nsel], dtype=torch.int32, device="cuda")
    q_idx, q_cnt = lists_to_padded(c.q_lists, H, N)
    dO = to_device(synth.make_grad_output(cfg), cfg.dtype)
    O, lse = ob.omni_block_attn_fwd(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, blk_idx, blk_budget, block)
    g1 = ob.omni_block_attn_bwd(c.desc, c.dQ, c.dK, c.dV, O, dO, lse, q_idx, q_cnt, blk_idx, blk_budget, block)
    kv_idx, budget = ob.omni_expand_blocks(c.desc, blk_idx, blk_budget, block)
    g2 = ob.omni_sparse_attn_bwd(c.desc, c.dQ, c.dK, c.dV, O, dO, lse, q_idx, q_cnt, kv_idx, budget, kv_idx.shape[-1])
    torch.cuda.synchronize()
    for name, x, y in zip(("dQ", "dK", "dV"), g1, g2):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16)), name
    assert float(g1[1].float().abs().max()) > 0


def test_c5_131k_decode_step():
    """One decode step on the 131072-token cache: seeded per-head lists of the bench's budget fraction (the
    oracle's own selection at this length takes a minute; the decode kernels do not care where a list came from)."""
    cfg = synth.C5_DECODE_131K
    layer = synth.make_layer(cfg)
    N, H, Hkv, D = cfg.n_tokens, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    batch, n_new = 2, 3
    steps = synth.make_decode_steps(cfg, layer, n_new, batch=batch)
    cap = N + n_new
    Kc = np.zeros((batch, Hkv, cap, D), dtype=np.float32)
    Vc = np.zeros_like(Kc)
    Kc[:, :, :N], Vc[:, :, :N] = layer["K"], layer["V"]
    for s in range(n_new):
        Kc[:, :, N + s], Vc[:, :, N + s] = steps["k_new"][s], steps["v_new"][s]
    ctx = np.array([N + n_new, N + 1], dtype=np.int32)         # two different context lengths
    q = steps["q"][n_new - 1]
    probe = oc.probe_keys(layer["K"], cfg.vis_begin, cfg.vis_end, cfg.sink_index).astype(np.float32)
    probe = np.repeat(probe, batch, axis=0)
    rng = np.random.default_rng(47)
    b = int(0.53 * N)
    vis = [[np.sort(rng.choice(np.arange(cfg.vis_begin, cfg.vis_end), int(rng.integers(b // 8, b)), replace=False)).astype(np.int32)
            for _ in range(H)] for _ in range(batch)]
    dq, dKc, dVc = (to_device(x, cfg.dtype) for x in (q, Kc, Vc))
    dctx = torch.from_numpy(ctx).cuda()
    dprobe = torch.from_numpy(probe).cuda()
    vis_idx, vis_cnt = lists_to_padded(vis, H, b)
    desc = ob.make_decode_desc(dq, dKc, cfg.vis_begin, cfg.vis_end, TAU)
    O, act = ob.omni_slim_decode(desc, dq, dKc, dVc, dctx, dprobe, vis_idx, vis_cnt, b)
    Od = ob.omni_dense_decode(desc, dq, dKc, dVc, dctx)
    torch.cuda.synchronize()
    Oo, acto, sc = oc.slim_decode(q, Kc, Vc, ctx, probe, vis, TAU, cfg.vis_begin, cfg.vis_end, cfg.scale)
    act = to_host(act)
    clear = np.abs(sc - TAU) > 1e-5
    np.testing.assert_array_equal(act[clear], acto[clear])
    same = act == acto
    assert same.mean() > 0.9
    assert np.max(np.abs(to_host(O)[same] - Oo[same])) <= TOL
    Odo = oc.dense_decode(q, Kc, Vc, ctx, cfg.scale)
    assert np.max(np.abs(to_host(Od) - Odo)) <= TOL
    # the same lists as group unions: gathered from the cache, from the compacted store, from the paged store
    shape_only = torch.empty((batch, H, N, D), dtype=torch.bfloat16, device="meta")
    ldesc = ob.make_layer_desc(shape_only, torch.empty((batch, Hkv, N, D), dtype=torch.bfloat16, device="meta"),
                               cfg.vis_begin, cfg.vis_end, cfg.sink_index, cfg.causal)
    grp_idx, grp_mask, grp_cnt = ob.omni_group_subset(ldesc, vis_idx, vis_cnt, b, _per_head=True)
    u_max = int(grp_cnt.max().cpu())
    grp_idx, grp_mask = grp_idx[:, :, :u_max].contiguous(), grp_mask[:, :, :u_max].contiguous()
    Og, actg = ob.omni_slim_decode_grouped(desc, dq, dKc, dVc, dctx, dprobe, grp_idx, grp_mask, grp_cnt)
    Kcomp, Vcomp = ob.omni_compact_cache(desc, dKc, dVc, grp_idx, grp_cnt)
    page_rows = 256
    need = ((grp_cnt + page_rows - 1) // page_rows).cpu().numpy()
    n_pages = int(need.sum())
    perm = np.random.default_rng(53).permutation(n_pages).astype(np.int32)
    table = np.full((batch, Hkv, -(-u_max // page_rows)), -1, dtype=np.int32)
    used = 0
    for bb in range(batch):
        for g in range(Hkv):
            table[bb, g, : need[bb, g]] = perm[used: used + need[bb, g]]
            used += int(need[bb, g])
    Kpool = torch.empty(n_pages, page_rows, D, dtype=torch.bfloat16, device="cuda")
    Vpool = torch.empty_like(Kpool)
    pool = ob.make_page_pool(Kpool, Vpool, torch.from_numpy(table).cuda())
    ob.omni_compact_cache_paged(desc, dKc, dVc, grp_idx, grp_cnt, pool)
    dKc[:, :, cfg.vis_begin:cfg.vis_end] = float("nan")         # the visual rows of the cache are not needed any more
    dVc[:, :, cfg.vis_begin:cfg.vis_end] = float("nan")
    Oc, actc = ob.omni_slim_decode_compact(desc, dq, dKc, dVc, dctx, dprobe, Kcomp, Vcomp, grp_idx, grp_mask, grp_cnt)
    Op, actp = ob.omni_slim_decode_paged(desc, dq, dKc, dVc, dctx, dprobe, pool, grp_idx, grp_mask, grp_cnt)
    torch.cuda.synchronize()
    for Ox, actx in ((Og, actg), (Oc, actc), (Op, actp)):
        np.testing.assert_array_equal(to_host(actx), act)
        got = to_host(Ox)
        assert np.all(np.isfinite(got))
        assert np.max(np.abs(got[same] - Oo[same])) <= TOL
    assert torch.equal(Og.view(torch.int16), Oc.view(torch.int16)) and torch.equal(Oc.view(torch.int16), Op.view(torch.int16))
