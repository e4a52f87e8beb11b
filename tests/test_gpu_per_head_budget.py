"""GPU parity of the per-head-budget variant: budget_mode 2 and the *_per_head calls against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import omni_oracle as oc
from paper_2511_12201_amd import binding as ob
from paper_2511_12201_amd import synth
from tests.helpers import (check_selection_on_gpu_scores, lists_to_padded, oracle_train, padded_to_lists, to_device,
                           to_host)
from tests.test_gpu_parity import (ALL_CFGS, CFG_BF16, CFG_BF16_64, CFG_F32, TOL_OUT, _check_fwd, _check_grads,
                                   case_for)

pytestmark = pytest.mark.gpu


def _ragged_budgets(cfg, rng, lo=0):
    """[B,Hq] budgets that span 0 / 1 / a ragged tile tail / everything."""
    N, H = cfg.n_tokens, cfg.n_q_heads
    fixed = [N, 1, lo, 65, N - 1, 130]
    bud = np.array([[fixed[h] if h < len(fixed) else int(rng.integers(1, N)) for h in range(H)]
                    for _ in range(cfg.batch)], dtype=np.int32)
    return bud


@pytest.mark.parametrize("cfg", ALL_CFGS, ids=lambda c: c.name)
@pytest.mark.parametrize("p", [0.95, 0.5, 1.0])
def test_per_head_budgets_from_given_scores_are_exact(cfg, p):
    c = case_for(cfg)
    a = torch.from_numpy(c.o_a32).cuda()
    r = ob.omni_budget_from_scores(c.desc, a, p, 2)
    torch.cuda.synchronize()
    want = oc.kv_budget(c.o_a32, p, 2)
    assert tuple(r.budget.shape) == (cfg.batch, cfg.n_q_heads)
    np.testing.assert_array_equal(to_host(r.budget), want["budget"])
    np.testing.assert_array_equal(to_host(r.flattest), want["flattest"])
    np.testing.assert_allclose(to_host(r.kurtosis), want["kurtosis"], rtol=1e-9)
    np.testing.assert_allclose(to_host(r.recall), want["recall"], atol=1e-6)


@pytest.mark.parametrize("cfg", ALL_CFGS, ids=lambda c: c.name)
def test_select_kv_per_head_is_bit_exact_on_given_scores(cfg):
    c = case_for(cfg)
    a = torch.from_numpy(c.o_a32).cuda()
    N = cfg.n_tokens
    rng = np.random.default_rng(31)
    for bud_np in (oc.kv_budget(c.o_a32, 0.95, 2)["budget"], _ragged_budgets(cfg, rng)):
        bud = torch.from_numpy(np.ascontiguousarray(bud_np)).cuda()
        kv_idx = ob.omni_select_kv_per_head(c.desc, a, bud, N)
        torch.cuda.synchronize()
        want = oc.select_kv(c.o_a32, bud_np)
        got = to_host(kv_idx)
        for b in range(cfg.batch):
            for h in range(cfg.n_q_heads):
                np.testing.assert_array_equal(got[b, h, : bud_np[b, h]], want[b][h], err_msg=f"head {h}")
    # capacity below a head's budget clamps that head only
    cap = 96
    bud_np = _ragged_budgets(cfg, rng, lo=2)
    got = to_host(ob.omni_select_kv_per_head(c.desc, a, torch.from_numpy(bud_np).cuda(), cap))
    want = oc.select_kv(c.o_a32, np.minimum(bud_np, cap))
    for h in range(cfg.n_q_heads):
        np.testing.assert_array_equal(got[0, h, : min(bud_np[0, h], cap)], want[0][h])


def test_shape_of_the_budget_array_is_checked_by_the_binding():
    c = case_for(CFG_BF16)
    a = torch.from_numpy(c.o_a32).cuda()
    with pytest.raises(ValueError):
        ob.omni_select_kv_per_head(c.desc, a, torch.ones(1, dtype=torch.int32, device="cuda"), 8)
    with pytest.raises(ValueError):
        ob.omni_select_kv(c.desc, a, torch.ones(1, CFG_BF16.n_q_heads, dtype=torch.int32, device="cuda"), 8)


def _run_fwd_bwd_per_head(c, q_lists, kv_lists, dO_np=None):
    """Forward on the GPU; the backward (when dO is given) on the oracle's stored forward output and log-sum-exp, so
    that both sides are the same function of the same inputs.  Returns (O, lse, grads, oracle's gradients)."""
    cfg = c.cfg
    q_idx, q_cnt = lists_to_padded(q_lists, cfg.n_q_heads, cfg.n_tokens)
    cap = max(1, max(len(x) for per in kv_lists for x in per))
    kv_idx, budget = lists_to_padded(kv_lists, cfg.n_q_heads, cap)
    O, lse = ob.omni_sparse_attn_fwd_per_head(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, kv_idx, budget, cap)
    grads = want = None
    if dO_np is not None:
        O_st, lse_o, want = oracle_train(oc, cfg.dtype, c.Q, c.K, c.V, dO_np, q_lists, kv_lists, cfg.causal, cfg.scale)
        dO = to_device(dO_np, cfg.dtype)
        grads = ob.omni_sparse_attn_bwd_per_head(c.desc, c.dQ, c.dK, c.dV, to_device(O_st, cfg.dtype), dO,
                                                 torch.from_numpy(lse_o).cuda(), q_idx, q_cnt, kv_idx, budget, cap)
    torch.cuda.synchronize()
    return to_host(O), to_host(lse), grads, want


@pytest.mark.parametrize("cfg", ALL_CFGS, ids=lambda c: c.name)
def test_attention_fwd_bwd_on_the_oracles_per_head_selection(cfg):
    c = case_for(cfg)
    bud = oc.kv_budget(c.o_a32, c.recall_p, 2)["budget"]
    assert bud.min() < bud.max()                               # the budgets really are ragged on this input
    kv_lists = oc.select_kv(c.o_a32, bud)
    dO = synth.make_grad_output(cfg)
    O, lse, grads, want = _run_fwd_bwd_per_head(c, c.o_qidx, kv_lists, dO)
    Oo, Lo = oc.sparse_attn_fwd(c.Q, c.K, c.V, c.o_qidx, kv_lists, cfg.causal, cfg.scale)
    _check_fwd(c, O, lse, Oo, Lo)
    _check_grads(cfg, grads, want, c.o_qidx, kv_lists)


@pytest.mark.parametrize("cfg", [CFG_BF16, CFG_BF16_64, CFG_F32], ids=lambda c: c.name)
def test_attention_fwd_bwd_with_ragged_budgets_including_an_empty_head(cfg):
    c = case_for(cfg)
    N, H = cfg.n_tokens, cfg.n_q_heads
    rng = np.random.default_rng(33)
    bud = _ragged_budgets(cfg, rng)                              # head 2 (where there is one) selects no key at all
    kv_lists = [[np.sort(rng.choice(N, int(bud[b, h]), replace=False)).astype(np.int32) for h in range(H)]
                for b in range(cfg.batch)]
    q_lists = [[np.arange(N, dtype=np.int32)] + [np.sort(rng.choice(N, int(rng.integers(1, 300)), replace=False)).astype(np.int32)
                                                for _ in range(H - 1)] for _ in range(cfg.batch)]
    dO = synth.make_grad_output(cfg)
    O, lse, grads, want = _run_fwd_bwd_per_head(c, q_lists, kv_lists, dO)
    Oo, Lo = oc.sparse_attn_fwd(c.Q, c.K, c.V, q_lists, kv_lists, cfg.causal, cfg.scale)
    _check_fwd(c, O, lse, Oo, Lo)
    empty = [h for h in range(H) if bud[0, h] == 0]
    for h in empty:
        assert np.all(lse[0, h] == -np.inf) and np.all(O[0, h] == 0)
    _check_grads(cfg, grads, want, q_lists, kv_lists)
    for h in empty:
        assert np.all(to_host(grads[0])[0, h] == 0)


def test_equal_per_head_budgets_reproduce_the_shared_budget_calls_bit_for_bit():
    cfg = CFG_BF16
    c = case_for(cfg)
    b = int(c.o_bud["budget"][0])
    kv_lists = [list(c.o_kvidx[bb]) for bb in range(cfg.batch)]
    q_idx, q_cnt = lists_to_padded(c.o_qidx, cfg.n_q_heads, cfg.n_tokens)
    kv_idx, per_head = lists_to_padded(kv_lists, cfg.n_q_heads, b)
    shared = torch.full((cfg.batch,), b, dtype=torch.int32, device="cuda")
    dO = to_device(synth.make_grad_output(cfg), cfg.dtype)
    O1, l1 = ob.omni_sparse_attn_fwd(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, kv_idx, shared, b)
    O2, l2 = ob.omni_sparse_attn_fwd_per_head(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, kv_idx, per_head, b)
    g1 = ob.omni_sparse_attn_bwd(c.desc, c.dQ, c.dK, c.dV, O1, dO, l1, q_idx, q_cnt, kv_idx, shared, b)
    g2 = ob.omni_sparse_attn_bwd_per_head(c.desc, c.dQ, c.dK, c.dV, O2, dO, l2, q_idx, q_cnt, kv_idx, per_head, b)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(l1, l2)
    for x, y in zip(g1, g2):
        assert torch.equal(x, y)


def test_visual_subset_per_head_matches_oracle():
    cfg = CFG_BF16
    c = case_for(cfg)
    bud = oc.kv_budget(c.o_a32, c.recall_p, 2)["budget"]
    kv_lists = oc.select_kv(c.o_a32, bud)
    cap = int(bud.max())
    kv_idx, budget = lists_to_padded(kv_lists, cfg.n_q_heads, cap)
    vis_idx, vis_cnt = ob.omni_visual_subset_per_head(c.desc, kv_idx, budget, cap)
    torch.cuda.synchronize()
    want = oc.visual_subset(kv_lists, cfg.vis_begin, cfg.vis_end)
    got = padded_to_lists(vis_idx, vis_cnt)
    for h in range(cfg.n_q_heads):
        np.testing.assert_array_equal(got[0][h], want[0][h])


def test_group_subset_per_head_is_the_union_of_the_ragged_lists_with_membership_bits():
    cfg = CFG_BF16
    c = case_for(cfg)
    H, Hkv = cfg.n_q_heads, cfg.n_kv_heads
    G = H // Hkv
    bud = oc.kv_budget(c.o_a32, c.recall_p, 2)["budget"]
    kv_lists = oc.select_kv(c.o_a32, bud)
    cap = int(bud.max())
    kv_idx, budget = lists_to_padded(kv_lists, H, cap)
    grp_idx, grp_mask, grp_cnt = ob.omni_group_subset_per_head(c.desc, kv_idx, budget, cap)
    torch.cuda.synchronize()
    vis = oc.visual_subset(kv_lists, cfg.vis_begin, cfg.vis_end)
    gi, gm, gc = to_host(grp_idx), to_host(grp_mask).view(np.uint32), to_host(grp_cnt)
    for g in range(Hkv):
        sets = [set(int(x) for x in vis[0][g * G + j]) for j in range(G)]
        union = sorted(set().union(*sets))
        n = int(gc[0, g])
        assert n == len(union)
        np.testing.assert_array_equal(gi[0, g, :n], np.array(union, dtype=np.int32))
        want = np.array([sum((1 << j) for j in range(G) if t in sets[j]) for t in union], dtype=np.uint32)
        np.testing.assert_array_equal(gm[0, g, :n], want)


@pytest.mark.parametrize("cfg", ALL_CFGS, ids=lambda c: c.name)
def test_free_running_per_head_pipeline_oracle_selection_on_the_gpu_scores_gives_the_gpu_sets(cfg):
    """Nothing teacher-forced on the GPU side: its own key scores, budgets and lists.  The oracle's per-head budgets and
    lists on those score arrays must be the GPU's bit for bit, and attention is compared on every head."""
    c = case_for(cfg)
    N, H = cfg.n_tokens, cfg.n_q_heads
    r = ob.omni_kv_budget(c.desc, c.dQ, c.dK, c.recall_p, c.probe_block, 2)
    kv_idx = ob.omni_select_kv_per_head(c.desc, r.key_scores, r.budget, N)
    q_idx, q_cnt = lists_to_padded(c.o_qidx, H, N)
    O, lse = ob.omni_sparse_attn_fwd_per_head(c.desc, c.dQ, c.dK, c.dV, q_idx, q_cnt, kv_idx, r.budget, N)
    torch.cuda.synchronize()
    a_gpu = to_host(r.key_scores)
    assert np.max(np.abs(a_gpu.astype(np.float64) - c.o_a32)) <= 1e-4 * c.o_a32.max()
    assert np.all(to_host(r.recall)[0] >= c.recall_p - 1e-4)   # every head meets the target with its own budget
    kv_lists = check_selection_on_gpu_scores(oc, c.o_scores32, a_gpu, c.o_qidx, to_host(r.flattest), to_host(r.budget),
                                             to_host(kv_idx), c.q_mode, c.q_param, c.recall_p, 2, cfg.vis_begin,
                                             cfg.vis_end)
    Oo, Lo = oc.sparse_attn_fwd(c.Q, c.K, c.V, c.o_qidx, kv_lists, cfg.causal, cfg.scale)
    Og, Lg = to_host(O), to_host(lse)
    assert np.max(np.abs(Og - Oo)) <= TOL_OUT[cfg.dtype]
    fin = np.isfinite(Lo)
    assert np.array_equal(np.isfinite(Lg), fin) and np.max(np.abs(Lg[fin] - Lo[fin])) <= 2e-3
