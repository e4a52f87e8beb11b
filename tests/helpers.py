"""Shared helpers for the GPU parity tests: host<->device marshalling and set comparison."""
from __future__ import annotations

import numpy as np
import torch

from paper_2511_12201_amd import synth


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 host array -> device tensor of the layer dtype (bf16 arrays must lie on the bf16 grid)."""
    if dtype == "bf16":
        return torch.from_numpy(synth.bf16_bits(x)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.detach().float().cpu().numpy()
    return t.detach().cpu().numpy()


def lists_to_padded(lists, n_heads: int, width: int):
    """list[batch][head] of index arrays -> (idx [B,H,width] int32 device, cnt [B,H] int32 device)."""
    B = len(lists)
    idx = np.zeros((B, n_heads, width), dtype=np.int32)
    cnt = np.zeros((B, n_heads), dtype=np.int32)
    for b in range(B):
        for h in range(n_heads):
            a = np.asarray(lists[b][h], dtype=np.int32)
            idx[b, h, : a.size] = a
            cnt[b, h] = a.size
    return torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda()


def padded_to_lists(idx: torch.Tensor, cnt: torch.Tensor):
    idx, cnt = idx.cpu().numpy(), cnt.cpu().numpy()
    return [[idx[b, h, : cnt[b, h]].copy() for h in range(idx.shape[1])] for b in range(idx.shape[0])]


def near_cut_only(got: np.ndarray, want: np.ndarray, values: np.ndarray, cut: float, rel: float) -> bool:
    """True iff every index in the symmetric difference has a value within rel of the cut."""
    diff = np.setxor1d(got, want)
    if diff.size == 0:
        return True
    return bool(np.all(np.abs(values[diff].astype(np.float64) - cut) <= rel * max(abs(cut), 1e-30)))


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of the bf16 grid (8 significant bits) at |x|; 0 where x is 0."""
    ax = np.abs(np.asarray(x, dtype=np.float64))
    e = np.floor(np.log2(np.where(ax > 0, ax, 1.0)))
    return np.where(ax > 0, np.exp2(e - 7), 0.0)


# bf16 gradients: the matrix cores take P and dS rounded to 8 significant bits (relative error up to 2^-9, independent
# from product to product), so a gradient element -- a sum of products with one rounded factor each -- is off by about
# 0.5 * 2^-9 * rss, rss = root of the sum of the squared products (the oracle computes it), whatever the summation
# order; the largest of ~10^6 elements reaches 4 of those in a CPU emulation of the roundings.  GRAD_RSS = 6 * 2^-9
# leaves half as much again.  Storing the result in bf16 adds half a spacing of the bf16 grid at the reference value.
GRAD_RSS = 6 * 2.0 ** -9


def grad_bar(ref: np.ndarray, dtype: str, rss: np.ndarray | None = None) -> np.ndarray:
    """Element-wise max-abs bar for gradients: 1e-4 (fp32); bf16: 2e-2, or where that is larger the rounding scale
    of the element, GRAD_RSS * rss + half a bf16 spacing at |ref| (without rss: one spacing)."""
    if dtype != "bf16":
        return np.full(np.shape(ref), 1e-4)
    if rss is None:
        return np.maximum(2e-2, bf16_ulp(ref))
    return np.maximum(2e-2, GRAD_RSS * rss + 0.5 * bf16_ulp(ref))


def budget_window_ok(a_head32: np.ndarray, b: int, p: float, n_queries: int, rel: float = 1e-6) -> bool:
    """b is a smallest count reaching mass p*N on this score vector, up to `rel` on the fp64 cumulative sums."""
    srt = np.sort(np.asarray(a_head32, dtype=np.float32).astype(np.float64))[::-1]
    cum = np.cumsum(srt)
    target = float(np.float32(p)) * n_queries
    reached = cum[b - 1] >= target * (1 - rel) or b == srt.size
    minimal = b == 1 or cum[b - 2] < target * (1 + rel)
    return bool(reached and minimal)


def check_selection_on_gpu_scores(oc, scores_gpu, key_scores_gpu, q_lists_gpu, flattest_gpu, budget_gpu, kv_idx_gpu,
                                  q_mode, q_param, recall_p, budget_mode, vis_begin, vis_end):
    """The oracle's selection run on the score arrays the GPU produced must give the GPU's sets bit for bit.

    scores_gpu, key_scores_gpu [B,Hq,N] float32 (host copies of the device arrays); q_lists_gpu list[b][h];
    flattest_gpu [B]; budget_gpu [B] or [B,Hq]; kv_idx_gpu [B,Hq,b_cap] host array.  The flattest head may differ
    only when the oracle's two smallest kurtoses lie within 1e-9 (relative) of each other, the budget only inside
    the 1e-6 window of the fp64 cumulative sums; the index lists must then still be the oracle's for the GPU's own
    head and budget.  Returns the key lists (list[b][h]) for the attention check.
    """
    B, H, N = key_scores_gpu.shape
    want_q = oc.select_queries(scores_gpu, q_mode, q_param, vis_begin, vis_end)
    for b in range(B):
        for h in range(H):
            np.testing.assert_array_equal(q_lists_gpu[b][h], want_q[b][h], err_msg=f"query set, batch {b} head {h}")
    want = oc.kv_budget(key_scores_gpu, recall_p, budget_mode)
    budget_gpu = np.asarray(budget_gpu)
    kv_lists = []
    for b in range(B):
        f = int(flattest_gpu[b])
        if f != int(want["flattest"][b]):
            k = want["kurtosis"][b]
            assert abs(k[f] - k.min()) <= 1e-9 * abs(k.min()), f"flattest head {f}, oracle {want['flattest'][b]}"
        per_head = []
        for h in range(H):
            if budget_mode == 2:
                bg, bo, src = int(budget_gpu[b, h]), int(want["budget"][b, h]), h
            elif budget_mode == 0:
                bg, bo, src = int(budget_gpu[b]), int(oc.budget_of(key_scores_gpu[b, f], recall_p, N)), f
            else:
                bg, bo, src = int(budget_gpu[b]), int(want["budget"][b]), None
            if bg != bo:
                assert src is not None and budget_window_ok(key_scores_gpu[b, src], bg, recall_p, N), \
                    f"budget {bg}, oracle {bo} (batch {b} head {h})"
            lists = oc.select_kv(key_scores_gpu[b:b + 1, h:h + 1], np.array([bg]))[0][0]
            np.testing.assert_array_equal(kv_idx_gpu[b, h, :bg], lists, err_msg=f"kv set, batch {b} head {h}")
            per_head.append(np.asarray(lists, dtype=np.int32))
        kv_lists.append(per_head)
    return kv_lists


def stored(x: np.ndarray, dtype: str) -> np.ndarray:
    """An fp64 result as a layer of this dtype stores it (float32 array; bf16 layers: on the bf16 grid)."""
    x32 = np.asarray(x, dtype=np.float32)
    return synth.round_to_bf16(x32) if dtype == "bf16" else x32


class Grads(tuple):
    """(dQ, dK, dV) of the oracle with .rss = the root-sum-square of each element's products (for grad_bar)."""
    rss = None


def oracle_train(oc, dtype, Q, K, V, dO, q_lists, kv_lists, causal, scale):
    """The oracle's forward as the layer stores it, and the gradients of a backward that is handed that output:
    (O_stored float32, lse float32, Grads).  The GPU backward is run on the same O and lse, so that both sides are
    the same function of the same inputs (rowsum(dO * O) reads the stored, rounded O on both)."""
    Oo, Lo = oc.sparse_attn_fwd(Q, K, V, q_lists, kv_lists, causal, scale)
    O_st = stored(Oo, dtype)
    want = Grads(oc.sparse_attn_bwd(Q, K, V, dO, q_lists, kv_lists, causal, scale, O=O_st))
    if dtype == "bf16":
        want.rss = oc.sparse_attn_bwd_term_rss(Q, K, V, dO, q_lists, kv_lists, causal, scale, O=O_st)
    return O_st, Lo.astype(np.float32), want
