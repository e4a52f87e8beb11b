"""CPU oracle for the OmniSparse per-layer hot path.  TEST INFRASTRUCTURE ONLY.

This module is a plain, slow, obviously-correct numpy implementation (fp64
arithmetic) of what the HIP library computes.  It exists so that tests, the
smoke check and the benchmark's cpu_baseline leg have something independent to
compare against.  It shares no code with the HIP path, imports nothing from the
package, and must never be imported by the product path.

Every function follows a passage of the paper (arxiv 2511.12201); the passage
is named in the docstring.  Conventions used throughout:

  * Q is [B, Hq, N, d]; K and V are [B, Hkv, N, d]; query head i reads the K/V
    (and probe keys) of KV head i // (Hq // Hkv).  The paper writes plain
    multi-head attention; its backbones use grouped KV heads, so the grouping
    is this build's reading.
  * Heads are 0-based: the paper's "first attention head" is head 0.
  * Tokens [vis_begin, vis_end) are the visual tokens X_v; everything else is
    text (Sec. "Overview").  The attention sink is token `sink_index`.
  * Floating-point decisions that produce integers (threshold compares, top-b
    membership, the budget) are taken on float32 score arrays, because float32
    is the storage type of those arrays at the library boundary.  The scores
    themselves are computed here in fp64 and rounded once.
  * Inputs may be float32 arrays holding bf16-representable values; they are
    widened to fp64 and never re-rounded.

All functions are pinned by tests/test_oracle_*.py (run with -m "not gpu")
against closed forms, library routines, brute force and the paper's printed
table arithmetic.  Model-quality effects (the accuracy tables) are
"parity unpinned": they need weights and datasets that are not available.
"""
from __future__ import annotations

import math

import numpy as np

NEG_INF = -np.inf


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def _group(Hq: int, Hkv: int) -> int:
    if Hq % Hkv:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    return Hq // Hkv


# --------------------------------------------------------------------------
# Query selection as lazy/active classification
# --------------------------------------------------------------------------

def probe_keys(K, vis_begin: int, vis_end: int, sink_index: int = 0):
    """Lazy and active reference keys, one pair per KV head.

    Sec. "Query Selection as Binary Lazy-Active Classification": the lazy
    reference is the key of the attention sink (the first token); the active
    reference is the average of all visual keys.  Returns [B, Hkv, 2, d] fp64,
    row 0 = lazy, row 1 = active.
    """
    K = _f64(K)
    lazy = K[:, :, sink_index, :]
    act = K[:, :, vis_begin:vis_end, :].mean(axis=2)
    return np.stack([lazy, act], axis=2)


def score_queries(Q, probe, scale: float):
    """Active-class probability of every query (probe-softmax equation).

    softmax over the two logits q.k_lazy*scale and q.k_act*scale; the second
    column (active) is returned.  [B, Hq, N] fp64.
    """
    Q = _f64(Q)
    probe = _f64(probe)
    B, Hq, N, _ = Q.shape
    G = _group(Hq, probe.shape[1])
    out = np.empty((B, Hq, N))
    for b in range(B):
        for i in range(Hq):
            z = (Q[b, i] @ probe[b, i // G].T) * scale        # [N, 2]
            m = z.max(axis=1, keepdims=True)
            e = np.exp(z - m)
            out[b, i] = e[:, 1] / e.sum(axis=1)
    return out


def select_queries(scores_f32, mode: int, param: float, vis_begin: int, vis_end: int):
    """Kept-query index lists (query-mask equation).

    mode 0: a visual query is active iff its score is strictly greater than
            tau = param.
    mode 1: (extension used by the tiny configuration) the ceil(param * N_v)
            visual queries of highest score are active, equal scores resolved
            towards the lower token index.
    Head 0 keeps every query.  Non-visual (text) queries are never classified
    and always kept: the probe scores are defined on the N_v visual queries
    only.  Returns a list over batch of lists over heads of ascending int32
    index arrays.
    """
    s = np.asarray(scores_f32, dtype=np.float32)
    B, Hq, N = s.shape
    n = np.arange(N)
    is_vis = (n >= vis_begin) & (n < vis_end)
    n_vis = vis_end - vis_begin
    out = []
    for b in range(B):
        per_head = []
        for i in range(Hq):
            if i == 0:
                keep = np.ones(N, dtype=bool)
            elif mode == 0:
                keep = (~is_vis) | (s[b, i] > np.float32(param))
            elif mode == 1:
                want = min(n_vis, max(0, math.ceil(float(np.float32(param)) * n_vis)))
                vis_scores = s[b, i, vis_begin:vis_end]
                order = np.lexsort((np.arange(n_vis), -vis_scores.astype(np.float64)))
                keep = ~is_vis
                keep[vis_begin + order[:want]] = True
            else:
                raise ValueError("mode must be 0 or 1")
            per_head.append(np.nonzero(keep)[0].astype(np.int32))
        out.append(per_head)
    return out


# --------------------------------------------------------------------------
# KV selection with one budget set by the flattest head
# --------------------------------------------------------------------------

def exact_key_scores(Q, K, causal: bool, scale: float):
    """Accumulated attention score of every key from the full attention map.

    Sec. "KV Selection with Head-level Dynamic Budget Allocation": a_{i,k} is
    the attention mass key k receives summed over all queries; each row of the
    map is a softmax, so the scores of a head sum to N.  [B, Hq, N] fp64.
    Quadratic in N: for small inputs and fidelity checks only.
    """
    Q = _f64(Q)
    K = _f64(K)
    B, Hq, N, _ = Q.shape
    G = _group(Hq, K.shape[1])
    out = np.empty((B, Hq, N))
    tri = np.tril(np.ones((N, N), dtype=bool)) if causal else None
    for b in range(B):
        for i in range(Hq):
            S = (Q[b, i] @ K[b, i // G].T) * scale
            if causal:
                S = np.where(tri, S, NEG_INF)
            S = S - S.max(axis=1, keepdims=True)
            P = np.exp(S)
            P /= P.sum(axis=1, keepdims=True)
            out[b, i] = P.sum(axis=0)
    return out


def pooled_key_scores(Q, K, probe_block: int, causal: bool, scale: float):
    """Accumulated key scores from the block-wise probe.

    Sec. "Block-wise probing and sparse flash attention kernel": the attention
    map is approximated by pooling the queries along the sequence in blocks of
    `probe_block` tokens, over all queries (not only the selected ones).  Keys
    stay at token level here so that the budget is a token count.  Pooled row j
    stands for its w_j member queries: under the causal mask it sees the keys
    up to the last token of its block, and its softmax row is added with weight
    w_j, which keeps the identity sum_k a_{i,k} = N.  [B, Hq, N] fp64.
    """
    Q = _f64(Q)
    K = _f64(K)
    B, Hq, N, _ = Q.shape
    G = _group(Hq, K.shape[1])
    starts = np.arange(0, N, probe_block)
    ends = np.minimum(starts + probe_block, N)           # exclusive
    w = (ends - starts).astype(np.float64)
    cols = np.arange(N)
    out = np.empty((B, Hq, N))
    for b in range(B):
        for i in range(Hq):
            qbar = np.stack([Q[b, i, s:e].mean(axis=0) for s, e in zip(starts, ends)])
            S = (qbar @ K[b, i // G].T) * scale             # [nblk, N]
            if causal:
                S = np.where(cols[None, :] < ends[:, None], S, NEG_INF)
            S = S - S.max(axis=1, keepdims=True)
            P = np.exp(S)
            P /= P.sum(axis=1, keepdims=True)
            out[b, i] = (w[:, None] * P).sum(axis=0)
    return out


def pooled_block_scores(Q, K, block: int, causal: bool, scale: float):
    """Accumulated scores of key BLOCKS from the probe with queries and keys both pooled.

    Sec. "Block-wise probing and sparse flash attention kernel" as the paper runs
    it: queries and keys are mean-pooled along the sequence in blocks of `block`
    tokens and the pooled map stands in for the full one.  A key block m of c_m
    tokens enters query block j's softmax with weight c_m (c_m equal keys at the
    block mean), and under the causal mask j sees the key blocks m <= j.  Row j
    is added with weight w_j = its number of queries, so the block scores sum to
    N; they are returned divided by the mean block mass N / n_blocks, i.e. summing
    to n_blocks, which lets the budget rule (share p of the total) run on them
    unchanged with "length = total".  [B, Hq, n_blocks] fp64.
    """
    Q = _f64(Q)
    K = _f64(K)
    B, Hq, N, _ = Q.shape
    G = _group(Hq, K.shape[1])
    starts = np.arange(0, N, block)
    ends = np.minimum(starts + block, N)
    cnt = (ends - starts).astype(np.float64)
    nb = starts.size
    out = np.empty((B, Hq, nb))
    blk = np.arange(nb)
    for b in range(B):
        for i in range(Hq):
            qbar = np.stack([Q[b, i, s:e].mean(axis=0) for s, e in zip(starts, ends)])
            kbar = np.stack([K[b, i // G, s:e].mean(axis=0) for s, e in zip(starts, ends)])
            S = (qbar @ kbar.T) * scale                      # [nb, nb]
            if causal:
                S = np.where(blk[None, :] <= blk[:, None], S, NEG_INF)
            S = S - S.max(axis=1, keepdims=True)
            P = cnt[None, :] * np.exp(S)
            P /= P.sum(axis=1, keepdims=True)
            out[b, i] = (cnt[:, None] * P).sum(axis=0) * (nb / N)
    return out


def expand_blocks(blk_idx, block: int, n_tokens: int):
    """Token lists of selected key blocks: blk_idx[b][i] ascending block ids -> ascending token ids."""
    out = []
    for per_b in blk_idx:
        heads = []
        for ids in per_b:
            toks = [np.arange(int(m) * block, min((int(m) + 1) * block, n_tokens), dtype=np.int32) for m in ids]
            heads.append(np.concatenate(toks) if toks else np.zeros(0, dtype=np.int32))
        out.append(heads)
    return out


def kurtosis(a_f32):
    """Excess kurtosis m4 / m2^2 - 3 of each head's score vector, fp64.

    Same section: the attention sparsity of a head is measured by the kurtosis
    of its accumulated scores.  The population form is used; the sample-size
    corrections of the cited estimators are increasing functions of it at equal
    length, so the arg-min over heads is the same.  A constant vector (m2 = 0)
    gets -2, the lower bound of the statistic.  [B, Hq].
    """
    a = _f64(a_f32)
    mu = a.mean(axis=-1, keepdims=True)
    c = a - mu
    m2 = (c ** 2).mean(axis=-1)
    m4 = (c ** 4).mean(axis=-1)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = m4 / (m2 * m2) - 3.0
    return np.where(m2 > 0, r, -2.0)


FLATTEST_TIE_REL = 1e-9


def flattest_head(kurt):
    """Head with the smallest kurtosis (budget equation: arg-min over heads).  [B].

    The paper does not say which head wins among equals.  Heads whose kurtosis
    lies within FLATTEST_TIE_REL (relative) of the smallest count as tied and the
    lowest index wins.  The window matters for vectors of two or three scores,
    where the statistic is the same constant for every head (-2 and -1.5) and an
    exact arg-min would be decided by the rounding of the moment sums.
    """
    kurt = np.asarray(kurt, dtype=np.float64)
    lo = kurt.min(axis=-1, keepdims=True)
    tied = kurt <= lo + FLATTEST_TIE_REL * np.abs(lo)
    return np.argmax(tied, axis=-1).astype(np.int32)


def budget_of(a_head_f32, recall_p: float, n_queries: int) -> int:
    """Smallest b whose b largest scores sum to at least p * N (budget equation).

    The sum runs in fp64 over the float32 scores sorted in descending order.  If
    rounding keeps even the full sum below the target, b is the vector length.
    """
    a = np.sort(_f64(np.asarray(a_head_f32, dtype=np.float32)))[::-1]
    target = float(np.float32(recall_p)) * float(n_queries)
    c = np.cumsum(a)
    hit = np.nonzero(c >= target)[0]
    return int(hit[0]) + 1 if hit.size else int(a.size)


def kv_budget(a_f32, recall_p: float, budget_mode: int = 0):
    """Kurtosis, flattest head, shared budget and per-head recall.

    budget_mode 0 is the paper's rule: the budget of the flattest head, applied
    to every head.  budget_mode 1 takes the largest per-head budget instead,
    which meets the recall target on every head by construction (the paper
    asserts this of mode 0; it holds when the flattest head is also the one
    that needs the most keys).  budget_mode 2 gives every head the budget of
    its own scores: the alternative the paper's introduction and KV-selection
    section weigh against the shared budget and set aside for its cost; budget
    is then [B,Hq].  recall[i] is the mass of head i's own b (b_i in mode 2)
    largest scores divided by N.  Returns dict(kurtosis [B,Hq] f64, flattest
    [B] i32, budget [B] i32 (mode 2: [B,Hq]), recall [B,Hq] f64).
    """
    a = np.asarray(a_f32, dtype=np.float32)
    B, Hq, N = a.shape
    kurt = kurtosis(a)
    flat = flattest_head(kurt)
    budget = np.empty((B, Hq) if budget_mode == 2 else B, dtype=np.int32)
    recall = np.empty((B, Hq))
    for b in range(B):
        if budget_mode == 0:
            budget[b] = budget_of(a[b, flat[b]], recall_p, N)
        elif budget_mode == 1:
            budget[b] = max(budget_of(a[b, i], recall_p, N) for i in range(Hq))
        elif budget_mode == 2:
            for i in range(Hq):
                budget[b, i] = budget_of(a[b, i], recall_p, N)
        else:
            raise ValueError("budget_mode must be 0, 1 or 2")
        for i in range(Hq):
            bi = budget[b, i] if budget_mode == 2 else budget[b]
            top = np.sort(_f64(a[b, i]))[::-1][:bi]
            recall[b, i] = top.sum() / N
    return dict(kurtosis=kurt, flattest=flat, budget=budget, recall=recall)


def select_kv(a_f32, budget):
    """Per head, the b keys of largest accumulated score (key-mask equation).

    Exactly b keys per head: when several keys share the b-th largest value the
    ones of lower token index are taken.  The value mask equals the key mask.
    budget is [B] (one b per batch item, the paper's rule) or [B,Hq] (a budget
    per head).  Returns a list over batch of int32 arrays [Hq, b], ascending
    along b; with per-head budgets, a list over batch of lists over heads of
    int32 arrays [b_i].
    """
    a = np.asarray(a_f32, dtype=np.float32)
    B, Hq, N = a.shape
    budget = np.asarray(budget)
    out = []
    for b in range(B):
        rows = []
        for i in range(Hq):
            bb = int(budget[b, i] if budget.ndim == 2 else budget[b])
            order = np.lexsort((np.arange(N), -a[b, i].astype(np.float64)))
            rows.append(np.sort(order[:bb]).astype(np.int32))
        out.append(rows if budget.ndim == 2 else np.stack(rows).reshape(Hq, -1))
    return out


# --------------------------------------------------------------------------
# Attention: dense definition, sparse forward / backward, slimmed decode
# --------------------------------------------------------------------------

def dense_attention(Q, K, V, causal: bool, scale: float):
    """softmax(Q K^T * scale) V per head (Sec. "Preliminary", attention equation).

    Returns O [B,Hq,N,d] and LSE [B,Hq,N], fp64.
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, Hq, N, d = Q.shape
    G = _group(Hq, K.shape[1])
    O = np.empty((B, Hq, N, d))
    L = np.empty((B, Hq, N))
    tri = np.tril(np.ones((N, N), dtype=bool)) if causal else None
    for b in range(B):
        for i in range(Hq):
            S = (Q[b, i] @ K[b, i // G].T) * scale
            if causal:
                S = np.where(tri, S, NEG_INF)
            m = S.max(axis=1, keepdims=True)
            P = np.exp(S - m)
            l = P.sum(axis=1, keepdims=True)
            O[b, i] = (P / l) @ V[b, i // G]
            L[b, i] = (m + np.log(l))[:, 0]
    return O, L


def _masked_scores(q_rows, k_rows, q_idx, kv_idx, causal, scale):
    S = (q_rows @ k_rows.T) * scale
    if causal:
        S = np.where(kv_idx[None, :] <= q_idx[:, None], S, NEG_INF)
    return S


def sparse_attn_fwd(Q, K, V, q_idx, kv_idx, causal: bool, scale: float):
    """Attention restricted to kept queries and selected keys.

    Sec. "Preliminary" (token-level sparse attention with masks M^Q, M^K, M^V)
    and the closing sentence of the query-selection section (lazy queries are
    skipped).  For head i and kept query n the keys are those of S_i that the
    causal mask allows (index <= n); the softmax is renormalised over them.
    A skipped query, or a kept query with no allowed key, has output row 0 and
    LSE = -inf.  q_idx, kv_idx: per batch, per head, int index arrays in any
    order.  Returns O [B,Hq,N,d], LSE [B,Hq,N], fp64.
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, Hq, N, d = Q.shape
    G = _group(Hq, K.shape[1])
    O = np.zeros((B, Hq, N, d))
    L = np.full((B, Hq, N), NEG_INF)
    for b in range(B):
        for i in range(Hq):
            qi = np.asarray(q_idx[b][i], dtype=np.int64)
            ki = np.asarray(kv_idx[b][i], dtype=np.int64)
            if qi.size == 0 or ki.size == 0:
                continue
            g = i // G
            S = _masked_scores(Q[b, i, qi], K[b, g, ki], qi, ki, causal, scale)
            m = S.max(axis=1, keepdims=True)
            ok = np.isfinite(m[:, 0])
            m = np.where(np.isfinite(m), m, 0.0)
            P = np.exp(S - m)
            l = P.sum(axis=1, keepdims=True)
            with np.errstate(divide="ignore", invalid="ignore"):
                o = (P / l) @ V[b, g, ki]
                lse = (m + np.log(l))[:, 0]
            O[b, i, qi[ok]] = o[ok]
            L[b, i, qi[ok]] = lse[ok]
    return O, L


def sparse_attn_bwd(Q, K, V, dO, q_idx, kv_idx, causal: bool, scale: float, O=None):
    """Gradient of sparse_attn_fwd w.r.t. Q, K, V with the index sets constant.

    The paper applies the same sparse attention in training and gives no
    relaxation of the selection, so the sets carry no gradient.  The formulas
    are the chain rule on O = softmax(S) V:  dV = P^T dO, dP = dO V^T,
    dS = P * (dP - rowsum(dO * O)), dQ = dS K * scale, dK = dS^T Q * scale.
    dK and dV add up over the query heads that share a KV head.  Rows that are
    not kept / not selected are 0.  Returns dQ [B,Hq,N,d], dK, dV [B,Hkv,N,d].

    O [B,Hq,N,d], when given, is the forward's output as the layer stored it
    (rounded to the layer's type) and is what rowsum(dO * O) reads, as in a
    training step, where the backward is handed the stored output; without it
    the unrounded product P V is used.
    """
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    if O is not None:
        O = _f64(O)
    B, Hq, N, d = Q.shape
    Hkv = K.shape[1]
    G = _group(Hq, Hkv)
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for b in range(B):
        for i in range(Hq):
            qi = np.asarray(q_idx[b][i], dtype=np.int64)
            ki = np.asarray(kv_idx[b][i], dtype=np.int64)
            if qi.size == 0 or ki.size == 0:
                continue
            g = i // G
            S = _masked_scores(Q[b, i, qi], K[b, g, ki], qi, ki, causal, scale)
            m = S.max(axis=1, keepdims=True)
            ok = np.isfinite(m[:, 0])
            m = np.where(np.isfinite(m), m, 0.0)
            P = np.exp(S - m)
            l = P.sum(axis=1, keepdims=True)
            with np.errstate(divide="ignore", invalid="ignore"):
                P = np.where(ok[:, None], P / l, 0.0)
            do = dO[b, i, qi] * ok[:, None]
            o = P @ V[b, g, ki] if O is None else O[b, i, qi]
            dP = do @ V[b, g, ki].T
            delta = (do * o).sum(axis=1, keepdims=True)
            dS = P * (dP - delta)
            dQ[b, i, qi] = (dS @ K[b, g, ki]) * scale
            np.add.at(dK[b, g], ki, (dS.T @ Q[b, i, qi]) * scale)
            np.add.at(dV[b, g], ki, P.T @ do)
    return dQ, dK, dV


def sparse_attn_bwd_term_rss(Q, K, V, dO, q_idx, kv_idx, causal: bool, scale: float, O=None):
    """Root of the sum of squares of the products that add up to each gradient element.

    Every element of dQ, dK, dV is a sum of products (dS[n,k] K[k,e] scale over
    the keys of a row; dS[n,k] Q[n,e] scale and P[n,k] dO[n,e] over the kept
    queries of all heads of the group).  An implementation that rounds one
    factor of each product to t bits is off by about 2^-t times this root (the
    roundings are independent), whatever order it adds in, so the parity tests
    scale their bar for reduced-precision arithmetic with it.  Same arguments
    and same chain rule as sparse_attn_bwd; returns (rQ, rK, rV), shaped like
    (dQ, dK, dV), all >= 0.
    """
    Q, K, V, dO = _f64(Q), _f64(K), _f64(V), _f64(dO)
    if O is not None:
        O = _f64(O)
    B, Hq, N, d = Q.shape
    G = _group(Hq, K.shape[1])
    sQ = np.zeros_like(Q)
    sK = np.zeros_like(K)
    sV = np.zeros_like(V)
    for b in range(B):
        for i in range(Hq):
            qi = np.asarray(q_idx[b][i], dtype=np.int64)
            ki = np.asarray(kv_idx[b][i], dtype=np.int64)
            if qi.size == 0 or ki.size == 0:
                continue
            g = i // G
            S = _masked_scores(Q[b, i, qi], K[b, g, ki], qi, ki, causal, scale)
            m = S.max(axis=1, keepdims=True)
            ok = np.isfinite(m[:, 0])
            m = np.where(np.isfinite(m), m, 0.0)
            P = np.exp(S - m)
            l = P.sum(axis=1, keepdims=True)
            with np.errstate(divide="ignore", invalid="ignore"):
                P = np.where(ok[:, None], P / l, 0.0)
            do = dO[b, i, qi] * ok[:, None]
            o = P @ V[b, g, ki] if O is None else O[b, i, qi]
            dS = P * (do @ V[b, g, ki].T - (do * o).sum(axis=1, keepdims=True))
            sQ[b, i, qi] = ((dS ** 2) @ (K[b, g, ki] ** 2)) * scale ** 2
            np.add.at(sK[b, g], ki, ((dS ** 2).T @ (Q[b, i, qi] ** 2)) * scale ** 2)
            np.add.at(sV[b, g], ki, (P ** 2).T @ (do ** 2))
    return np.sqrt(sQ), np.sqrt(sK), np.sqrt(sV)


def visual_subset(kv_idx, vis_begin: int, vis_end: int):
    """The selected keys that are visual tokens, per head, ascending.

    Sec. "KV Cache Slimming": the selected KV pairs are stored at token level
    with the same budget b for every head; decode treats text and answer KV
    densely, so only the visual part of each head's set is kept as a list.
    """
    out = []
    for per_head in kv_idx:
        out.append([np.sort(h[(h >= vis_begin) & (h < vis_end)]).astype(np.int32) for h in per_head])
    return out


def slim_decode(q, Kc, Vc, ctx_len, probe, vis_idx, tau: float,
                vis_begin: int, vis_end: int, scale: float):
    """One decode step with KV cache slimming (decoding-attention equation).

    Per head the decoding query is scored against the stored probe keys exactly
    like a prefill query; it is active iff score > tau or the head is head 0.
    An active head attends its stored visual keys, a lazy head none; every head
    attends all non-visual cache rows below ctx_len (text and decoded answer).
    q [B,Hq,d]; Kc, Vc [B,Hkv,cap,d]; ctx_len [B]; probe [B,Hkv,2,d];
    vis_idx per batch per head.  Returns O [B,Hq,d] fp64, active [B,Hq] uint8,
    score [B,Hq] fp64.
    """
    q, Kc, Vc, probe = _f64(q), _f64(Kc), _f64(Vc), _f64(probe)
    B, Hq, d = q.shape
    G = _group(Hq, Kc.shape[1])
    O = np.zeros((B, Hq, d))
    act = np.zeros((B, Hq), dtype=np.uint8)
    sc = score_queries(q[:, :, None, :], probe, scale)[:, :, 0]
    for b in range(B):
        L = int(ctx_len[b])
        dense_part = np.concatenate([np.arange(0, min(vis_begin, L)), np.arange(min(vis_end, L), L)])
        for i in range(Hq):
            g = i // G
            a = (i == 0) or (np.float32(sc[b, i]) > np.float32(tau))
            act[b, i] = 1 if a else 0
            vis = np.asarray(vis_idx[b][i], dtype=np.int64)
            vis = vis[vis < L]
            keys = np.concatenate([vis, dense_part]) if a else dense_part
            keys = keys.astype(np.int64)
            if keys.size == 0:
                continue
            s = (Kc[b, g, keys] @ q[b, i]) * scale
            p = np.exp(s - s.max())
            p /= p.sum()
            O[b, i] = p @ Vc[b, g, keys]
    return O, act, sc


def dense_decode(q, Kc, Vc, ctx_len, scale: float):
    """Plain decode attention over cache rows [0, ctx_len) (attention equation)."""
    q, Kc, Vc = _f64(q), _f64(Kc), _f64(Vc)
    B, Hq, d = q.shape
    G = _group(Hq, Kc.shape[1])
    O = np.zeros((B, Hq, d))
    for b in range(B):
        L = int(ctx_len[b])
        for i in range(Hq):
            g = i // G
            s = (Kc[b, g, :L] @ q[b, i]) * scale
            p = np.exp(s - s.max())
            p /= p.sum()
            O[b, i] = p @ Vc[b, g, :L]
    return O


# --------------------------------------------------------------------------
# Work accounting (used for the reported FLOP figures)
# --------------------------------------------------------------------------

def count_pairs(q_idx, kv_idx, causal: bool) -> int:
    """Number of (query, key) pairs the sparse attention evaluates.

    Attention FLOPs are 4 * d * pairs.  The paper's ablation table is
    consistent with lazy queries costing nothing and the cost being the product
    of kept queries and selected keys (without the causal mask).
    """
    total = 0
    for per_q, per_k in zip(q_idx, kv_idx):
        for qi, ki in zip(per_q, per_k):
            qi = np.asarray(qi, dtype=np.int64)
            ki = np.sort(np.asarray(ki, dtype=np.int64))
            if causal:
                total += int(np.searchsorted(ki, qi, side="right").sum())
            else:
                total += int(qi.size) * int(ki.size)
    return total
