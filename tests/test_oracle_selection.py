"""Pins for the oracle's query scoring / selection and KV budget / selection (CPU only)."""
import itertools
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

from oracle import omni_oracle as oc
from paper_2511_12201_amd import synth


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ------------------------------------------------------------------ probe keys and scores

def test_probe_keys_are_sink_and_visual_mean():
    K = _rand((2, 3, 17, 8), 0)
    pk = oc.probe_keys(K, 2, 11, sink_index=1)
    assert pk.shape == (2, 3, 2, 8)
    np.testing.assert_array_equal(pk[:, :, 0], K[:, :, 1])
    manual = sum(K[:, :, n] for n in range(2, 11)) / 9.0
    np.testing.assert_allclose(pk[:, :, 1], manual, rtol=0, atol=1e-15)
    # one visual token: the active key is that key
    np.testing.assert_array_equal(oc.probe_keys(K, 5, 6)[:, :, 1], K[:, :, 5])


def test_scores_closed_form_sigmoid_and_library_softmax():
    B, Hq, Hkv, N, d = 2, 6, 2, 33, 16
    Q = _rand((B, Hq, N, d), 1)
    K = _rand((B, Hkv, N, d), 2)
    scale = 1.0 / math.sqrt(d)
    pk = oc.probe_keys(K, 3, 30)
    s = oc.score_queries(Q, pk, scale)
    G = Hq // Hkv
    for b in range(B):
        for i in range(Hq):
            zl = Q[b, i] @ pk[b, i // G, 0] * scale
            za = Q[b, i] @ pk[b, i // G, 1] * scale
            # two-way softmax == logistic of the logit difference
            np.testing.assert_allclose(s[b, i], scipy.special.expit(za - zl), rtol=1e-12, atol=1e-15)
            lib = torch.softmax(torch.tensor(np.stack([zl, za], 1)), dim=1)[:, 1].numpy()
            np.testing.assert_allclose(s[b, i], lib, rtol=1e-12, atol=1e-15)
    # the wrong column (lazy) or the wrong KV head must not pass
    assert not np.allclose(s, 1.0 - s)


def test_scores_special_cases():
    d = 8
    Q = _rand((1, 2, 9, d), 3)
    K = _rand((1, 1, 9, d), 4)
    pk = oc.probe_keys(K, 0, 9)
    pk[:, :, 1] = pk[:, :, 0]                        # equal references: no preference
    np.testing.assert_allclose(oc.score_queries(Q, pk, 0.3), 0.5, atol=1e-15)
    pk = oc.probe_keys(K, 0, 9)
    np.testing.assert_allclose(oc.score_queries(np.zeros_like(Q), pk, 0.3), 0.5, atol=1e-15)
    # a query equal to a large multiple of (k_act - k_lazy) is active with probability ~1
    diff = pk[0, 0, 1] - pk[0, 0, 0]
    Q2 = np.tile(50.0 * diff, (1, 2, 9, 1))
    assert oc.score_queries(Q2, pk, 0.3).min() > 0.999


def test_scores_large_logits_do_not_overflow():
    Q = np.full((1, 1, 2, 4), 300.0)
    pk = np.zeros((1, 1, 2, 4))
    pk[0, 0, 0] = 5.0
    pk[0, 0, 1] = -5.0
    s = oc.score_queries(Q, pk, 1.0)
    assert np.all(np.isfinite(s)) and np.all(s < 1e-300 + 1e-12)


# ------------------------------------------------------------------ query selection

def test_select_queries_threshold_limits_and_strictness():
    sc = np.random.default_rng(5).random((2, 4, 40)).astype(np.float32)
    v0, v1 = 4, 30
    allkept = oc.select_queries(sc, 0, 0.0, v0, v1)       # scores are > 0
    for b in range(2):
        for i in range(4):
            np.testing.assert_array_equal(allkept[b][i], np.arange(40))
    none = oc.select_queries(sc, 0, 1.0, v0, v1)
    text = np.concatenate([np.arange(0, v0), np.arange(v1, 40)])
    for b in range(2):
        np.testing.assert_array_equal(none[b][0], np.arange(40))       # first head keeps everything
        for i in range(1, 4):
            np.testing.assert_array_equal(none[b][i], text)            # text queries are never dropped
    # strict inequality: a score equal to tau is lazy
    sc2 = np.full((1, 2, 6), 0.25, dtype=np.float32)
    sc2[0, 1, 3] = np.nextafter(np.float32(0.25), np.float32(1))
    out = oc.select_queries(sc2, 0, 0.25, 0, 6)
    np.testing.assert_array_equal(out[0][1], [3])
    np.testing.assert_array_equal(out[0][0], np.arange(6))


def test_select_queries_threshold_matches_bruteforce():
    rng = np.random.default_rng(6)
    sc = rng.random((1, 3, 25)).astype(np.float32)
    tau = 0.4
    out = oc.select_queries(sc, 0, tau, 5, 20)
    for i in range(1, 3):
        want = [n for n in range(25) if not (5 <= n < 20) or sc[0, i, n] > np.float32(tau)]
        assert out[0][i].tolist() == want
        assert out[0][i].dtype == np.int32


def test_select_queries_top_fraction_count_ties_and_bruteforce():
    rng = np.random.default_rng(7)
    sc = rng.integers(0, 5, (1, 3, 31)).astype(np.float32) / 8.0     # many ties
    v0, v1, rho = 3, 27, 0.3
    out = oc.select_queries(sc, 1, rho, v0, v1)
    want_cnt = math.ceil(rho * (v1 - v0))
    for i in range(1, 3):
        kept = out[0][i]
        vis_kept = [n for n in kept if v0 <= n < v1]
        assert len(vis_kept) == want_cnt
        assert all(n in kept for n in list(range(0, v0)) + list(range(v1, 31)))
        # brute force: sort (score desc, index asc) by hand
        order = sorted(range(v0, v1), key=lambda n: (-sc[0, i, n], n))[:want_cnt]
        assert sorted(order) == vis_kept
        assert list(kept) == sorted(kept)
    np.testing.assert_array_equal(out[0][0], np.arange(31))


# ------------------------------------------------------------------ accumulated key scores

def test_exact_key_scores_match_library_softmax_column_sums():
    B, Hq, Hkv, N, d = 1, 4, 2, 23, 8
    Q, K = _rand((B, Hq, N, d), 8), _rand((B, Hkv, N, d), 9)
    for causal in (True, False):
        a = oc.exact_key_scores(Q, K, causal, 0.35)
        for i in range(Hq):
            S = torch.tensor(Q[0, i] @ K[0, i // 2].T * 0.35)
            if causal:
                S = S.masked_fill(~torch.tril(torch.ones(N, N, dtype=torch.bool)), float("-inf"))
            ref = torch.softmax(S, dim=1).sum(dim=0).numpy()        # mass RECEIVED by each key
            np.testing.assert_allclose(a[0, i], ref, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(a.sum(-1), N, rtol=1e-12)
    # causal: the last key is seen only by the last query, the first key by all
    a = oc.exact_key_scores(Q, K, True, 0.35)
    assert np.all(a[..., -1] < 1.0) and np.all(a[..., 0] > a[..., -1])


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("block", [1, 4, 7, 64])
def test_pooled_key_scores_sum_to_number_of_queries(block, causal):
    Q, K = _rand((2, 4, 29, 8), 10), _rand((2, 2, 29, 8), 11)
    a = oc.pooled_key_scores(Q, K, block, causal, 0.3)
    np.testing.assert_allclose(a.sum(-1), 29.0, rtol=1e-12)
    assert np.all(a >= 0)


@pytest.mark.parametrize("causal", [True, False])
def test_pooled_probe_with_block_one_is_the_exact_map(causal):
    Q, K = _rand((1, 4, 19, 8), 12), _rand((1, 2, 19, 8), 13)
    np.testing.assert_allclose(oc.pooled_key_scores(Q, K, 1, causal, 0.4),
                               oc.exact_key_scores(Q, K, causal, 0.4), rtol=1e-12, atol=1e-14)


def test_pooled_probe_uniform_keys_closed_form():
    # identical keys: every pooled row spreads its weight evenly over the keys it sees
    N, blk = 11, 4
    Q = _rand((1, 1, N, 4), 14)
    K = np.tile(_rand((1, 1, 1, 4), 15), (1, 1, N, 1))
    a = oc.pooled_key_scores(Q, K, blk, True, 1.0)[0, 0]
    ends = [4, 8, 11]
    w = [4, 4, 3]
    want = np.array([sum(wj / e for wj, e in zip(w, ends) if k < e) for k in range(N)])
    np.testing.assert_allclose(a, want, rtol=1e-13)
    a_nc = oc.pooled_key_scores(Q, K, blk, False, 1.0)[0, 0]
    np.testing.assert_allclose(a_nc, 1.0, rtol=1e-13)


def test_pooled_probe_uses_mean_query_and_group_key_head():
    # one block covering everything, non causal: a = N * softmax(mean(q) . K)
    Q, K = _rand((1, 2, 6, 4), 16), _rand((1, 2, 6, 4), 17)
    a = oc.pooled_key_scores(Q, K, 6, False, 0.5)
    for i in range(2):
        z = torch.tensor(K[0, i] @ Q[0, i].mean(0) * 0.5)
        np.testing.assert_allclose(a[0, i], 6 * torch.softmax(z, 0).numpy(), rtol=1e-12)


# ------------------------------------------------------------------ probe with pooled queries AND keys (block granular)

@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("block", [1, 4, 7, 64])
def test_block_scores_sum_to_number_of_blocks(block, causal):
    Q, K = _rand((2, 4, 29, 8), 40), _rand((2, 2, 29, 8), 41)
    a = oc.pooled_block_scores(Q, K, block, causal, 0.3)
    nb = math.ceil(29 / block)
    assert a.shape == (2, 4, nb)
    np.testing.assert_allclose(a.sum(-1), float(nb), rtol=1e-12)
    assert np.all(a >= 0)


@pytest.mark.parametrize("causal", [True, False])
def test_block_probe_with_block_one_is_the_exact_map(causal):
    Q, K = _rand((1, 4, 19, 8), 42), _rand((1, 2, 19, 8), 43)
    np.testing.assert_allclose(oc.pooled_block_scores(Q, K, 1, causal, 0.4),
                               oc.exact_key_scores(Q, K, causal, 0.4), rtol=1e-12, atol=1e-14)


def test_block_probe_uniform_keys_closed_form():
    # identical keys: query block j spreads its w_j queries over the visible key blocks in proportion to their sizes
    N, blk = 11, 4
    Q = _rand((1, 1, N, 4), 44)
    K = np.tile(_rand((1, 1, 1, 4), 45), (1, 1, N, 1))
    a = oc.pooled_block_scores(Q, K, blk, True, 1.0)[0, 0]
    c = [4, 4, 3]
    seen = [4, 8, 11]                                     # tokens in the key blocks m <= j
    mass = np.array([sum(c[j] * c[m] / seen[j] for j in range(3) if m <= j) for m in range(3)])
    np.testing.assert_allclose(a, mass * 3 / N, rtol=1e-13)
    a_nc = oc.pooled_block_scores(Q, K, blk, False, 1.0)[0, 0]
    np.testing.assert_allclose(a_nc, np.array(c) * 3 / N, rtol=1e-13)


def test_block_probe_is_softmax_of_pooled_logits():
    # equal blocks, non causal: mass of key block m = sum_j w_j softmax_m(qbar_j . kbar_m)
    Q, K = _rand((1, 2, 12, 4), 46), _rand((1, 1, 12, 4), 47)
    a = oc.pooled_block_scores(Q, K, 4, False, 0.5)
    for i in range(2):
        qb = Q[0, i].reshape(3, 4, 4).mean(1)
        kb = K[0, 0].reshape(3, 4, 4).mean(1)
        P = torch.softmax(torch.tensor(qb @ kb.T * 0.5), dim=1).numpy()
        np.testing.assert_allclose(a[0, i], (4 * P).sum(0) * 3 / 12, rtol=1e-12)


def test_expand_blocks_gives_ascending_token_ranges():
    out = oc.expand_blocks([[np.array([0, 2]), np.array([2]), np.array([], dtype=np.int32)]], 4, 11)
    np.testing.assert_array_equal(out[0][0], [0, 1, 2, 3, 8, 9, 10])
    np.testing.assert_array_equal(out[0][1], [8, 9, 10])
    assert out[0][2].size == 0


# ------------------------------------------------------------------ kurtosis / flattest head

def test_kurtosis_matches_library_and_known_values():
    a = np.abs(_rand((2, 5, 101), 18)).astype(np.float32)
    k = oc.kurtosis(a)
    ref = scipy.stats.kurtosis(a.astype(np.float64), axis=-1, fisher=True, bias=True)
    np.testing.assert_allclose(k, ref, rtol=1e-10)
    two_point = np.array([[[1.0, 3.0] * 10]], dtype=np.float32)
    np.testing.assert_allclose(oc.kurtosis(two_point), -2.0, atol=1e-12)
    const = np.ones((1, 1, 8), dtype=np.float32)
    assert oc.kurtosis(const)[0, 0] == -2.0
    g = np.random.default_rng(19).standard_normal((1, 1, 200000)).astype(np.float32)
    assert abs(oc.kurtosis(g)[0, 0]) < 0.05
    # invariant to positive affine maps
    np.testing.assert_allclose(oc.kurtosis(a * 7.0 + 2.0), k, rtol=1e-5)


def test_flattest_head_is_argmin_with_lowest_index_on_ties_and_estimators_agree():
    kurt = np.array([[3.0, 1.0, 1.0, 2.0], [0.5, 4.0, 0.7, 0.5]])
    np.testing.assert_array_equal(oc.flattest_head(kurt), [1, 0])
    # the bias-corrected estimator of the cited comparison orders heads identically
    a = np.abs(_rand((1, 9, 64), 20)) ** 3
    g2 = oc.kurtosis(a)[0]
    G2 = scipy.stats.kurtosis(a[0], axis=-1, fisher=True, bias=False)
    assert np.argmin(g2) == np.argmin(G2)
    assert oc.flattest_head(oc.kurtosis(a))[0] == np.argmin(g2)
    # a flat head has lower kurtosis than a peaked one
    flat = np.ones(64) + 0.01 * np.arange(64)
    peak = np.ones(64) * 0.1
    peak[5] = 50.0
    assert oc.flattest_head(oc.kurtosis(np.stack([peak, flat])[None]))[0] == 1


def test_flattest_head_ties_within_the_window_go_to_the_lowest_index():
    # two and three scores: the statistic is -2 and -3/2 whatever the values (for deviations that sum to zero,
    # sum c^4 = (sum c^2)^2 / 2 when there are three of them), so every head ties and head 0 is taken
    rng = np.random.default_rng(77)
    for n, const in ((2, -2.0), (3, -1.5)):
        for _ in range(50):
            a = rng.uniform(0.01, 3.0, (2, 6, n)).astype(np.float32)
            k = oc.kurtosis(a)
            np.testing.assert_allclose(k, const, rtol=0, atol=1e-12)
            np.testing.assert_array_equal(oc.flattest_head(k), [0, 0])
    # inside the window the lowest index wins, outside it the smaller value does
    np.testing.assert_array_equal(oc.flattest_head(np.array([[1.0 + 5e-10, 1.0, 1.0 - 1e-12]])), [0])
    np.testing.assert_array_equal(oc.flattest_head(np.array([[1.0 + 1e-6, 1.0, 1.0 + 1e-12]])), [1])
    np.testing.assert_array_equal(oc.flattest_head(np.array([[-1.5 + 1e-6, -1.5 - 2e-16, -1.5]])), [1])


# ------------------------------------------------------------------ budget

def _brute_budget(a, p, n):
    a = np.asarray(a, dtype=np.float64)
    target = float(np.float32(p)) * n
    for b in range(1, a.size + 1):
        best = max(sum(c) for c in itertools.combinations(a, b)) if a.size <= 10 else np.sort(a)[::-1][:b].sum()
        if best >= target:
            return b
    return a.size


def test_budget_is_minimal_bruteforce():
    rng = np.random.default_rng(21)
    for trial in range(20):
        n = int(rng.integers(3, 10))
        a = rng.random(n).astype(np.float32)
        a *= np.float32(n / a.sum())
        p = float(rng.choice([0.2, 0.5, 0.82, 0.95]))
        b = oc.budget_of(a, p, n)
        assert b == _brute_budget(a, p, n)
        srt = np.sort(a.astype(np.float64))[::-1]
        assert srt[:b].sum() >= float(np.float32(p)) * n
        assert b == 1 or srt[: b - 1].sum() < float(np.float32(p)) * n


def test_budget_limits():
    a = np.array([4.0, 1.0, 1.0, 1.0, 1.0], dtype=np.float32)      # sums to 8 = N
    assert oc.budget_of(a, 0.5, 8) == 1                              # 4 >= 4: compare is >=
    assert oc.budget_of(a, 0.51, 8) == 2
    assert oc.budget_of(a, 1.0, 8) == 5
    assert oc.budget_of(a, 1.0, 9) == 5                              # unreachable target -> all keys


def test_kv_budget_modes_and_recall():
    cfg = synth.C2_16K.scaled(frames=4, n_text=16, n_q_heads=8, n_kv_heads=2, head_dim=32)
    L = synth.make_layer(cfg)
    a = oc.pooled_key_scores(L["Q"], L["K"], 64, True, cfg.scale).astype(np.float32)
    N = cfg.n_tokens
    for p in (0.5, 0.82, 0.95):
        r0 = oc.kv_budget(a, p, 0)
        r1 = oc.kv_budget(a, p, 1)
        f = int(r0["flattest"][0])
        assert f == int(np.argmin(r0["kurtosis"][0]))
        assert r0["budget"][0] == oc.budget_of(a[0, f], p, N)
        # the flattest head always meets the target; mode 1 meets it on every head
        assert r0["recall"][0, f] >= float(np.float32(p)) - 1e-12
        assert np.all(r1["recall"][0] >= float(np.float32(p)) - 1e-12)
        assert r1["budget"][0] >= r0["budget"][0]
        per_head = [oc.budget_of(a[0, i], p, N) for i in range(cfg.n_q_heads)]
        assert r1["budget"][0] == max(per_head)
        # recall is the mass of the head's own top-b
        for i in range(cfg.n_q_heads):
            top = np.sort(a[0, i].astype(np.float64))[::-1][: r0["budget"][0]].sum() / N
            assert abs(top - r0["recall"][0, i]) < 1e-12


def test_shared_budget_meets_recall_on_every_head_of_the_synthetic_layer():
    # the generator makes head 0 clearly the flattest; the paper's rule then covers all heads
    cfg = synth.C2_16K.scaled(frames=8, n_text=32)
    L = synth.make_layer(cfg)
    a = oc.pooled_key_scores(L["Q"], L["K"], 256, True, cfg.scale).astype(np.float32)
    r = oc.kv_budget(a, 0.95, 0)
    assert r["flattest"][0] == 0
    assert np.all(r["recall"][0] >= float(np.float32(0.95)) - 1e-9)
    assert 0.05 * cfg.n_tokens < r["budget"][0] < 0.8 * cfg.n_tokens


def test_per_head_budgets_are_each_minimal_and_bracket_the_shared_ones():
    # budget_mode 2: every head gets the smallest prefix of its own sorted scores
    # that reaches p*N (brute force), so each head meets the target and no head
    # could drop a key; modes 0 and 1 are one entry / the maximum of that row
    cfg = synth.C2_16K.scaled(frames=4, n_text=16, n_q_heads=8, n_kv_heads=2, head_dim=32)
    L = synth.make_layer(cfg)
    a = oc.pooled_key_scores(L["Q"], L["K"], 64, True, cfg.scale).astype(np.float32)
    N = cfg.n_tokens
    for p in (0.5, 0.82, 0.95):
        r2 = oc.kv_budget(a, p, 2)
        assert r2["budget"].shape == (1, cfg.n_q_heads) and r2["budget"].dtype == np.int32
        target = float(np.float32(p)) * N
        for i in range(cfg.n_q_heads):
            bi = int(r2["budget"][0, i])
            assert bi == _brute_budget(a[0, i], p, N)
            srt = np.sort(a[0, i].astype(np.float64))[::-1]
            assert srt[:bi].sum() >= target
            assert bi == 1 or srt[: bi - 1].sum() < target
            assert abs(srt[:bi].sum() / N - r2["recall"][0, i]) < 1e-12
        assert np.all(r2["recall"][0] >= float(np.float32(p)) - 1e-12)
        r0 = oc.kv_budget(a, p, 0)
        r1 = oc.kv_budget(a, p, 1)
        assert r0["budget"][0] == r2["budget"][0, int(r0["flattest"][0])]
        assert r1["budget"][0] == r2["budget"][0].max()
        np.testing.assert_array_equal(r2["kurtosis"], r0["kurtosis"])
    with pytest.raises(ValueError):
        oc.kv_budget(a, 0.5, 3)


def test_select_kv_with_per_head_budgets_is_ragged_and_matches_the_shared_rule_per_head():
    rng = np.random.default_rng(27)
    a = rng.random((2, 3, 9)).astype(np.float32)
    budget = np.array([[1, 9, 4], [3, 3, 0]], dtype=np.int32)
    out = oc.select_kv(a, budget)
    assert len(out) == 2 and all(len(rows) == 3 for rows in out)
    for b in range(2):
        for i in range(3):
            bi = int(budget[b, i])
            got = out[b][i]
            assert got.dtype == np.int32 and got.shape == (bi,)
            # head by head it is the shared-budget selection at that head's b
            if bi:
                np.testing.assert_array_equal(got, oc.select_kv(a[b:b + 1], [bi])[0][i])
                best = max(a[b, i, list(c)].astype(np.float64).sum()
                           for c in itertools.combinations(range(9), bi))
                assert a[b, i, got].astype(np.float64).sum() == pytest.approx(best, rel=0, abs=1e-12)


# ------------------------------------------------------------------ top-b key selection

def test_select_kv_maximises_retained_mass_bruteforce():
    rng = np.random.default_rng(22)
    for trial in range(6):
        N = int(rng.integers(5, 12))
        a = rng.random((1, 2, N)).astype(np.float32)
        b = int(rng.integers(1, N + 1))
        idx = oc.select_kv(a, [b])[0]
        assert idx.shape == (2, b) and idx.dtype == np.int32
        for i in range(2):
            assert list(idx[i]) == sorted(set(idx[i].tolist()))
            got = a[0, i, idx[i]].astype(np.float64).sum()
            best = max(a[0, i, list(c)].astype(np.float64).sum() for c in itertools.combinations(range(N), b))
            assert got == pytest.approx(best, rel=0, abs=1e-12)
            cut = np.sort(a[0, i])[::-1][b - 1]
            assert np.all(a[0, i, idx[i]] >= cut)
            rest = np.setdiff1d(np.arange(N), idx[i])
            assert rest.size == 0 or np.all(a[0, i, rest] <= cut)


def test_select_kv_ties_take_lowest_index_and_full_budget():
    a = np.array([[[0.5, 0.9, 0.5, 0.5, 0.1, 0.5]]], dtype=np.float32)
    np.testing.assert_array_equal(oc.select_kv(a, [3])[0][0], [0, 1, 2])
    np.testing.assert_array_equal(oc.select_kv(a, [1])[0][0], [1])
    np.testing.assert_array_equal(oc.select_kv(a, [6])[0][0], np.arange(6))


def test_visual_subset_keeps_only_visual_indices():
    kv = [[np.array([0, 3, 5, 9, 12], dtype=np.int32), np.array([1, 2], dtype=np.int32)]]
    out = oc.visual_subset(kv, 3, 10)
    np.testing.assert_array_equal(out[0][0], [3, 5, 9])
    assert out[0][1].size == 0
