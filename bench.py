#!/usr/bin/env python3
"""Benchmark of the OmniSparse hot path on one MI355X.

A step is one pass of the sparse prefill path over one synthetic 64k-token layer
(28 query / 4 KV heads, head_dim 128, bf16, causal): query scoring, query
selection, key-score probe + budget, KV selection, sparse attention forward.
Inputs are resident in HBM before the timed region.  Prints one JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_64k|c2_16k] [--no-extras]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the sparse forward kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# file, scaled by the calibration copy (profiles/attn_fwd_c3_64k_hbm_traffic.txt); None where not profiled.
MEASURED_TRAFFIC = {"c3_64k": 5.39e9}

TAU = 0.08
RECALL_P = 0.95
PROBE_BLOCK = 256


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def pair_counts(q_lists, kv_lists, causal: bool, tile_m: int = 128, tile_n: int = 64):
    """Valid (query, key) pairs and pairs covered by the launched tile_m x tile_n tiles."""
    valid = issued = 0
    for qi, ki in zip(q_lists, kv_lists):
        if qi.size == 0 or ki.size == 0:
            continue
        if causal:
            per_q = np.searchsorted(ki, qi, side="right")
        else:
            per_q = np.full(qi.size, ki.size)
        valid += int(per_q.sum())
        last = per_q[np.minimum(np.arange(tile_m - 1, qi.size + tile_m - 1, tile_m), qi.size - 1)]
        issued += int((np.ceil(last / tile_n) * tile_n).sum()) * tile_m
    return valid, issued


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps before the timed ones (the clocks of the first few steps under load are lower)")
    ap.add_argument("--workload", default="c3_64k", choices=["c3_64k", "c2_16k"])
    ap.add_argument("--no-extras", action="store_true", help="skip dense baseline / oracle timing")
    ap.add_argument("--only", choices=["train", "decode", "mfma", "dense"],
                    help="run just the training-step extra, the decode extra or the matrix-core rate probe and print "
                         "its JSON (for profiling; the headline line is the default run)")
    ap.add_argument("--decode-steps", type=int, default=256, help="with --only decode: decode steps per mode")
    ap.add_argument("--decode-modes", default="", help="with --only decode: comma-separated subset of "
                    "slim,slim_stateless,slim_grouped,slim_compact,slim_paged,dense (for counter runs; prints the times only)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy (a kernel of known HBM traffic, to scale rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (the path is a single-GPU kernel library); "
            "run with --gpus 1")
        sys.exit(2)

    import torch
    from paper_2511_12201_amd import binding as ob
    from paper_2511_12201_amd import synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)
    ob.load_library()
    if args.only == "mfma":
        print(json.dumps({"mfma_only_probe": mfma_probe(ob, repeats=3)}), flush=True)
        return
    if args.only == "dense":
        print(json.dumps({"dense": bench_dense(torch, ob, synth)}), flush=True)
        return
    if args.only:
        modes = tuple(m for m in args.decode_modes.split(",") if m) or DECODE_MODES
        fn = bench_train if args.only == "train" else (
            lambda *a: bench_decode(*a, n_steps=args.decode_steps, batches=(1, 8), modes=modes))
        print(json.dumps({args.only: fn(torch, ob, synth)}), flush=True)
        return
    cfg = synth.C3_64K if args.workload == "c3_64k" else synth.C2_16K
    N, Hq, D = cfg.n_tokens, cfg.n_q_heads, cfg.head_dim

    t0 = time.time()
    layer = synth.make_layer(cfg)
    log(f"[bench] generated {cfg.name} in {time.time() - t0:.1f}s")
    dev = {k: torch.from_numpy(synth.bf16_bits(layer[k])).view(torch.bfloat16).cuda() for k in "QKV"}
    Q, K, V = dev["Q"], dev["K"], dev["V"]
    desc = ob.make_layer_desc(Q, K, cfg.vis_begin, cfg.vis_end, cfg.sink_index, cfg.causal)

    # outputs allocated once; the step itself allocates nothing
    B = cfg.batch
    f32, i32 = torch.float32, torch.int32
    probe = torch.empty(B, cfg.n_kv_heads, 2, D, dtype=f32, device="cuda")
    scores = torch.empty(B, Hq, N, dtype=f32, device="cuda")
    q_idx = torch.empty(B, Hq, N, dtype=i32, device="cuda")
    q_cnt = torch.empty(B, Hq, dtype=i32, device="cuda")
    bud = ob.BudgetResult(torch.empty(B, Hq, N, dtype=f32, device="cuda"),
                          torch.empty(B, Hq, dtype=torch.float64, device="cuda"),
                          torch.empty(B, dtype=i32, device="cuda"), torch.empty(B, dtype=i32, device="cuda"),
                          torch.empty(B, Hq, dtype=f32, device="cuda"))
    b_cap = N
    kv_idx = torch.empty(B, Hq, b_cap, dtype=i32, device="cuda")
    O = torch.empty_like(Q)
    lse = torch.empty(B, Hq, N, dtype=f32, device="cuda")

    sel = ob.SelectionResult(probe, scores, q_idx, q_cnt, bud, kv_idx)

    def selection():
        # omni_score_queries + omni_select_queries + omni_kv_budget + omni_select_kv in their fused form
        ob.omni_prefill_select(desc, Q, K, 0, TAU, RECALL_P, PROBE_BLOCK, 0, b_cap, out=sel)

    def step():
        selection()
        ob.omni_sparse_attn_fwd(desc, Q, K, V, q_idx, q_cnt, kv_idx, bud.budget, b_cap, O, lse)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        ob.debug_copy(src, dst)             # calibration_copy_kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the timed region: HIP events around the dominant kernel only (an event pair costs a few microseconds on the
    # stream; the other kernels are timed in a pass of their own below)
    ob.profile_enable(True, ["attn_fwd"])
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kern = {}
    ms, n = ob.profile_read("attn_fwd")
    kern["attn_fwd"] = ms / n
    others = ("pack_kv", "clear_out", "pool_q", "probe_lse", "probe_sum", "score")
    ob.profile_enable(True, others)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    for name in others:
        ms, n = ob.profile_read(name)
        if n:
            kern[name] = ms / n
    ob.profile_enable(False)
    log(f"[bench] step {ms_per_step:.3f} ms; kernels {kern}")

    # selection-only time (same launches, attention left out)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(args.steps):
        selection()
    ev1.record()
    torch.cuda.synchronize()
    sel_ms = ev0.elapsed_time(ev1) / args.steps

    # work accounting from the realised selection
    cnt = q_cnt.cpu().numpy()[0]
    b = int(bud.budget.cpu().numpy()[0])
    qi = q_idx.cpu().numpy()[0]
    ki = kv_idx.cpu().numpy()[0]
    q_lists = [qi[h, : cnt[h]] for h in range(Hq)]
    kv_lists = [ki[h, :b] for h in range(Hq)]
    valid, issued = pair_counts(q_lists, kv_lists, cfg.causal, tile_m=256)
    dense_pairs = Hq * N * (N + 1) // 2
    flops_alg = 4.0 * D * valid
    flops_issued = 4.0 * D * issued
    attn_ms = kern.get("attn_fwd", float("nan"))
    ach = flops_alg / (attn_ms * 1e-3) / 1e12
    ach_issued = flops_issued / (attn_ms * 1e-3) / 1e12

    out = {
        "metric": "sparse_prefill_ms_64k" if cfg is synth.C3_64K else "sparse_prefill_ms_16k",
        "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: 1 layer, batch 1, {Hq} q heads / {cfg.n_kv_heads} kv heads, head_dim {D}, "
                               f"N={N} ({cfg.frames} frames x {cfg.tok_per_frame} visual + {cfg.n_text} text), causal, "
                               f"tau={TAU}, recall p={RECALL_P}, probe block {PROBE_BLOCK}",
                   "step": "prefill_select (= score_queries + select_queries + kv_budget + select_kv) + sparse_attn_fwd",
                   "arithmetic": "bf16 inputs; Q.K^T on the bf16 matrix cores, softmax in fp32, weights rounded to f16 and "
                                 "multiplied with V (converted from bf16 to f16, exact inside +-65504) on the f16 matrix "
                                 "cores, fp32 accumulation"},
        "roofline": {"bound": "mfma", "kernel": "attn_fwd_bf16_kernel<128> (sparse)", "achieved": round(ach, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_BF16_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC.get(cfg.name),
                     "traffic_source": "profiles/attn_fwd_c3_64k_hbm_traffic.txt (rocprofv3 counter runs of this command; "
                                       "not measured in this run)",
                     "kernel_ms": round(attn_ms, 4),
                     "achieved_on_issued_tiles": round(ach_issued, 2),
                     "frac_on_issued_tiles": round(ach_issued / PEAK_BF16_TFLOPS, 4)},
        "selection_ms": round(sel_ms, 4),
        "kernel_ms": {k: round(v, 4) for k, v in kern.items()},
        "kept_query_fraction": round(float(cnt.sum()) / (Hq * N), 4),
        "budget_fraction": round(b / N, 4),
        "flops_fraction_of_dense": round(valid / dense_pairs, 4),
        "recall_min": round(float(bud.recall.min().item()), 4),
        "flattest_head": int(bud.flattest.cpu()[0]),
        "paper_context": "paper reports 2.7x prefill speedup and 2.4x decode memory reduction for the whole "
                         "LLaVA-Video-7b model on one H100 (not this metric)",
    }
    # the one pass over Q (query scores + pooled queries): Q in, scores and the split pooled queries out
    pool_bytes = Q.numel() * 2 + Hq * N * 4 + Hq * ((N + PROBE_BLOCK - 1) // PROBE_BLOCK) * D * 4
    if "pool_q" in kern:
        out["score_and_pool_pass_hbm"] = {"GB/s": round(pool_bytes / kern["pool_q"] / 1e6, 1),
                                          "frac": round(pool_bytes / kern["pool_q"] / 1e6 / PEAK_HBM_GBS, 4)}

    if not args.no_extras:
        # the same step through omni_sparse_prefill (key lists formed inside the attention's gather: one launch and one
        # pass over the lists fewer), outputs bit-identical; interleaved with the two-call step so that both see the
        # same clocks
        O1, lse1 = torch.empty_like(O), torch.empty_like(lse)

        def one_call():
            ob.omni_sparse_prefill(desc, Q, K, V, 0, TAU, RECALL_P, PROBE_BLOCK, 0, b_cap, out=sel, O=O1, lse=lse1)

        t_two = t_one = 0.0
        for fn in (step, one_call):
            for _ in range(args.warmup):
                fn()
        for _ in range(2):
            for which, fn in ((0, step), (1, one_call)):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(args.steps):
                    fn()
                torch.cuda.synchronize()
                dt = (time.perf_counter() - t0) * 1e3 / args.steps / 2
                t_two, t_one = (t_two + dt, t_one) if which == 0 else (t_two, t_one + dt)
        out["one_call_step"] = {"what": "omni_sparse_prefill: selection + gather + attention in one call",
                                "ms_per_step": round(t_one, 4), "two_call_ms_per_step_same_session": round(t_two, 4),
                                "output_bit_identical": bool(torch.equal(O1, O) and torch.equal(lse1, lse))}
        del O1, lse1
        # the same step replayed from a captured HIP graph (no call of it allocates, synchronises or memsets):
        # what the launch gaps between its ~25 kernels cost
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            for _ in range(3):
                graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            out["hip_graph_replay_ms_per_step"] = round((time.perf_counter() - t0) * 1e3 / args.steps, 4)
            del graph
        except Exception as e:
            out["hip_graph_replay_ms_per_step"] = {"error": repr(e)}
        # dense attention baseline from the same library, same inputs
        Od = torch.empty_like(Q)
        ob.omni_dense_attn_fwd(desc, Q, K, V, Od, lse)
        torch.cuda.synchronize()
        reps = 3
        ev0.record()
        for _ in range(reps):
            ob.omni_dense_attn_fwd(desc, Q, K, V, Od, lse)
        ev1.record()
        torch.cuda.synchronize()
        dense_ms = ev0.elapsed_time(ev1) / reps
        out["dense_attn_ms"] = round(dense_ms, 4)
        out["dense_tflops"] = round(4.0 * D * dense_pairs / (dense_ms * 1e-3) / 1e12, 2)
        out["speedup_vs_dense"] = round(dense_ms / ms_per_step, 3)
        del Od
        # what the matrix cores sustain with nothing else running: nominal (constant operands) and with
        # operands that toggle like data, where the clock is held down by the power limit
        out["mfma_only_probe"] = mfma_probe(ob)
        tf_r = out["mfma_only_probe"]["random_operands"]["TFLOP/s"]
        out["roofline"]["frac_of_sustained_random_operand_rate"] = round(ach / tf_r, 4)
        # the same launch (same lists, same instruction stream) on all-zero Q, K, V: what the kernel's schedule does
        # when the operands do not toggle and the power limit lets the clock stay up (context, not the metric)
        Zq, Zk = torch.zeros_like(Q), torch.zeros_like(K)
        ob.omni_sparse_attn_fwd(desc, Zq, Zk, Zk, q_idx, q_cnt, kv_idx, bud.budget, b_cap, O, lse)
        torch.cuda.synchronize()
        ob.profile_enable(True)
        for _ in range(5):
            ob.omni_sparse_attn_fwd(desc, Zq, Zk, Zk, q_idx, q_cnt, kv_idx, bud.budget, b_cap, O, lse)
        torch.cuda.synchronize()
        zms, zn = ob.profile_read("attn_fwd")
        ob.profile_enable(False)
        zms /= max(1, zn)
        out["roofline"]["constant_operand_run"] = {
            "what": "same kernel, same lists, Q = K = V = 0 (results discarded)", "kernel_ms": round(zms, 4),
            "frac_on_issued_tiles": round(flops_issued / (zms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
        del Zq, Zk
        try:
            out["block_granular_variant"] = bench_block_variant(torch, ob, cfg, desc, Q, K, V, probe, scores, q_idx, q_cnt,
                                                                bud, O, lse, args.steps)
        except Exception as e:
            out["block_granular_variant"] = {"error": repr(e)}
        try:
            out["per_head_budget_variant"] = bench_per_head_variant(torch, ob, cfg, desc, Q, K, V, probe, scores, q_idx,
                                                                    q_cnt, bud, O, lse, args.steps)
        except Exception as e:
            out["per_head_budget_variant"] = {"error": repr(e)}
        out["cpu_baseline"] = cpu_baseline(cfg, layer, q_lists, kv_lists, valid, ms_per_step)
        del Q, K, V, O, dev
        torch.cuda.empty_cache()
        # shared budget against per-head budgets over the recall target, on the bench's generator and on the
        # configuration text's generator without the salience term and the sharpness of head 0 (synth `plain`)
        try:
            t0 = time.time()
            plain_cfg = cfg.scaled(name=cfg.name + "_plain", plain=True)
            out["recall_sweep"] = {
                "what": "budget b/N, recall reached and ms per step (selection + sparse forward) for the paper's "
                        "shared budget (flattest head), the largest per-head budget, and one budget per head; "
                        "over-selection = shared budget minus the heads' own budgets, in percent of N (the paper "
                        "reports about 5 at recall 0.2 and 20 at 0.8 between its flattest and sharpest heads)",
                "bench_generator": bench_recall_sweep(torch, ob, synth, cfg, layer=layer),
                "plain_generator": bench_recall_sweep(torch, ob, synth, plain_cfg)}
            log(f"[bench] recall_sweep done in {time.time() - t0:.1f}s")
        except Exception as e:
            out["recall_sweep"] = {"error": repr(e)}
        del layer
        for name, fn in (("train_step_32k", bench_train),
                         ("train_step_32k_per_head_budgets", lambda *a: bench_train(*a, per_head=True)),
                         ("decode_131k", bench_decode),
                         ("decode_131k_per_head_budgets", lambda *a: bench_decode(*a, per_head=True, batches=(1, 8))),
                         ("decode_131k_plain_generator", lambda *a: bench_decode(*a, batches=(1, 8), plain=True))):
            try:
                t0 = time.time()
                out[name] = fn(torch, ob, synth)
                log(f"[bench] {name} done in {time.time() - t0:.1f}s")
            except Exception as e:      # the headline line must survive a failing extra
                out[name] = {"error": repr(e)}

    print(json.dumps(out), flush=True)


def _upload(torch, synth, x):
    return torch.from_numpy(synth.bf16_bits(x)).view(torch.bfloat16).cuda()


def bench_block_variant(torch, ob, cfg, desc, Q, K, V, probe, scores, q_idx, q_cnt, bud, O, lse, steps):
    """The paper's own granularity: queries and keys pooled in blocks of 256, budget and lists in key blocks."""
    N, Hq = cfg.n_tokens, cfg.n_q_heads
    block = PROBE_BLOCK
    nb = (N + block - 1) // block
    bdesc = ob.block_level_desc(desc, block)
    blk_idx = torch.empty(cfg.batch, Hq, nb, dtype=torch.int32, device="cuda")
    kv_idx = torch.empty(cfg.batch, Hq, nb * block, dtype=torch.int32, device="cuda")
    budget = torch.empty(cfg.batch, dtype=torch.int32, device="cuda")
    res = None

    def step():
        nonlocal res
        ob.omni_score_queries(desc, Q, K, probe, scores)
        ob.omni_select_queries(desc, scores, 0, TAU, q_idx, q_cnt)
        a_blk = ob.omni_block_scores(desc, Q, K, block)
        res = ob.omni_budget_from_scores(bdesc, a_blk, RECALL_P, 0)
        ob.omni_select_kv(bdesc, a_blk, res.budget, nb, blk_idx)
        ob.omni_expand_blocks(desc, blk_idx, res.budget, block, kv_idx, budget)
        ob.omni_sparse_attn_fwd(desc, Q, K, V, q_idx, q_cnt, kv_idx, budget, nb * block, O, lse)

    for _ in range(3):
        step()
    torch.cuda.synchronize()
    ob.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    attn_ms, n = ob.profile_read("attn_fwd")
    ob.profile_enable(False)

    # the same lists walked in place: one token-ordered K/V copy per KV head, no gather, no token lists
    O2, lse2 = torch.empty_like(O), torch.empty_like(lse)

    def step_in_place():
        ob.omni_score_queries(desc, Q, K, probe, scores)
        ob.omni_select_queries(desc, scores, 0, TAU, q_idx, q_cnt)
        a_blk = ob.omni_block_scores(desc, Q, K, block)
        r = ob.omni_budget_from_scores(bdesc, a_blk, RECALL_P, 0)
        ob.omni_select_kv(bdesc, a_blk, r.budget, nb, blk_idx)
        ob.omni_block_attn_fwd(desc, Q, K, V, q_idx, q_cnt, blk_idx, r.budget, block, O2, lse2)

    for _ in range(3):
        step_in_place()
    torch.cuda.synchronize()
    same = bool(torch.equal(O.view(torch.int16), O2.view(torch.int16)))
    ob.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step_in_place()
    torch.cuda.synchronize()
    ms2 = (time.perf_counter() - t0) * 1e3 / steps
    attn2_ms, n2 = ob.profile_read("attn_fwd")
    ob.profile_enable(False)
    b_tok = int(budget.cpu()[0])
    # share of the token-level accumulated scores (the main path's probe) that the block lists capture, per head
    a_tok = bud.key_scores[0]
    idx = kv_idx[0, :, :b_tok].long().clamp(max=N - 1)
    real = kv_idx[0, :, :b_tok] < N
    recall = (torch.gather(a_tok, 1, idx) * real).sum(1) / N
    cnt = q_cnt.cpu().numpy()[0]
    qi, ki = q_idx.cpu().numpy()[0], kv_idx.cpu().numpy()[0]
    kl = [ki[h, :b_tok][ki[h, :b_tok] < N] for h in range(Hq)]
    valid, _ = pair_counts([qi[h, : cnt[h]] for h in range(Hq)], kl, cfg.causal, tile_m=256)
    return {"what": f"queries and keys pooled in blocks of {block}; recall target {RECALL_P} on the block scores; "
                    "same kept queries, same attention kernel on the token lists of the selected blocks",
            "ms_per_step": round(ms, 4), "attn_fwd_ms": round(attn_ms / max(1, n), 4),
            "in_place": {"what": "block lists walked inside one token-ordered K/V copy per KV head (no gather)",
                         "ms_per_step": round(ms2, 4), "attn_fwd_ms": round(attn2_ms / max(1, n2), 4),
                         "output_bit_identical": same},
            "budget_blocks": int(res.budget.cpu()[0]), "budget_fraction": round(b_tok / N, 4),
            "token_level_recall_min": round(float(recall.min()), 4), "token_level_recall_mean": round(float(recall.mean()), 4),
            "attn_algorithmic_tflops": round(4.0 * cfg.head_dim * valid / (attn_ms / max(1, n) * 1e-3) / 1e12, 1)}


def bench_per_head_variant(torch, ob, cfg, desc, Q, K, V, probe, scores, q_idx, q_cnt, bud, O, lse, steps):
    """The alternative the paper sets aside: every head searches its own budget (same probe, same recall target)."""
    N, Hq = cfg.n_tokens, cfg.n_q_heads
    res = ob.BudgetResult(bud.key_scores, torch.empty_like(bud.kurtosis), torch.empty_like(bud.flattest),
                          torch.empty(cfg.batch, Hq, dtype=torch.int32, device="cuda"), torch.empty_like(bud.recall))
    kv_idx = torch.empty(cfg.batch, Hq, N, dtype=torch.int32, device="cuda")

    sel = ob.SelectionResult(probe, scores, q_idx, q_cnt, res, kv_idx)

    def selection():
        ob.omni_prefill_select(desc, Q, K, 0, TAU, RECALL_P, PROBE_BLOCK, 2, N, out=sel)

    def step():
        selection()
        ob.omni_sparse_attn_fwd_per_head(desc, Q, K, V, q_idx, q_cnt, kv_idx, res.budget, N, O, lse)

    for _ in range(3):
        step()
    torch.cuda.synchronize()
    ob.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    attn_ms, n = ob.profile_read("attn_fwd")
    ob.profile_enable(False)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(steps):
        selection()
    ev1.record()
    torch.cuda.synchronize()
    b = res.budget.cpu().numpy()[0]
    cnt = q_cnt.cpu().numpy()[0]
    qi, ki = q_idx.cpu().numpy()[0], kv_idx.cpu().numpy()[0]
    valid, _ = pair_counts([qi[h, : cnt[h]] for h in range(Hq)], [ki[h, : b[h]] for h in range(Hq)], cfg.causal, tile_m=256)
    attn = attn_ms / max(1, n)
    return {"what": f"budget_mode 2: each head keeps the fewest keys that reach recall {RECALL_P} on its own scores",
            "ms_per_step": round(ms, 4), "selection_ms": round(ev0.elapsed_time(ev1) / steps, 4),
            "attn_fwd_ms": round(attn, 4),
            "budget_fraction_min_mean_max": [round(float(b.min()) / N, 4), round(float(b.mean()) / N, 4),
                                             round(float(b.max()) / N, 4)],
            "recall_min": round(float(res.recall.min().item()), 4),
            "flops_fraction_of_dense": round(valid / (Hq * N * (N + 1) // 2), 4),
            "attn_algorithmic_tflops": round(4.0 * cfg.head_dim * valid / (attn * 1e-3) / 1e12, 1)}


def bench_dense(torch, ob, synth, reps: int = 3):
    """The dense baseline alone (omni_dense_attn_fwd on the 64k layer), for counter runs."""
    cfg = synth.C3_64K
    layer = synth.make_layer(cfg)
    Q, K, V = (_upload(torch, synth, layer[k]) for k in "QKV")
    desc = ob.make_layer_desc(Q, K, cfg.vis_begin, cfg.vis_end, cfg.sink_index, cfg.causal)
    O = torch.empty_like(Q)
    lse = torch.empty(cfg.batch, cfg.n_q_heads, cfg.n_tokens, dtype=torch.float32, device="cuda")
    ob.omni_dense_attn_fwd(desc, Q, K, V, O, lse)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(reps):
        ob.omni_dense_attn_fwd(desc, Q, K, V, O, lse)
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / reps
    pairs = cfg.n_q_heads * cfg.n_tokens * (cfg.n_tokens + 1) // 2
    return {"workload": "c3_64k dense causal attention", "ms": round(ms, 4),
            "tflops": round(4.0 * cfg.head_dim * pairs / (ms * 1e-3) / 1e12, 2)}


RECALL_SWEEP = (0.2, 0.5, 0.8, 0.82, 0.95)


def bench_recall_sweep(torch, ob, synth, cfg, steps: int = 5, layer=None):
    """Shared budget against per-head budgets as a function of the recall target (the measurement of the paper's
    paragraph on over-selection for sharp heads, its sparsity-difference figure): budgets, recall reached, and the
    time of the whole step, for budget_mode 0 (flattest head, the paper's rule), 1 (largest per-head budget) and 2
    (one budget per head)."""
    layer = layer or synth.make_layer(cfg)
    Q, K, V = (_upload(torch, synth, layer[k]) for k in "QKV")
    N, Hq = cfg.n_tokens, cfg.n_q_heads
    desc = ob.make_layer_desc(Q, K, cfg.vis_begin, cfg.vis_end, cfg.sink_index, cfg.causal)
    O = torch.empty_like(Q)
    lse = torch.empty(cfg.batch, Hq, N, dtype=torch.float32, device="cuda")
    rows = []
    for p in RECALL_SWEEP:
        row = {"recall_target": p}
        per_head_budgets = None
        for mode, name in ((2, "per_head"), (0, "flattest_head"), (1, "max_over_heads")):
            sel = None

            def step():
                nonlocal sel
                sel = ob.omni_prefill_select(desc, Q, K, 0, TAU, p, PROBE_BLOCK, mode, N, out=sel)
                ob.omni_sparse_attn_fwd(desc, Q, K, V, sel.q_idx, sel.q_cnt, sel.kv_idx, sel.budget.budget, N, O, lse,
                                        _per_head=mode == 2)

            step()
            step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / steps
            b = sel.budget.budget.cpu().numpy().reshape(-1).astype(np.float64)
            r = {"ms_per_step": round(ms, 3), "recall_min": round(float(sel.budget.recall.min().item()), 4)}
            if mode == 2:
                per_head_budgets = b
                r["budget_fraction_min_mean_max"] = [round(b.min() / N, 4), round(b.mean() / N, 4), round(b.max() / N, 4)]
            else:
                r["budget_fraction"] = round(b[0] / N, 4)
                r["flattest_head"] = int(sel.budget.flattest.cpu()[0])
                # keys selected beyond what the heads need themselves, in percent of the sequence: on average over
                # the heads, and for the sharpest head (the figure's flattest-minus-sharpest sparsity difference)
                r["over_selection_pct_of_N"] = {"mean_head": round(100 * (b[0] - per_head_budgets.mean()) / N, 2),
                                                "sharpest_head": round(100 * (b[0] - per_head_budgets.min()) / N, 2)}
                r["heads_below_target"] = int((sel.budget.recall.cpu().numpy() < p - 1e-6).sum())
            row[name] = r
        rows.append(row)
    del Q, K, V, O, lse
    torch.cuda.empty_cache()
    return rows


def bench_train(torch, ob, synth, steps: int = 5, per_head: bool = False):
    """Training step of one layer at N=32768: selection recomputed, sparse forward, sparse backward."""
    cfg = synth.C4_TRAIN_32K
    layer = synth.make_layer(cfg)
    Q, K, V = (_upload(torch, synth, layer[k]) for k in "QKV")
    dO = _upload(torch, synth, synth.make_grad_output(cfg))
    N, Hq, D = cfg.n_tokens, cfg.n_q_heads, cfg.head_dim
    desc = ob.make_layer_desc(Q, K, cfg.vis_begin, cfg.vis_end, cfg.sink_index, cfg.causal)
    f32, i32 = torch.float32, torch.int32
    O, dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    lse = torch.empty(1, Hq, N, dtype=f32, device="cuda")
    sel = None

    def step():
        nonlocal sel
        sel = ob.omni_prefill_select(desc, Q, K, 0, TAU, RECALL_P, PROBE_BLOCK, 2 if per_head else 0, N, out=sel)
        bud, q_idx, q_cnt, kv_idx = sel.budget, sel.q_idx, sel.q_cnt, sel.kv_idx
        ob.omni_sparse_attn_fwd(desc, Q, K, V, q_idx, q_cnt, kv_idx, bud.budget, N, O, lse, _per_head=per_head)
        ob.omni_sparse_attn_bwd(desc, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, bud.budget, N, dQ, dK, dV,
                                _per_head=per_head)

    step()
    step()
    torch.cuda.synchronize()
    ob.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    kern = {}
    for name in ("attn_fwd", "bwd_dkdv", "bwd_dq", "bwd_reduce", "pack_kv"):
        t, n = ob.profile_read(name)
        if n:
            kern[name] = round(t / n, 4)
    ob.profile_enable(False)
    bud, q_idx, q_cnt, kv_idx = sel.budget, sel.q_idx, sel.q_cnt, sel.kv_idx
    cnt = q_cnt.cpu().numpy()[0]
    bh = bud.budget.cpu().numpy().reshape(-1)
    bh = bh if per_head else np.full(Hq, bh[0])
    b = float(bh.mean())
    qi, ki = q_idx.cpu().numpy()[0], kv_idx.cpu().numpy()[0]
    valid, _ = pair_counts([qi[h, : cnt[h]] for h in range(Hq)], [ki[h, : bh[h]] for h in range(Hq)], cfg.causal)
    bwd_ms = kern.get("bwd_dkdv", 0) + kern.get("bwd_dq", 0)
    res = {"workload": f"{cfg.name}: N={N}, bf16, selection + sparse fwd + sparse bwd"
                       + (", one budget per head" if per_head else ""), "ms_per_step": round(ms, 4),
           "kernel_ms": kern, "kept_query_fraction": round(float(cnt.sum()) / (Hq * N), 4),
           "budget_fraction": round(b / N, 4),
           "bwd_algorithmic_tflops": round(10.0 * D * valid / (bwd_ms * 1e-3) / 1e12, 2) if bwd_ms else None,
           # 8 GEMMs per pair are issued (S is recomputed by the dK, dV and dQ kernels), 5 are the algorithm's
           "bwd_issued_gemm_tflops": round(16.0 * D * valid / (bwd_ms * 1e-3) / 1e12, 2) if bwd_ms else None,
           "fwd_algorithmic_tflops": round(4.0 * D * valid / (kern["attn_fwd"] * 1e-3) / 1e12, 2)}
    return res


def mfma_probe(ob, repeats: int = 1):
    """Register-resident bf16 MFMAs and nothing else: constant operands, pseudo-random operands, and pseudo-random
    operands with the matrix cores idle a third of the time.  With repeats > 1 every mode's runs are listed."""
    names = ("constant_operands", "random_operands", "random_operands_two_thirds_duty")
    runs = {n: [] for n in names}
    for _ in range(repeats):
        for mode, n in enumerate(names):
            tf, mhz = ob.debug_mfma_rate(mode)
            runs[n].append({"TFLOP/s": round(tf, 1), "shader_MHz": round(mhz)})
    return {n: (v[0] if repeats == 1 else v) for n, v in runs.items()}


DECODE_MODES = ("slim", "slim_stateless", "slim_grouped", "slim_compact", "slim_paged", "dense")


def bench_decode(torch, ob, synth, n_steps: int = 256, per_head: bool = False, batches=(1, 2, 4, 8), modes=DECODE_MODES,
                 plain: bool = False):
    """Decode with KV cache slimming on a 131072-token cache, batch 1..8, 256 steps each."""
    cfg = synth.C5_DECODE_131K
    if plain:             # the generator without the salience term: the heads of a group pick less alike
        cfg = cfg.scaled(name=cfg.name + "_plain", plain=True)
    layer = synth.make_layer(cfg)
    Q, K, V = (_upload(torch, synth, layer[k]) for k in "QKV")
    N, Hq, Hkv, D = cfg.n_tokens, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    desc = ob.make_layer_desc(Q, K, cfg.vis_begin, cfg.vis_end, cfg.sink_index, cfg.causal)
    probe, _ = ob.omni_score_queries(desc, Q, K)
    bud = ob.omni_kv_budget(desc, Q, K, RECALL_P, PROBE_BLOCK, 2 if per_head else 0)
    b = int(bud.budget.max().cpu())
    b_mean = float(bud.budget.float().mean().cpu())
    kv_idx = ob.omni_select_kv(desc, bud.key_scores, bud.budget, b, _per_head=per_head)
    vis_idx1, vis_cnt1 = ob.omni_visual_subset(desc, kv_idx, bud.budget, b, _per_head=per_head)
    grp_idx1, grp_mask1, grp_cnt1 = ob.omni_group_subset(desc, kv_idx, bud.budget, b, _per_head=per_head)
    torch.cuda.synchronize()
    del Q, bud
    cap = N + n_steps
    res = {"workload": f"{cfg.name}: cache {N} tokens + {n_steps} decoded, bf16, tau={TAU}"
                       + (", one budget per head" if per_head else ""),
           "budget_fraction": round(b_mean / N, 4),
           "timing": "us_per_token = GPU time of the decode call's kernels (HIP events, first 64 steps); the Python loop "
                     "around it (cache append, ctypes launches) is host-bound and listed separately",
           "per_batch": {}}
    vis_cnt_host = vis_cnt1.cpu().numpy()[0]
    vis_idx_host = vis_idx1.cpu().numpy()[0]
    member = np.zeros((Hq, N), dtype=bool)            # member[h, n]: head h stores visual row n
    for h in range(Hq):
        member[h, vis_idx_host[h, : vis_cnt_host[h]]] = True
    for B in batches:
        steps = synth.make_decode_steps(cfg, layer, n_steps, batch=B)
        q_all = _upload(torch, synth, steps["q"])                      # [S,B,Hq,D]
        k_new = _upload(torch, synth, steps["k_new"])
        v_new = _upload(torch, synth, steps["v_new"])
        Kc = torch.zeros(B, Hkv, cap, D, dtype=torch.bfloat16, device="cuda")
        Vc = torch.zeros_like(Kc)
        Kc[:, :, :N] = K
        Vc[:, :, :N] = V
        vis_idx = vis_idx1.expand(B, -1, -1).contiguous()
        vis_cnt = vis_cnt1.expand(B, -1).contiguous()
        grp_idx, grp_mask = grp_idx1.expand(B, -1, -1).contiguous(), grp_mask1.expand(B, -1, -1).contiguous()
        grp_cnt = grp_cnt1.expand(B, -1).contiguous()
        probe_b = probe.expand(B, -1, -1, -1).contiguous()
        ctx = torch.full((B,), N, dtype=torch.int32, device="cuda")
        O = torch.empty(B, Hq, D, dtype=torch.bfloat16, device="cuda")
        act = torch.empty(B, Hq, dtype=torch.uint8, device="cuda")
        ddesc = ob.make_decode_desc(q_all[0], Kc, cfg.vis_begin, cfg.vis_end, TAU)
        # omni_slim_decode as a serving loop calls it: the lists are fixed at prefill (static_lists), merged once per KV
        # group by omni_slim_decode_prepare; "slim_stateless" reads the per-head lists anew on every step
        sdesc = ob.make_decode_desc(q_all[0], Kc, cfg.vis_begin, cfg.vis_end, TAU, static_lists=True)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        # the compacted store: the rows of the group lists side by side (built once after prefill)
        u_max = int(grp_cnt.max().cpu())
        g_idx_c, g_mask_c = grp_idx[:, :, :u_max].contiguous(), grp_mask[:, :, :u_max].contiguous()
        Kcomp, Vcomp = ob.omni_compact_cache(ddesc, Kc, Vc, g_idx_c, grp_cnt)
        torch.cuda.synchronize()
        ev0.record()
        ob.omni_compact_cache(ddesc, Kc, Vc, g_idx_c, grp_cnt, Kcomp, Vcomp)
        ev1.record()
        torch.cuda.synchronize()
        compact_us = ev0.elapsed_time(ev1) * 1e3
        # the same store in pages of 256 rows handed out in a seeded random order, as a block allocator would
        page_rows = 256
        need = ((grp_cnt + page_rows - 1) // page_rows).cpu().numpy()
        n_pages = int(need.sum())
        perm = np.random.default_rng(5).permutation(n_pages).astype(np.int32)
        table = np.full((B, Hkv, (u_max + page_rows - 1) // page_rows), -1, dtype=np.int32)
        used = 0
        for bb in range(B):
            for g in range(Hkv):
                table[bb, g, : need[bb, g]] = perm[used: used + need[bb, g]]
                used += int(need[bb, g])
        Kpool = torch.empty(n_pages, page_rows, D, dtype=torch.bfloat16, device="cuda")
        Vpool = torch.empty_like(Kpool)
        pool = ob.make_page_pool(Kpool, Vpool, torch.from_numpy(table).cuda())
        ob.omni_compact_cache_paged(ddesc, Kc, Vc, g_idx_c, grp_cnt, pool)
        timing, ktime = {}, {}
        for mode in modes:
            ctx.fill_(N + 1)
            if mode == "slim":                # once after prefill: the lists merged per KV group, in a workspace of their own
                ws_static = ob.Workspace()
                ob.omni_slim_decode_prepare(sdesc, vis_idx, vis_cnt, b, ws=ws_static)
            for _ in range(3):                                    # untimed warm-up of the entry points
                ob.omni_slim_decode_grouped(ddesc, q_all[0], Kc, Vc, ctx, probe_b, grp_idx, grp_mask, grp_cnt, O, act)
                ob.omni_slim_decode(ddesc, q_all[0], Kc, Vc, ctx, probe_b, vis_idx, vis_cnt, b, O, act)
                if mode == "slim":
                    ob.omni_slim_decode(sdesc, q_all[0], Kc, Vc, ctx, probe_b, vis_idx, vis_cnt, b, O, act, ws=ws_static)
                ob.omni_dense_decode(ddesc, q_all[0], Kc, Vc, ctx, O)
            ctx.fill_(N)
            torch.cuda.synchronize()
            ob.profile_enable(True)
            ev0.record()
            for s in range(n_steps):
                Kc[:, :, N + s] = k_new[s]
                Vc[:, :, N + s] = v_new[s]
                ctx += 1
                if mode == "slim":
                    ob.omni_slim_decode(sdesc, q_all[s], Kc, Vc, ctx, probe_b, vis_idx, vis_cnt, b, O, act, ws=ws_static)
                elif mode == "slim_stateless":
                    ob.omni_slim_decode(ddesc, q_all[s], Kc, Vc, ctx, probe_b, vis_idx, vis_cnt, b, O, act)
                elif mode == "slim_grouped":
                    ob.omni_slim_decode_grouped(ddesc, q_all[s], Kc, Vc, ctx, probe_b, grp_idx, grp_mask, grp_cnt, O, act)
                elif mode == "slim_compact":
                    ob.omni_slim_decode_compact(ddesc, q_all[s], Kc, Vc, ctx, probe_b, Kcomp, Vcomp, g_idx_c, g_mask_c,
                                                grp_cnt, O, act)
                elif mode == "slim_paged":
                    ob.omni_slim_decode_paged(ddesc, q_all[s], Kc, Vc, ctx, probe_b, pool, g_idx_c, g_mask_c, grp_cnt, O, act)
                else:
                    ob.omni_dense_decode(ddesc, q_all[s], Kc, Vc, ctx, O)
            ev1.record()
            torch.cuda.synchronize()
            timing[mode] = ev0.elapsed_time(ev1) * 1e3 / n_steps          # us per decode step
            kms, kn = ob.profile_read("decode")                               # last 64 launches: row-streaming kernels only
            ktime[mode] = kms * 1e3 / max(1, kn)
            ob.profile_enable(False)
        # the same call replayed from a captured HIP graph (rows kernel + slice combine back to back, no host in
        # between): what a serving loop pays per token and layer once its step is captured
        graph_us = {}
        if set(modes) == set(DECODE_MODES):
            def replay_us(fn):
                fn()
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    fn()
                g.replay()
                torch.cuda.synchronize()
                ev0.record()
                for _ in range(64):
                    g.replay()
                ev1.record()
                torch.cuda.synchronize()
                return ev0.elapsed_time(ev1) * 1e3 / 64
            graph_us["slim_grouped"] = replay_us(lambda: ob.omni_slim_decode_grouped(
                ddesc, q_all[0], Kc, Vc, ctx, probe_b, grp_idx, grp_mask, grp_cnt, O, act))
            graph_us["dense"] = replay_us(lambda: ob.omni_dense_decode(ddesc, q_all[0], Kc, Vc, ctx, O))
        if set(modes) != set(DECODE_MODES):               # a counter run on some of the modes: times only
            res["per_batch"][str(B)] = {f"{k}_us_per_token": round(v, 2) for k, v in ktime.items()}
            del Kc, Vc, Kpool, Vpool, Kcomp, Vcomp
            torch.cuda.empty_cache()
            continue
        # K/V rows a step asks for (last step's activity).  Plain decode: every row once per KV group.  Slimmed
        # decode with per-head lists: every active head its own stored visual rows (heads of a group that store
        # the same row both ask for it), plus the non-visual rows once per group.  Grouped lists: the union over
        # the active heads of a group instead.
        a = act.cpu().numpy()
        G = Hq // Hkv
        n_text = (N - cfg.vis_end) + cfg.vis_begin + n_steps
        rows_head = rows_union = 0
        for bb in range(B):
            for g in range(Hkv):
                heads = [h for h in range(g * G, (g + 1) * G) if a[bb, h]]
                if heads:
                    rows_union += int(np.any(member[heads], axis=0).sum())
                    rows_head += int(member[heads].sum())
                rows_union += n_text
                rows_head += n_text
        rows_dense = B * Hkv * (N + n_steps)
        row_bytes = 2 * D * 2
        gbps = lambda rows, us: round(rows * row_bytes / (us * 1e-6) / 1e9, 1)
        res["per_batch"][str(B)] = {
            "slim_us_per_token": round(ktime["slim"], 2), "dense_us_per_token": round(ktime["dense"], 2),
            "speedup": round(ktime["dense"] / ktime["slim"], 3),
            "speedup_grouped": round(ktime["dense"] / ktime["slim_grouped"], 3),
            "slim_stateless_us_per_token": round(ktime["slim_stateless"], 2),
            "slim_grouped_us_per_token": round(ktime["slim_grouped"], 2),
            "slim_compact_us_per_token": round(ktime["slim_compact"], 2),
            "slim_paged_us_per_token": round(ktime["slim_paged"], 2),
            "compaction_us_once": round(compact_us, 1),
            # what a serving stack has to keep per layer: the whole cache, or the compacted visual rows (with their
            # token index and membership word) plus the non-visual rows
            "kv_store_bytes": {"full_cache": int(rows_dense * row_bytes),
                               "compacted": int(int(grp_cnt.sum().cpu()) * (row_bytes + 8) + B * Hkv * n_text * row_bytes)},
            "python_loop_us_per_token": {k: round(v, 1) for k, v in timing.items()},
            "hip_graph_us_per_token": {k: round(v, 1) for k, v in graph_us.items()},
            "active_head_fraction_last_step": round(float(a.mean()), 4),
            # rows the lists name: per head (a row stored by several active heads of a group counted for each) and as
            # the group's union, which is what every slimmed variant reads (omni_slim_decode merges the heads' lists)
            "rows_requested_vs_dense": {"per_head_lists": round(rows_head / rows_dense, 4),
                                        "group_union": round(rows_union / rows_dense, 4)},
            "GBps_of_requested_rows": {"slim": gbps(rows_union, ktime["slim"]), "slim_grouped": gbps(rows_union, ktime["slim_grouped"]),
                                       "dense": gbps(rows_dense, ktime["dense"])},
            "dense_frac_of_hbm_peak": round(rows_dense * row_bytes / (ktime["dense"] * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)}
        del Kc, Vc, Kpool, Vpool, Kcomp, Vcomp
        torch.cuda.empty_cache()
    return res


def cpu_baseline(cfg, layer, q_lists, kv_lists, total_pairs, gpu_ms):
    """The oracle as it stands, timed on a bounded sample of the same step and scaled to the full step."""
    from oracle import omni_oracle as oc      # the only place the benchmark touches the oracle
    Q, K, V = layer["Q"], layer["K"], layer["V"]
    G = cfg.n_q_heads // cfg.n_kv_heads
    heads = list(range(2 * G))                      # two whole KV groups
    t0 = time.perf_counter()
    Qs, Ks = Q[:, heads], K[:, :2]
    pk = oc.probe_keys(Ks, cfg.vis_begin, cfg.vis_end, cfg.sink_index)
    sc = oc.score_queries(Qs, pk, cfg.scale).astype(np.float32)
    oc.select_queries(sc, 0, TAU, cfg.vis_begin, cfg.vis_end)
    a = oc.pooled_key_scores(Qs, Ks, PROBE_BLOCK, cfg.causal, cfg.scale).astype(np.float32)
    r = oc.kv_budget(a, RECALL_P, 0)
    oc.select_kv(a, r["budget"])
    t_sel = time.perf_counter() - t0
    # attention on samples of the kept queries of heads 1..6 with the realised selection
    att_heads = [1, 2, 3, 4, 5, 6]
    empty = np.zeros(0, dtype=np.int32)
    samples = {h: q_lists[h][:: max(1, q_lists[h].size // 8192)][:8192] for h in att_heads}
    t0 = time.perf_counter()
    q_arg = [[samples.get(h, empty) for h in range(G)]]
    kv_arg = [[kv_lists[h] if h in samples else empty for h in range(G)]]
    oc.sparse_attn_fwd(Q[:, :G], K[:, :1], V[:, :1], q_arg, kv_arg, cfg.causal, cfg.scale)
    t_att = time.perf_counter() - t0
    sample_pairs = sum(int(np.searchsorted(kv_lists[h], samples[h], side="right").sum()) if cfg.causal
                       else samples[h].size * kv_lists[h].size for h in att_heads)
    sample_q_total = sum(s.size for s in samples.values())
    est_ms = (t_sel * cfg.n_q_heads / len(heads) + t_att * total_pairs / max(1, sample_pairs)) * 1e3
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": round(est_ms, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
            "sample": f"selection pipeline on query heads 0..{len(heads) - 1} ({t_sel:.1f}s, scaled x{cfg.n_q_heads / len(heads):g}) + "
                      f"sparse attention of {sample_q_total} kept queries of heads {att_heads} against their selected keys "
                      f"({t_att:.1f}s, {sample_pairs} of {total_pairs} pairs, scaled by pairs)"}


if __name__ == "__main__":
    main()
