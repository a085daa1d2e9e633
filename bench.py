#!/usr/bin/env python3
"""Benchmark of the Dodo hot path on one MI355X.

One "step" is one pass of the whole path over one batch of the LLaMA-7B-shaped
prefill workload (bf16, batch 8, 4096 context tokens per sequence, 10x
compression, 512-token query block after 128 local tokens):

    dodo_score -> dodo_select_topk -> dodo_gather_nuggets
      -> dodo_nugget_attention (512-row query block, MFMA kernel)
      -> dodo_nugget_attention (one decode token per sequence, split-K kernel)

All inputs are resident in HBM before the timed region.  Prints ONE JSON line:
whole-step query tokens/s, the per-kernel durations measured with events on
the launch stream inside the timed region, the roofline of the dominant
kernel, and the oracle timed on the host cores on a bounded sample of the same
workload (a reported baseline, not a target).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2, help="workload id (2 = LLaMA-7B prefill, the metric's config)")
    ap.add_argument("--suite", action="store_true",
                    help="instead of the default line: decode step over 32 layers (workload 3), compress phase over "
                         "40 layers (workload 4), 64 decode steps (workload 5)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-events", action="store_true", help="no per-kernel events inside the timed region")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (reference for the HBM traffic counters)")
    return ap.parse_args()


def algorithmic_work(wl, ks, E):
    """Algorithmic bytes / flop per launch (what the method itself must move or compute)."""
    N, d, B = wl.N, wl.d_model, wl.B
    Hd = wl.H_kv * wl.d_h
    Kt = sum(ks)
    Sq = sum(wl.q_lens)
    vis_pairs = sum(sum(k + (m - q + i + 1) for i in range(q)) for k, m, q in zip(ks, wl.local_lens, wl.q_lens))
    out = {
        "score": {"bytes": N * d * E + d * E + 4 * N, "flop": 2 * N * d},
        "select": {"bytes": 4 * N + 4 * Kt + 8 * (B + 1), "flop": 0},
        "gather": {"bytes": 2 * (2 * Kt * Hd * E) + 4 * Kt, "flop": 0},
        "attn_block": {"bytes": E * (2 * Sq * wl.H * wl.d_h + 2 * sum(k + m for k, m in zip(ks, wl.local_lens)) * Hd),
                       "flop": 4 * wl.d_h * wl.H * vis_pairs},
    }
    dec_rows = sum(k + m + 1 for k, m in zip(ks, wl.local_lens))
    out["attn_decode"] = {"bytes": E * (2 * B * wl.H * wl.d_h + 2 * dec_rows * Hd), "flop": 4 * wl.d_h * wl.H * dec_rows}
    return out


def cpu_baseline(wl, host, ks, scale):
    """Times the oracle, as it stands, on sequence 0 of the batch (all sequences have the same shape):
    score + select + gather of its context and attention for all its query tokens, all heads."""
    import numpy as np
    import oracle
    n0, q0, m0, k0 = wl.seq_lens[0], wl.q_lens[0], wl.local_lens[0], ks[0]
    cu_s, cu_k = oracle.cu_from_lengths([n0]), oracle.cu_from_lengths([k0])
    cu_q, cu_m = oracle.cu_from_lengths([q0]), oracle.cu_from_lengths([m0])
    t0 = time.perf_counter()
    s = oracle.score(host["hidden"][:n0], host["w"])
    idx = oracle.select_topk(s, cu_s, cu_k, oracle.FORCE_LAST)
    Kn, Vn = oracle.gather(host["K"][:n0], host["V"][:n0], idx, cu_s, cu_k)
    t1 = time.perf_counter()
    oracle.attention(host["Q"][:q0], Kn, Vn, host["Kl"][:m0], host["Vl"][:m0], cu_q, cu_k, cu_m, scale)
    oracle.attention(host["Qd"][:1], Kn, Vn, host["Kld"][:m0 + 1], host["Vld"][:m0 + 1], oracle.cu_from_lengths([1]),
                     cu_k, oracle.cu_from_lengths([m0 + 1]), scale)
    t2 = time.perf_counter()
    total = t2 - t0
    return {"value": (q0 + 1) / total, "unit": "query tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"sequence 0 of {wl.B} (n={n0}, k={k0}, q={q0}+1 decode token, all {wl.H} heads): "
                      f"score+select+gather {t1 - t0:.2f} s, attention {t2 - t1:.2f} s; "
                      "per-sequence cost is identical, so tokens/s carries over to the whole batch"}


def suite(args):
    """Measurements beyond the default line: the decode step of workload 3 over all 32 layers, the
    compress phase of workload 4 over all 40 layers, and 64 decode steps of workload 5.  One JSON line."""
    import torch
    import paper_2310_02409_amd as D
    import workloads as W

    dev = torch.device("cuda:0")
    out = {"suite": True, "n_gpus": 1, "data": "synthetic", "dtype": "bf16"}

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3)
        ts.sort()
        return sum(ts) / len(ts), ts[0]

    # ---- workload 3: one token step across 32 layers, a nugget cache and a local window per layer
    wl = W.config(3)
    B, L = wl.B, wl.layers
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt, Sm = sum(ks), sum(wl.local_lens) + B
    cu_q, cu_l = W.cumulative([1] * B, dev), W.cumulative([m + 1 for m in wl.local_lens], dev)
    mk = lambda tid, n, h: W.normal(wl.seed, tid, (n, h, wl.d_h), 1.0, wl.dtype, dev)
    layers = [dict(Kn=mk(100 + 8 * l, Kt, wl.H_kv), Vn=mk(101 + 8 * l, Kt, wl.H_kv), Kl=mk(102 + 8 * l, Sm, wl.H_kv),
                   Vl=mk(103 + 8 * l, Sm, wl.H_kv), Q=mk(104 + 8 * l, B, wl.H)) for l in range(L)]
    O = torch.empty_like(layers[0]["Q"])
    max_m = max(wl.local_lens) + 1
    scale = wl.d_h ** -0.5

    def step3():
        for t in layers:
            D.dodo_nugget_attention(t["Q"], t["Kn"], t["Vn"], t["Kl"], t["Vl"], cu_q, cu_k, cu_l, 1, max(ks), max_m,
                                    scale, D.TOKEN_MAJOR, O)
    avg, mn = timed(step3, 10)
    by = 2 * (2 * (Kt + Sm) * wl.H_kv * wl.d_h + 2 * B * wl.H * wl.d_h) * L
    out["c3_decode_step_32_layers"] = {
        "launches": L, "avg_us": round(avg, 1), "min_us": round(mn, 1), "query_tokens_per_s": round(B / avg * 1e6),
        "GBps": round(by / avg * 1e-3, 1), "frac_of_8TBps": round(by / avg * 1e-3 / HBM_PEAK_GBS, 4),
        "bytes_per_step": by, "note": "64 ragged sequences, 20x compression, 256 local tokens + the token itself; "
                                      "32 launches of dodo_nugget_attention on 32 distinct caches (18.9 GB, no reuse)"}
    del layers
    torch.cuda.empty_cache()

    # ---- workload 4: score + select + gather over 40 layers
    wl = W.config(4)
    B, L = wl.B, wl.layers
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt = sum(ks)
    cu_s = W.cumulative(wl.seq_lens, dev)
    lay = [W.make_inputs(wl, dev, layer=l, which=["hidden", "w", "K", "V"]) for l in range(L)]
    # the layers' K and V in one allocation each ([L, N, H_kv, d_h]) so that one launch can pack all of them
    K_all = torch.empty((L,) + tuple(lay[0]["K"].shape), dtype=wl.dtype, device=dev)
    V_all = torch.empty_like(K_all)
    for l in range(L):
        K_all[l].copy_(lay[l]["K"])
        V_all[l].copy_(lay[l]["V"])
        lay[l]["K"], lay[l]["V"] = K_all[l], V_all[l]
    scores = torch.empty((L, wl.N), dtype=torch.float32, device=dev)
    idx = torch.empty((L, Kt), dtype=torch.int32, device=dev)
    Kn = torch.empty((L, Kt, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev)
    Vn = torch.empty_like(Kn)
    # all layers' sequences as one batch of L*B sequences for the single-launch select
    cu_s_all = W.cumulative(wl.seq_lens * L, dev)
    cu_k_all = W.cumulative(ks * L, dev)

    def per_layer():
        for l in range(L):
            D.dodo_score(lay[l]["hidden"], lay[l]["w"], 0.0, scores[l])
            D.dodo_select_topk(scores[l], cu_s, cu_k, max(wl.seq_lens), max(ks), Kt, D.FORCE_LAST, idx[l])
            D.dodo_gather_nuggets(lay[l]["K"], lay[l]["V"], idx[l], cu_s, cu_k, Kt, D.TOKEN_MAJOR, Kn[l], Vn[l])

    def batched_select():
        for l in range(L):
            D.dodo_score(lay[l]["hidden"], lay[l]["w"], 0.0, scores[l])
        D.dodo_select_topk(scores.view(-1), cu_s_all, cu_k_all, max(wl.seq_lens), max(ks), L * Kt, D.FORCE_LAST,
                           idx.view(-1))
        for l in range(L):
            D.dodo_gather_nuggets(lay[l]["K"], lay[l]["V"], idx[l], cu_s, cu_k, Kt, D.TOKEN_MAJOR, Kn[l], Vn[l])

    def shared_indices():
        # the Scorer reads one fixed layer and its indices serve every layer (Sec. 2.1): 3 launches in all
        D.dodo_score(lay[0]["hidden"], lay[0]["w"], 0.0, scores[0])
        D.dodo_select_topk(scores[0], cu_s, cu_k, max(wl.seq_lens), max(ks), Kt, D.FORCE_LAST, idx[0])
        D.dodo_gather_nuggets_layers(K_all, V_all, idx[0], cu_s, cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn)

    def shared_indices_gather_per_layer():
        D.dodo_score(lay[0]["hidden"], lay[0]["w"], 0.0, scores[0])
        D.dodo_select_topk(scores[0], cu_s, cu_k, max(wl.seq_lens), max(ks), Kt, D.FORCE_LAST, idx[0])
        for l in range(L):
            D.dodo_gather_nuggets(lay[l]["K"], lay[l]["V"], idx[0], cu_s, cu_k, Kt, D.TOKEN_MAJOR, Kn[l], Vn[l])
    E = 2
    by3 = (wl.N * wl.d_model * E + wl.d_model * E + 4 * wl.N + 4 * wl.N + 4 * Kt) + L * 4 * Kt * wl.H_kv * wl.d_h * E
    a3, m3 = timed(shared_indices, 5)
    a4, m4 = timed(shared_indices_gather_per_layer, 5)
    by = L * (wl.N * wl.d_model * E + wl.d_model * E + 4 * wl.N + 4 * wl.N + 4 * Kt + 4 * Kt * wl.H_kv * wl.d_h * E)
    a1, m1 = timed(per_layer, 5)
    a2, m2 = timed(batched_select, 5)
    out["c4_compress_40_layers"] = {
        "per_layer_rounds": {"launches": 3 * L, "avg_us": round(a1, 1), "min_us": round(m1, 1),
                             "GBps": round(by / a1 * 1e-3, 1)},
        "one_select_launch_for_all_layers": {"launches": 2 * L + 1, "avg_us": round(a2, 1), "min_us": round(m2, 1),
                                             "GBps": round(by / a2 * 1e-3, 1)},
        "shared_indices_one_gather_launch": {"launches": 3, "avg_us": round(a3, 1), "min_us": round(m3, 1),
                                             "GBps": round(by3 / a3 * 1e-3, 1), "bytes": by3},
        "shared_indices_gather_per_layer": {"launches": L + 2, "avg_us": round(a4, 1), "min_us": round(m4, 1),
                                            "GBps": round(by3 / a4 * 1e-3, 1), "bytes": by3},
        "bytes": by, "note": "16 x 2048 tokens, d = 5120, 20x compression. First two forms: per-layer scores and "
                             "selections (the second selects the 640 (layer, sequence) segments in one launch). Last "
                             "two: one scored layer whose indices pack all 40 layers, as in the paper (Sec. 2.1), "
                             "with one gather launch for all layers or one per layer"}
    del lay, Kn, Vn, K_all, V_all
    torch.cuda.empty_cache()

    # ---- workload 5: 64 decode steps after the 1024-token prefill (the local buffer grows by one row per step)
    wl = W.config(5)
    B = wl.B
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt = sum(ks)
    steps, m0 = 64, wl.q_lens[0]
    mk = lambda tid, n, h: W.normal(wl.seed, tid, (n, h, wl.d_h), 1.0, wl.dtype, dev)
    Kn, Vn = mk(200, Kt, wl.H_kv), mk(201, Kt, wl.H_kv)
    Kl, Vl = mk(202, B * (m0 + steps), wl.H_kv), mk(203, B * (m0 + steps), wl.H_kv)  # room for every step's rows
    Q = mk(204, B, wl.H)
    O = torch.empty_like(Q)
    cu_q = W.cumulative([1] * B, dev)
    # step t sees m0 + t + 1 local rows of each sequence: cumulative arrays with a fixed pitch are not packed,
    # so each step gets its own packed copy of the window (made outside the timed region)
    wins = []
    for t in range(steps):
        m = m0 + t + 1
        rows = torch.cat([torch.arange(b * (m0 + steps), b * (m0 + steps) + m, device=dev) for b in range(B)])
        wins.append((Kl[rows].contiguous(), Vl[rows].contiguous(), W.cumulative([m] * B, dev), m))
    ws_bytes = D.dodo_nugget_attention_workspace_bytes(B, wl.H, wl.d_h, 1, max(ks), m0 + steps, D.BF16)
    ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    def decode64():
        for kl, vl, cu_l, m in wins:
            D.dodo_nugget_attention(Q, Kn, Vn, kl, vl, cu_q, cu_k, cu_l, 1, max(ks), m0 + steps, scale, D.TOKEN_MAJOR, O,
                                    ws=ws)
    avg, mn = timed(decode64, 5)
    by = sum(2 * (2 * (Kt + B * w[3]) * wl.H_kv * wl.d_h + 2 * B * wl.H * wl.d_h) for w in wins)
    out["c5_decode_64_steps"] = {
        "launches": steps, "avg_us": round(avg, 1), "min_us": round(mn, 1), "us_per_step": round(avg / steps, 2),
        "query_tokens_per_s": round(B * steps / avg * 1e6), "GBps": round(by / avg * 1e-3, 1),
        "frac_of_8TBps": round(by / avg * 1e-3 / HBM_PEAK_GBS, 4),
        "note": "2 sequences, 3277 nuggets each, local buffer 1024 + t + 1 rows at step t; the same 107 MB nugget "
                "cache is re-read every step and stays in the 256 MB last-level cache, so this is not an HBM figure"}
    del Kn, Vn, Kl, Vl, wins
    torch.cuda.empty_cache()

    # ---- segment form of the autoregressive objective: workload 2's 8 x 4096 tokens as 64 segments of 512 tokens
    # that see the nuggets before (segment start - 128) and the uncompressed tokens from there on
    wl = W.config(2)
    B, seg_len, tau = wl.B, 512, 128
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt = sum(ks)
    cu_s = W.cumulative(wl.seq_lens, dev)
    mk = lambda tid, n, h: W.normal(wl.seed, tid, (n, h, wl.d_h), 1.0, wl.dtype, dev)
    Q, K, V = mk(300, wl.N, wl.H), mk(301, wl.N, wl.H_kv), mk(302, wl.N, wl.H_kv)
    Kn, Vn = mk(303, Kt, wl.H_kv), mk(304, Kt, wl.H_kv)
    sc = W.normal(wl.seed, 305, (wl.N,), 1.0, torch.float32, dev)
    idx = torch.empty(Kt, dtype=torch.int32, device=dev)
    D.dodo_select_topk(sc, cu_s, cu_k, max(wl.seq_lens), max(ks), Kt, D.FORCE_LAST, idx)
    E = sum(-(-n // seg_len) for n in wl.seq_lens)
    plan = D.dodo_segment_plan(idx, cu_s, cu_k, seg_len, tau, E)
    O = torch.empty_like(Q)
    a_plan, m_plan = timed(lambda: D.dodo_segment_plan(idx, cu_s, cu_k, seg_len, tau, E), 10)
    a_att, m_att = timed(lambda: D.dodo_nugget_attention_segments(Q, Kn, Vn, K, V, plan[0], plan[1], plan[2], plan[3],
                                                                  plan[4], seg_len, max(ks), seg_len + tau, scale,
                                                                  D.TOKEN_MAJOR, O), 10)
    cu_q_h, nl_h, ll_h = plan[0].cpu().tolist(), plan[2].cpu().tolist(), plan[4].cpu().tolist()
    pairs = 0
    for e in range(E):
        q = cu_q_h[e + 1] - cu_q_h[e]
        pairs += q * nl_h[e] + sum(min(ll_h[e], ll_h[e] - q + i + 1) for i in range(q))
    flop = 4.0 * pairs * wl.d_h * wl.H
    out["segment_form_8x4096_seg512_tau128"] = {
        "entries": E, "plan_avg_us": round(a_plan, 1), "attention_avg_us": round(a_att, 1),
        "attention_min_us": round(m_att, 1), "visible_pairs_per_head": pairs,
        "TFLOPs": round(flop / a_att * 1e-6, 1), "frac_of_bf16_peak": round(flop / a_att * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
        "query_tokens_per_s": round(wl.N / a_att * 1e6),
        "note": "forward attention of the training-time segment mask (Sec. 2.4): 32 heads x 128, 10x compression; "
                "every token of the 8 texts is a query row"}
    print(json.dumps(out))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.suite:
        suite(args)
        return
    import torch
    import paper_2310_02409_amd as D
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    wl = W.config(args.workload)
    E = 2 if wl.dtype == torch.bfloat16 else 4
    g = W.make_inputs(wl, dev)
    B = wl.B
    # decode sub-step: one new token per sequence; its local buffer is the prefill's plus the token itself
    dec_local = [m + 1 for m in wl.local_lens]
    g["Qd"] = W.normal(wl.seed, 10, (B, wl.H, wl.d_h), 1.0, wl.dtype, dev)
    g["Kld"] = W.normal(wl.seed, 11, (sum(dec_local), wl.H_kv, wl.d_h), 1.0, wl.dtype, dev)
    g["Vld"] = W.normal(wl.seed, 12, (sum(dec_local), wl.H_kv, wl.d_h), 1.0, wl.dtype, dev)
    cu_qd, cu_ld = W.cumulative([1] * B, dev), W.cumulative(dec_local, dev)
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt, max_n, max_k = sum(ks), max(wl.seq_lens), max(ks)
    max_q, max_m = max(wl.q_lens), max(wl.local_lens)
    scale = wl.d_h ** -0.5

    # every output and workspace is allocated once, outside the timed region
    scores = torch.empty(wl.N, dtype=torch.float32, device=dev)
    idx = torch.empty(Kt, dtype=torch.int32, device=dev)
    Kn = torch.empty((Kt, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev)
    Vn = torch.empty_like(Kn)
    O = torch.empty_like(g["Q"])
    Od = torch.empty_like(g["Qd"])
    ws_bytes = D.dodo_nugget_attention_workspace_bytes(B, wl.H, wl.d_h, 1, max_k, max(dec_local), D.BF16 if E == 2 else D.F32)
    ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    names = ["score", "select", "gather", "attn_block", "attn_decode"]

    def step(events=None):
        if events is not None:
            events[0].record()
        D.dodo_score(g["hidden"], g["w"], 0.0, scores)
        if events is not None:
            events[1].record()
        D.dodo_select_topk(scores, g["cu_seqlens"], cu_k, max_n, max_k, Kt, D.FORCE_LAST, idx)
        if events is not None:
            events[2].record()
        D.dodo_gather_nuggets(g["K"], g["V"], idx, g["cu_seqlens"], cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn)
        if events is not None:
            events[3].record()
        D.dodo_nugget_attention(g["Q"], Kn, Vn, g["Kl"], g["Vl"], g["cu_q"], cu_k, g["cu_local"], max_q, max_k, max_m,
                                scale, D.TOKEN_MAJOR, O)
        if events is not None:
            events[4].record()
        D.dodo_nugget_attention(g["Qd"], Kn, Vn, g["Kld"], g["Vld"], cu_qd, cu_k, cu_ld, 1, max_k, max(dec_local),
                                scale, D.TOKEN_MAJOR, Od, ws=ws)
        if events is not None:
            events[5].record()

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)  # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    work = algorithmic_work(wl, ks, E)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # Instrumented pre-pass (not part of the timed region): events between all calls give the
    # per-kernel breakdown and name the dominant kernel.  Each interval also contains the launch gap
    # to the previous kernel, so short kernels read a few microseconds longer than in a kernel trace.
    kernels = {}
    dom = None
    if not args.no_events:
        pre_steps = max(10, min(50, args.steps))
        pev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(pre_steps)]
        for k in range(pre_steps):
            step(pev[k])
        torch.cuda.synchronize()
        for j, name in enumerate(names):
            us = sorted(e[j].elapsed_time(e[j + 1]) * 1e3 for e in pev)
            avg = sum(us) / len(us)
            kernels[name] = {"avg_us": round(avg, 2), "median_us": round(us[len(us) // 2], 2), "min_us": round(us[0], 2),
                             "GBps": round(work[name]["bytes"] / avg * 1e-3, 1),
                             "TFLOPs": round(work[name]["flop"] / avg * 1e-6, 2)}
        kernels["attn_block"]["query_tokens_per_s"] = round(sum(wl.q_lens) / kernels["attn_block"]["avg_us"] * 1e6)
        kernels["attn_decode"]["query_tokens_per_s"] = round(B / kernels["attn_decode"]["avg_us"] * 1e6)
        tg = kernels["select"]["avg_us"] + kernels["gather"]["avg_us"]
        kernels["topk_plus_gather_GBps"] = round((work["select"]["bytes"] + work["gather"]["bytes"]) / tg * 1e-3, 1)
        kernels["note"] = "instrumented pre-pass with events between all calls"
        dom = max(names, key=lambda n: kernels[n]["avg_us"])

        # The autoregressive mode's selection (threshold rule), outside the step and its timing: Lambda from
        # the step's own scores as the sample, threshold selection of the whole batch, and one decode step
        # (append the leaving token of every sequence, then attend over the caches with room to grow).
        cap = max_k + 64
        lam = D.dodo_threshold_from_sample(scores, wl.keep_num, wl.keep_den)
        Kc = torch.zeros((B, cap, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev)
        Vc = torch.zeros_like(Kc)
        counts = torch.zeros(B, dtype=torch.int32, device=dev)
        Kc[:, :max_k] = Kn.view(B, -1, wl.H_kv, wl.d_h)[:, :max_k] if len(set(ks)) == 1 else 0
        Vc[:, :max_k] = Vn.view(B, -1, wl.H_kv, wl.d_h)[:, :max_k] if len(set(ks)) == 1 else 0
        counts.fill_(max_k if len(set(ks)) == 1 else 0)
        starts = (torch.arange(B, dtype=torch.int32, device=dev) * cap).contiguous()
        leave_s = scores[: B].clone()
        leave_K, leave_V = g["K"][: B].contiguous(), g["V"][: B].contiguous()
        ar_calls = {
            "threshold_from_sample": lambda: D.dodo_threshold_from_sample(scores, wl.keep_num, wl.keep_den, out=lam),
            "select_threshold": lambda: D.dodo_select_threshold(scores, g["cu_seqlens"], lam),
            "stream_append": lambda: (counts.fill_(max_k if len(set(ks)) == 1 else 0),
                                      D.dodo_stream_append(leave_s, lam, leave_K, leave_V, counts, Kc, Vc)),
            "attn_decode_cached": lambda: D.dodo_nugget_attention_cached(
                g["Qd"], Kc.view(B * cap, wl.H_kv, wl.d_h), Vc.view(B * cap, wl.H_kv, wl.d_h), g["Kld"], g["Vld"], cu_qd,
                starts, counts, cu_ld, 1, cap, max(dec_local), scale, D.TOKEN_MAJOR, Od, ws=ws_c),
        }
        ws_c_bytes = D.dodo_nugget_attention_workspace_bytes(B, wl.H, wl.d_h, 1, cap, max(dec_local),
                                                             D.BF16 if E == 2 else D.F32)
        ws_c = torch.zeros(max(ws_c_bytes, 16), dtype=torch.uint8, device=dev)
        ar = {}
        for name, fn in ar_calls.items():
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
            for a, b in evs:
                a.record()
                fn()
                b.record()
            torch.cuda.synchronize()
            us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
            ar[name] = {"avg_us": round(sum(us) / len(us), 2), "min_us": round(us[0], 2)}
        # the pooling baseline's compaction (same output shape as the gather)
        for _ in range(3):
            D.dodo_meanpool_nuggets(g["K"], g["V"], g["cu_seqlens"], cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
        for a, b in evs:
            a.record()
            D.dodo_meanpool_nuggets(g["K"], g["V"], g["cu_seqlens"], cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn)
            b.record()
        torch.cuda.synchronize()
        us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        mp_bytes = 2 * (wl.N + Kt) * wl.H_kv * wl.d_h * E
        kernels["meanpool_baseline"] = {"avg_us": round(sum(us) / len(us), 2), "min_us": round(us[0], 2),
                                        "GBps": round(mp_bytes / (sum(us) / len(us)) * 1e-3, 1)}
        D.dodo_gather_nuggets(g["K"], g["V"], idx, g["cu_seqlens"], cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn)  # restore the cache
        # gather-free attention: the nuggets are read in place through the index list (no packed cache)
        def _timed_us(fn, reps=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, b in evs:
                a.record()
                fn()
                b.record()
            torch.cuda.synchronize()
            us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
            return round(sum(us) / len(us), 2), round(us[0], 2)
        gf = {}
        a, m = _timed_us(lambda: D.dodo_nugget_attention_indexed(
            g["Q"], g["K"], g["V"], idx, g["cu_seqlens"], g["Kl"], g["Vl"], g["cu_q"], cu_k, g["cu_local"], max_q, max_k,
            max_m, max_n, scale, O=O))
        gf["attn_block_indexed"] = {"avg_us": a, "min_us": m}
        a, m = _timed_us(lambda: D.dodo_nugget_attention_indexed(
            g["Qd"], g["K"], g["V"], idx, g["cu_seqlens"], g["Kld"], g["Vld"], cu_qd, cu_k, cu_ld, 1, max_k,
            max(dec_local), max_n, scale, O=Od, ws=ws))
        gf["attn_decode_indexed"] = {"avg_us": a, "min_us": m}
        gf["note"] = ("same results, bit for bit, as gather + attention; compare with gather + attn_block and "
                      "gather + attn_decode above")
        kernels["gather_free"] = gf
        # score gradient of the straight-through estimator for this layer (backward of the block attention's
        # nugget columns), fed with the O of the step and a fresh lse
        if E == 2:
            lse_b = torch.empty((g["Q"].shape[0], wl.H), dtype=torch.float32, device=dev)
            D.dodo_nugget_attention(g["Q"], Kn, Vn, g["Kl"], g["Vl"], g["cu_q"], cu_k, g["cu_local"], max_q, max_k, max_m,
                                    scale, D.TOKEN_MAJOR, O, lse=lse_b)
            dO = W.normal(wl.seed, 99, tuple(g["Q"].shape), 1.0, wl.dtype, dev)
            ste_ws = torch.empty(D.dodo_ste_score_grad_workspace_bytes(g["Q"].shape[0], wl.H, Kt), dtype=torch.uint8,
                                 device=dev)
            ste_grad = torch.empty(Kt, dtype=torch.float32, device=dev)
            a, m = _timed_us(lambda: D.dodo_ste_score_grad(g["Q"], Kn, Vn, dO, O, lse_b, g["cu_q"], cu_k, max_q, max_k,
                                                           scale, scale, D.TOKEN_MAJOR, grad=ste_grad, ws=ste_ws))
            ste_flop = 4.0 * sum(q * k for q, k in zip(wl.q_lens, ks)) * wl.d_h * wl.H
            kernels["ste_score_grad"] = {"avg_us": a, "min_us": m, "TFLOPs": round(ste_flop / a * 1e-6, 1),
                                         "frac_of_bf16_peak": round(ste_flop / a * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 3),
                                         "note": "whole call: row dots, the MFMA kernel, the sum over heads (training "
                                                 "path, not part of the step)"}
            del dO, ste_ws
        # the scorer as a 2-layer feedforward network (d -> d -> 1) over the step's hidden states
        if E == 2:
            d_model = g["hidden"].shape[1]
            gen = torch.Generator(device="cpu").manual_seed(wl.seed + 77)
            W1 = (torch.randn(d_model, d_model, generator=gen) * d_model ** -0.5).to(torch.bfloat16).to(dev)
            b1 = (torch.randn(d_model, generator=gen) * 0.5).to(dev)
            w2 = (torch.randn(d_model, generator=gen) * d_model ** -0.5).to(torch.bfloat16).to(dev)
            mlp_ws = torch.empty(max(D.dodo_score_mlp_workspace_bytes(D.BF16, wl.N, d_model, d_model), 16),
                                 dtype=torch.uint8, device=dev)
            mlp_out = torch.empty(wl.N, dtype=torch.float32, device=dev)
            for _ in range(2):
                D.dodo_score_mlp(g["hidden"], W1, b1, w2, 0.0, D.RELU, mlp_out, mlp_ws)
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
            for a, b in evs:
                a.record()
                D.dodo_score_mlp(g["hidden"], W1, b1, w2, 0.0, D.RELU, mlp_out, mlp_ws)
                b.record()
            torch.cuda.synchronize()
            us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
            mlp_flop = 2.0 * wl.N * d_model * d_model
            kernels["scorer_2layer"] = {"avg_us": round(sum(us) / len(us), 2), "min_us": round(us[0], 2),
                                        "TFLOPs": round(mlp_flop / (sum(us) / len(us)) * 1e-6, 1),
                                        "frac_of_bf16_peak": round(mlp_flop / (sum(us) / len(us)) * 1e-6 / 2500.0, 3),
                                        "note": "ReLU, d_hid = d; replaces the linear head when used (not part of the step)"}
            del W1, mlp_ws
        ar["note"] = ("threshold rule of the autoregressive mode, timed apart from the step: sample = the step's "
                      f"{wl.N} scores; stream_append includes a fill of the {B} counters; caches of {cap} rows per sequence")
        kernels["autoregressive_mode"] = ar

    # Timed region: exactly `steps` steps; the only events inside it bracket the dominant kernel.
    dom_idx = names.index(dom) if dom is not None else -1

    def timed_step(e0, e1):
        calls = [
            lambda: D.dodo_score(g["hidden"], g["w"], 0.0, scores),
            lambda: D.dodo_select_topk(scores, g["cu_seqlens"], cu_k, max_n, max_k, Kt, D.FORCE_LAST, idx),
            lambda: D.dodo_gather_nuggets(g["K"], g["V"], idx, g["cu_seqlens"], cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn),
            lambda: D.dodo_nugget_attention(g["Q"], Kn, Vn, g["Kl"], g["Vl"], g["cu_q"], cu_k, g["cu_local"], max_q,
                                            max_k, max_m, scale, D.TOKEN_MAJOR, O),
            lambda: D.dodo_nugget_attention(g["Qd"], Kn, Vn, g["Kld"], g["Vld"], cu_qd, cu_k, cu_ld, 1, max_k,
                                            max(dec_local), scale, D.TOKEN_MAJOR, Od, ws=ws),
        ]
        for j, c in enumerate(calls):
            if j == dom_idx:
                e0.record()
                c()
                e1.record()
            else:
                c()

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        timed_step(*ev[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    q_tokens = sum(wl.q_lens) + B
    value = q_tokens / (ms_per_step * 1e-3)

    roof = None
    if dom is not None:
        us = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
        avg = sum(us) / len(us)
        if dom == "attn_block":
            ach = work[dom]["flop"] / avg * 1e-6
            roof = {"kernel": dom, "bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None}
            # a kernel near the ridge: what the two peaks allow together at its algorithmic intensity
            intensity = work[dom]["flop"] / work[dom]["bytes"]
            attainable = min(MFMA_BF16_PEAK_TFLOPS, intensity * HBM_PEAK_GBS * 1e-3)
            roof["intensity_flop_per_byte"] = round(intensity, 1)
            roof["attainable"] = round(attainable, 1)
            roof["frac_of_attainable"] = round(ach / attainable, 4)
            roof["hbm_GBps_at_this_time"] = round(work[dom]["bytes"] / avg * 1e-3, 1)
        else:
            ach = work[dom]["bytes"] / avg * 1e-3
            roof = {"kernel": dom, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None}
        roof["avg_us"] = round(avg, 2)
        roof["launches"] = len(us)
        tpath = os.path.join(ROOT, "profiles", "traffic.json")
        if os.path.exists(tpath):  # HBM bytes per launch from the committed counter runs, if recorded for this kernel
            roof["traffic"] = json.load(open(tpath)).get(wl.name, {}).get(dom)

    cpu = None
    if not args.no_cpu_baseline:
        host = {k: W.to_numpy(v) for k, v in g.items() if k in ("hidden", "w", "K", "V", "Q", "Kl", "Vl")}
        n0, m0 = wl.seq_lens[0], wl.local_lens[0]
        host = {k: (v[:n0] if k in ("hidden", "K", "V") else v) for k, v in host.items()}
        host["Qd"], host["Kld"], host["Vld"] = (W.to_numpy(g[k][:m0 + 1]) for k in ("Qd", "Kld", "Vld"))
        cpu = cpu_baseline(wl, host, ks, scale)
        cpu["value"] = round(cpu["value"], 2)

    line = {
        "metric": "nugget-attention query tokens/s (whole hot-path step: score+TopK+gather+block attention+decode token)",
        "value": round(value, 1), "unit": "query tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if E == 2 else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "batch": B, "context": wl.seq_lens[0] if len(set(wl.seq_lens)) == 1 else "ragged",
                   "nuggets_per_seq": ks[0], "query_block": max_q, "local_tokens": wl.tau[0], "d_model": wl.d_model,
                   "heads": wl.H, "head_dim": wl.d_h, "layers": 1, "decode_tokens_per_seq": 1},
        "roofline": roof, "cpu_baseline": cpu, "kernels": kernels,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
