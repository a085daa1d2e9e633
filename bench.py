#!/usr/bin/env python3
"""Benchmark of the Dodo hot path on one MI355X.

Headline (the timed region): the LLaMA-13B-shaped autoencoding workload, the largest of the five that runs on one
GPU -- bf16, batch 16, 2048 context tokens per sequence at 20x compression (103 nuggets), 40 layers, then a
2048-token causal query block per sequence.  One "step" is one pass of the whole path over that batch, every
layer on its own tensors (80 GB of inputs, nothing is re-read from a cache):

    for each of the 40 layers:
        dodo_score -> dodo_select_topk -> dodo_gather_nuggets        (compress the layer's context)
        dodo_nugget_attention                                        (2048-row query block over nuggets + itself)

`value` = query tokens of the batch (16 x 2048) per second of whole-step time.  `roofline` describes the dominant
kernel, the query-block attention, from events around each of its launches inside the timed region.

`kernels` then holds, per workload (c2 prefill, c3 32-layer decode, c4, c5 long context), every kernel's time,
GB/s or TFLOP/s and fraction of the HBM / bf16 matrix peak; bandwidth-bound kernels are timed over four rotating
buffer sets (more than the 256 MB last-level cache holds), and a read-only stream and a copy kernel written in the
same style are timed in the same run as what this device's memory system gives such code (`ceilings`).
`cpu_baseline` is the oracle timed on one host core on a bounded sample (a reported baseline, not a target).
All inputs are synthetic and resident in HBM before any timed region.  Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
E = 2                           # bytes per element (bf16 workloads)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workloads", default="c4,c2,c3,c5",
                    help="which per-workload kernel tables to measure (c4, the headline, always runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip the kernels beyond the four-call path (threshold rule, pooling baseline, gather-free "
                         "attention, score gradient, 2-layer scorer, segment form)")
    return ap.parse_args()


# ------------------------------------------------------------------------------------------------ helpers
def work_score(N, d):
    return {"bytes": N * d * E + d * E + 4 * N, "flop": 2 * N * d}


def work_select(N, Kt, B):
    return {"bytes": 4 * N + 4 * Kt + 8 * (B + 1), "flop": 0}


def work_gather(Kt, Hd):
    return {"bytes": 2 * (2 * Kt * Hd * E) + 4 * Kt, "flop": 0}


def work_attention(q_lens, k_lens, m_lens, H, H_kv, d_h):
    """Algorithmic work of the attention: masked pairs are not counted, every K/V row is counted once."""
    pairs = 0
    for q, k, m in zip(q_lens, k_lens, m_lens):
        lo = m - q + 1  # local rows visible to the first query row (may be <= 0)
        pairs += q * k + sum(max(0, min(m, lo + i)) for i in range(q))
    return {"bytes": E * (2 * sum(q_lens) * H * d_h + 2 * (sum(k_lens) + sum(m_lens)) * H_kv * d_h),
            "flop": 4 * d_h * H * pairs}


def hbm_row(us, work):
    gbs = work["bytes"] / us * 1e-3
    return {"avg_us": round(us, 2), "GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            "bound": "hbm", "bytes": work["bytes"]}


def mfma_row(us, work):
    tf = work["flop"] / us * 1e-6
    return {"avg_us": round(us, 2), "TFLOPs": round(tf, 1), "frac_of_bf16_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
            "bound": "mfma", "flop": work["flop"], "GBps": round(work["bytes"] / us * 1e-3, 1)}


class Clock:
    """Event timing on torch's current stream, which is the stream every library call is given."""

    def __init__(self, torch):
        self.torch = torch

    def batched(self, calls, rounds=6, inner=3):
        """Average and minimum time per call, in microseconds, of the calls in `calls` (one per rotating buffer
        set) launched back to back `inner` times between one pair of events."""
        torch = self.torch
        for c in calls:
            c()
        torch.cuda.synchronize()
        per = []
        for _ in range(rounds):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(inner):
                for c in calls:
                    c()
            e1.record()
            torch.cuda.synchronize()
            per.append(e0.elapsed_time(e1) * 1e3 / (inner * len(calls)))
        return sum(per) / len(per), min(per)


    def pipeline(self, sets, fns, rounds=3):
        """The calls of `fns` (name -> callable(set)) in path order on one rotating buffer set after another, with
        an event between all calls: average microseconds per call as it runs inside the path (each interval also
        holds the gap to the previous launch)."""
        torch = self.torch
        names = list(fns)
        evs = []
        for _ in range(rounds):
            for g in sets:
                e = [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)]
                for j, n in enumerate(names):
                    e[j].record()
                    fns[n](g)
                e[-1].record()
                evs.append(e)
        torch.cuda.synchronize()
        return {n: sum(e[j].elapsed_time(e[j + 1]) for e in evs) * 1e3 / len(evs) for j, n in enumerate(names)}


def add_pipeline_times(table, times, work):
    """Adds the in-path time of every kernel to its row (and, for the matrix-core kernel, the fraction it gives)."""
    for n, us in times.items():
        table[n]["in_pipeline_us"] = round(us, 2)
        if table[n].get("bound") == "mfma":
            table[n]["frac_of_bf16_peak_in_pipeline"] = round(work[n]["flop"] / us * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4)


# ------------------------------------------------------------------------------------------------ ceilings
def measure_ceilings(torch, D, clock, dev):
    """What the memory system gives a plain streaming kernel here, at a large size and at the size of the small
    workloads' kernels (where launch, ramp-up and drain weigh): four rotating buffers each."""
    out = {"nominal_hbm_peak_GBps": HBM_PEAK_GBS,
           "note": "4 rotating buffers per size; copy = bytes read + bytes written; the small size is about what the "
                   "gather and decode kernels of workloads 2 and 5 move per launch"}
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    for label, n in (("512MiB", 512 << 20), ("128MiB", 128 << 20)):
        bufs = [torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(4)]
        dst = [torch.empty(n // 2, dtype=torch.uint8, device=dev) for _ in range(4)]
        rd, _ = clock.batched([lambda b=b: D.dodo_probe_read(b, sink) for b in bufs], rounds=4, inner=2)
        cp, _ = clock.batched([lambda b=b, d=d: D.dodo_probe_copy(b[: n // 2], d) for b, d in zip(bufs, dst)], rounds=4, inner=2)
        rt, _ = clock.batched([lambda b=b, d=d: d.copy_(b[: n // 2]) for b, d in zip(bufs, dst)], rounds=4, inner=2)
        out[label] = {"read_stream_GBps": round(n / rd * 1e-3, 1), "read_stream_us": round(rd, 2),
                      "copy_kernel_GBps": round(n / cp * 1e-3, 1), "copy_kernel_us": round(cp, 2),
                      "runtime_copy_GBps": round(n / rt * 1e-3, 1)}
        del bufs, dst
        torch.cuda.empty_cache()
    return out


# ------------------------------------------------------------------------------------------------ workload 4 (headline)
def run_c4(torch, D, W, clock, dev, args):
    wl = W.config(4)
    B, L = wl.B, wl.layers
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt, max_n, max_k = sum(ks), max(wl.seq_lens), max(ks)
    max_q, max_m = max(wl.q_lens), max(wl.local_lens)
    Sq = sum(wl.q_lens)
    scale = wl.d_h ** -0.5
    lay = [W.make_inputs(wl, dev, layer=l) for l in range(L)]
    cu_s, cu_q, cu_l = lay[0]["cu_seqlens"], lay[0]["cu_q"], lay[0]["cu_local"]
    scores = torch.empty((L, wl.N), dtype=torch.float32, device=dev)
    idx = torch.empty((L, Kt), dtype=torch.int32, device=dev)
    Kn = torch.empty((L, Kt, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev)
    Vn = torch.empty_like(Kn)
    O = torch.empty_like(lay[0]["Q"])
    names = ["score", "select", "gather", "attn_block"]

    def layer_calls(l):
        t = lay[l]
        return [
            lambda: D.dodo_score(t["hidden"], t["w"], 0.0, scores[l]),
            lambda: D.dodo_select_topk(scores[l], cu_s, cu_k, max_n, max_k, Kt, D.FORCE_LAST, idx[l]),
            lambda: D.dodo_gather_nuggets(t["K"], t["V"], idx[l], cu_s, cu_k, Kt, D.TOKEN_MAJOR, Kn[l], Vn[l]),
            lambda: D.dodo_nugget_attention(t["Q"], Kn[l], Vn[l], t["Kl"], t["Vl"], cu_q, cu_k, cu_l, max_q, max_k,
                                            max_m, scale, D.TOKEN_MAJOR, O),
        ]
    calls = [layer_calls(l) for l in range(L)]

    def step(attn_events=None):
        for l in range(L):
            c = calls[l]
            c[0]()
            c[1]()
            c[2]()
            if attn_events is not None:
                attn_events[l][0].record()
                c[3]()
                attn_events[l][1].record()
            else:
                c[3]()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # instrumented pre-pass (not the timed region): events between all calls of two steps
    ev = [[[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(L)] for _ in range(2)]
    for s in range(2):
        for l in range(L):
            for j in range(4):
                ev[s][l][j].record()
                calls[l][j]()
            ev[s][l][4].record()
    torch.cuda.synchronize()
    per = {n: [] for n in names}
    for s in range(2):
        for l in range(L):
            for j, n in enumerate(names):
                per[n].append(ev[s][l][j].elapsed_time(ev[s][l][j + 1]) * 1e3)
    work = {"score": work_score(wl.N, wl.d_model), "select": work_select(wl.N, Kt, B),
            "gather": work_gather(Kt, wl.H_kv * wl.d_h),
            "attn_block": work_attention(wl.q_lens, ks, wl.local_lens, wl.H, wl.H_kv, wl.d_h)}
    table = {}
    for n in names:
        us = sum(per[n]) / len(per[n])
        table[n] = mfma_row(us, work[n]) if n == "attn_block" else hbm_row(us, work[n])
        table[n]["min_us"] = round(min(per[n]), 2)
    table["select"].pop("frac_of_hbm_peak")  # latency-bound integer kernel: 16 workgroups
    table["select"]["bound"] = "latency"
    tg = table["select"]["avg_us"] + table["gather"]["avg_us"]
    table["topk_plus_gather_GBps"] = round((work["select"]["bytes"] + work["gather"]["bytes"]) / tg * 1e-3, 1)
    table["attn_block"]["query_tokens_per_s_per_layer"] = round(Sq / table["attn_block"]["avg_us"] * 1e6)
    for n, j in (("score", 0), ("gather", 2), ("attn_block", 3)):  # the same kernels launched back to back on 4 layers
        a, _ = clock.batched([calls[l][j] for l in range(4)])
        table[n]["back_to_back_us"] = round(a, 2)
        if n == "attn_block":
            table[n]["frac_of_bf16_peak_back_to_back"] = round(work[n]["flop"] / a * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4)
        else:
            table[n]["frac_of_hbm_peak_back_to_back"] = round(work[n]["bytes"] / a * 1e-3 / HBM_PEAK_GBS, 4)
    table["note"] = ("per layer; avg_us from events between all calls of two untimed steps (each interval includes the gap "
                     "to the previous launch), 40 layers on 40 distinct tensor sets; back_to_back_us = the kernel alone, "
                     "launched back to back on 4 layers' tensors")

    # the compress phase of all 40 layers with the layers' tensors in one allocation each
    H_all = torch.stack([t["hidden"] for t in lay])
    w_all = torch.stack([t["w"] for t in lay])
    K_all = torch.stack([t["K"] for t in lay])
    V_all = torch.stack([t["V"] for t in lay])
    cu_s_all, cu_k_all = W.cumulative(wl.seq_lens * L, dev), W.cumulative(ks * L, dev)

    def compress_3_launches():  # per-layer scores and selections: every (layer, sequence) is a sequence of one batch
        D.dodo_score_layers(H_all, w_all, None, scores)
        D.dodo_select_topk(scores.view(-1), cu_s_all, cu_k_all, max_n, max_k, L * Kt, D.FORCE_LAST, idx.view(-1))
        D.dodo_gather_nuggets(K_all.view(L * wl.N, wl.H_kv, wl.d_h), V_all.view(L * wl.N, wl.H_kv, wl.d_h), idx.view(-1),
                              cu_s_all, cu_k_all, L * Kt, D.TOKEN_MAJOR, Kn.view(L * Kt, wl.H_kv, wl.d_h),
                              Vn.view(L * Kt, wl.H_kv, wl.d_h))

    def compress_shared_indices():  # the paper's form (Sec. 2.1): one scored layer, its indices pack every layer
        D.dodo_score(lay[0]["hidden"], lay[0]["w"], 0.0, scores[0])
        D.dodo_select_topk(scores[0], cu_s, cu_k, max_n, max_k, Kt, D.FORCE_LAST, idx[0])
        D.dodo_gather_nuggets_layers(K_all, V_all, idx[0], cu_s, cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn)

    def compress_per_layer():
        for l in range(L):
            calls[l][0]()
            calls[l][1]()
            calls[l][2]()
    by_all = L * (work["score"]["bytes"] + work["select"]["bytes"] + work["gather"]["bytes"])
    by_shared = work["score"]["bytes"] + work["select"]["bytes"] + L * work["gather"]["bytes"]
    comp = {}
    for name, fn, by, launches in (("per_layer_calls", compress_per_layer, by_all, 3 * L),
                                   ("layered_calls", compress_3_launches, by_all, 3),
                                   ("shared_indices", compress_shared_indices, by_shared, 3)):
        a, m_ = clock.batched([fn], rounds=4, inner=1)
        comp[name] = {"launches": launches, "avg_us": round(a, 1), "min_us": round(m_, 1), "GBps": round(by / a * 1e-3, 1),
                      "frac_of_hbm_peak": round(by / a * 1e-3 / HBM_PEAK_GBS, 4), "bytes": by}
    comp["note"] = ("compress phase of all 40 layers: per_layer_calls = 120 launches (score, select, gather per layer); "
                    "layered_calls = dodo_score_layers + one select and one gather over the 640 (layer, sequence) segments; "
                    "shared_indices = one scored layer whose indices pack all 40 layers (dodo_gather_nuggets_layers)")
    table["compress_40_layers"] = comp
    del H_all, w_all, K_all, V_all

    # ---- timed region: exactly `steps` steps; events only around the dominant kernel's launches
    steps = args.steps
    aev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)]
           for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(aev[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    us = [a.elapsed_time(b) * 1e3 for st in aev for a, b in st]
    avg = sum(us) / len(us)
    ach = work["attn_block"]["flop"] / avg * 1e-6
    intensity = work["attn_block"]["flop"] / work["attn_block"]["bytes"]
    roof = {"kernel": "block_attention_kernel (dodo_nugget_attention, 2048-row causal query blocks)", "bound": "mfma",
            "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None, "avg_us": round(avg, 2),
            "min_us": round(min(us), 2), "launches": len(us), "flop_per_launch": work["attn_block"]["flop"],
            "bytes_per_launch": work["attn_block"]["bytes"], "intensity_flop_per_byte": round(intensity, 1)}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):  # HBM bytes per launch from the committed counter runs
        roof["traffic"] = json.load(open(tpath)).get(wl.name, {}).get("attn_block")
    head = {"ms_per_step": ms_per_step, "value": Sq / (ms_per_step * 1e-3), "roofline": roof,
            "config": {"workload": wl.name, "batch": B, "context": wl.seq_lens[0], "nuggets_per_seq": ks[0],
                       "query_block": max_q, "local_tokens": wl.tau[0], "d_model": wl.d_model, "heads": wl.H,
                       "head_dim": wl.d_h, "layers": L, "launches_per_step": 4 * L}}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline_c4(W, wl, lay[0], ks, scale)
    del lay, calls, Kn, Vn, scores
    torch.cuda.empty_cache()
    return head, table, cpu


def cpu_baseline_c4(W, wl, t, ks, scale):
    """The oracle, as it stands, on one host core: sequence 0 of layer 0 (compress its 2048-token context, then
    the attention of its 40 heads x 2048 rows)."""
    import oracle
    n0, q0, m0, k0 = wl.seq_lens[0], wl.q_lens[0], wl.local_lens[0], ks[0]
    host = {k: W.to_numpy(t[k][:n0]) for k in ("hidden", "K", "V")}
    host["w"] = W.to_numpy(t["w"])
    host.update({k: W.to_numpy(t[k][:q0]) for k in ("Q",)})
    host.update({k: W.to_numpy(t[k][:m0]) for k in ("Kl", "Vl")})
    cu_s, cu_k = oracle.cu_from_lengths([n0]), oracle.cu_from_lengths([k0])
    cu_q, cu_m = oracle.cu_from_lengths([q0]), oracle.cu_from_lengths([m0])
    t0 = time.perf_counter()
    s = oracle.score(host["hidden"], host["w"])
    idx = oracle.select_topk(s, cu_s, cu_k, oracle.FORCE_LAST)
    Kn, Vn = oracle.gather(host["K"], host["V"], idx, cu_s, cu_k)
    t1 = time.perf_counter()
    heads = wl.H  # about 47 GFLOP in double precision
    rows = [(0, h, i) for h in range(heads) for i in range(q0)]
    oracle.attention_rows(host["Q"], Kn, Vn, host["Kl"], host["Vl"], cu_q, cu_k, cu_m, scale, rows)
    t2 = time.perf_counter()
    per_layer_seq = (t1 - t0) + (t2 - t1) * wl.H / heads  # one sequence, one layer, all heads
    total = per_layer_seq * wl.layers
    return {"value": round(q0 / total, 3), "unit": "query tokens/s", "cores": 1, "kind": "oracle",
            "sample": f"layer 0, sequence 0 of {wl.B} (n={n0}, k={k0}, q={q0}): score+select+gather {t1 - t0:.2f} s, "
                      f"attention of {heads} heads x {q0} rows {t2 - t1:.2f} s; extrapolated to "
                      f"{wl.layers} layers (every layer and sequence costs the same), single thread"}


# ------------------------------------------------------------------------------------------------ workload 2
def run_c2(torch, D, W, clock, dev, args):
    wl = W.config(2)
    B, S = wl.B, 4  # four rotating sets of every input
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt, max_n, max_k = sum(ks), max(wl.seq_lens), max(ks)
    max_q, max_m = max(wl.q_lens), max(wl.local_lens)
    scale = wl.d_h ** -0.5
    dec_local = [m + 1 for m in wl.local_lens]
    cu_qd, cu_ld = W.cumulative([1] * B, dev), W.cumulative(dec_local, dev)
    sets = []
    for s in range(S):
        g = W.make_inputs(wl, dev, layer=s)
        g["Qd"] = W.normal(wl.seed, 1000 + 16 * s, (B, wl.H, wl.d_h), 1.0, wl.dtype, dev)
        g["Kld"] = W.normal(wl.seed, 1001 + 16 * s, (sum(dec_local), wl.H_kv, wl.d_h), 1.0, wl.dtype, dev)
        g["Vld"] = W.normal(wl.seed, 1002 + 16 * s, (sum(dec_local), wl.H_kv, wl.d_h), 1.0, wl.dtype, dev)
        g["scores"] = torch.empty(wl.N, dtype=torch.float32, device=dev)
        g["idx"] = torch.empty(Kt, dtype=torch.int32, device=dev)
        g["Kn"] = torch.empty((Kt, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev)
        g["Vn"] = torch.empty_like(g["Kn"])
        g["O"], g["Od"] = torch.empty_like(g["Q"]), torch.empty_like(g["Qd"])
        sets.append(g)
    ws_bytes = D.dodo_nugget_attention_workspace_bytes(B, wl.H, wl.d_h, 1, max_k, max(dec_local), D.BF16)
    ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    cu_s, cu_q, cu_l = sets[0]["cu_seqlens"], sets[0]["cu_q"], sets[0]["cu_local"]
    fns = {
        "score": lambda g: D.dodo_score(g["hidden"], g["w"], 0.0, g["scores"]),
        "select": lambda g: D.dodo_select_topk(g["scores"], cu_s, cu_k, max_n, max_k, Kt, D.FORCE_LAST, g["idx"]),
        "gather": lambda g: D.dodo_gather_nuggets(g["K"], g["V"], g["idx"], cu_s, cu_k, Kt, D.TOKEN_MAJOR, g["Kn"], g["Vn"]),
        "attn_block": lambda g: D.dodo_nugget_attention(g["Q"], g["Kn"], g["Vn"], g["Kl"], g["Vl"], cu_q, cu_k, cu_l, max_q,
                                                        max_k, max_m, scale, D.TOKEN_MAJOR, g["O"]),
        "attn_decode": lambda g: D.dodo_nugget_attention(g["Qd"], g["Kn"], g["Vn"], g["Kld"], g["Vld"], cu_qd, cu_k, cu_ld,
                                                         1, max_k, max(dec_local), scale, D.TOKEN_MAJOR, g["Od"], ws=ws),
    }
    for g in sets:  # fill every set's intermediate tensors once
        for n in fns:
            fns[n](g)
    work = {"score": work_score(wl.N, wl.d_model), "select": work_select(wl.N, Kt, B),
            "gather": work_gather(Kt, wl.H_kv * wl.d_h),
            "attn_block": work_attention(wl.q_lens, ks, wl.local_lens, wl.H, wl.H_kv, wl.d_h),
            "attn_decode": work_attention([1] * B, ks, dec_local, wl.H, wl.H_kv, wl.d_h)}
    table = {}
    for n, f in fns.items():
        a, m = clock.batched([lambda g=g, f=f: f(g) for g in sets])
        table[n] = mfma_row(a, work[n]) if n == "attn_block" else hbm_row(a, work[n])
        table[n]["min_us"] = round(m, 2)
    table["select"].pop("frac_of_hbm_peak")
    table["select"]["bound"] = "latency"
    add_pipeline_times(table, clock.pipeline(sets, fns), work)
    tg = table["select"]["avg_us"] + table["gather"]["avg_us"]
    table["topk_plus_gather_GBps"] = round((work["select"]["bytes"] + work["gather"]["bytes"]) / tg * 1e-3, 1)
    table["attn_block"]["query_tokens_per_s"] = round(sum(wl.q_lens) / table["attn_block"]["in_pipeline_us"] * 1e6)
    table["attn_decode"]["query_tokens_per_s"] = round(B / table["attn_decode"]["avg_us"] * 1e6)
    # the five calls as one pipeline on one buffer set after another
    a, m = clock.batched([lambda g=g: [f(g) for f in fns.values()] for g in sets])
    table["pipeline_5_calls"] = {"avg_us": round(a, 2), "min_us": round(m, 2),
                                 "query_tokens_per_s": round((sum(wl.q_lens) + B) / a * 1e6)}
    table["note"] = ("batch 8 x 4096 context tokens, 10x, 512-row query block after 128 local tokens, one layer; 4 rotating "
                     "buffer sets; avg_us = the kernel launched back to back on the sets, in_pipeline_us = between events "
                     "inside the five-call path (the matrix-core kernel is power-limited when it runs back to back, the "
                     "short kernels carry the launch gap when timed inside the path)")
    nxt = None if args.no_next_rows else next_rows_c2(torch, D, W, clock, dev, wl, sets[0], cu_k, ks, ws, cu_qd, cu_ld, dec_local)
    del sets
    torch.cuda.empty_cache()
    return table, nxt


def next_rows_c2(torch, D, W, clock, dev, wl, g, cu_k, ks, ws, cu_qd, cu_ld, dec_local):
    """Kernels beyond the four-call path, at workload 2's shapes (one buffer set: not HBM figures)."""
    B = wl.B
    Kt, max_n, max_k = sum(ks), max(wl.seq_lens), max(ks)
    max_q, max_m = max(wl.q_lens), max(wl.local_lens)
    scale = wl.d_h ** -0.5
    out = {}

    def t(fn, rounds=5, inner=2):
        a, m = clock.batched([fn], rounds=rounds, inner=inner)
        return {"avg_us": round(a, 2), "min_us": round(m, 2)}
    # threshold rule of the autoregressive mode (Sec. 2.4)
    cap = max_k + 64
    lam = D.dodo_threshold_from_sample(g["scores"], wl.keep_num, wl.keep_den)
    thr_ws = torch.empty(max(D.dodo_threshold_from_sample_workspace_bytes(wl.N), 16), dtype=torch.uint8, device=dev)
    Kc = torch.zeros((B, cap, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev)
    Vc = torch.zeros_like(Kc)
    Kc[:, :max_k] = g["Kn"].view(B, -1, wl.H_kv, wl.d_h)
    Vc[:, :max_k] = g["Vn"].view(B, -1, wl.H_kv, wl.d_h)
    counts = torch.full((B,), max_k, dtype=torch.int32, device=dev)
    starts = (torch.arange(B, dtype=torch.int32, device=dev) * cap).contiguous()
    leave_s, leave_K, leave_V = g["scores"][:B].clone(), g["K"][:B].contiguous(), g["V"][:B].contiguous()
    ws_c = torch.zeros(max(D.dodo_nugget_attention_workspace_bytes(B, wl.H, wl.d_h, 1, cap, max(dec_local), D.BF16), 16),
                       dtype=torch.uint8, device=dev)
    ar = {
        "threshold_from_sample": t(lambda: D.dodo_threshold_from_sample(g["scores"], wl.keep_num, wl.keep_den, out=lam, ws=thr_ws)),
        "select_threshold": t(lambda: D.dodo_select_threshold(g["scores"], g["cu_seqlens"], lam)),
        "stream_append": t(lambda: (counts.fill_(max_k), D.dodo_stream_append(leave_s, lam, leave_K, leave_V, counts, Kc, Vc))),
        "attn_decode_cached": t(lambda: D.dodo_nugget_attention_cached(
            g["Qd"], Kc.view(B * cap, wl.H_kv, wl.d_h), Vc.view(B * cap, wl.H_kv, wl.d_h), g["Kld"], g["Vld"], cu_qd, starts,
            counts, cu_ld, 1, cap, max(dec_local), scale, D.TOKEN_MAJOR, g["Od"], ws=ws_c)),
        "note": f"sample = the step's {wl.N} scores; stream_append includes a fill of the {B} counters; caches of {cap} rows",
    }
    out["autoregressive_mode"] = ar
    # pooling baseline's compaction (Sec. 5.1)
    Kp, Vp = torch.empty_like(g["Kn"]), torch.empty_like(g["Vn"])
    r = t(lambda: D.dodo_meanpool_nuggets(g["K"], g["V"], g["cu_seqlens"], cu_k, Kt, D.TOKEN_MAJOR, Kp, Vp))
    r["GBps"] = round(2 * (wl.N + Kt) * wl.H_kv * wl.d_h * E / r["avg_us"] * 1e-3, 1)
    out["meanpool_baseline"] = r
    # gather-free attention
    out["gather_free"] = {
        "attn_block_indexed": t(lambda: D.dodo_nugget_attention_indexed(
            g["Q"], g["K"], g["V"], g["idx"], g["cu_seqlens"], g["Kl"], g["Vl"], g["cu_q"], cu_k, g["cu_local"], max_q, max_k,
            max_m, max_n, scale, O=g["O"])),
        "attn_decode_indexed": t(lambda: D.dodo_nugget_attention_indexed(
            g["Qd"], g["K"], g["V"], g["idx"], g["cu_seqlens"], g["Kld"], g["Vld"], cu_qd, cu_k, cu_ld, 1, max_k,
            max(dec_local), max_n, scale, O=g["Od"], ws=ws)),
        "note": "same results, bit for bit, as gather + attention"}
    # score gradient of the straight-through estimator (Eq. 17-18)
    lse_b = torch.empty((g["Q"].shape[0], wl.H), dtype=torch.float32, device=dev)
    D.dodo_nugget_attention(g["Q"], g["Kn"], g["Vn"], g["Kl"], g["Vl"], g["cu_q"], cu_k, g["cu_local"], max_q, max_k, max_m,
                            scale, D.TOKEN_MAJOR, g["O"], lse=lse_b)
    dO = W.normal(wl.seed, 99, tuple(g["Q"].shape), 1.0, wl.dtype, dev)
    ste_ws = torch.empty(D.dodo_ste_score_grad_workspace_bytes(g["Q"].shape[0], wl.H, Kt), dtype=torch.uint8, device=dev)
    ste_grad = torch.empty(Kt, dtype=torch.float32, device=dev)
    r = t(lambda: D.dodo_ste_score_grad(g["Q"], g["Kn"], g["Vn"], dO, g["O"], lse_b, g["cu_q"], cu_k, max_q, max_k, scale,
                                        scale, D.TOKEN_MAJOR, grad=ste_grad, ws=ste_ws))
    ste_flop = 4.0 * sum(q * k for q, k in zip(wl.q_lens, ks)) * wl.d_h * wl.H
    r.update(TFLOPs=round(ste_flop / r["avg_us"] * 1e-6, 1),
             frac_of_bf16_peak=round(ste_flop / r["avg_us"] * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 3),
             note="whole call: row dots, the MFMA kernel, the sum over heads")
    out["ste_score_grad"] = r
    # 2-layer scorer (App. B), d -> d -> 1
    d = wl.d_model
    gen = torch.Generator(device="cpu").manual_seed(wl.seed + 77)
    W1 = (torch.randn(d, d, generator=gen) * d ** -0.5).to(torch.bfloat16).to(dev)
    b1 = (torch.randn(d, generator=gen) * 0.5).to(dev)
    w2 = (torch.randn(d, generator=gen) * d ** -0.5).to(torch.bfloat16).to(dev)
    mlp_ws = torch.empty(max(D.dodo_score_mlp_workspace_bytes(D.BF16, wl.N, d, d), 16), dtype=torch.uint8, device=dev)
    mlp_out = torch.empty(wl.N, dtype=torch.float32, device=dev)
    r = t(lambda: D.dodo_score_mlp(g["hidden"], W1, b1, w2, 0.0, D.RELU, mlp_out, mlp_ws), rounds=4, inner=2)
    mlp_flop = 2.0 * wl.N * d * d
    r.update(TFLOPs=round(mlp_flop / r["avg_us"] * 1e-6, 1),
             frac_of_bf16_peak=round(mlp_flop / r["avg_us"] * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 3), note="ReLU, d_hid = d")
    out["scorer_2layer"] = r
    # segment form of the autoregressive objective: the 8 x 4096 tokens as 64 segments of 512 with tau = 128
    seg_len, tau = 512, 128
    mk = lambda tid, n, h: W.normal(wl.seed, tid, (n, h, wl.d_h), 1.0, wl.dtype, dev)
    Qs = mk(300, wl.N, wl.H)
    Os = torch.empty_like(Qs)
    n_seg = sum(-(-n // seg_len) for n in wl.seq_lens)
    plan = D.dodo_segment_plan(g["idx"], g["cu_seqlens"], cu_k, seg_len, tau, n_seg)
    r = t(lambda: D.dodo_nugget_attention_segments(Qs, g["Kn"], g["Vn"], g["K"], g["V"], plan[0], plan[1], plan[2], plan[3],
                                                   plan[4], seg_len, max_k, seg_len + tau, scale, D.TOKEN_MAJOR, Os),
          rounds=4, inner=2)
    cu_q_h, nl_h, ll_h = plan[0].cpu().tolist(), plan[2].cpu().tolist(), plan[4].cpu().tolist()
    pairs = 0
    for e in range(n_seg):
        q = cu_q_h[e + 1] - cu_q_h[e]
        pairs += q * nl_h[e] + sum(min(ll_h[e], ll_h[e] - q + i + 1) for i in range(q))
    flop = 4.0 * pairs * wl.d_h * wl.H
    r.update(entries=n_seg, TFLOPs=round(flop / r["avg_us"] * 1e-6, 1),
             frac_of_bf16_peak=round(flop / r["avg_us"] * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
             plan=t(lambda: D.dodo_segment_plan(g["idx"], g["cu_seqlens"], cu_k, seg_len, tau, n_seg)))
    out["segment_form_8x4096_seg512_tau128"] = r
    # grouped-query decode (8 query heads per KV head): one workgroup per (sequence, KV head) reads every row once
    # for the 8 heads and multiplies on the matrix cores
    Bg, Hg, Hkvg, kg, mg = 64, 64, 8, 410, 257
    gsets = []
    for s_ in range(4):
        mk = lambda tid, n, h: W.normal(wl.seed, 3000 + 8 * s_ + tid, (n, h, wl.d_h), 1.0, wl.dtype, dev)
        gsets.append(dict(Q=mk(0, Bg, Hg), Kn=mk(1, Bg * kg, Hkvg), Vn=mk(2, Bg * kg, Hkvg), Kl=mk(3, Bg * mg, Hkvg),
                          Vl=mk(4, Bg * mg, Hkvg)))
    cuq, cuk, cul = W.cumulative([1] * Bg, dev), W.cumulative([kg] * Bg, dev), W.cumulative([mg] * Bg, dev)
    Og = torch.empty_like(gsets[0]["Q"])
    a, m_ = clock.batched([lambda t_=t_: D.dodo_nugget_attention(t_["Q"], t_["Kn"], t_["Vn"], t_["Kl"], t_["Vl"], cuq, cuk, cul, 1,
                                                                  kg, mg, scale, D.TOKEN_MAJOR, Og) for t_ in gsets])
    wg = work_attention([1] * Bg, [kg] * Bg, [mg] * Bg, Hg, Hkvg, wl.d_h)
    r = hbm_row(a, wg)
    r.update(min_us=round(m_, 2), note=f"batch {Bg}, {Hg} query heads over {Hkvg} KV heads, {kg} nuggets + {mg} local rows; "
                                       "algorithmic bytes count every K/V row once")
    out["gqa_decode_64_heads_8_kv_heads"] = r

    def shared_rows(Bs, Hs, Hkvs, qs, ks_, ms_, tid0):
        """Several query vectors per K/V row at another shape: 4 rotating sets, the workspace the grouped kernel asks for."""
        sets = []
        for s_ in range(4):
            mk = lambda tid, n, h: W.normal(wl.seed, tid0 + 8 * s_ + tid, (n, h, wl.d_h), 1.0, wl.dtype, dev)
            sets.append(dict(Q=mk(0, Bs * qs, Hs), Kn=mk(1, Bs * ks_, Hkvs), Vn=mk(2, Bs * ks_, Hkvs), Kl=mk(3, Bs * ms_, Hkvs),
                             Vl=mk(4, Bs * ms_, Hkvs)))
        cq, ck, cl = W.cumulative([qs] * Bs, dev), W.cumulative([ks_] * Bs, dev), W.cumulative([ms_] * Bs, dev)
        Os = torch.empty_like(sets[0]["Q"])
        need = D.dodo_nugget_attention_workspace_bytes_grouped(Bs, Hs, Hkvs, wl.d_h, qs, ks_, ms_, D.BF16)
        wsb = torch.zeros(max(need, 16), dtype=torch.uint8, device=dev)
        a_, m2 = clock.batched([lambda t_=t_: D.dodo_nugget_attention(t_["Q"], t_["Kn"], t_["Vn"], t_["Kl"], t_["Vl"], cq, ck, cl,
                                                                      qs, ks_, ms_, scale, D.TOKEN_MAJOR, Os, ws=wsb)
                                for t_ in sets])
        row = hbm_row(a_, work_attention([qs] * Bs, [ks_] * Bs, [ms_] * Bs, Hs, Hkvs, wl.d_h))
        row.update(min_us=round(m2, 2))
        return row
    r = shared_rows(2, 64, 8, 1, 3277, 1089, 3200)
    r["note"] = "batch 2, 64 query heads over 8 KV heads, 3277 nuggets + 1089 local rows: the keys of a (sequence, KV head) pair are split over 16 workgroups; latency-bound (36 MB)"
    out["gqa_decode_long_context_batch_2"] = r
    r = shared_rows(64, 32, 32, 4, kg, mg, 3300)
    r["note"] = "batch 64, multi-head attention, query blocks of 4 rows (each row of a head reads the same K/V rows)"
    out["query_block_of_4_rows"] = r
    # query-block attention with 64-wide heads (64 heads x 64: the same flop count as the 32 x 128 workload)
    mk = lambda tid, n, h: W.normal(wl.seed, 3100 + tid, (n, h, 64), 1.0, wl.dtype, dev)
    Q6, Kn6, Vn6 = mk(0, sum(wl.q_lens), 64), mk(1, Kt, 64), mk(2, Kt, 64)
    Kl6, Vl6 = mk(3, sum(wl.local_lens), 64), mk(4, sum(wl.local_lens), 64)
    O6 = torch.empty_like(Q6)
    r = t(lambda: D.dodo_nugget_attention(Q6, Kn6, Vn6, Kl6, Vl6, g["cu_q"], cu_k, g["cu_local"], max_q, max_k, max_m, 0.125,
                                          D.TOKEN_MAJOR, O6))
    w6 = work_attention(wl.q_lens, ks, wl.local_lens, 64, 64, 64)
    r.update(TFLOPs=round(w6["flop"] / r["avg_us"] * 1e-6, 1),
             frac_of_bf16_peak=round(w6["flop"] / r["avg_us"] * 1e-6 / MFMA_BF16_PEAK_TFLOPS, 4),
             note="workload 2's shape with 64 heads of 64 channels: half the matrix work per key and query row, the same "
                  "softmax work, so the vector pipe bounds it")
    out["attn_block_64_wide_heads"] = r
    return out


# ------------------------------------------------------------------------------------------------ workload 3
def run_c3(torch, D, W, clock, dev, args):
    wl = W.config(3)
    B, L = wl.B, wl.layers
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt, Sm = sum(ks), sum(wl.local_lens)
    dec_local = wl.local_lens  # 256 uncompressed tokens + the new token itself
    cu_q, cu_l = W.cumulative([1] * B, dev), W.cumulative(dec_local, dev)
    mk = lambda tid, n, h: W.normal(wl.seed, tid, (n, h, wl.d_h), 1.0, wl.dtype, dev)
    layers = [dict(Kn=mk(100 + 8 * l, Kt, wl.H_kv), Vn=mk(101 + 8 * l, Kt, wl.H_kv), Kl=mk(102 + 8 * l, Sm, wl.H_kv),
                   Vl=mk(103 + 8 * l, Sm, wl.H_kv), Q=mk(104 + 8 * l, B, wl.H)) for l in range(L)]
    O = torch.empty_like(layers[0]["Q"])
    max_m, max_k = max(dec_local), max(ks)
    scale = wl.d_h ** -0.5

    def step():
        for t in layers:
            D.dodo_nugget_attention(t["Q"], t["Kn"], t["Vn"], t["Kl"], t["Vl"], cu_q, cu_k, cu_l, 1, max_k, max_m, scale,
                                    D.TOKEN_MAJOR, O)
    a, m = clock.batched([step], rounds=6, inner=1)
    w1 = work_attention([1] * B, ks, dec_local, wl.H, wl.H_kv, wl.d_h)
    table = {"attn_decode": hbm_row(a / L, w1)}
    table["attn_decode"]["min_us"] = round(m / L, 2)
    table["decode_step_32_layers"] = {"launches": L, "avg_us": round(a, 1), "min_us": round(m, 1),
                                      "query_tokens_per_s": round(B / a * 1e6), "bytes_per_step": w1["bytes"] * L,
                                      "GBps": round(w1["bytes"] * L / a * 1e-3, 1),
                                      "frac_of_hbm_peak": round(w1["bytes"] * L / a * 1e-3 / HBM_PEAK_GBS, 4)}
    del layers
    torch.cuda.empty_cache()
    # the ragged compress phase of one layer (set-up of the decode): 3.2 GB of hidden states, 6.4 GB of K/V
    g = W.make_inputs(wl, dev, layer=0, which=["hidden", "w", "K", "V"])
    scores = torch.empty(wl.N, dtype=torch.float32, device=dev)
    idx = torch.empty(Kt, dtype=torch.int32, device=dev)
    Kn = torch.empty((Kt, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev)
    Vn = torch.empty_like(Kn)
    cu_s = g["cu_seqlens"]
    a, _ = clock.batched([lambda: D.dodo_score(g["hidden"], g["w"], 0.0, scores)], rounds=4, inner=2)
    table["score"] = hbm_row(a, work_score(wl.N, wl.d_model))
    a, _ = clock.batched([lambda: D.dodo_select_topk(scores, cu_s, cu_k, max(wl.seq_lens), max_k, Kt, D.FORCE_LAST, idx)],
                         rounds=4, inner=2)
    table["select"] = {"avg_us": round(a, 2), "bound": "latency", "bytes": work_select(wl.N, Kt, B)["bytes"]}
    a, _ = clock.batched([lambda: D.dodo_gather_nuggets(g["K"], g["V"], idx, cu_s, cu_k, Kt, D.TOKEN_MAJOR, Kn, Vn)],
                         rounds=4, inner=2)
    table["gather"] = hbm_row(a, work_gather(Kt, wl.H_kv * wl.d_h))
    table["note"] = ("batch 64, ragged contexts in [4096, 8192] at 20x, 256 local tokens + the token itself; decode = one "
                     "token step over 32 layers on 32 distinct caches (no reuse); compress = one layer's context (its "
                     "inputs alone exceed the last-level cache)")
    del g, Kn, Vn
    torch.cuda.empty_cache()
    return table


# ------------------------------------------------------------------------------------------------ workload 5
def run_c5(torch, D, W, clock, dev, args):
    wl = W.config(5)
    B, S = wl.B, 4
    cu_k, ks = D.cu_nuggets_from_lengths(wl.seq_lens, wl.keep_num, wl.keep_den, dev)
    Kt, max_n, max_k = sum(ks), max(wl.seq_lens), max(ks)
    max_q, max_m = max(wl.q_lens), max(wl.local_lens)
    scale = wl.d_h ** -0.5
    m_dec = max_m + 32 + 1  # decode step 32 of 64: 1024 prefill rows + 32 earlier tokens + the token itself
    cu_qd, cu_ld = W.cumulative([1] * B, dev), W.cumulative([m_dec] * B, dev)
    sets = []
    for s in range(S):
        g = W.make_inputs(wl, dev, layer=s)
        g["Qd"] = W.normal(wl.seed, 1000 + 16 * s, (B, wl.H, wl.d_h), 1.0, wl.dtype, dev)
        g["Kld"] = W.normal(wl.seed, 1001 + 16 * s, (B * m_dec, wl.H_kv, wl.d_h), 1.0, wl.dtype, dev)
        g["Vld"] = W.normal(wl.seed, 1002 + 16 * s, (B * m_dec, wl.H_kv, wl.d_h), 1.0, wl.dtype, dev)
        g["scores"] = torch.empty(wl.N, dtype=torch.float32, device=dev)
        g["qscores"] = torch.empty(wl.N, dtype=torch.float32, device=dev)
        g["idx"] = torch.empty(Kt, dtype=torch.int32, device=dev)
        g["Kn"] = torch.empty((Kt, wl.H_kv, wl.d_h), dtype=wl.dtype, device=dev)
        g["Vn"] = torch.empty_like(g["Kn"])
        g["O"], g["Od"] = torch.empty_like(g["Q"]), torch.empty_like(g["Qd"])
        sets.append(g)
    cu_s, cu_q, cu_l = sets[0]["cu_seqlens"], sets[0]["cu_q"], sets[0]["cu_local"]
    ws_bytes = D.dodo_nugget_attention_workspace_bytes(B, wl.H, wl.d_h, 1, max_k, m_dec + 64, D.BF16)
    ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    sel_ws = torch.zeros(max(D.dodo_select_topk_workspace_bytes(B, max_n), 16), dtype=torch.uint8, device=dev)
    for g in sets:
        D.dodo_score(g["hidden"], g["w"], 0.0, g["scores"])
        g["qscores"].copy_(W.quantise16(g["scores"]))  # the workload's 16-level tie stress (input preparation)
    fns = {
        "score": lambda g: D.dodo_score(g["hidden"], g["w"], 0.0, g["scores"]),
        "select": lambda g: D.dodo_select_topk(g["qscores"], cu_s, cu_k, max_n, max_k, Kt, D.FORCE_LAST, g["idx"], ws=sel_ws),
        "gather": lambda g: D.dodo_gather_nuggets(g["K"], g["V"], g["idx"], cu_s, cu_k, Kt, D.TOKEN_MAJOR, g["Kn"], g["Vn"]),
        "attn_block": lambda g: D.dodo_nugget_attention(g["Q"], g["Kn"], g["Vn"], g["Kl"], g["Vl"], cu_q, cu_k, cu_l, max_q,
                                                        max_k, max_m, scale, D.TOKEN_MAJOR, g["O"]),
        "attn_decode": lambda g: D.dodo_nugget_attention(g["Qd"], g["Kn"], g["Vn"], g["Kld"], g["Vld"], cu_qd, cu_k, cu_ld, 1,
                                                         max_k, m_dec, scale, D.TOKEN_MAJOR, g["Od"], ws=ws),
    }
    for g in sets:
        for n in fns:
            fns[n](g)
    work = {"score": work_score(wl.N, wl.d_model), "select": work_select(wl.N, Kt, B),
            "gather": work_gather(Kt, wl.H_kv * wl.d_h),
            "attn_block": work_attention(wl.q_lens, ks, wl.local_lens, wl.H, wl.H_kv, wl.d_h),
            "attn_decode": work_attention([1] * B, ks, [m_dec] * B, wl.H, wl.H_kv, wl.d_h)}
    table = {}
    for n, f in fns.items():
        a, m = clock.batched([lambda g=g, f=f: f(g) for g in sets])
        table[n] = mfma_row(a, work[n]) if n == "attn_block" else hbm_row(a, work[n])
        table[n]["min_us"] = round(m, 2)
    table["select"].pop("frac_of_hbm_peak")
    table["select"]["bound"] = "latency"
    add_pipeline_times(table, clock.pipeline(sets, fns), work)
    assert int(sel_ws.view(torch.int32)[0]) == 0, "dodo_select_topk reported a failed wait"
    tg = table["select"]["avg_us"] + table["gather"]["avg_us"]
    table["topk_plus_gather_GBps"] = round((work["select"]["bytes"] + work["gather"]["bytes"]) / tg * 1e-3, 1)
    table["attn_block"]["query_tokens_per_s"] = round(sum(wl.q_lens) / table["attn_block"]["in_pipeline_us"] * 1e6)
    table["attn_decode"]["note"] = "decode step 32 of 64 on 4 rotating caches: every launch reads its cache from HBM"
    # the 64 decode steps of one generation: the local buffer grows by a row per step, the same cache every step
    g = sets[0]
    steps = 64
    Kl_all = W.normal(wl.seed, 2000, (B * (max_m + steps), wl.H_kv, wl.d_h), 1.0, wl.dtype, dev)
    Vl_all = W.normal(wl.seed, 2001, (B * (max_m + steps), wl.H_kv, wl.d_h), 1.0, wl.dtype, dev)
    wins = []
    for t in range(steps):
        m = max_m + t + 1
        rows = torch.cat([torch.arange(b * (max_m + steps), b * (max_m + steps) + m, device=dev) for b in range(B)])
        wins.append((Kl_all[rows].contiguous(), Vl_all[rows].contiguous(), W.cumulative([m] * B, dev), m))

    def decode64():
        for kl, vl, cu, m in wins:
            D.dodo_nugget_attention(g["Qd"], g["Kn"], g["Vn"], kl, vl, cu_qd, cu_k, cu, 1, max_k, max_m + steps, scale,
                                    D.TOKEN_MAJOR, g["Od"], ws=ws)
    a, m = clock.batched([decode64], rounds=5, inner=1)
    by = sum(work_attention([1] * B, ks, [w[3]] * B, wl.H, wl.H_kv, wl.d_h)["bytes"] for w in wins)
    table["decode_64_steps"] = {"launches": steps, "avg_us": round(a, 1), "us_per_step": round(a / steps, 2),
                                "query_tokens_per_s": round(B * steps / a * 1e6), "GBps": round(by / a * 1e-3, 1),
                                "cache_resident": True,
                                "note": "the same 107 MB nugget cache is re-read every step and stays in the 256 MB "
                                        "last-level cache: not an HBM figure"}
    table["note"] = ("batch 2 x 32768 context tokens, 10x (3277 nuggets), scores quantised to 16 levels; 1024-row query "
                     "block; 4 rotating buffer sets; avg_us / in_pipeline_us as for workload 2")
    del sets, wins, Kl_all, Vl_all
    torch.cuda.empty_cache()
    return table


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2310_02409_amd as D
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    clock = Clock(torch)
    want = [w.strip() for w in args.workloads.split(",") if w.strip()]
    kernels = {}
    head, kernels["c4_llama13b_autoencode"], cpu = run_c4(torch, D, W, clock, dev, args)
    nxt = None
    if "c2" in want:
        kernels["c2_llama7b_prefill"], nxt = run_c2(torch, D, W, clock, dev, args)
    if "c3" in want:
        kernels["c3_llama7b_decode"] = run_c3(torch, D, W, clock, dev, args)
    if "c5" in want:
        kernels["c5_long_context"] = run_c5(torch, D, W, clock, dev, args)
    ceilings = measure_ceilings(torch, D, clock, dev)

    # the targets named for this path, from the tables above: bandwidth-bound kernels back to back over rotating
    # buffers (no launch gap in the figure), the matrix-core kernel as it runs inside the path
    targets = {}
    for wname, t in kernels.items():
        for k in ("gather", "attn_decode"):
            if k in t and isinstance(t[k], dict):
                f = t[k].get("frac_of_hbm_peak_back_to_back", t[k].get("frac_of_hbm_peak"))
                if f is not None:
                    targets[f"{wname}.{k}"] = {"frac_of_hbm_peak": f, "target": 0.60, "met": f >= 0.60}
        if "attn_block" in t:
            a = t["attn_block"]
            f = a.get("frac_of_bf16_peak_in_pipeline", a["frac_of_bf16_peak"]) if wname != "c4_llama13b_autoencode" \
                else a["frac_of_bf16_peak"]
            targets[f"{wname}.attn_block"] = {"frac_of_bf16_peak": f, "target": 0.40, "met": f >= 0.40}
    targets["note"] = ("from this run's event timings: an interval between events holds the kernel and the gap to the "
                       "next launch (about 1 us), so the 13-30 us kernels read 3-7% lower here than in a kernel trace "
                       "of the same command (profiles/bench_default_kernel_trace.md)")
    line = {
        "metric": "nugget-attention query tokens/s (whole hot-path step: 40 layers of score+TopK+gather+query-block attention)",
        "value": round(head["value"], 1), "unit": "query tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic", "config": head["config"], "roofline": head["roofline"], "cpu_baseline": cpu,
        "kernels": kernels, "ceilings": ceilings, "targets": targets, "next_rows": nxt,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
